"""Host code under AddressSanitizer + UndefinedBehaviorSanitizer, no GPU needed:
  * the CPU oracle (gcc -fsanitize=address,undefined) against all of its pins;
  * the library's host side - argument validation, workspace layout, job footprints - (hipcc with the sanitizers on
    the host pass only) against the host-only ABI tests.
Each runs the existing test files in a child interpreter with the sanitizer runtime preloaded and the sanitized
library selected through the environment; any report makes the child fail."""
import os
import subprocess
import sys
from pathlib import Path

ROOT = Path(__file__).resolve().parent.parent


def _run(files, env_extra, runtime):
    env = dict(os.environ)
    env.update(env_extra)
    old = env.get("LD_PRELOAD", "")
    env["LD_PRELOAD"] = str(runtime) + ((":" + old) if old else "")      # the sanitizer runtime has to come first
    # the interpreter itself is not instrumented: its own allocations are not this test's business
    env["ASAN_OPTIONS"] = "detect_leaks=0:abort_on_error=1:halt_on_error=1"
    env["UBSAN_OPTIONS"] = "halt_on_error=1:print_stacktrace=1"
    cmd = [sys.executable, "-m", "pytest", "-x", "-q", "-p", "no:cacheprovider", *files]
    p = subprocess.run(cmd, cwd=ROOT, env=env, capture_output=True, text=True, timeout=900)
    tail = (p.stdout + p.stderr)[-3000:]
    assert p.returncode == 0, tail
    assert "ERROR: AddressSanitizer" not in tail and "runtime error:" not in tail, tail
    return tail


def test_oracle_pins_under_address_and_undefined_behaviour_sanitizers():
    import oracle
    lib = oracle.build_sanitized()
    runtime = subprocess.run(["gcc", "-print-file-name=libasan.so"], capture_output=True, text=True).stdout.strip()
    assert os.path.isabs(runtime) and os.path.exists(runtime), runtime
    files = sorted(str(p.relative_to(ROOT)) for p in (ROOT / "tests").glob("test_oracle_*.py")
                   if p.name != "test_oracle_mutations.py")      # the mutants build and load their own libraries
    tail = _run(files, {"LOOKM_ORACLE_LIB": str(lib)}, runtime)
    assert " passed" in tail


def test_library_host_code_under_address_and_undefined_behaviour_sanitizers():
    from paper_2406_18139_amd import build
    lib = build.build_host_sanitized()
    tail = _run(["tests/test_abi_host.py"], {"LOOKM_LIB": str(lib)}, build.asan_runtime())
    assert " passed" in tail
