"""Host-side checks that need no GPU: the library loads, exports every symbol the header declares,
and rejects bad arguments before launching anything."""
import ctypes
import re
from pathlib import Path

import numpy as np
import pytest

from paper_2406_18139_amd import lookm

ROOT = Path(__file__).resolve().parent.parent


def declared_symbols():
    text = (ROOT / "include" / "lookm.h").read_text()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(lookm_[a-z_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = lookm.lib()
    names = declared_symbols()
    assert set(names) == set(lookm.EXPORTS)
    for n in names:
        assert hasattr(L, n), n


def test_version_and_status_strings():
    assert "lookm" in lookm.version()
    for code in range(-6, 1):
        assert lookm.status_string(code) not in ("", "unknown status")
    assert lookm.status_string(-99) == "unknown status"


def test_protected_count_matches_definition():
    rng = np.random.default_rng(0)
    for _ in range(20):
        L = int(rng.integers(1, 200))
        M = int(rng.integers(0, L + 1))
        mask = rng.integers(0, 2, L).astype(np.uint8)
        ref = sum(1 for j in range(L) if mask[j] == 0 or j >= L - M)
        assert lookm.protected_count(mask, M) == ref
    with pytest.raises(lookm.LookmError):
        lookm.protected_count(np.ones(4, np.uint8), 5)


def test_workspace_bytes():
    assert lookm.workspace_bytes(32, 12644, 128, 2276, lookm.BF16) > 4 * 32 * 12644
    assert lookm.workspace_bytes(32, 12644, 128, 2276, lookm.BF16) % 256 == 0
    assert lookm.workspace_bytes(0, 10, 128, 5, lookm.BF16) == 0
    assert lookm.workspace_bytes(1, 10, 100, 5, lookm.BF16) == 0      # head_dim not a multiple of 8
    assert lookm.workspace_bytes(1, 10, 128, 11, lookm.BF16) == 0     # budget > L
    assert lookm.workspace_bytes(1, 40000, 128, 5, lookm.BF16) == 0   # beyond LOOKM_MAX_L


FAKE = 0x10000   # non-null, 256-byte aligned, never dereferenced: every call below fails validation first


def compress(q=FAKE, k=FAKE, v=FAKE, mask=FAKE, H=2, L=64, d=64, dt=0, B=32, M=8, mode=1, ko=FAKE, vo=FAKE,
             kept=FAKE, scores=None, status=FAKE, ws=FAKE, wsn=1 << 30, stream=None):
    return lookm.lib().lookm_compress(q, k, v, mask, H, L, d, dt, B, M, mode, ko, vo, kept, scores, status, ws, wsn, stream)


def test_compress_rejects_bad_arguments_without_touching_the_gpu():
    assert compress(q=None) == lookm.ERR_INVALID_ARG
    assert compress(status=None) == lookm.ERR_INVALID_ARG
    assert compress(H=0) == lookm.ERR_INVALID_ARG
    assert compress(dt=7) == lookm.ERR_INVALID_ARG
    assert compress(mode=9) == lookm.ERR_INVALID_ARG
    assert compress(k=FAKE + 4) == lookm.ERR_INVALID_ARG               # misaligned
    assert compress(d=100) == lookm.ERR_UNSUPPORTED
    assert compress(d=512) == lookm.ERR_UNSUPPORTED
    assert compress(L=100000) == lookm.ERR_UNSUPPORTED
    assert compress(B=65) == lookm.ERR_BUDGET_RANGE
    assert compress(B=4, M=8) == lookm.ERR_BUDGET_RANGE
    assert compress(M=65, B=64) == lookm.ERR_BUDGET_RANGE
    assert compress(M=-1) == lookm.ERR_INVALID_ARG
    assert compress(ws=None) == lookm.ERR_WORKSPACE
    assert compress(ws=FAKE + 16) == lookm.ERR_WORKSPACE
    assert compress(wsn=100) == lookm.ERR_WORKSPACE


def test_stage_calls_reject_bad_arguments():
    L = lookm.lib()
    assert L.lookm_scores(None, FAKE, 1, 8, 8, 0, FAKE, FAKE, 1 << 20, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_scores(FAKE, FAKE, 1, 8, 12, 0, FAKE, FAKE, 1 << 20, None) == lookm.ERR_UNSUPPORTED
    assert L.lookm_scores(FAKE, FAKE, 1, 8, 8, 0, FAKE, FAKE, 8, None) == lookm.ERR_WORKSPACE
    assert L.lookm_scores_lse(FAKE, FAKE, None, 1, 8, 8, 0, FAKE, FAKE, 1 << 20, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_scores_grouped(FAKE, FAKE, 6, 4, 8, 8, 0, FAKE, FAKE, 1 << 20, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_scores_window(FAKE, FAKE, 1, 8, 8, 0, 0, FAKE, FAKE, 1 << 20, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_scores_window(FAKE, FAKE, 1, 8, 8, 0, 9, FAKE, FAKE, 1 << 20, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_compress_lse(FAKE, FAKE, FAKE, FAKE, None, 2, 64, 64, 0, 32, 8, 1, FAKE, FAKE, FAKE, None, FAKE, FAKE,
                                1 << 30, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_select(FAKE, FAKE, 1, 8, 9, 0, FAKE, FAKE, FAKE, None) == lookm.ERR_BUDGET_RANGE
    assert L.lookm_select(FAKE, None, 1, 8, 4, 0, FAKE, FAKE, FAKE, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_nearest(FAKE, FAKE, FAKE, 1, 8, 8, 0, 0, FAKE, FAKE, FAKE, 1 << 20, None) == lookm.ERR_BUDGET_RANGE
    assert L.lookm_nearest(FAKE, FAKE, FAKE, 1, 8, 8, 0, 4, FAKE, FAKE, None, 0, None) == lookm.ERR_WORKSPACE
    assert L.lookm_merge(FAKE, FAKE, FAKE, FAKE, FAKE, FAKE, 1, 8, 8, 0, 4, 5, FAKE, FAKE, FAKE, 1 << 20, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_merge(FAKE, FAKE, FAKE, None, FAKE, FAKE, 1, 8, 8, 0, 4, 1, FAKE, FAKE, FAKE, 1 << 20, None) == lookm.ERR_INVALID_ARG


def fake_job(**kw):
    f = dict(q=FAKE, k=FAKE, v=FAKE, modality_mask=FAKE, row_lse=None, H=2, L=64, d=64, dt=0, budget=32, recent_window=8,
             merge_mode=1, rule=0, score_window=0, kv_heads=0, k_out=FAKE, v_out=FAKE, kept_idx=FAKE, scores_out=None, status_out=FAKE,
             workspace=FAKE, workspace_bytes=1 << 30)
    f.update(kw)
    return lookm.Job(**f)


def test_batch_validates_every_job_before_any_launch():
    import ctypes
    L = lookm.lib()
    bad = ctypes.c_int(-1)

    def run(jobs):
        arr = (lookm.Job * len(jobs))(*jobs)
        return L.lookm_compress_batch(arr, len(jobs), ctypes.byref(bad), None)

    assert L.lookm_compress_batch(None, 0, None, None) == lookm.OK              # nothing to do
    assert L.lookm_compress_batch(None, 2, None, None) == lookm.ERR_INVALID_ARG
    # every job below is invalid, so nothing is ever enqueued; the LAST job decides code and index
    assert run([fake_job(q=None)]) == lookm.ERR_INVALID_ARG and bad.value == 0
    assert run([fake_job(rule=5)]) == lookm.ERR_INVALID_ARG
    assert run([fake_job(budget=99)]) == lookm.ERR_BUDGET_RANGE
    assert run([fake_job(score_window=65)]) == lookm.ERR_INVALID_ARG
    assert run([fake_job(H=6, kv_heads=4)]) == lookm.ERR_INVALID_ARG          # 4 key heads do not divide 6 query heads
    assert run([fake_job(row_lse=FAKE + 2)]) == lookm.ERR_INVALID_ARG
    # the struct's last field: a layout that disagreed with the header would report something else
    assert run([fake_job(workspace_bytes=64)]) == lookm.ERR_WORKSPACE and bad.value == 0
    assert run([fake_job(d=100), fake_job()]) == lookm.ERR_UNSUPPORTED and bad.value == 0


def test_two_stream_batch_and_workspace_offsets_validate_on_the_host():
    L = lookm.lib()
    bad = ctypes.c_int(-1)
    arr = (lookm.Job * 1)(fake_job(budget=99))
    # the second stream must differ from the first (NULL is the default stream on both sides here)
    assert L.lookm_compress_batch_two_streams(arr, 1, ctypes.byref(bad), None, None) == lookm.ERR_INVALID_ARG
    assert L.lookm_compress_batch_two_streams(arr, 1, ctypes.byref(bad), None, FAKE) == lookm.ERR_BUDGET_RANGE
    assert L.lookm_compress_batch_two_streams(None, 0, None, None, FAKE) == lookm.OK
    none = ctypes.c_size_t(-1).value
    offs = [L.lookm_workspace_offset(32, 32, 12644, 128, 2276, lookm.BF16, item) for item in (0, 1, 2)]
    assert all(o != none and o % 256 == 0 for o in offs) and len(set(offs)) == 3
    assert max(offs) + 4 * 32 * (12644 - 2276) <= lookm.workspace_bytes(32, 12644, 128, 2276, lookm.BF16)
    assert L.lookm_workspace_offset(32, 32, 12644, 128, 2276, lookm.BF16, 3) == none
    assert L.lookm_workspace_offset(32, 5, 12644, 128, 2276, lookm.BF16, 0) == none      # 5 does not divide 32
    assert L.lookm_workspace_offset(32, 32, 12644, 128, 20000, lookm.BF16, 0) == none


def test_budget_from_ratios_matches_the_oracle():
    import oracle
    for L in (1, 17, 256, 4096, 12644, 32768):
        for a1 in (0.0, 0.01, 0.1, 0.25):
            for a2 in (0.0, 0.04, 0.1, 0.5, 0.74):
                assert lookm.budget_from_ratios(L, a1, a2) == oracle.budget_from_ratios(L, a1, a2)
    with pytest.raises(lookm.LookmError) as e:
        lookm.budget_from_ratios(100, 0.6, 0.6)
    assert e.value.code == lookm.ERR_BUDGET_RANGE
    with pytest.raises(lookm.LookmError) as e:
        lookm.budget_from_ratios(100, -0.1, 0.6)
    assert e.value.code == lookm.ERR_INVALID_ARG
    L = lookm.lib()
    assert L.lookm_select_rule_(FAKE, FAKE, 1, 8, 4, 0, 3, FAKE, FAKE, FAKE, None) == lookm.ERR_INVALID_ARG


def test_decode_rejects_bad_arguments():
    L = lookm.lib()
    ok = L.lookm_decode_workspace_bytes(32, 128)
    assert ok > 0 and L.lookm_decode_workspace_bytes(32, 100) == 0 and L.lookm_decode_workspace_bytes(0, 128) == 0
    def call(**kw):
        a = dict(q=FAKE, k=FAKE, v=FAKE, H=2, rows=64, S=64, d=64, dt=0, out=FAKE, ws=FAKE, wsn=1 << 24, st=None)
        a.update(kw)
        return L.lookm_decode_attention(*[a[n] for n in ("q", "k", "v", "H", "rows", "S", "d", "dt", "out", "ws", "wsn", "st")])

    assert call(q=None) == lookm.ERR_INVALID_ARG
    assert call(S=0) == lookm.ERR_INVALID_ARG and call(S=65) == lookm.ERR_INVALID_ARG
    assert call(d=20) == lookm.ERR_UNSUPPORTED
    assert call(dt=3) == lookm.ERR_INVALID_ARG
    assert call(out=FAKE + 8) == lookm.ERR_INVALID_ARG
    assert call(wsn=16) == lookm.ERR_WORKSPACE and call(ws=None) == lookm.ERR_WORKSPACE


def test_noalloc_decode_rejects_bad_arguments_and_sizes_beyond_its_scratch():
    L = lookm.lib()
    def call(**kw):
        a = dict(q=FAKE, k=FAKE, v=FAKE, H=2, rows=64, S=64, d=64, dt=0, out=FAKE, st=None)
        a.update(kw)
        return L.lookm_decode_attention_noalloc(*[a[n] for n in ("q", "k", "v", "H", "rows", "S", "d", "dt", "out", "st")])

    assert call(out=None) == lookm.ERR_INVALID_ARG
    assert call(S=65) == lookm.ERR_INVALID_ARG and call(dt=2) == lookm.ERR_INVALID_ARG
    assert call(d=12) == lookm.ERR_UNSUPPORTED
    assert call(k=FAKE + 2) == lookm.ERR_INVALID_ARG
    # 64 heads x 256 pieces x (256 + 2) floats = 16.9 MB of partial results: more than the 8 MiB the library holds
    assert call(H=64, rows=100000, S=100000, d=256, dt=1) == lookm.ERR_WORKSPACE


def test_probe_rejects_bad_arguments():
    import ctypes
    L = lookm.lib()
    out = ctypes.c_float(0.0)
    def call(rnd=1, wps=3, iters=16, reps=2, o=ctypes.byref(out), ws=FAKE, wsn=1 << 20):
        return L.lookm_probe_mfma(rnd, wps, iters, reps, o, ws, wsn, None)

    assert call(o=None) == lookm.ERR_INVALID_ARG and call(ws=None) == lookm.ERR_INVALID_ARG
    assert call(wps=0) == lookm.ERR_INVALID_ARG and call(wps=4) == lookm.ERR_INVALID_ARG
    assert call(iters=0) == lookm.ERR_INVALID_ARG and call(iters=(1 << 20) + 1) == lookm.ERR_INVALID_ARG
    assert call(reps=0) == lookm.ERR_INVALID_ARG and call(reps=1001) == lookm.ERR_INVALID_ARG
    assert call(rnd=-1) == lookm.ERR_INVALID_ARG and call(rnd=3) == lookm.ERR_INVALID_ARG


def test_binding_refuses_cpu_tensors():
    import torch
    t = torch.zeros(1, 8, 8)
    with pytest.raises(ValueError):
        lookm.lookm_scores(t, t, workspace=torch.zeros(1 << 16, dtype=torch.uint8))
