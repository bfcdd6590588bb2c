"""CPU oracle for LOOK-M prefill-time KV-cache compression (TEST INFRASTRUCTURE ONLY).

Thin ctypes loader around ``lookm_oracle.c`` (plain C, binary64 arithmetic, written from
the paper's Sections 3.2-3.3, Eq. 4-12).  Nothing in the product package may import this
module: it exists so that tests, the smoke check and the benchmark's ``cpu_baseline`` leg
have an independent statement of what the HIP path must compute.

All array arguments are NumPy arrays; tensors of the caller's dtype (bf16 / fp32) are
widened exactly to float32 before they get here (see ``as_f32``).
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from pathlib import Path

import numpy as np

_HERE = Path(__file__).resolve().parent
_SRC = _HERE / "lookm_oracle.c"
_LIB = _HERE / "liblookm_oracle.so"

OK = 0
ERR_ARG = -1
ERR_BUDGET_RANGE = -3
ERR_BUDGET_BELOW_PROTECTED = -4

MODES = {"none": 0, "averaged": 1, "pivotal": 2, "weighted": 3}

CFLAGS = ["-O2", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared"]


def build(force: bool = False) -> Path:
    """Compile the C oracle with gcc (no fast-math, no contraction)."""
    if force or not _LIB.exists() or _LIB.stat().st_mtime < _SRC.stat().st_mtime:
        tmp = _LIB.with_suffix(f".so.tmp{os.getpid()}")
        subprocess.check_call(["gcc", *CFLAGS, str(_SRC), "-o", str(tmp), "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


def build_sanitized() -> Path:
    """The oracle with AddressSanitizer and UndefinedBehaviorSanitizer (oracle/_build/liblookm_oracle_san.so), for the
    test that runs the pins against it; load it through LOOKM_ORACLE_LIB with gcc's libasan preloaded."""
    out_dir = _HERE / "_build"
    out_dir.mkdir(exist_ok=True)
    out = out_dir / "liblookm_oracle_san.so"
    subprocess.check_call(["gcc", "-O1", "-g", "-ffp-contract=off", "-fopenmp", "-fPIC", "-shared",
                           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", str(_SRC), "-o", str(out),
                           "-lm"])
    return out


_lib = None


def lib() -> ctypes.CDLL:
    global _lib
    if _lib is None:
        # LOOKM_ORACLE_LIB: tests that plant a mistake in a copy of the source point this at the
        # mutant's library to show that the pins notice it
        override = os.environ.get("LOOKM_ORACLE_LIB")
        L = ctypes.CDLL(override if override else str(build()))
        fp = ctypes.POINTER(ctypes.c_float)
        dp = ctypes.POINTER(ctypes.c_double)
        ip = ctypes.POINTER(ctypes.c_int32)
        up = ctypes.POINTER(ctypes.c_uint8)
        I = ctypes.c_int
        L.oracle_scores_head.argtypes = [fp, fp, I, I, dp]
        L.oracle_scores_head.restype = None
        L.oracle_scores.argtypes = [fp, fp, I, I, I, dp]
        L.oracle_scores.restype = None
        L.oracle_scores_window.argtypes = [fp, fp, I, I, I, I, dp]
        L.oracle_scores_window.restype = None
        L.oracle_scores_grouped.argtypes = [fp, fp, I, I, I, I, dp]
        L.oracle_scores_grouped.restype = I
        L.oracle_decode.argtypes = [fp, fp, fp, I, I, I, I, dp]
        L.oracle_decode.restype = None
        L.oracle_row_lse.argtypes = [fp, fp, I, I, I, dp]
        L.oracle_row_lse.restype = None
        L.oracle_protected_count.argtypes = [up, I, I]
        L.oracle_protected_count.restype = I
        L.oracle_select_head.argtypes = [dp, up, I, I, I, ip, ip]
        L.oracle_select_head.restype = I
        L.oracle_select_rule_head.argtypes = [dp, up, I, I, I, I, ip, ip]
        L.oracle_select_rule_head.restype = I
        L.oracle_budget_from_ratios.argtypes = [I, ctypes.c_double, ctypes.c_double, ip, ip]
        L.oracle_budget_from_ratios.restype = I
        L.oracle_nearest_head.argtypes = [fp, I, ip, I, ip, I, ip, dp]
        L.oracle_nearest_head.restype = None
        L.oracle_merge_head.argtypes = [fp, I, ip, I, ip, I, ip, dp, I, dp]
        L.oracle_merge_head.restype = I
        L.oracle_compress.argtypes = [fp, fp, fp, up, I, I, I, I, I, I, dp, ip, ip, ip, dp, dp, dp]
        L.oracle_compress.restype = I
        L.oracle_compress_rule.argtypes = [fp, fp, fp, up, I, I, I, I, I, I, I, dp, ip, ip, ip, dp, dp, dp]
        L.oracle_compress_rule.restype = I
        L.oracle_num_threads.argtypes = []
        L.oracle_num_threads.restype = I
        _lib = L
    return _lib


def _p(a: np.ndarray, ct):
    return a.ctypes.data_as(ctypes.POINTER(ct))


def as_f32(x) -> np.ndarray:
    """Exact widening of a torch (bf16/fp32/fp64-representable) or NumPy array to contiguous float32."""
    if hasattr(x, "detach"):
        x = x.detach().cpu().float().numpy()
    return np.ascontiguousarray(x, dtype=np.float32)


def _mask(m) -> np.ndarray:
    if hasattr(m, "detach"):
        m = m.detach().cpu().numpy()
    return np.ascontiguousarray(m, dtype=np.uint8)


class OracleError(ValueError):
    def __init__(self, code: int):
        super().__init__(f"oracle status {code}")
        self.code = code


def num_threads() -> int:
    return int(lib().oracle_num_threads())


def scores(q, k) -> np.ndarray:
    """Eq. 4: accumulated attention scores.  q, k: [H, L, d] (or [L, d]) -> float64 [H, L] (or [L])."""
    q, k = as_f32(q), as_f32(k)
    single = q.ndim == 2
    if single:
        q, k = q[None], k[None]
    H, L, d = q.shape
    out = np.empty((H, L), dtype=np.float64)
    lib().oracle_scores(_p(q, ctypes.c_float), _p(k, ctypes.c_float), H, L, d, _p(out, ctypes.c_double))
    return out[0] if single else out


def scores_grouped(q, k) -> np.ndarray:
    """Grouped-query attention: q [H, L, d], k [kv_heads, L, d] -> float64 [kv_heads, L], Eq. 4 summed over the query
    heads that share a key head."""
    q, k = as_f32(q), as_f32(k)
    H, L, d = q.shape
    kvh = k.shape[0]
    out = np.empty((kvh, L), dtype=np.float64)
    rc = lib().oracle_scores_grouped(_p(q, ctypes.c_float), _p(k, ctypes.c_float), H, kvh, L, d, _p(out, ctypes.c_double))
    if rc != OK:
        raise OracleError(rc)
    return out


def compress_grouped(q, k, v, mask, budget: int, recent_window: int, mode, rule="protect_text") -> dict:
    """The whole path with grouped query heads: scores_grouped, then selection, matching and merging per KEY head
    with the single-head functions above.  q: [H, L, d]; k, v: [kv_heads, L, d]."""
    k32, v32 = as_f32(k), as_f32(v)
    m = _mask(mask)
    sc = scores_grouped(q, k)
    kvh, L, d = k32.shape
    B = int(budget)
    out = dict(scores=sc, kept=np.empty((kvh, B), np.int32), evicted=np.empty((kvh, L - B), np.int32),
               assign=np.empty((kvh, L - B), np.int32), sim=np.empty((kvh, L - B), np.float64),
               k_out=np.empty((kvh, B, d), np.float64), v_out=np.empty((kvh, B, d), np.float64))
    for h in range(kvh):
        out["kept"][h], out["evicted"][h] = select(sc[h], m, B, recent_window, rule)
        out["assign"][h], out["sim"][h] = nearest(k32[h], out["kept"][h], out["evicted"][h])
        out["k_out"][h] = merge(k32[h], out["kept"][h], out["evicted"][h], out["assign"][h], out["sim"][h], mode)
        out["v_out"][h] = merge(v32[h], out["kept"][h], out["evicted"][h], out["assign"][h], out["sim"][h], mode)
    return out


def scores_window(q, k, window: int) -> np.ndarray:
    """Accumulated attention of the last ``window`` query rows only.  q, k: [H, L, d] (or [L, d]) -> float64."""
    q, k = as_f32(q), as_f32(k)
    single = q.ndim == 2
    if single:
        q, k = q[None], k[None]
    H, L, d = q.shape
    if not 1 <= int(window) <= L:
        raise OracleError(-1)
    out = np.empty((H, L), dtype=np.float64)
    lib().oracle_scores_window(_p(q, ctypes.c_float), _p(k, ctypes.c_float), H, L, d, int(window),
                               _p(out, ctypes.c_double))
    return out[0] if single else out


def decode(q, k, v, S: int | None = None) -> np.ndarray:
    """Eq. 3: Softmax(q K^T / sqrt(d)) V for one new token per head.  q: [H, d]; k, v: [H, rows, d]; the first S rows
    (default all) are attended.  -> float64 [H, d]."""
    q, k, v = as_f32(q), as_f32(k), as_f32(v)
    H, rows, d = k.shape
    S = rows if S is None else int(S)
    if not (1 <= S <= rows) or q.shape != (H, d) or v.shape != k.shape:
        raise OracleError(-1)
    out = np.empty((H, d), dtype=np.float64)
    f = ctypes.c_float
    lib().oracle_decode(_p(q, f), _p(k, f), _p(v, f), H, rows, S, d, _p(out, ctypes.c_double))
    return out


def row_lse(q, k) -> np.ndarray:
    """Natural-log log-sum-exp of every causal row of q k^T / sqrt(d) (the normaliser of A_p in Eq. 4).
    q, k: [H, L, d] (or [L, d]) -> float64 [H, L] (or [L])."""
    q, k = as_f32(q), as_f32(k)
    single = q.ndim == 2
    if single:
        q, k = q[None], k[None]
    H, L, d = q.shape
    out = np.empty((H, L), dtype=np.float64)
    lib().oracle_row_lse(_p(q, ctypes.c_float), _p(k, ctypes.c_float), H, L, d, _p(out, ctypes.c_double))
    return out[0] if single else out


def protected_count(mask, recent_window: int) -> int:
    m = _mask(mask)
    return int(lib().oracle_protected_count(_p(m, ctypes.c_uint8), m.shape[0], int(recent_window)))


RULES = {"protect_text": 0, "literal": 1}


def budget_from_ratios(L: int, alpha_recent: float, alpha_important: float):
    """Section 4 "Implementation Details": M = alpha_1 L, N = alpha_2 L -> (recent_window M, budget S = N + M)."""
    M = np.zeros(1, np.int32)
    N = np.zeros(1, np.int32)
    rc = lib().oracle_budget_from_ratios(int(L), float(alpha_recent), float(alpha_important),
                                         _p(M, ctypes.c_int32), _p(N, ctypes.c_int32))
    if rc < 0:
        raise OracleError(rc)
    return int(M[0]), int(rc)


def select(scores_1d, mask, budget: int, recent_window: int, rule="protect_text"):
    """Eq. 5-8 for one head: -> (kept [B] int32 ascending, evicted [L-B] int32 ascending).
    rule "protect_text": all text tokens must fit in the budget; "literal": Eq. 8 as printed, for any budget."""
    s = np.ascontiguousarray(scores_1d, dtype=np.float64)
    m = _mask(mask)
    L = s.shape[0]
    B = int(budget)
    kept = np.empty(max(B, 0), dtype=np.int32)
    ev = np.empty(max(L - B, 0), dtype=np.int32)
    rule = RULES[rule] if isinstance(rule, str) else int(rule)
    rc = lib().oracle_select_rule_head(_p(s, ctypes.c_double), _p(m, ctypes.c_uint8), L, B, int(recent_window), rule,
                                       _p(kept, ctypes.c_int32), _p(ev, ctypes.c_int32))
    if rc != OK:
        raise OracleError(rc)
    return kept, ev


def nearest(k_2d, kept, evicted):
    """Eq. 9 for one head: -> (assign [Le] int32 slot index into kept, sim [Le] float64)."""
    k = as_f32(k_2d)
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    ev = np.ascontiguousarray(evicted, dtype=np.int32)
    assign = np.empty(ev.shape[0], dtype=np.int32)
    sim = np.empty(ev.shape[0], dtype=np.float64)
    lib().oracle_nearest_head(_p(k, ctypes.c_float), k.shape[1], _p(kept, ctypes.c_int32), kept.shape[0],
                              _p(ev, ctypes.c_int32), ev.shape[0], _p(assign, ctypes.c_int32), _p(sim, ctypes.c_double))
    return assign, sim


def merge(x_2d, kept, evicted, assign, sim, mode) -> np.ndarray:
    """Eq. 10-12 for one head and one tensor (K or V): -> float64 [B, d]."""
    x = as_f32(x_2d)
    kept = np.ascontiguousarray(kept, dtype=np.int32)
    ev = np.ascontiguousarray(evicted, dtype=np.int32)
    assign = np.ascontiguousarray(assign, dtype=np.int32)
    sim = np.ascontiguousarray(sim, dtype=np.float64)
    mode = MODES[mode] if isinstance(mode, str) else int(mode)
    out = np.empty((kept.shape[0], x.shape[1]), dtype=np.float64)
    rc = lib().oracle_merge_head(_p(x, ctypes.c_float), x.shape[1], _p(kept, ctypes.c_int32), kept.shape[0],
                                 _p(ev, ctypes.c_int32), ev.shape[0], _p(assign, ctypes.c_int32),
                                 _p(sim, ctypes.c_double), mode, _p(out, ctypes.c_double))
    if rc != OK:
        raise OracleError(rc)
    return out


def compress(q, k, v, mask, budget: int, recent_window: int, mode, rule="protect_text") -> dict:
    """The whole path over all heads.  q, k, v: [H, L, d].  Returns a dict of NumPy arrays:
    scores [H, L] f64, kept [H, B] i32, evicted [H, Le] i32, assign [H, Le] i32, sim [H, Le] f64,
    k_out / v_out [H, B, d] f64 (unrounded)."""
    q, k, v = as_f32(q), as_f32(k), as_f32(v)
    m = _mask(mask)
    H, L, d = q.shape
    B = int(budget)
    M = int(recent_window)
    mode = MODES[mode] if isinstance(mode, str) else int(mode)
    Le = max(L - B, 0)
    Bn = max(B, 0)
    out = dict(
        scores=np.empty((H, L), np.float64), kept=np.empty((H, Bn), np.int32),
        evicted=np.empty((H, Le), np.int32), assign=np.empty((H, Le), np.int32),
        sim=np.empty((H, Le), np.float64), k_out=np.empty((H, Bn, d), np.float64),
        v_out=np.empty((H, Bn, d), np.float64))
    f, dd, i32 = ctypes.c_float, ctypes.c_double, ctypes.c_int32
    rule = RULES[rule] if isinstance(rule, str) else int(rule)
    rc = lib().oracle_compress_rule(_p(q, f), _p(k, f), _p(v, f), _p(m, ctypes.c_uint8), H, L, d, B, M, mode, rule,
                               _p(out["scores"], dd), _p(out["kept"], i32), _p(out["evicted"], i32),
                               _p(out["assign"], i32), _p(out["sim"], dd), _p(out["k_out"], dd), _p(out["v_out"], dd))
    if rc != OK:
        raise OracleError(rc)
    return out
