"""ctypes binding of liblookm.so: argument marshalling only.

Every function has the name and the semantics of the C entry point it forwards to (see
include/lookm.h).  PyTorch is used for device memory and for the current HIP stream; all of the
method's arithmetic runs in the library's kernels.  There is no CPU fallback: a missing library
or a non-GPU tensor raises.
"""
from __future__ import annotations

import ctypes
from dataclasses import dataclass
from pathlib import Path
from typing import Optional

import torch

import os

_PKG = Path(__file__).resolve().parent
# LOOKM_LIB: another build of the same library (the host-sanitizer build the CPU tests make); default: the in-tree one
LIB_PATH = Path(os.environ["LOOKM_LIB"]) if os.environ.get("LOOKM_LIB") else _PKG / "liblookm.so"

OK = 0
ERR_INVALID_ARG = -1
ERR_UNSUPPORTED = -2
ERR_BUDGET_RANGE = -3
ERR_BUDGET_BELOW_PROTECTED = -4
ERR_WORKSPACE = -5
ERR_DEVICE = -6

MERGE_MODES = {"none": 0, "averaged": 1, "pivotal": 2, "weighted": 3}
F32, BF16 = 0, 1
SELECT_RULES = {"protect_text": 0, "literal": 1}

EXPORTS = ["lookm_version", "lookm_status_string", "lookm_protected_count", "lookm_workspace_bytes",
           "lookm_compress", "lookm_scores", "lookm_select", "lookm_nearest", "lookm_merge",
           "lookm_compress_profile", "lookm_scores_lse", "lookm_compress_lse", "lookm_budget_from_ratios",
           "lookm_select_rule_", "lookm_compress_batch", "lookm_scores_window", "lookm_job_profile", "lookm_decode_workspace_bytes",
           "lookm_decode_attention", "lookm_scores_grouped", "lookm_probe_mfma", "lookm_init",
           "lookm_compress_batch_two_streams", "lookm_workspace_offset", "lookm_decode_attention_noalloc"]

KERNELS = ["score_lse", "score_lse_fold", "score_colsum", "score_colsum_fold", "select", "rnorm", "nearest",
           "nearest_fold", "bucket", "merge"]   # LOOKM_K_* order


class Job(ctypes.Structure):
    """struct lookm_job of include/lookm.h, field for field."""
    _fields_ = [("q", ctypes.c_void_p), ("k", ctypes.c_void_p), ("v", ctypes.c_void_p),
                ("modality_mask", ctypes.c_void_p), ("row_lse", ctypes.c_void_p),
                ("H", ctypes.c_int), ("L", ctypes.c_int), ("d", ctypes.c_int), ("dt", ctypes.c_int),
                ("budget", ctypes.c_int), ("recent_window", ctypes.c_int), ("merge_mode", ctypes.c_int),
                ("rule", ctypes.c_int), ("score_window", ctypes.c_int), ("kv_heads", ctypes.c_int),
                ("k_out", ctypes.c_void_p), ("v_out", ctypes.c_void_p), ("kept_idx", ctypes.c_void_p),
                ("scores_out", ctypes.c_void_p), ("status_out", ctypes.c_void_p),
                ("workspace", ctypes.c_void_p), ("workspace_bytes", ctypes.c_size_t)]


class LookmError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {status_string(code)} ({code})")


_lib = None


def lib() -> ctypes.CDLL:
    """Loads liblookm.so (built by ``python -m paper_2406_18139_amd.build``); raises if it is missing."""
    global _lib
    if _lib is None:
        if not LIB_PATH.exists():
            raise FileNotFoundError(f"{LIB_PATH} is not built; run `python -m paper_2406_18139_amd.build`")
        L = ctypes.CDLL(str(LIB_PATH))
        vp, I, sz = ctypes.c_void_p, ctypes.c_int, ctypes.c_size_t
        L.lookm_version.restype = ctypes.c_char_p
        L.lookm_version.argtypes = []
        L.lookm_status_string.restype = ctypes.c_char_p
        L.lookm_status_string.argtypes = [I]
        L.lookm_protected_count.restype = I
        L.lookm_protected_count.argtypes = [vp, I, I]
        L.lookm_workspace_bytes.restype = sz
        L.lookm_workspace_bytes.argtypes = [I, I, I, I, I]
        L.lookm_compress.restype = I
        L.lookm_compress.argtypes = [vp, vp, vp, vp, I, I, I, I, I, I, I, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lookm_compress_profile.restype = I
        L.lookm_compress_profile.argtypes = [vp, vp, vp, vp, I, I, I, I, I, I, I, vp, vp, vp, vp, vp, vp, sz, vp, I,
                                             ctypes.POINTER(ctypes.c_float)]
        L.lookm_scores_lse.restype = I
        L.lookm_scores_lse.argtypes = [vp, vp, vp, I, I, I, I, vp, vp, sz, vp]
        L.lookm_compress_lse.restype = I
        L.lookm_compress_lse.argtypes = [vp, vp, vp, vp, vp, I, I, I, I, I, I, I, vp, vp, vp, vp, vp, vp, sz, vp]
        L.lookm_scores.restype = I
        L.lookm_scores.argtypes = [vp, vp, I, I, I, I, vp, vp, sz, vp]
        L.lookm_select.restype = I
        L.lookm_select.argtypes = [vp, vp, I, I, I, I, vp, vp, vp, vp]
        L.lookm_nearest.restype = I
        L.lookm_nearest.argtypes = [vp, vp, vp, I, I, I, I, I, vp, vp, vp, sz, vp]
        L.lookm_merge.restype = I
        L.lookm_merge.argtypes = [vp, vp, vp, vp, vp, vp, I, I, I, I, I, I, vp, vp, vp, sz, vp]
        L.lookm_budget_from_ratios.restype = I
        L.lookm_budget_from_ratios.argtypes = [I, ctypes.c_double, ctypes.c_double, ctypes.POINTER(I), ctypes.POINTER(I)]
        L.lookm_select_rule_.restype = I
        L.lookm_select_rule_.argtypes = [vp, vp, I, I, I, I, I, vp, vp, vp, vp]
        L.lookm_scores_grouped.restype = I
        L.lookm_scores_grouped.argtypes = [vp, vp, I, I, I, I, I, vp, vp, sz, vp]
        L.lookm_scores_window.restype = I
        L.lookm_scores_window.argtypes = [vp, vp, I, I, I, I, I, vp, vp, sz, vp]
        L.lookm_decode_workspace_bytes.restype = sz
        L.lookm_decode_workspace_bytes.argtypes = [I, I]
        L.lookm_decode_attention.restype = I
        L.lookm_decode_attention.argtypes = [vp, vp, vp, I, I, I, I, I, vp, vp, sz, vp]
        L.lookm_decode_attention_noalloc.restype = I
        L.lookm_decode_attention_noalloc.argtypes = [vp, vp, vp, I, I, I, I, I, vp, vp]
        L.lookm_job_profile.restype = I
        L.lookm_job_profile.argtypes = [ctypes.POINTER(Job), I, ctypes.POINTER(ctypes.c_float), vp]
        L.lookm_compress_batch.restype = I
        L.lookm_compress_batch.argtypes = [ctypes.POINTER(Job), I, ctypes.POINTER(I), vp]
        L.lookm_compress_batch_two_streams.restype = I
        L.lookm_compress_batch_two_streams.argtypes = [ctypes.POINTER(Job), I, ctypes.POINTER(I), vp, vp]
        L.lookm_init.restype = I
        L.lookm_init.argtypes = []
        L.lookm_workspace_offset.restype = sz
        L.lookm_workspace_offset.argtypes = [I, I, I, I, I, I, I]
        L.lookm_probe_mfma.restype = I
        L.lookm_probe_mfma.argtypes = [I, I, I, I, ctypes.POINTER(ctypes.c_float), vp, sz, vp]
        _lib = L
    return _lib


def version() -> str:
    return lib().lookm_version().decode()


def status_string(code: int) -> str:
    return lib().lookm_status_string(int(code)).decode()


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return F32
    if t.dtype == torch.bfloat16:
        return BF16
    raise TypeError(f"unsupported dtype {t.dtype}")


def _dev(t: torch.Tensor, name: str) -> int:
    if not t.is_cuda:
        raise ValueError(f"{name} must live on the GPU (no CPU path exists)")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    return t.data_ptr()


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _mode(m) -> int:
    return MERGE_MODES[m] if isinstance(m, str) else int(m)


def _rule(r) -> int:
    return SELECT_RULES[r] if isinstance(r, str) else int(r)


def budget_from_ratios(L: int, alpha_recent: float, alpha_important: float):
    """lookm_budget_from_ratios -> (recent_window, budget)."""
    M, B = ctypes.c_int(0), ctypes.c_int(0)
    rc = lib().lookm_budget_from_ratios(int(L), float(alpha_recent), float(alpha_important), ctypes.byref(M),
                                        ctypes.byref(B))
    if rc != OK:
        raise LookmError(rc, "lookm_budget_from_ratios")
    return M.value, B.value


def protected_count(mask_host, recent_window: int) -> int:
    """lookm_protected_count on a host mask (torch CPU tensor / numpy array / bytes-like of uint8)."""
    m = torch.as_tensor(mask_host, dtype=torch.uint8).contiguous().cpu()
    rc = lib().lookm_protected_count(m.data_ptr(), m.numel(), int(recent_window))
    if rc < 0:
        raise LookmError(rc, "lookm_protected_count")
    return rc


def workspace_bytes(H: int, L: int, d: int, budget: int, dt: int) -> int:
    return int(lib().lookm_workspace_bytes(H, L, d, budget, dt))


def alloc_workspace(H: int, L: int, d: int, budget: int, dt: int, device) -> torch.Tensor:
    n = workspace_bytes(H, L, d, budget, dt)
    if n == 0:
        raise LookmError(ERR_INVALID_ARG, "lookm_workspace_bytes")
    return torch.empty(n + 256, dtype=torch.uint8, device=device)


def _ws_ptr(ws: torch.Tensor):
    p = ws.data_ptr()
    a = (p + 255) // 256 * 256
    return a, ws.numel() - (a - p)


@dataclass
class Compressed:
    k_out: torch.Tensor       # [H, B, d]
    v_out: torch.Tensor       # [H, B, d]
    kept_idx: torch.Tensor    # [H, B] int32
    scores: Optional[torch.Tensor]   # [H, L] float32 or None
    status: torch.Tensor      # [1] int32 (device)


def lookm_compress(q, k, v, modality_mask, budget: int, recent_window: int, merge_mode,
                   want_scores: bool = False, out: Optional[Compressed] = None,
                   workspace: Optional[torch.Tensor] = None, check: bool = True,
                   row_lse: Optional[torch.Tensor] = None, rule="protect_text", score_window: int = 0) -> Compressed:
    """One layer's compression.  q, k, v: GPU tensors [H, L, d]; modality_mask: GPU uint8 [L].
    ``check=True`` synchronises to read the device status word and raises on failure.
    With ``row_lse`` (GPU float32 [H, L]) the call forwards to lookm_compress_lse; with a selection rule other
    than the default, an observation window for the scores, or fewer key / value heads than query heads (grouped
    query heads: k, v [kv_heads, L, d]), it forwards to lookm_compress_batch as a single job (the entry point that
    takes them)."""
    if _rule(rule) != 0 or int(score_window) != 0 or k.shape[0] != q.shape[0]:
        H, L, d = q.shape
        if out is None:
            out = alloc_outputs(k.shape[0], L, d, int(budget), q.dtype, q.device, want_scores)
        if workspace is None:
            workspace = alloc_workspace(H, L, d, min(max(int(budget), 0), L), _dt(q), q.device)
        lookm_compress_batch([make_job(q, k, v, modality_mask, budget, recent_window, merge_mode, out, workspace,
                                       row_lse=row_lse, rule=rule, score_window=score_window)])
        if check:
            st = int(out.status.item())
            if st != OK:
                raise LookmError(st, "lookm_compress_batch (device)")
        return out
    H, L, d = q.shape
    dt = _dt(q)
    B = int(budget)
    dev = q.device
    if out is None:
        out = alloc_outputs(H, L, d, B, q.dtype, dev, want_scores)
    if workspace is None:
        workspace = alloc_workspace(H, L, d, min(max(B, 0), L), dt, dev)
    wp, wn = _ws_ptr(workspace)
    tail = (H, L, d, dt, B, int(recent_window), _mode(merge_mode),
            _dev(out.k_out, "k_out"), _dev(out.v_out, "v_out"), _dev(out.kept_idx, "kept_idx"),
            _dev(out.scores, "scores") if out.scores is not None else None,
            _dev(out.status, "status"), wp, wn, _stream())
    head = (_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(modality_mask, "modality_mask"))
    if row_lse is None:
        rc = lib().lookm_compress(*head, *tail)
    else:
        if row_lse.dtype != torch.float32 or tuple(row_lse.shape) != (H, L):
            raise ValueError("row_lse must be float32 [H, L]")
        rc = lib().lookm_compress_lse(*head, _dev(row_lse, "row_lse"), *tail)
    if rc != OK:
        raise LookmError(rc, "lookm_compress")
    if check:
        st = int(out.status.item())
        if st != OK:
            raise LookmError(st, "lookm_compress (device)")
    return out


def make_job(q, k, v, modality_mask, budget: int, recent_window: int, merge_mode, out: Compressed,
             workspace: torch.Tensor, row_lse: Optional[torch.Tensor] = None, rule="protect_text",
             score_window: int = 0) -> Job:
    """A struct lookm_job over the given tensors (which the caller keeps alive until the work has run)."""
    H, L, d = q.shape
    if row_lse is not None and (row_lse.dtype != torch.float32 or tuple(row_lse.shape) != (H, L)):
        raise ValueError("row_lse must be float32 [H, L]")
    kv_heads = 0 if k.shape[0] == H else int(k.shape[0])        # grouped query heads when k has fewer heads than q
    wp, wn = _ws_ptr(workspace)
    return Job(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(modality_mask, "modality_mask"),
               _dev(row_lse, "row_lse") if row_lse is not None else None, H, L, d, _dt(q), int(budget),
               int(recent_window), _mode(merge_mode), _rule(rule), int(score_window), kv_heads,
               _dev(out.k_out, "k_out"),
               _dev(out.v_out, "v_out"),
               _dev(out.kept_idx, "kept_idx"), _dev(out.scores, "scores") if out.scores is not None else None,
               _dev(out.status, "status"), wp, wn)


def lookm_compress_batch(jobs, aux_stream: Optional[torch.cuda.Stream] = None) -> None:
    """lookm_compress_batch over a list of Job structs (see make_job), on the current stream; with ``aux_stream``
    (a second stream of the caller's) lookm_compress_batch_two_streams."""
    n = len(jobs)
    arr = (Job * max(n, 1))(*jobs)
    bad = ctypes.c_int(-1)
    if aux_stream is None:
        rc = lib().lookm_compress_batch(arr, n, ctypes.byref(bad), _stream())
    else:
        rc = lib().lookm_compress_batch_two_streams(arr, n, ctypes.byref(bad), _stream(), aux_stream.cuda_stream)
    if rc != OK:
        raise LookmError(rc, f"lookm_compress_batch (job {bad.value})")


def lookm_init() -> None:
    rc = lib().lookm_init()
    if rc != OK:
        raise LookmError(rc, "lookm_init")


WS_ITEMS = {"evicted": (0, torch.int32), "assign": (1, torch.int32), "sim": (2, torch.float32)}


def workspace_view(workspace: torch.Tensor, item: str, H: int, kv_heads: int, L: int, d: int, budget: int, dt: int):
    """The intermediate array ``item`` ("evicted", "assign", "sim") that a finished compression call left in
    ``workspace`` (lookm_workspace_offset): a [kv_heads, L - budget] view, no copy."""
    code, dtype = WS_ITEMS[item]
    off = int(lib().lookm_workspace_offset(H, kv_heads, L, d, int(budget), dt, code))
    if off == ctypes.c_size_t(-1).value:
        raise LookmError(ERR_INVALID_ARG, "lookm_workspace_offset")
    base, _ = _ws_ptr(workspace)
    start = base - workspace.data_ptr() + off
    n = kv_heads * (L - int(budget))
    return workspace[start:start + 4 * n].view(dtype).view(kv_heads, L - int(budget))


def alloc_outputs(H: int, L: int, d: int, budget: int, dtype, device, want_scores: bool = False) -> Compressed:
    nb = max(int(budget), 0)
    return Compressed(torch.empty((H, nb, d), dtype=dtype, device=device),
                      torch.empty((H, nb, d), dtype=dtype, device=device),
                      torch.empty((H, nb), dtype=torch.int32, device=device),
                      torch.empty((H, L), dtype=torch.float32, device=device) if want_scores else None,
                      torch.zeros(1, dtype=torch.int32, device=device))


def lookm_compress_profile(q, k, v, modality_mask, budget: int, recent_window: int, merge_mode, reps: int,
                           out: Compressed, workspace: torch.Tensor) -> dict:
    """lookm_compress run ``reps`` times with an event after every kernel; returns {kernel: average ms}.
    Synchronises the current stream."""
    H, L, d = q.shape
    wp, wn = _ws_ptr(workspace)
    ms = (ctypes.c_float * len(KERNELS))()
    rc = lib().lookm_compress_profile(_dev(q, "q"), _dev(k, "k"), _dev(v, "v"), _dev(modality_mask, "modality_mask"),
                                      H, L, d, _dt(q), int(budget), int(recent_window), _mode(merge_mode),
                                      _dev(out.k_out, "k_out"), _dev(out.v_out, "v_out"),
                                      _dev(out.kept_idx, "kept_idx"),
                                      _dev(out.scores, "scores") if out.scores is not None else None,
                                      _dev(out.status, "status"), wp, wn, _stream(), int(reps), ms)
    if rc != OK:
        raise LookmError(rc, "lookm_compress_profile")
    return {name: float(ms[i]) for i, name in enumerate(KERNELS)}


def lookm_decode_attention(q, k_cache, v_cache, S: Optional[int] = None, out: Optional[torch.Tensor] = None,
                           workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """Eq. 3 for one new token per head.  q: GPU [H, d]; k_cache, v_cache: GPU [H, rows, d]; the first S rows
    (default all) are attended.  Returns [H, d] in the inputs' dtype."""
    H, rows, d = k_cache.shape
    S = rows if S is None else int(S)
    dt = _dt(q)
    if out is None:
        out = torch.empty((H, d), dtype=q.dtype, device=q.device)
    if workspace is None:
        workspace = torch.empty(int(lib().lookm_decode_workspace_bytes(H, d)) + 256, dtype=torch.uint8, device=q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib().lookm_decode_attention(_dev(q, "q"), _dev(k_cache, "k_cache"), _dev(v_cache, "v_cache"), H, rows, S, d,
                                      dt, _dev(out, "out"), wp, wn, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_decode_attention")
    return out


def lookm_decode_attention_noalloc(q, k_cache, v_cache, out: torch.Tensor, S: Optional[int] = None) -> torch.Tensor:
    """lookm_decode_attention_noalloc: the same step with the library's static scratch; ``out`` ([H, d], the inputs'
    dtype) is the caller's, nothing is allocated here or in the library."""
    H, rows, d = k_cache.shape
    S = rows if S is None else int(S)
    rc = lib().lookm_decode_attention_noalloc(_dev(q, "q"), _dev(k_cache, "k_cache"), _dev(v_cache, "v_cache"), H, rows,
                                              S, d, _dt(q), _dev(out, "out"), _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_decode_attention_noalloc")
    return out


def lookm_probe_mfma(random_operands, waves_per_simd: int = 3, iters: int = 4096, reps: int = 20,
                     workspace: Optional[torch.Tensor] = None) -> float:
    """lookm_probe_mfma: sustained TFLOP/s of the bf16 MFMA from registers alone (a measurement aid).
    random_operands: 0 / False constant operands, 1 / True random operands (both v_mfma_f32_32x32x16_bf16),
    2 random operands through v_mfma_f32_16x16x32_bf16.  Synchronises the current stream."""
    if workspace is None:
        workspace = torch.empty((1 << 20) + 256, dtype=torch.uint8, device="cuda")
    wp, wn = _ws_ptr(workspace)
    out = ctypes.c_float(0.0)
    rc = lib().lookm_probe_mfma(int(random_operands), int(waves_per_simd), int(iters), int(reps),
                                ctypes.byref(out), wp, wn, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_probe_mfma")
    return float(out.value)


def lookm_job_profile(job: Job, reps: int) -> dict:
    """lookm_job_profile: the job run ``reps`` times with an event after every kernel -> {kernel: average ms}."""
    ms = (ctypes.c_float * len(KERNELS))()
    rc = lib().lookm_job_profile(ctypes.byref(job), int(reps), ms, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_job_profile")
    return {name: float(ms[i]) for i, name in enumerate(KERNELS)}


def lookm_scores(q, k, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    H, L, d = q.shape
    dt = _dt(q)
    scores = torch.empty((H, L), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(H, L, d, 0, dt, q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib().lookm_scores(_dev(q, "q"), _dev(k, "k"), H, L, d, dt, scores.data_ptr(), wp, wn, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_scores")
    return scores


def lookm_scores_grouped(q, k, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    """q: [H, L, d], k: [kv_heads, L, d] -> scores [kv_heads, L] (Eq. 4 summed over each key head's query heads)."""
    H, L, d = q.shape
    kvh = k.shape[0]
    dt = _dt(q)
    scores = torch.empty((kvh, L), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(H, L, d, 0, dt, q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib().lookm_scores_grouped(_dev(q, "q"), _dev(k, "k"), H, kvh, L, d, dt, scores.data_ptr(), wp, wn, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_scores_grouped")
    return scores


def lookm_scores_window(q, k, window: int, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    H, L, d = q.shape
    dt = _dt(q)
    scores = torch.empty((H, L), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(H, L, d, 0, dt, q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib().lookm_scores_window(_dev(q, "q"), _dev(k, "k"), H, L, d, dt, int(window), scores.data_ptr(), wp, wn,
                                   _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_scores_window")
    return scores


def lookm_scores_lse(q, k, row_lse, workspace: Optional[torch.Tensor] = None) -> torch.Tensor:
    H, L, d = q.shape
    dt = _dt(q)
    if row_lse.dtype != torch.float32 or tuple(row_lse.shape) != (H, L):
        raise ValueError("row_lse must be float32 [H, L]")
    scores = torch.empty((H, L), dtype=torch.float32, device=q.device)
    if workspace is None:
        workspace = alloc_workspace(H, L, d, 0, dt, q.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib().lookm_scores_lse(_dev(q, "q"), _dev(k, "k"), _dev(row_lse, "row_lse"), H, L, d, dt,
                                scores.data_ptr(), wp, wn, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_scores_lse")
    return scores


def lookm_select(scores, modality_mask, budget: int, recent_window: int, check: bool = True, rule="protect_text"):
    H, L = scores.shape
    B = int(budget)
    dev = scores.device
    kept = torch.empty((H, max(B, 0)), dtype=torch.int32, device=dev)
    evicted = torch.empty((H, max(L - B, 0)), dtype=torch.int32, device=dev)
    status = torch.zeros(1, dtype=torch.int32, device=dev)
    if _rule(rule) == 0:
        rc = lib().lookm_select(_dev(scores, "scores"), _dev(modality_mask, "modality_mask"), H, L, B,
                                int(recent_window), kept.data_ptr(), evicted.data_ptr(), status.data_ptr(), _stream())
    else:
        rc = lib().lookm_select_rule_(_dev(scores, "scores"), _dev(modality_mask, "modality_mask"), H, L, B,
                                      int(recent_window), _rule(rule), kept.data_ptr(), evicted.data_ptr(),
                                      status.data_ptr(), _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_select")
    if check:
        st = int(status.item())
        if st != OK:
            raise LookmError(st, "lookm_select (device)")
    return kept, evicted


def lookm_nearest(k, kept_idx, evicted_idx, workspace: Optional[torch.Tensor] = None):
    H, L, d = k.shape
    B = kept_idx.shape[1]
    dt = _dt(k)
    Le = L - B
    assign = torch.empty((H, Le), dtype=torch.int32, device=k.device)
    sim = torch.empty((H, Le), dtype=torch.float32, device=k.device)
    if workspace is None:
        workspace = alloc_workspace(H, L, d, B, dt, k.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib().lookm_nearest(_dev(k, "k"), _dev(kept_idx, "kept_idx"), _dev(evicted_idx, "evicted_idx"), H, L, d, dt,
                             B, assign.data_ptr(), sim.data_ptr(), wp, wn, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_nearest")
    return assign, sim


def lookm_merge(k, v, kept_idx, evicted_idx, assign, sim, merge_mode, workspace: Optional[torch.Tensor] = None):
    H, L, d = k.shape
    B = kept_idx.shape[1]
    dt = _dt(k)
    k_out = torch.empty((H, B, d), dtype=k.dtype, device=k.device)
    v_out = torch.empty((H, B, d), dtype=k.dtype, device=k.device)
    if workspace is None:
        workspace = alloc_workspace(H, L, d, B, dt, k.device)
    wp, wn = _ws_ptr(workspace)
    rc = lib().lookm_merge(_dev(k, "k"), _dev(v, "v"), _dev(kept_idx, "kept_idx"), _dev(evicted_idx, "evicted_idx"),
                           _dev(assign, "assign"), _dev(sim, "sim"), H, L, d, dt, B, _mode(merge_mode),
                           k_out.data_ptr(), v_out.data_ptr(), wp, wn, _stream())
    if rc != OK:
        raise LookmError(rc, "lookm_merge")
    return k_out, v_out
