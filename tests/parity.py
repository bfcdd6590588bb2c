"""Helpers shared by the GPU parity tests: run the HIP path through the C ABI binding, run the CPU
oracle on the same seeded inputs, and compare.

Top-k and argmax are discontinuous, so where floating point decides an integer both sides have to decide
in the same precision.  The protocol:
  * stage-exact, EVERY head: the oracle's selection applied to the kernel's own fp32 scores must reproduce
    the kernel's kept and evicted lists bit for bit; the oracle's merge applied to the matching the call
    itself computed (read back from its workspace) must reproduce the output rows within the metric's
    tolerance, compared with the oracle's UNROUNDED fp64 rows (2e-2 absolute for bf16); the stage call
    lookm_nearest must reproduce that in-path matching bit for bit; the matching equal to the fp64 oracle's
    on the call's own kept and evicted lists (a differing row is counted if its cosine lies within TIE_COS of
    the oracle's best, and is an error otherwise; the tests assert zero), cosines within SIM_ATOL;
  * end-to-end, on the sampled heads the fp64 oracle's score loop is run for: scores within tolerance; kept
    sets equal to the fp64 oracle's (a differing position is only tolerated - and counted - when its oracle
    score lies within TIE_SCORE (relative) of the oracle's threshold score; the tests assert the count is
    zero).
Every run appends its statistics to STATS; with LOOKM_PARITY_STATS=<file> in the environment the test session
writes them there as a table (tests/conftest.py).
"""
from __future__ import annotations

import os
from concurrent.futures import ThreadPoolExecutor

import numpy as np
import torch

import oracle
from paper_2406_18139_amd import lookm
from paper_2406_18139_amd import workloads as W

TIE_SCORE = 1e-5
TIE_COS = 1e-5
SCORE_RTOL = 1e-3          # bar stated for the metric; the kernels are far inside it
SIM_ATOL = 2e-6            # cosine handed on to weighted merging (fp32 value of a 20-bit key, or the exact pass)
MERGE_ATOL = {torch.bfloat16: 2e-2, torch.float32: 1e-4}

STATS = []                 # one dict per run_and_check call (and per hand-rolled check that calls record())


def record(**kw):
    STATS.append(kw)
    return kw


def to_gpu(*ts):
    return [t.cuda() for t in ts]


def check_scores(gpu_scores: np.ndarray, ref: np.ndarray, rtol=SCORE_RTOL):
    rel = np.abs(gpu_scores - ref) / ref
    assert np.all(np.isfinite(gpu_scores))
    assert rel.max() <= rtol, f"score relative error {rel.max():.3e} > {rtol}"
    return float(rel.max())


def check_select_stage(kept_gpu, evicted_gpu, scores_gpu, mask, B, M, rule="protect_text"):
    """Both sides deciding on the kernel's own scores: kept (and, when given, evicted) lists must be identical.
    All heads."""
    for h in range(kept_gpu.shape[0]):
        kp, ev = oracle.select(scores_gpu[h].astype(np.float64), mask, B, M, rule)
        assert kp.tolist() == kept_gpu[h].tolist(), f"head {h}: selection differs from the oracle on the kernel's own scores"
        if evicted_gpu is not None:
            assert ev.tolist() == evicted_gpu[h].tolist(), f"head {h}: evicted list differs from the oracle's"


def check_kept(kept_gpu, scores_gpu, ref_scores, ref_kept, mask, B, M, rule="protect_text"):
    """Returns the number of heads whose kept set differs from the fp64 oracle's (all inside the tie band)."""
    H = kept_gpu.shape[0]
    check_select_stage(kept_gpu, None, scores_gpu, mask, B, M, rule)
    differing = 0
    for h in range(H):
        if kept_gpu[h].tolist() != ref_kept[h].tolist():
            differing += 1
            a, b = set(kept_gpu[h].tolist()), set(ref_kept[h].tolist())
            sym = sorted(a ^ b)
            # the tokens that competed by score: image tokens before the window, or, under the literal rule
            # with a budget below the protected count, text tokens before the window
            competing = 1 if B >= oracle.protected_count(mask, M) else 0
            kept_cmp = [j for j in ref_kept[h] if mask[j] == competing and j < len(mask) - M]
            thr = min(ref_scores[h][j] for j in kept_cmp)
            for j in sym:
                rel = abs(ref_scores[h][j] - thr) / thr
                assert rel <= TIE_SCORE, f"head {h}: position {j} differs outside the tie band (rel {rel:.2e})"
    return differing


def boundary_margin(ref_scores_h, ref_kept_h, mask, B, M):
    """Relative gap between the lowest conserved and the highest evicted competing score of one head (fp64 oracle):
    how far the selection threshold is from a tie.  None when nothing competes."""
    L = len(mask)
    competing = 1 if B >= oracle.protected_count(mask, M) else 0
    comp = np.flatnonzero((mask == competing) & (np.arange(L) < L - M))
    kept = np.intersect1d(comp, ref_kept_h)
    ev = np.setdiff1d(comp, ref_kept_h)
    if len(kept) == 0 or len(ev) == 0:
        return None
    lo, hi = ref_scores_h[kept].min(), ref_scores_h[ev].max()
    return float((lo - hi) / lo)


def check_nearest(k_head_f32: np.ndarray, kept, evicted, assign_gpu, sim_gpu, with_error=False):
    """k_head_f32: [L, d] float32 (exact widening).  Returns the number of tie-band disagreements (and, with
    ``with_error``, the largest cosine error over the rows that agree)."""
    a_ref, s_ref = oracle.nearest(k_head_f32, kept, evicted)
    bad = np.flatnonzero(a_ref != assign_gpu)
    k64 = k_head_f32.astype(np.float64)
    for e in bad:
        ki, kj = k64[evicted[e]], k64[kept[assign_gpu[e]]]
        c = (ki @ kj) / (np.sqrt(ki @ ki) * np.sqrt(kj @ kj))
        assert s_ref[e] - c <= TIE_COS, f"evicted {evicted[e]}: kernel chose cos {c:.7f}, best is {s_ref[e]:.7f}"
    ok = a_ref == assign_gpu
    np.testing.assert_allclose(sim_gpu[ok], s_ref[ok], rtol=0, atol=SIM_ATOL)
    if with_error:
        return int(bad.size), float(np.abs(sim_gpu[ok] - s_ref[ok]).max()) if ok.any() else 0.0
    return int(bad.size)


def check_merge(x_head_f32, kept, evicted, assign, sim, mode, out_gpu, dtype):
    ref = oracle.merge(x_head_f32, kept, evicted, assign, sim.astype(np.float64), mode)
    err = np.abs(out_gpu.astype(np.float64) - ref)
    assert err.max() <= MERGE_ATOL[dtype], f"merged rows off by {err.max():.3e}"
    # rows without members are bit copies
    n = np.bincount(assign, minlength=len(kept)) if mode != "none" and len(evicted) else np.zeros(len(kept), int)
    untouched = n == 0
    np.testing.assert_array_equal(out_gpu[untouched].astype(np.float64), x_head_f32[kept][untouched].astype(np.float64))
    return float(err.max())


def run_and_check(w, mode, heads=None, layer=0, oracle_heads=None, B=None, M=None, rule="protect_text", label=None):
    """Full path on the GPU for workload ``w`` (all heads, or ``heads``): the stage-exact checks on every head, the
    fp64 oracle on ``oracle_heads`` (indices into the generated heads; default all).  Returns the statistics."""
    q, k, v, mask = W.generate(w, layer, heads)
    B = w.budget() if B is None else B
    M = w.M if M is None else M
    return run_and_check_tensors(q, k, v, mask, B, M, mode, rule, label or w.name, layer, oracle_heads)


def run_and_check_tensors(q, k, v, mask, B, M, mode, rule="protect_text", label="", layer=0, oracle_heads=None):
    """The same for inputs made by the caller (CPU tensors q, k, v [H, L, d] and mask [L])."""
    qg, kg, vg, mg = to_gpu(q, k, v, mask)
    H, L, d = q.shape
    ws = lookm.alloc_workspace(H, L, d, B, lookm._dt(qg), qg.device)
    # first without the scores: the second score pass may then skip the keys that do not compete in the selection
    # (matrix-core path, default rule); the cache must come out bit for bit as when every score is computed
    lean = lookm.lookm_compress(qg, kg, vg, mg, B, M, mode, want_scores=False, rule=rule, workspace=ws)
    lean = (lean.kept_idx.clone(), lean.k_out.clone(), lean.v_out.clone())
    res = lookm.lookm_compress(qg, kg, vg, mg, B, M, mode, want_scores=True, rule=rule, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(lean[0], res.kept_idx) and torch.equal(lean[1], res.k_out) and torch.equal(lean[2], res.v_out), \
        "the call without scores_out gives a different cache"
    st = check_outputs(q, k, v, mask, B, M, mode, rule, res, ws, oracle_heads)
    st = dict(workload=label, layer=layer, mode=mode, rule=rule, H=H, L=L, B=B, M=M, **st)
    return record(**st)


def check_outputs(q, k, v, mask, B, M, mode, rule, res, ws, oracle_heads=None):
    """The checks of run_and_check on a finished call: q, k, v, mask the CPU inputs, ``res`` the call's outputs
    (with scores), ``ws`` its workspace (None when a later call has reused it: the matching is then taken from the
    stage call lookm_nearest on the call's kept set, which computes the same values)."""
    H, L, d = q.shape
    kept_g = res.kept_idx.cpu().numpy()
    scores_g = res.scores.cpu().numpy()
    mask_np = mask.numpy()
    # structure, every head
    assert kept_g.shape == (H, B)
    assert np.all(np.diff(kept_g, axis=1) > 0) and kept_g.min() >= 0 and kept_g.max() < L
    prot = np.flatnonzero((mask_np == 0) | (np.arange(L) >= L - M))
    if B < len(prot):                      # literal rule below the protected count: only the window is sure,
        prot = np.arange(L - M, L)         # and no image token before it may be conserved
        for h in range(H):
            assert not np.any(mask_np[kept_g[h][kept_g[h] < L - M]] == 1), f"head {h}: an image token was conserved"
    for h in range(H):
        assert np.isin(prot, kept_g[h]).all(), f"head {h}: a protected position was evicted"
    np.testing.assert_allclose(scores_g.astype(np.float64).sum(1), L, rtol=2e-5)

    oh = list(range(H)) if oracle_heads is None else list(oracle_heads)
    stats = dict(heads=H, heads_oracle=len(oh), kept_diff_heads=0, min_margin=None, nearest_tie_rows=0,
                 rows_matched=0, score_relerr=0.0, sim_abserr=0.0, merge_abserr=0.0)
    merging = mode != "none" and 0 < B < L
    dt = lookm._dt(res.k_out)
    if merging and ws is None:
        ev_ws = np.stack([np.setdiff1d(np.arange(L, dtype=np.int32), kept_g[h]) for h in range(H)])
        a2, s2 = lookm.lookm_nearest(k.cuda(), res.kept_idx, torch.from_numpy(ev_ws).cuda())
        assign_g, sim_g = a2.cpu().numpy(), s2.cpu().numpy()
    elif merging:
        # what the call itself computed, read back from its workspace
        ev_ws = lookm.workspace_view(ws, "evicted", H, H, L, d, B, dt).cpu().numpy()
        assign_g = lookm.workspace_view(ws, "assign", H, H, L, d, B, dt).cpu().numpy()
        sim_g = lookm.workspace_view(ws, "sim", H, H, L, d, B, dt).cpu().numpy()
        assert assign_g.min() >= 0 and assign_g.max() < B
        # the stage call reproduces the in-path matching bit for bit
        a2, s2 = lookm.lookm_nearest(k.cuda(), res.kept_idx, torch.from_numpy(ev_ws).cuda())
        assert np.array_equal(a2.cpu().numpy(), assign_g) and np.array_equal(s2.cpu().numpy(), sim_g)
    else:
        ev_ws = np.stack([np.setdiff1d(np.arange(L, dtype=np.int32), kept_g[h]) for h in range(H)]) if B < L \
            else np.zeros((H, 0), np.int32)
        assign_g = np.zeros(ev_ws.shape, np.int32)
        sim_g = np.ones(ev_ws.shape, np.float32)
    # stage-exact, every head
    check_select_stage(kept_g, ev_ws, scores_g, mask_np, B, M, rule)
    k_out = res.k_out.float().cpu().numpy()
    v_out = res.v_out.float().cpu().numpy()
    kf, vf = k.float().numpy(), v.float().numpy()
    for h in range(H):
        for x, o in ((kf, k_out), (vf, v_out)):
            stats["merge_abserr"] = max(stats["merge_abserr"],
                                        check_merge(x[h], kept_g[h], ev_ws[h], assign_g[h], sim_g[h], mode, o[h], q.dtype))
    # end to end against the fp64 oracle, sampled heads
    if oh:                                 # one head per thread: the C oracle runs outside the interpreter lock
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            ref_scores = np.stack(list(pool.map(lambda h: oracle.scores(q[h], k[h]), oh)))
    for n, h in enumerate(oh):
        stats["score_relerr"] = max(stats["score_relerr"], check_scores(scores_g[h].astype(np.float64), ref_scores[n]))
        ref_kept, _ = oracle.select(ref_scores[n], mask_np, B, M, rule)
        stats["kept_diff_heads"] += check_kept(kept_g[h:h + 1], scores_g[h:h + 1], ref_scores[n:n + 1], ref_kept[None],
                                               mask_np, B, M, rule)
        mg = boundary_margin(ref_scores[n], ref_kept, mask_np, B, M)
        if mg is not None:
            stats["min_margin"] = mg if stats["min_margin"] is None else min(stats["min_margin"], mg)
    # the matching against the oracle's, every head (the oracle is given the call's own kept and evicted lists, so
    # this holds whatever the selection did); the C oracle runs outside the interpreter lock, one head per thread
    if merging:
        with ThreadPoolExecutor(max_workers=min(16, os.cpu_count() or 1)) as pool:
            outcomes = list(pool.map(lambda h: check_nearest(kf[h], kept_g[h], ev_ws[h], assign_g[h], sim_g[h],
                                                             with_error=True), range(H)))
        stats["rows_matched"] = H * (L - B)
        stats["nearest_tie_rows"] = sum(t for t, _ in outcomes)
        stats["sim_abserr"] = max(e for _, e in outcomes)
    return stats
