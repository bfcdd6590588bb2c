#!/usr/bin/env python3
"""Benchmark of the LOOK-M prefill-time KV-cache compression path on one MI355X.

A "step" is one lookm_compress call: every kernel of the path (two score passes, selection, key
norms, cosine matching, similarity sets, merge + compaction) over all heads of one layer of the
headline workload (20 images x 576 tokens interleaved with 21 text spans, L = 12 644, 32 heads,
head_dim 128, bf16, budget = text + recent + 10 % of the evictable image tokens, pivotal merging).
Inputs are seeded synthetic tensors, resident in HBM before the timed region.

Prints ONE JSON line: throughput (prompt KV tokens compressed per second per layer), the roofline of
the dominant kernel (measured live with HIP events on the launch stream), per-kernel figures, and the
CPU oracle timed on a bounded sample of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import torch

from paper_2406_18139_amd import lookm
from paper_2406_18139_amd import workloads as W

PEAK_MFMA_BF16 = 2.5e15   # dense bf16 MFMA, FLOP/s
PEAK_HBM = 8.0e12         # B/s


PREWARM_SECONDS = 0.3     # untimed calls before the counted warm-up, sized by time


def prewarm(step, seconds: float = PREWARM_SECONDS):
    """Runs ``step`` until ``seconds`` of wall-clock have passed (at least 3 calls): after an idle period the GPU
    needs some tens of milliseconds under load before its clocks settle, whatever warm-up count the caller asked for.
    Returns (calls, milliseconds)."""
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    n = 0
    while n < 3 or time.perf_counter() - t0 < seconds:
        for _ in range(4):
            step()
        torch.cuda.synchronize()
        n += 4
    return n, (time.perf_counter() - t0) * 1e3


def algorithmic_work(w: W.Workload, score_window: int = 0, all_scores: bool = True) -> dict:
    """Work the method needs per launch of each kernel (all heads of one layer); nothing a particular
    tiling adds (masked halves of diagonal tiles, padding, re-reads) is counted.  ``all_scores`` False: the caller
    does not ask for the scores themselves, so pass 2 only owes the scores of the keys that compete in the selection
    (image tokens before the recent window, Eq. 5-8)."""
    H, L, d, B = w.H, w.L, w.d, w.budget()
    Le = L - B
    e = 2 if w.dtype == "bf16" else 4
    r0 = L - score_window if score_window > 0 else 0
    pairs = L * (L + 1) // 2 - r0 * (r0 + 1) // 2          # causal pairs of the query rows that count
    pairs2 = pairs                                         # pairs pass 2 owes
    if not all_scores and w.dtype == "bf16" and d == 128:
        m = w.mask()
        pairs2 = sum(L - max(j, r0) for j in range(L - w.M) if m[j] == 1)
    return {
        "score_lse": ("mfma", 2.0 * d * pairs * H),
        "score_lse_fold": ("hbm", H * 4.0 * L * 3),        # two partials in, one value out (at least one chunk)
        "score_colsum": ("mfma", 2.0 * d * pairs2 * H),
        "score_colsum_fold": ("hbm", H * 4.0 * L * 2),
        "select": ("hbm", H * (4.0 * L + 4.0 * B + 4.0 * Le) + L),
        "rnorm": ("hbm", H * (L * d * e + 4.0 * L)),
        "nearest": ("mfma", 2.0 * d * Le * B * H),
        "nearest_fold": ("hbm", H * (Le * (8.0 + 4.0 + 4.0 + 4.0 + 4.0))),   # one partial, position, norm in; assign + sim out
        "bucket": ("hbm", H * (4.0 * Le + 4.0 * (B + 1) + 4.0 * Le)),
        "merge": ("hbm", H * (2.0 * L * d * e + 2.0 * B * d * e + 4.0 * B + 12.0 * Le + 4.0 * (B + 1))),
    }


def stack(args) -> int:
    """The full 7B-shaped stack: 32 layers x 4 ragged prompts (4K, 6K, 9K, 12K tokens), weighted merging.  A step is
    the compression of all 128 (prompt, layer) caches by ONE lookm_compress_batch call on one stream.  Inputs are drawn
    on the GPU with a seeded generator (same recipe as the host generator) and all stay resident (about 25 GB)."""
    dev = torch.device("cuda:0")
    prompts = W.stack_prompts()
    layers = W.STACK_LAYERS
    per_prompt = []
    for w in prompts:
        B = w.budget()
        out = lookm.alloc_outputs(w.H, w.L, w.d, B, w.torch_dtype(), dev)
        ws = lookm.alloc_workspace(w.H, w.L, w.d, B, lookm.BF16, dev)
        per_prompt.append([(w, B, *W.generate_on_device(w, layer, dev), out, ws) for layer in range(layers)])
    # Layer-major order, as a prefill produces the caches: layer 0 of every prompt, then layer 1, ...  The layers of a
    # prompt share its workspace and outputs and therefore run in order; different prompts are independent, and the
    # library alternates them between the two streams it is given (see lookm_compress_batch_two_streams).
    jobs = [per_prompt[p][layer] for layer in range(layers) for p in range(len(prompts))]
    torch.cuda.synchronize()
    batch = [lookm.make_job(q, k, v, mask, B, w.M, "weighted", out, ws) for w, B, q, k, v, mask, out, ws in jobs]

    aux = torch.cuda.Stream() if args.two_streams else None

    def step():
        lookm.lookm_compress_batch(batch, aux_stream=aux)

    prewarm_calls, prewarm_ms = prewarm(step, 0.2)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    ms = (time.perf_counter() - t0) / args.steps * 1e3
    bad = [int(pp[0][6].status.item()) for pp in per_prompt]
    if any(bad):
        print(f"bench.py: device status {bad}", file=sys.stderr)
        return 1
    # Roofline: the score passes are 87 % of the stack's arithmetic.  Per-kernel durations of one job per prompt
    # (layer 0) come from HIP events recorded by the library on the launch stream; the dominant kernel of the stack
    # is the first score pass of the longest prompt.
    score_flop = 0.0
    for w in prompts:                      # pass 1 over all pairs, pass 2 over the competing keys' pairs (no scores_out)
        wk = algorithmic_work(w, all_scores=False)
        score_flop += (wk["score_lse"][1] + wk["score_colsum"][1]) * layers
    per_prompt_kernels = {}
    dom = None
    for pi, w in enumerate(prompts):
        kms = lookm.lookm_job_profile(batch[pi], 5)
        kms.pop("rnorm", None)
        per_prompt_kernels[w.name] = {k_: round(v_, 5) for k_, v_ in kms.items()}
        name = max(kms, key=kms.get)
        if dom is None or kms[name] > dom[2]:
            dom = (w, name, kms[name])
    dw, dname, dms = dom
    dwork = algorithmic_work(dw, all_scores=False)[dname]
    dach = dwork[1] / (dms * 1e-3)
    dpeak = PEAK_MFMA_BF16 if dwork[0] == "mfma" else PEAK_HBM
    roofline = {"kernel": f"{dname} of prompt {dw.name} (L={dw.L})", "bound": dwork[0],
                "achieved": round(dach / (1e12 if dwork[0] == "mfma" else 1e9), 3),
                "peak": dpeak / (1e12 if dwork[0] == "mfma" else 1e9),
                "unit": "TFLOP/s" if dwork[0] == "mfma" else "GB/s", "frac": round(dach / dpeak, 4), "traffic": None,
                "score_passes_whole_stack": {"flop": score_flop,
                                             "frac_mfma_peak_over_step_time": round(score_flop / (ms * 1e-3) / PEAK_MFMA_BF16, 4)}}
    tokens = sum(w.L for w in prompts)
    per_token = layers * prompts[0].H * prompts[0].d * 2 * 2          # K and V, bf16, all layers and heads
    total_b = tokens * per_token
    saved_b = sum(w.L - w.budget() for w in prompts) * per_token
    print(json.dumps({
        "metric": "compression time of the full stack (32 layers x 4 ragged prompts)", "value": round(ms, 3), "unit": "ms",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "prewarm": {"calls": prewarm_calls, "ms": round(prewarm_ms, 1)}, "ms_per_step": round(ms, 3),
        "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic (drawn on the GPU)",
        "config": {"workload": "stack: 32 layers x 32 heads x d128 bf16, prompts of "
                               + ", ".join(str(w.L) for w in prompts) + " tokens, budgets "
                               + ", ".join(str(w.budget()) for w in prompts) + ", recent_window 32, merge=weighted",
                   "streams": 2 if args.two_streams else 1},
        "roofline": roofline, "kernels_ms_layer0": per_prompt_kernels,
        "tokens_per_s_all_layers": round(tokens * layers / (ms * 1e-3), 1),
        "cache_bytes": total_b, "cache_bytes_after": total_b - saved_b, "cache_bytes_saved": saved_b,
        "fraction_saved": round(saved_b / total_b, 4)}))
    return 0


def decode(args) -> int:
    """The step after the path (Eq. 3): one new token per head attends to the cache of the headline prompt, once
    uncompressed (L rows) and once compressed (B rows).  A step is one lookm_decode_attention call over all 32 heads
    of one layer; the figure Table 4 of the paper is about is the ratio of the two."""
    dev = torch.device("cuda:0")
    w = W.LONG
    B = w.budget()
    g = torch.Generator(device=dev)
    g.manual_seed(w.seed())
    dt = w.torch_dtype()
    q = torch.randn((w.H, w.d), generator=g, device=dev).to(dt)
    k = torch.randn((w.H, w.L, w.d), generator=g, device=dev).to(dt)
    v = torch.randn((w.H, w.L, w.d), generator=g, device=dev).to(dt)
    out = torch.empty((w.H, w.d), dtype=dt, device=dev)
    ws = torch.empty(int(lookm.lib().lookm_decode_workspace_bytes(w.H, w.d)) + 256, dtype=torch.uint8, device=dev)
    # the headline budget, and the two total budgets of the paper's efficiency table (20 % and 5 % of the prompt)
    cases = (("full", w.L), ("compressed", B), ("budget_20pct", int(0.20 * w.L + 0.5)), ("budget_5pct", int(0.05 * w.L + 0.5)))
    res = {}
    for name, S in cases:
        kk, vv = k[:, :S].contiguous(), v[:, :S].contiguous()    # same bytes per row as a compressed cache
        # The two launches of a step are captured into a HIP graph and replayed: a decoding loop is launch-bound
        # from Python (about 30 us per eager call), and a serving loop would replay a graph as well.
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            lookm.lookm_decode_attention(q, kk, vv, out=out, workspace=ws)
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph):
            lookm.lookm_decode_attention(q, kk, vv, out=out, workspace=ws)
        for _ in range(args.warmup):
            graph.replay()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            graph.replay()
        torch.cuda.synchronize()
        ms = (time.perf_counter() - t0) / args.steps * 1e3
        nbytes = 2.0 * w.H * S * w.d * 2 + 2.0 * w.H * w.d * 2
        res[name] = {"rows": S, "ms": round(ms, 5), "GB/s": round(nbytes / (ms * 1e-3) / 1e9, 1),
                     "frac_hbm_peak": round(nbytes / (ms * 1e-3) / PEAK_HBM, 4),
                     "cache_GiB_32_layers": round(32 * 2.0 * w.H * S * w.d * 2 / 2**30, 3)}
    c = res["compressed"]
    print(json.dumps({
        "metric": "decode-step attention over the compressed cache of the 12K-token prompt (one layer, 32 heads)",
        "value": round(c["ms"] * 1e3, 2), "unit": "us", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": c["ms"], "higher_is_better": False, "scaling": "weak", "vs_baseline": None, "dtype": w.dtype,
        "data": "synthetic (drawn on the GPU)",
        "config": {"workload": f"decode: {w.H} heads x d{w.d} {w.dtype}, cache of {B} rows (compressed) vs {w.L} rows (full)"},
        "roofline": {"kernel": "decode (partial + merge launches)", "bound": "hbm", "achieved": c["GB/s"], "peak": 8000.0,
                     "unit": "GB/s", "frac": c["frac_hbm_peak"], "traffic": None},
        "full_cache": res["full"], "compressed_cache": c,
        "budget_20pct": res["budget_20pct"], "budget_5pct": res["budget_5pct"],
        "speedup_over_full_cache": round(res["full"]["ms"] / c["ms"], 2)}))
    return 0


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=None, help="timed steps (default 100; 10 for --workload stack)")
    ap.add_argument("--warmup", type=int, default=None, help="untimed steps (default 25; 2 for --workload stack)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--workload", default="long", choices=["long", "long_total", "long_noprior", "llava7b", "stack", "decode"])
    ap.add_argument("--reuse-lse", action="store_true",
                    help="supply the prefill's row log-sum-exp (lookm_compress_lse): the first score pass is skipped")
    ap.add_argument("--score-window", type=int, default=0,
                    help="variant: scores from the last W query rows only (lookm_scores_window), via a lookm_job")
    ap.add_argument("--one-stream", dest="two_streams", action="store_false",
                    help="--workload stack: enqueue all jobs on one stream (default: lookm_compress_batch_two_streams)")
    ap.add_argument("--with-scores", action="store_true",
                    help="also return the scores A_s of every key (scores_out): the second score pass then runs over "
                         "all keys, not only over the image tokens that compete in the selection")
    ap.add_argument("--split-heads", type=int, default=0,
                    help="issue the layer as this many jobs over equal groups of heads through ONE "
                         "lookm_compress_batch_two_streams call (0: one lookm_compress call on one stream)")
    ap.add_argument("--probe-mfma", action="store_true",
                    help="only measure the sustained rate of the bf16 MFMA instruction from registers (constant and "
                         "random operands, 1-3 waves per SIMD) and exit")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run a plain 1 GiB device-to-device copy kernel (to scale HBM byte counters) and exit")
    args = ap.parse_args()
    # One layer takes under 2 ms, and the first ~15 calls after an idle GPU run up to 20 % slower while its clocks
    # ramp up (seen in the kernel trace): the default warm-up covers that, the timed steps are steady state.
    if args.steps is None:
        args.steps = 10 if args.workload == "stack" else 100
    if args.warmup is None:
        args.warmup = 2 if args.workload == "stack" else 25
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus above 1 is not supported "
              "(the path shards over heads / layers / prompts with no exchange).", file=sys.stderr)
        return 2
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible; the compression path has no CPU fallback.", file=sys.stderr)
        return 2

    if args.calibrate_copy:
        n = 1 << 28                                       # 2^28 floats = 1 GiB read + 1 GiB written per copy
        src = torch.arange(n, dtype=torch.float32, device="cuda:0")
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibration": "copy", "bytes_read": 4 * n, "bytes_written": 4 * n, "copies": 3}))
        return 0

    if args.probe_mfma:
        res = {}
        for mode, name in ((0, "32x32x16_constant"), (1, "32x32x16_random"), (2, "16x16x32_random")):
            for wps in (1, 2, 3):
                res[f"{name}_operands_{wps}_waves_per_simd"] = round(
                    lookm.lookm_probe_mfma(mode, wps, iters=2048 * 3 // wps, reps=20), 1)
        print(json.dumps({"probe": "bf16 MFMA from registers, blocks of 64 x 32 x 128 multiply-adds: 16 of "
                                   "v_mfma_f32_32x32x16_bf16 in two chains, or 32 of v_mfma_f32_16x16x32_bf16 on eight "
                                   "accumulators",
                          "unit": "TFLOP/s", "datasheet_peak": PEAK_MFMA_BF16 / 1e12, "sustained": res}))
        return 0

    if args.workload == "stack":
        return stack(args)
    if args.workload == "decode":
        return decode(args)

    w = {"long": W.LONG, "long_total": W.LONG_TOTAL, "long_noprior": W.LONG_NOPRIOR, "llava7b": W.LLAVA7B}[args.workload]
    mode = w.modes[0]
    B, M = w.budget(), w.M
    q, k, v, mask = W.generate(w)
    dev = torch.device("cuda:0")
    qg, kg, vg, mg = (t.to(dev) for t in (q, k, v, mask))
    out = lookm.alloc_outputs(w.H, w.L, w.d, B, qg.dtype, dev, want_scores=args.with_scores)
    ws = lookm.alloc_workspace(w.H, w.L, w.d, B, lookm.BF16 if w.dtype == "bf16" else lookm.F32, dev)

    row_lse = None
    if args.reuse_lse:
        # what a flash-style prefill would hand over; prepared here with library ops, outside the timed region
        row_lse = torch.empty((w.H, w.L), dtype=torch.float32, device=dev)
        causal = torch.ones((w.L, w.L), dtype=torch.bool, device=dev).triu(1)
        for h in range(w.H):
            logits = (qg[h].float() @ kg[h].float().T) / (w.d ** 0.5)
            row_lse[h] = torch.logsumexp(logits.masked_fill_(causal, float("-inf")), dim=-1)
        del causal, logits

    variant = args.reuse_lse or args.score_window > 0
    job = lookm.make_job(qg, kg, vg, mg, B, M, mode, out, ws, row_lse=row_lse, score_window=args.score_window)

    split_jobs, aux = None, None
    if args.split_heads > 1:
        # the same layer as independent jobs over groups of heads (own workspace, own slice of the outputs), handed to
        # the library in one call with a second stream: the short kernels of one group run under the long ones of another
        n = args.split_heads
        assert w.H % n == 0
        g = w.H // n
        aux = torch.cuda.Stream()
        dtc = lookm.BF16 if w.dtype == "bf16" else lookm.F32
        split_jobs, split_keep = [], []
        for i in range(n):
            sl = slice(i * g, (i + 1) * g)
            o = lookm.Compressed(out.k_out[sl], out.v_out[sl], out.kept_idx[sl], None,
                                 torch.zeros(1, dtype=torch.int32, device=dev))
            wsi = lookm.alloc_workspace(g, w.L, w.d, B, dtc, dev)
            split_keep.append((o, wsi))
            split_jobs.append(lookm.make_job(qg[sl], kg[sl], vg[sl], mg, B, M, mode, o, wsi,
                                             row_lse=None if row_lse is None else row_lse[sl],
                                             score_window=args.score_window))

    def step():
        if split_jobs is not None:
            lookm.lookm_compress_batch(split_jobs, aux_stream=aux)
        elif variant:
            lookm.lookm_compress_batch([job])
        else:
            lookm.lookm_compress(qg, kg, vg, mg, B, M, mode, out=out, workspace=ws, check=False)

    prewarm_calls, prewarm_ms = prewarm(step)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    ms_per_step = dt / args.steps * 1e3
    status = int(out.status.item()) if split_jobs is None else min(int(o.status.item()) for o, _ in split_keep)
    if status != 0:
        print(f"bench.py: device status {status}", file=sys.stderr)
        return 1

    # per-kernel durations: HIP events recorded by the library on the launch stream, same inputs
    kms = lookm.lookm_job_profile(job, max(min(args.steps, 30), 1))
    work = algorithmic_work(w, args.score_window, all_scores=args.with_scores)
    if args.reuse_lse:
        kms.pop("score_lse"), kms.pop("score_lse_fold")          # not launched: the prefill's values are used
    kernels = {}
    event_gap_ms = None
    if w.dtype == "bf16" and w.d == 128:
        # on the matrix-core path the key norms come out of score pass 2 and no norm kernel is launched: its slot
        # is an empty interval between two events, i.e. what the event records themselves cost on the stream
        event_gap_ms = kms.pop("rnorm")
    for name, ms in kms.items():
        bound, amount = work[name]
        peak = PEAK_MFMA_BF16 if bound == "mfma" else PEAK_HBM
        ach = amount / (ms * 1e-3) if ms > 0 else 0.0
        kernels[name] = {"ms": round(ms, 5), "bound": bound,
                         "achieved": round(ach / (1e12 if bound == "mfma" else 1e9), 3),
                         "unit": "TFLOP/s" if bound == "mfma" else "GB/s", "frac": round(ach / peak, 4)}
    dominant = max(kms, key=kms.get)
    dbound, damount = work[dominant]
    dpeak = PEAK_MFMA_BF16 if dbound == "mfma" else PEAK_HBM
    dach = damount / (kms[dominant] * 1e-3)
    # HBM bytes per launch of that kernel, from the committed rocprofv3 --pmc summary (scaled by the copy
    # calibration); None when no summary covers this workload / kernel
    traffic, traffic_source = None, None
    tfile = os.path.join(os.path.dirname(os.path.abspath(__file__)), "profiles", f"hbm_traffic_{w.name}.json")
    if os.path.exists(tfile) and not variant and split_jobs is None:
        with open(tfile) as f:
            stored = json.load(f)
        traffic = stored.get("bytes_per_launch", {}).get(dominant)
        if traffic is not None:
            traffic_source = (f"stored counter figure, not of this run: profiles/hbm_traffic_{w.name}.json "
                              f"({stored.get('measured', 'date not recorded')}; rocprofv3 --pmc FETCH_SIZE, WRITE_SIZE, "
                              "scaled by the copy calibration)")
    roofline = {"kernel": dominant, "bound": dbound,
                "achieved": round(dach / (1e12 if dbound == "mfma" else 1e9), 3),
                "peak": dpeak / (1e12 if dbound == "mfma" else 1e9),
                "unit": "TFLOP/s" if dbound == "mfma" else "GB/s",
                "frac": round(dach / dpeak, 4), "traffic": traffic, "traffic_source": traffic_source}
    score_ms = kms.get("score_lse", 0.0) + kms.get("score_lse_fold", 0.0) + kms["score_colsum"] + kms["score_colsum_fold"]
    smc_ms = kms["select"] + kms["bucket"] + kms["merge"]
    smc_bytes = work["select"][1] + work["bucket"][1] + work["merge"][1]
    groups = {
        "score_passes": {"ms": round(score_ms, 4), "frac_mfma_peak": round(
            ((0.0 if args.reuse_lse else work["score_lse"][1]) + work["score_colsum"][1]) / (score_ms * 1e-3)
            / PEAK_MFMA_BF16, 4)},
        "select_bucket_merge": {"ms": round(smc_ms, 4), "GB/s": round(smc_bytes / (smc_ms * 1e-3) / 1e9, 1),
                                "frac_hbm_peak": round(smc_bytes / (smc_ms * 1e-3) / PEAK_HBM, 4)},
    }

    cpu_baseline = None
    if not args.no_cpu_baseline and not variant:
        import oracle
        threads = oracle.num_threads()
        n_heads = max(1, min(w.H, threads))
        t1 = time.perf_counter()
        oracle.compress(q[:n_heads], k[:n_heads], v[:n_heads], mask.numpy(), B, M, mode)
        sec = time.perf_counter() - t1
        layer_sec = sec * w.H / n_heads
        cpu_baseline = {"value": round(w.L / layer_sec, 3), "unit": "tokens/s/layer", "cores": min(threads, n_heads),
                        "kind": "oracle", "seconds": round(sec, 2),
                        "sample": f"heads 0..{n_heads - 1} of {w.H} of the same layer (one head per thread), "
                                  f"scaled by {w.H}/{n_heads} to the whole layer"}

    # context for the MFMA-bound rooflines: what the matrix cores of this GPU sustain on the same instruction with
    # operands that change every instruction, from registers alone (measured after the timed region)
    mfma_sustained = None
    if w.dtype == "bf16":
        mfma_sustained = round(lookm.lookm_probe_mfma(2, 3, iters=2048, reps=20), 1)
        roofline["sustained_mfma_probe"] = {"value": mfma_sustained, "unit": "TFLOP/s",
                                            "what": "v_mfma_f32_16x16x32_bf16 (the score kernels' instruction) from "
                                                    "registers, random operands, 3 waves per SIMD (lookm_probe_mfma)",
                                            "same_with_32x32x16": round(lookm.lookm_probe_mfma(1, 3, iters=2048, reps=20), 1)}

    metric = "prompt KV tokens compressed/sec per layer (12K ctx)"
    if args.reuse_lse:
        metric += ", row log-sum-exp supplied by the prefill"
    if args.score_window > 0:
        metric += f", scores from the last {args.score_window} query rows only"
    line = {
        "metric": metric,
        "value": round(w.L / (ms_per_step * 1e-3), 1),
        "unit": "tokens/s/layer",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "prewarm": {"calls": prewarm_calls, "ms": round(prewarm_ms, 1),
                    "what": "untimed calls before the counted warm-up, until the clocks have settled"},
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": w.dtype, "data": "synthetic",
        "config": {"workload": f"{w.name}: {w.H} heads x d{w.d} {w.dtype}, {w.n_img} images x {w.img_tokens} tokens + "
                               f"{len(w.spans)} text spans, L={w.L}, budget B={B} (k_img={w.k_img()}), "
                               f"recent_window={M}, merge={mode}",
                   "H": w.H, "L": w.L, "d": w.d, "budget": B, "recent_window": M, "merge_mode": mode,
                   "row_lse_supplied": bool(args.reuse_lse), "score_window": args.score_window,
                   "split_heads": args.split_heads},
        "roofline": roofline,
        "cpu_baseline": cpu_baseline,
        "kernels": kernels,
        "groups": groups,
        "event_gap_ms": None if event_gap_ms is None else round(event_gap_ms, 5),
    }
    print(json.dumps(line))
    return 0


if __name__ == "__main__":
    sys.exit(main())
