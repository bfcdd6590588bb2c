"""The library enqueues kernels only - no allocation, no memset, no synchronisation on the compression and decode
paths - so a caller can capture them into a HIP graph.  Captured once and replayed several times with eager work and
synchronisations in between, every replay has to reproduce the eager results bit for bit."""
import pytest
import torch

from paper_2406_18139_amd import lookm
from paper_2406_18139_amd import workloads as W

pytestmark = pytest.mark.gpu


def _eager_noise(dev):
    # unrelated eager work between replays: touches the allocator and the default stream
    x = torch.randn(1 << 16, device=dev)
    (x * 2 + 1).sum().item()


def test_compress_replays_in_a_hip_graph():
    w = W.LLAVA7B
    q, k, v, mask = W.generate(w)
    dev = torch.device("cuda:0")
    qg, kg, vg, mg = (t.to(dev) for t in (q, k, v, mask))
    B, M, mode = w.budget(), w.M, w.modes[0]
    dt = lookm.BF16 if w.dtype == "bf16" else lookm.F32
    ref = lookm.lookm_compress(qg, kg, vg, mg, B, M, mode)
    out = lookm.alloc_outputs(w.H, w.L, w.d, B, qg.dtype, dev)
    ws = lookm.alloc_workspace(w.H, w.L, w.d, B, dt, dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                      # one warm-up call on the capture stream, as torch asks
        lookm.lookm_compress(qg, kg, vg, mg, B, M, mode, out=out, workspace=ws, check=False)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lookm.lookm_compress(qg, kg, vg, mg, B, M, mode, out=out, workspace=ws, check=False)
    for rep in range(4):
        out.k_out.zero_(); out.v_out.zero_(); out.kept_idx.zero_(); out.status.fill_(-99)
        _eager_noise(dev)
        graph.replay()
        torch.cuda.synchronize()
        assert int(out.status.item()) == 0, rep
        assert torch.equal(out.kept_idx, ref.kept_idx), rep
        assert torch.equal(out.k_out, ref.k_out) and torch.equal(out.v_out, ref.v_out), rep
        _eager_noise(dev)


def test_decode_replays_in_a_hip_graph():
    dev = torch.device("cuda:0")
    H, S, d = 32, 2276, 128
    g = torch.Generator(device=dev).manual_seed(11)
    q = torch.randn((H, d), generator=g, device=dev).to(torch.bfloat16)
    k = torch.randn((H, S, d), generator=g, device=dev).to(torch.bfloat16)
    v = torch.randn((H, S, d), generator=g, device=dev).to(torch.bfloat16)
    ref = lookm.lookm_decode_attention(q, k, v)
    out = torch.empty_like(ref)
    ws = torch.empty(int(lookm.lib().lookm_decode_workspace_bytes(H, d)) + 256, dtype=torch.uint8, device=dev)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lookm.lookm_decode_attention(q, k, v, out=out, workspace=ws)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lookm.lookm_decode_attention(q, k, v, out=out, workspace=ws)
    for rep in range(4):
        out.zero_()
        _eager_noise(dev)
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, ref), rep
    # new inputs in the same buffers: the graph reads them at replay time
    q.copy_(torch.randn((H, d), generator=g, device=dev).to(torch.bfloat16))
    ref2 = lookm.lookm_decode_attention(q, k, v)
    graph.replay()
    torch.cuda.synchronize()
    assert torch.equal(out, ref2)


def test_batch_replays_in_a_hip_graph():
    """Under capture the batch call creates no stream or event: its jobs go onto the captured stream in order."""
    w = W.LLAVA7B
    dev = torch.device("cuda:0")
    B, M = w.budget(), w.M
    layers = []
    for i in range(3):
        q, k, v, mask = W.generate(w, heads=[i, i + 5])
        layers.append(tuple(t.to(dev) for t in (q, k, v, mask)))
    H, L, d = layers[0][0].shape
    ref = [lookm.lookm_compress(*t, B, M, "pivotal") for t in layers]
    outs = [lookm.alloc_outputs(H, L, d, B, layers[0][0].dtype, dev) for _ in layers]
    wss = [lookm.alloc_workspace(H, L, d, B, lookm._dt(layers[0][0]), dev) for _ in layers]
    jobs = [lookm.make_job(*t, B, M, "pivotal", o, x) for t, o, x in zip(layers, outs, wss)]
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        lookm.lookm_compress_batch(jobs)            # warm-up on a side stream
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lookm.lookm_compress_batch(jobs)
    for rep in range(3):
        for o in outs:
            o.k_out.zero_(); o.v_out.zero_(); o.kept_idx.zero_(); o.status.fill_(-99)
        _eager_noise(dev)
        graph.replay()
        torch.cuda.synchronize()
        for a, b in zip(ref, outs):
            assert int(b.status.item()) == 0, rep
            assert torch.equal(a.kept_idx, b.kept_idx) and torch.equal(a.k_out, b.k_out) and torch.equal(a.v_out, b.v_out), rep


def test_capture_of_a_shape_no_earlier_call_has_used():
    """Kernel attributes are set for every template instance on the library's first use of a device (or by
    lookm_init), never lazily inside a launcher: a shape whose kernels no earlier call has launched - here 20 000
    evicted keys, the similarity-set sort with the most entries per thread - can be captured directly."""
    dev = torch.device("cuda:0")
    lookm.lookm_init()
    H, L, d, B, M = 2, 21000, 128, 1000, 16
    g = torch.Generator(device=dev).manual_seed(3)
    q, k, v = (torch.randn((H, L, d), generator=g, device=dev).to(torch.bfloat16) for _ in range(3))
    mask = torch.ones(L, dtype=torch.uint8, device=dev)
    out = lookm.alloc_outputs(H, L, d, B, q.dtype, dev)
    ws = lookm.alloc_workspace(H, L, d, B, lookm.BF16, dev)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        lookm.lookm_compress(q, k, v, mask, B, M, "averaged", out=out, workspace=ws, check=False)
    graph.replay()
    torch.cuda.synchronize()
    ref = lookm.lookm_compress(q, k, v, mask, B, M, "averaged")
    for rep in range(2):
        out.k_out.zero_(); out.kept_idx.zero_(); out.status.fill_(-99)
        _eager_noise(dev)
        graph.replay()
        torch.cuda.synchronize()
        assert int(out.status.item()) == 0
        assert torch.equal(out.kept_idx, ref.kept_idx) and torch.equal(out.k_out, ref.k_out) and torch.equal(out.v_out, ref.v_out)
