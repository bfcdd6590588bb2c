"""GPU parity, stage by stage, through the C ABI: each kernel against the oracle function for the
same step, on sizes that span several tiles and a ragged tail, plus the degenerate cases."""
import numpy as np
import pytest
import torch

import oracle
from paper_2406_18139_amd import lookm
from tests import parity

pytestmark = pytest.mark.gpu


def rand_qk(H, L, d, dtype, seed, scale=1.0):
    g = torch.Generator().manual_seed(seed)
    q = (torch.randn(H, L, d, generator=g) * scale).to(dtype)
    k = (torch.randn(H, L, d, generator=g) * scale).to(dtype)
    return q, k


@pytest.mark.parametrize("H,L,d,dtype", [
    (3, 700, 128, torch.bfloat16),      # matrix-core path: 3 strips of 256, ragged tail
    (2, 256, 128, torch.bfloat16),      # exactly one strip
    (1, 1, 128, torch.bfloat16),        # single token
    (2, 65, 128, torch.bfloat16),
    (2, 333, 64, torch.bfloat16),       # portable path, bf16
    (2, 256, 64, torch.float32),        # the tiny configuration's shape
    (1, 130, 8, torch.float32),
    (1, 97, 256, torch.float32),
])
def test_scores_match_oracle(H, L, d, dtype):
    q, k = rand_qk(H, L, d, dtype, seed=L * 7 + d)
    s = lookm.lookm_scores(q.cuda(), k.cuda()).cpu().numpy().astype(np.float64)
    ref = oracle.scores(q, k)
    rel = np.abs(s - ref) / ref
    print(f"scores H={H} L={L} d={d} {dtype}: max rel err {rel.max():.3e}")
    assert rel.max() < 2e-5        # far inside the 1e-3 bar
    np.testing.assert_allclose(s.sum(1), L, rtol=1e-5)


@pytest.mark.parametrize("L", [2, 31, 63, 64, 127, 128, 129, 191, 255, 257, 320, 511, 513, 767, 1023, 1025, 1300])
def test_scores_around_tile_and_strip_boundaries(L):
    """Lengths on both sides of the 32-row block, 64-row tile and 256-row strip boundaries of the matrix-core
    kernels: ragged last tiles, waves with nothing to do, tiles skipped above the diagonal."""
    q, k = rand_qk(2, L, 128, torch.bfloat16, seed=1000 + L)
    s = lookm.lookm_scores(q.cuda(), k.cuda()).cpu().numpy().astype(np.float64)
    ref = oracle.scores(q, k)
    assert np.all(np.isfinite(s))
    assert (np.abs(s - ref) / ref).max() < 2e-5
    np.testing.assert_allclose(s.sum(1), L, rtol=1e-5)


def test_scores_large_logits_and_determinism():
    q, k = rand_qk(2, 600, 128, torch.bfloat16, seed=5, scale=4.0)   # logits up to ~ +-60
    a = lookm.lookm_scores(q.cuda(), k.cuda())
    b = lookm.lookm_scores(q.cuda(), k.cuda())
    assert torch.equal(a, b)
    ref = oracle.scores(q, k)
    s = a.cpu().numpy().astype(np.float64)
    assert np.all(np.isfinite(s))
    big = ref > 1e-6
    assert (np.abs(s - ref)[big] / ref[big]).max() < 1e-4
    np.testing.assert_allclose(s.sum(1), 600, rtol=1e-5)


def test_scores_logits_that_jump_late_in_the_row():
    # pass 1 sums a block against the row's current reference and only takes a new maximum when that overflows:
    # tiny keys first, then a few keys whose logits lie hundreds of binades higher (and lower), forces the refresh
    # in the middle of rows, in interior and in diagonal tiles
    H, L, d = 2, 900, 128
    g = torch.Generator().manual_seed(12)
    q = torch.randn(H, L, d, generator=g)
    k = torch.randn(H, L, d, generator=g) * 0.02
    for j in (130, 131, 400, 777, 899):
        k[:, j] *= 1500.0                                   # logits of about +-300
    q, k = q.to(torch.bfloat16), k.to(torch.bfloat16)
    a = lookm.lookm_scores(q.cuda(), k.cuda())
    assert torch.equal(a, lookm.lookm_scores(q.cuda(), k.cuda()))
    s = a.cpu().numpy().astype(np.float64)
    ref = oracle.scores(q, k)
    assert np.all(np.isfinite(s))
    big = ref > 1e-6
    assert (np.abs(s - ref)[big] / ref[big]).max() < 1e-4
    assert np.abs(s - ref)[~big].max() < 1e-9
    np.testing.assert_allclose(s.sum(1), L, rtol=1e-5)


def test_scores_zero_queries_closed_form():
    L = 1000
    q = torch.zeros(1, L, 128, dtype=torch.bfloat16)
    k = torch.randn(1, L, 128, generator=torch.Generator().manual_seed(1)).to(torch.bfloat16)
    s = lookm.lookm_scores(q.cuda(), k.cuda()).cpu().numpy()[0].astype(np.float64)
    inv = 1.0 / np.arange(1, L + 1)
    np.testing.assert_allclose(s, np.cumsum(inv[::-1])[::-1], rtol=2e-6)


@pytest.mark.parametrize("H,L,d,dtype", [(3, 700, 128, torch.bfloat16), (2, 333, 64, torch.bfloat16),
                                         (2, 256, 64, torch.float32)])
def test_scores_from_a_supplied_row_lse(H, L, d, dtype):
    # the row log-sum-exp a prefill kernel would hold (here: the oracle's, rounded to fp32) replaces pass 1
    q, k = rand_qk(H, L, d, dtype, seed=L + d)
    lse = torch.from_numpy(oracle.row_lse(q, k)).float()
    s = lookm.lookm_scores_lse(q.cuda(), k.cuda(), lse.cuda()).cpu().numpy().astype(np.float64)
    ref = oracle.scores(q, k)
    rel = np.abs(s - ref) / ref
    print(f"scores from row_lse H={H} L={L} d={d} {dtype}: max rel err {rel.max():.3e}")
    assert rel.max() < 2e-5
    own = lookm.lookm_scores(q.cuda(), k.cuda()).cpu().numpy().astype(np.float64)
    assert (np.abs(own - s) / ref).max() < 1e-5       # both routes agree


@pytest.mark.parametrize("H,L,d,dtype,windows", [
    (2, 700, 128, torch.bfloat16, (1, 63, 64, 65, 300, 699, 700)),      # matrix cores: inside one tile, across chunks
    (2, 3000, 128, torch.bfloat16, (17, 256, 1000, 2999)),
    (1, 333, 64, torch.bfloat16, (5, 200)),                             # portable kernels
    (2, 256, 64, torch.float32, (16, 255)),
])
def test_window_scores_match_oracle(H, L, d, dtype, windows):
    q, k = rand_qk(H, L, d, dtype, seed=L + d)
    qg, kg = q.cuda(), k.cuda()
    for w in windows:
        s = lookm.lookm_scores_window(qg, kg, w).cpu().numpy().astype(np.float64)
        ref = oracle.scores_window(q, k, w)
        assert np.all(np.isfinite(s))
        # columns that only far-away rows look at can be tiny: relative where it matters, absolute below
        np.testing.assert_allclose(s, ref, rtol=2e-5, atol=1e-12)
        np.testing.assert_allclose(s.sum(1), w, rtol=2e-5)
    full = lookm.lookm_scores(qg, kg)
    assert torch.equal(lookm.lookm_scores_window(qg, kg, L), full)       # the whole prompt: the same launches


@pytest.mark.parametrize("H,kvh,L,d,dtype", [
    (8, 2, 700, 128, torch.bfloat16),       # matrix cores, groups of four
    (6, 3, 1500, 128, torch.bfloat16),
    (4, 1, 300, 64, torch.bfloat16),        # portable kernels, one key head for all query heads
    (4, 2, 256, 64, torch.float32),
])
def test_grouped_scores_match_oracle(H, kvh, L, d, dtype):
    g = torch.Generator().manual_seed(H * 100 + L)
    q = torch.randn(H, L, d, generator=g).to(dtype)
    k = torch.randn(kvh, L, d, generator=g).to(dtype)
    s = lookm.lookm_scores_grouped(q.cuda(), k.cuda()).cpu().numpy().astype(np.float64)
    ref = oracle.scores_grouped(q, k)
    np.testing.assert_allclose(s, ref, rtol=2e-5)
    # the same sum taken from single-head launches: one query head per key head, repeated keys
    grp = H // kvh
    single = lookm.lookm_scores(q.cuda(), k.repeat_interleave(grp, 0).cuda()).view(kvh, grp, L)
    np.testing.assert_allclose(s, single.double().sum(1).cpu().numpy(), rtol=1e-6)


def select_case(scores, mask, B, M):
    sg = torch.from_numpy(np.asarray(scores, np.float32)).cuda()
    mg = torch.from_numpy(np.asarray(mask, np.uint8)).cuda()
    kept, ev = lookm.lookm_select(sg, mg, B, M)
    return kept.cpu().numpy(), ev.cpu().numpy()


@pytest.mark.parametrize("seed", range(8))
def test_select_matches_oracle_with_ties(seed):
    rng = np.random.default_rng(seed)
    H = 3
    L = int(rng.integers(1, 5000))
    M = int(rng.integers(0, min(L, 70) + 1))
    mask = (rng.random(L) < 0.8).astype(np.uint8)
    coarse = seed % 2 == 0
    scores = (rng.integers(1, 40, (H, L)) / 8.0 if coarse else rng.random((H, L)) + 1e-3).astype(np.float32)
    P = oracle.protected_count(mask, M)
    for B in sorted({P, min(L, P + 1), (P + L) // 2, max(P, L - 1), L}):
        kept, ev = select_case(scores, mask, B, M)
        for h in range(H):
            rk, re_ = oracle.select(scores[h].astype(np.float64), mask, B, M)
            assert kept[h].tolist() == rk.tolist(), (L, M, B, h)
            assert ev[h].tolist() == re_.tolist(), (L, M, B, h)


def test_select_scores_in_a_narrow_range_or_all_equal():
    # keys are re-based to the head's own range before the radix digits are taken
    rng = np.random.default_rng(5)
    L, M = 3000, 10
    mask = (rng.random(L) < 0.9).astype(np.uint8)
    P = oracle.protected_count(mask, M)
    narrow = (1.0 + rng.integers(0, 50, (1, L)) * 2.0 ** -23).astype(np.float32)     # 50 adjacent floats
    # positive, as Eq. 4 scores are, and within what the oracle's literal binary64 add of Eq. 5 resolves
    wide = (10.0 ** rng.uniform(-7, 7, (1, L))).astype(np.float32)
    same = np.full((1, L), 0.37, np.float32)
    two = np.where(rng.random((1, L)) < 0.5, np.float32(1.0e-7), np.float32(3.0e7)).astype(np.float32)
    for scores in (narrow, wide, same, two):
        for B in (P + 1, P + 700, L - 1):
            kept, ev = select_case(scores, mask, B, M)
            rk, re_ = oracle.select(scores[0].astype(np.float64), mask, B, M)
            assert kept[0].tolist() == rk.tolist() and ev[0].tolist() == re_.tolist(), B


@pytest.mark.parametrize("seed", range(4))
def test_select_literal_rule_matches_oracle_for_every_budget(seed):
    # Eq. 8 as printed: below |T u R| the text tokens compete by score and no image token is conserved
    rng = np.random.default_rng(40 + seed)
    H = 2
    L = int(rng.integers(50, 3000))
    M = int(rng.integers(0, 40))
    mask = (rng.random(L) < 0.5).astype(np.uint8)
    scores = (rng.integers(1, 60, (H, L)) / 8.0 if seed % 2 else rng.random((H, L)) + 1e-3).astype(np.float32)
    sg = torch.from_numpy(scores).cuda()
    mg = torch.from_numpy(mask).cuda()
    P = oracle.protected_count(mask, M)
    budgets = sorted({M, M + 1, (M + P) // 2, P - 1, P, P + 1, (P + L) // 2, L} & set(range(M, L + 1)))
    for B in budgets:
        kept, ev = lookm.lookm_select(sg, mg, B, M, rule="literal")
        kept, ev = kept.cpu().numpy(), ev.cpu().numpy()
        for h in range(H):
            rk, re_ = oracle.select(scores[h].astype(np.float64), mask, B, M, "literal")
            assert kept[h].tolist() == rk.tolist() and ev[h].tolist() == re_.tolist(), (L, M, B, h)
        if B < P:
            with pytest.raises(lookm.LookmError) as e:
                lookm.lookm_select(sg, mg, B, M)                     # the default rule still refuses
            assert e.value.code == lookm.ERR_BUDGET_BELOW_PROTECTED


def test_select_degenerate_cases():
    L = 300
    scores = np.random.default_rng(0).random((2, L)).astype(np.float32)
    ones = np.ones(L, np.uint8)
    kept, ev = select_case(scores, ones, 0, 0)                      # nothing conserved
    assert kept.shape == (2, 0) and ev[0].tolist() == list(range(L))
    kept, ev = select_case(scores, ones, L, L)                      # the window is the whole prompt
    assert kept[1].tolist() == list(range(L)) and ev.shape == (2, 0)
    kept, _ = select_case(scores, np.zeros(L, np.uint8), L, 0)      # all text
    assert kept[0].tolist() == list(range(L))
    kept, _ = select_case(scores, ones, 40, 0)                      # text prior off: plain top-B
    for h in range(2):
        assert kept[h].tolist() == np.sort(np.argsort(-scores[h], kind="stable")[:40]).tolist()
    neg = -scores                                                   # negative and zero scores order correctly
    neg[:, 5] = 0.0
    neg[:, 6] = -0.0
    kept, _ = select_case(neg, ones, 3, 0)
    for h in range(2):
        assert kept[h].tolist() == oracle.select(neg[h].astype(np.float64), ones, 3, 0)[0].tolist()


def test_select_reports_budget_below_protected():
    L = 64
    mask = np.zeros(L, np.uint8)
    mask[10:50] = 1
    sg = torch.rand(2, L, device="cuda")
    with pytest.raises(lookm.LookmError) as e:
        lookm.lookm_select(sg, torch.from_numpy(mask).cuda(), 20, 4)   # 24 text + 4 recent (text) -> 24 > 20
    assert e.value.code == lookm.ERR_BUDGET_BELOW_PROTECTED


def split(L, B, seed):
    rng = np.random.default_rng(seed)
    kept = np.sort(rng.choice(L, B, replace=False)).astype(np.int32)
    return kept, np.setdiff1d(np.arange(L, dtype=np.int32), kept)


@pytest.mark.parametrize("H,L,B,d,dtype", [
    (2, 900, 200, 128, torch.bfloat16),    # matrix-core path: ragged conserved and evicted tiles
    (2, 600, 64, 128, torch.bfloat16),
    (1, 300, 1, 128, torch.bfloat16),      # one conserved key
    (1, 300, 299, 128, torch.bfloat16),    # one evicted key
    (1, 32768, 32000, 128, torch.bfloat16),  # the longest prompt the library takes, nearly all of it conserved: nine chunks of 112 blocks
    (2, 500, 130, 64, torch.bfloat16),     # portable path
    (2, 256, 154, 64, torch.float32),
    (1, 100, 30, 8, torch.float32),
])
def test_nearest_matches_oracle(H, L, B, d, dtype):
    g = torch.Generator().manual_seed(L + B)
    cent = torch.randn(H, 16, d, generator=g)
    k = (cent[:, torch.randint(0, 16, (L,), generator=g)] + 0.3 * torch.randn(H, L, d, generator=g)).to(dtype)
    kept = np.stack([split(L, B, 10 + h)[0] for h in range(H)])
    ev = np.stack([split(L, B, 10 + h)[1] for h in range(H)])
    a, s = lookm.lookm_nearest(k.cuda(), torch.from_numpy(kept).cuda(), torch.from_numpy(ev).cuda())
    a, s = a.cpu().numpy(), s.cpu().numpy()
    kf = k.float().numpy()
    ties = sum(parity.check_nearest(kf[h], kept[h], ev[h], a[h], s[h]) for h in range(H))
    print(f"nearest H={H} L={L} B={B} d={d}: {ties} tie-band rows")
    assert ties == 0


def test_nearest_exact_ties_and_zero_keys():
    L, d = 200, 128
    g = torch.Generator().manual_seed(3)
    k = torch.randn(1, L, d, generator=g).to(torch.bfloat16)
    kept, ev = split(L, 50, 4)
    k[0, kept[7]] = k[0, kept[3]]                   # duplicate conserved keys: lower slot must win
    k[0, kept[30]] = k[0, kept[3]] * 2
    k[0, ev[5]] = k[0, kept[3]] * 0.5
    k[0, ev[9]] = 0                                 # zero evicted key: cosine 0 with everything -> slot 0
    k[0, kept[0]] = 0                               # zero conserved key
    a, s = lookm.lookm_nearest(k.cuda(), torch.from_numpy(kept)[None].cuda(), torch.from_numpy(ev)[None].cuda())
    a, s = a.cpu().numpy()[0], s.cpu().numpy()[0]
    ra, rs = oracle.nearest(k[0], kept, ev)
    assert a[5] == 3 and ra[5] == 3 and abs(s[5] - 1.0) < 1e-6
    assert a[9] == 0 and ra[9] == 0 and s[9] == 0.0
    assert np.array_equal(a, ra)


def test_nearest_when_every_cosine_is_negative():
    """Evicted keys that point away from every conserved key: the best cosine is negative, where the integer order
    of float bits is the reverse of their value order - those rows are decided by the exact pass over all slots."""
    L, d, B = 700, 128, 300
    g = torch.Generator().manual_seed(5)
    v = torch.randn(d, generator=g)
    k = torch.empty(1, L, d)
    kept, ev = split(L, B, 6)
    k[0, kept] = v + 0.3 * torch.randn(B, d, generator=g)
    k[0, ev] = -v + 0.3 * torch.randn(L - B, d, generator=g)
    k = k.to(torch.bfloat16)
    a, s = lookm.lookm_nearest(k.cuda(), torch.from_numpy(kept)[None].cuda(), torch.from_numpy(ev)[None].cuda())
    ra, rs = oracle.nearest(k[0].float().numpy(), kept, ev)
    assert rs.max() < 0
    assert np.array_equal(a.cpu().numpy()[0], ra)
    np.testing.assert_allclose(s.cpu().numpy()[0], rs, rtol=0, atol=parity.SIM_ATOL)


@pytest.mark.parametrize("H,Le", [(1, 512), (16, 12288), (3, 30000)])
def test_nearest_near_ties_between_far_apart_blocks(H, Le):
    """Pairs (and triples) of conserved keys whose cosines to an evicted key differ by a few 1e-7 - less than the
    matrix cores' fp32 values can tell apart - sitting 8, 16 or 32 blocks of 32 slots apart.  The matching must
    still be the binary64 one on every row: every block that holds a contender has to reach the exact pass.  With
    16 heads x 48 strips the conserved axis is ONE chunk of 64 blocks, so the members of a pair fall into the same
    block class of the same lane (two contenders that a set of class bits would show as one); with one head the
    axis is cut into 8 chunks and the members sit in different chunks; the third shape has chunks of 12 blocks.
    The twin of a key differs from it in one component (0 against 2^-7), where the evicted keys hold +-2^-7: the
    dot product moves by 2^-14 in about a hundred."""
    d, B = 128, 2048
    g = torch.Generator().manual_seed(11)
    kept_k = torch.randn(B, d, generator=g)
    kept_k[:, 5] = 0
    n_src = 256
    for s in range(n_src):
        for off in ((256,), (512,), (1024,), (256, 512))[s % 4]:
            kept_k[s + off] = kept_k[s]
            kept_k[s + off, 5] = 2.0 ** -7
    src = torch.arange(Le) % n_src
    ev_k = kept_k[src] + 0.05 * torch.randn(Le, d, generator=g)
    ev_k[:, 5] = (2.0 ** -7) * (1 - 2 * (torch.arange(Le) // n_src % 2)).float()
    k1 = torch.cat([kept_k, ev_k]).to(torch.bfloat16)
    k = k1[None].expand(H, -1, -1).contiguous()                       # every head holds the same keys
    kept = np.tile(np.arange(B, dtype=np.int32), (H, 1))
    ev = np.tile(np.arange(B, B + Le, dtype=np.int32), (H, 1))
    a, s = lookm.lookm_nearest(k.cuda(), torch.from_numpy(kept).cuda(), torch.from_numpy(ev).cuda())
    a, s = a.cpu().numpy(), s.cpu().numpy()
    assert all(np.array_equal(a[h], a[0]) and np.array_equal(s[h], s[0]) for h in range(H))
    rows = np.arange(0, Le, max(1, Le // 800))                        # the oracle on a sample of a long list
    ra, rs = oracle.nearest(k1.float().numpy(), kept[0], ev[0][rows])
    twins = int(np.sum(ra >= n_src))
    print(f"near ties: {len(rows)} rows checked, {twins} matched to a twin, {int(np.sum(a[0][rows] != ra))} differ")
    assert len(rows) // 8 < twins < len(rows)                         # both members of a pair win somewhere
    assert np.array_equal(a[0][rows], ra)
    np.testing.assert_allclose(s[0][rows], rs, rtol=0, atol=parity.SIM_ATOL)


@pytest.mark.parametrize("B,Le", [(1024, 4000), (64, 3000), (8, 2000), (2, 600)])
def test_nearest_keys_without_a_similar_conserved_key(B, Le):
    """Evicted keys unrelated to every conserved key: best cosines of 0.35 (1024 conserved keys) down to 0.1 (two).
    The rounding errors of the fp32 dot products grow like 1 / cos relative to the value, so the band inside which
    the matching is decided exactly widens with them, and below a cosine of 0.08 every slot is decided exactly.
    Every conserved key has a twin 2^-14 away in the dot product, so near ties are the rule here; every row must
    still get the binary64 answer."""
    d = 128
    g = torch.Generator().manual_seed(B)
    half = torch.randn(B // 2, d, generator=g)
    half[:, 5] = 0
    twin = half.clone()
    twin[:, 5] = 2.0 ** -7
    kept_k = torch.cat([half, twin])
    ev_k = torch.randn(Le, d, generator=g)
    ev_k[:, 5] = (2.0 ** -7) * (1 - 2 * (torch.arange(Le) % 2)).float()
    k = torch.cat([kept_k, ev_k])[None].to(torch.bfloat16)
    kept = np.arange(B, dtype=np.int32)[None]
    ev = np.arange(B, B + Le, dtype=np.int32)[None]
    a, s = lookm.lookm_nearest(k.cuda(), torch.from_numpy(kept).cuda(), torch.from_numpy(ev).cuda())
    a, s = a.cpu().numpy()[0], s.cpu().numpy()[0]
    ra, rs = oracle.nearest(k[0].float().numpy(), kept[0], ev[0])
    print(f"dissimilar keys, B={B}: best cosines {rs.min():.3f} .. {rs.max():.3f}, {int(np.sum(a != ra))} rows differ")
    assert np.array_equal(a, ra)
    np.testing.assert_allclose(s, rs, rtol=0, atol=parity.SIM_ATOL)


@pytest.mark.parametrize("H,B,Le", [(16, 2048, 12288), (32, 3072, 9216), (2, 1000, 3000)])
def test_nearest_near_ties_scattered_over_the_conserved_axis(H, B, Le):
    """Near-tied conserved keys at random slots (any lane, any entry of a block, any chunk; some in threes), with
    cosine gaps from 3e-8 to 4e-6 - from far below to just above what the matrix-core values resolve - and an
    evicted key for each that prefers one or the other by the sign of one small component.  Chunks of 64, 48 and 8
    blocks: every counter width of the block marks.  The matching must be the binary64 one on every checked row."""
    d = 128
    rng = np.random.default_rng(B + Le)
    g = torch.Generator().manual_seed(B)
    kept_k = torch.randn(B, d, generator=g)
    kept_k[:, 5] = 0
    n_src = B // 5
    slots = rng.permutation(B)
    src_slot, twin_slot, third_slot = slots[:n_src], slots[n_src:2 * n_src], slots[2 * n_src:3 * n_src]
    p_exp = rng.integers(6, 10, n_src)
    for i in range(n_src):
        kept_k[twin_slot[i]] = kept_k[src_slot[i]]
        kept_k[twin_slot[i], 5] = 2.0 ** -int(p_exp[i])
        if i % 3 == 0:
            kept_k[third_slot[i]] = kept_k[src_slot[i]]
            kept_k[third_slot[i], 5] = -(2.0 ** -int(p_exp[i]))
    which = torch.from_numpy(rng.integers(0, n_src, Le))
    ev_k = kept_k[torch.from_numpy(src_slot)[which]] + 0.05 * torch.randn(Le, d, generator=g)
    q_exp = torch.from_numpy(rng.integers(5, 10, Le)).float()
    sign = torch.from_numpy(rng.choice([-1.0, 1.0], Le)).float()
    ev_k[:, 5] = sign * 2.0 ** -q_exp
    k1 = torch.cat([kept_k, ev_k]).to(torch.bfloat16)
    k = k1[None].expand(H, -1, -1).contiguous()
    kept = np.tile(np.arange(B, dtype=np.int32), (H, 1))
    ev = np.tile(np.arange(B, B + Le, dtype=np.int32), (H, 1))
    a, s = lookm.lookm_nearest(k.cuda(), torch.from_numpy(kept).cuda(), torch.from_numpy(ev).cuda())
    a, s = a.cpu().numpy(), s.cpu().numpy()
    assert all(np.array_equal(a[h], a[0]) and np.array_equal(s[h], s[0]) for h in range(H))
    rows = np.arange(0, Le, max(1, Le // 1500))
    ra, rs = oracle.nearest(k1.float().numpy(), kept[0], ev[0][rows])
    print(f"scattered near ties: {len(rows)} rows checked, {int(np.sum(a[0][rows] != ra))} differ")
    assert np.array_equal(a[0][rows], ra)
    np.testing.assert_allclose(s[0][rows], rs, rtol=0, atol=parity.SIM_ATOL)


@pytest.mark.parametrize("mode", ["averaged", "pivotal", "weighted", "none"])
@pytest.mark.parametrize("H,L,B,d,dtype", [
    (2, 700, 150, 128, torch.bfloat16),
    (2, 256, 154, 64, torch.float32),
    (1, 120, 40, 8, torch.float32),
    (1, 300, 77, 256, torch.bfloat16),
    (2, 9000, 2100, 16, torch.bfloat16),     # register-resident sort, 8 entries per thread
    (1, 7000, 5200, 8, torch.float32),       # budget too large for 16 counter rows in LDS: general sort
    (1, 20000, 1500, 8, torch.bfloat16),     # more than 16 K evicted tokens: general sort
])
def test_merge_matches_oracle(mode, H, L, B, d, dtype):
    g = torch.Generator().manual_seed(L * 3 + B)
    k = torch.randn(H, L, d, generator=g).to(dtype)
    v = (torch.randn(H, L, d, generator=g) * 2).to(dtype)
    rng = np.random.default_rng(B)
    kept = np.stack([split(L, B, 20 + h)[0] for h in range(H)])
    ev = np.stack([split(L, B, 20 + h)[1] for h in range(H)])
    # skewed assignment: a few slots collect many members, many collect none
    assign = np.minimum((rng.random((H, L - B)) ** 3 * B).astype(np.int32), B - 1)
    sim = rng.uniform(0.1, 1.0, (H, L - B)).astype(np.float32)
    ko, vo = lookm.lookm_merge(k.cuda(), v.cuda(), torch.from_numpy(kept).cuda(), torch.from_numpy(ev).cuda(),
                               torch.from_numpy(assign).cuda(), torch.from_numpy(sim).cuda(), mode)
    ko, vo = ko.float().cpu().numpy(), vo.float().cpu().numpy()
    for h in range(H):
        parity.check_merge(k[h].float().numpy(), kept[h], ev[h], assign[h], sim[h], mode, ko[h], dtype)
        parity.check_merge(v[h].float().numpy(), kept[h], ev[h], assign[h], sim[h], mode, vo[h], dtype)


def test_merge_everything_into_one_slot():
    # the worst skew: all evicted rows matched to one conserved row
    H, L, B, d = 1, 2000, 10, 128
    g = torch.Generator().manual_seed(9)
    k = torch.randn(H, L, d, generator=g).to(torch.bfloat16)
    kept, ev = split(L, B, 1)
    assign = np.full((1, L - B), 4, np.int32)
    sim = np.full((1, L - B), 0.5, np.float32)
    ko, vo = lookm.lookm_merge(k.cuda(), k.cuda(), torch.from_numpy(kept)[None].cuda(), torch.from_numpy(ev)[None].cuda(),
                               torch.from_numpy(assign).cuda(), torch.from_numpy(sim).cuda(), "averaged")
    parity.check_merge(k[0].float().numpy(), kept, ev, assign[0], sim[0], "averaged", ko[0].float().cpu().numpy(),
                       torch.bfloat16)
    assert torch.equal(ko, vo)


def test_mfma_probe_reports_a_plausible_rate():
    """The measurement aid runs, and the rate it reports lies between a tenth of the datasheet peak and the peak."""
    for mode in (0, 1, 2):        # constant / random operands with 32x32x16, random operands with 16x16x32
        t = lookm.lookm_probe_mfma(mode, 3, iters=256, reps=6)
        assert 250.0 < t < 2600.0, (mode, t)
