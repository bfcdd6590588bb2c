"""Pins for the oracle's accumulated attention score (Eq. 4 of the paper, scale of Eq. 3).

Each check is independent of the oracle's own code: a closed form, a library softmax,
or a separately written dense NumPy evaluation.
"""
import math

import numpy as np
import pytest
import torch

import oracle


def dense_scores_numpy(q, k):
    """Materialises the L x L causal attention matrix and sums its columns."""
    q = np.asarray(q, np.float64)
    k = np.asarray(k, np.float64)
    L, d = q.shape
    logits = (q @ k.T) / math.sqrt(d)
    logits = np.where(np.tril(np.ones((L, L), bool)), logits, -np.inf)
    logits = logits - logits.max(axis=1, keepdims=True)
    w = np.exp(logits)
    w /= w.sum(axis=1, keepdims=True)
    return w.sum(axis=0)


@pytest.mark.parametrize("L,d,seed", [(1, 8, 0), (2, 4, 1), (17, 16, 2), (64, 64, 3), (96, 128, 4), (130, 32, 5)])
def test_matches_dense_numpy(L, d, seed):
    rng = np.random.default_rng(seed)
    q = rng.standard_normal((L, d)).astype(np.float32)
    k = rng.standard_normal((L, d)).astype(np.float32)
    np.testing.assert_allclose(oracle.scores(q, k), dense_scores_numpy(q, k), rtol=1e-12, atol=1e-14)


@pytest.mark.parametrize("L,d", [(50, 64), (128, 128)])
def test_matches_library_softmax(L, d):
    g = torch.Generator().manual_seed(L * 1000 + d)
    q = torch.randn(L, d, generator=g)
    k = torch.randn(L, d, generator=g) * 2.0
    logits = (q.double() @ k.double().T) / math.sqrt(d)
    causal = torch.full((L, L), float("-inf"), dtype=torch.float64).triu(1)
    ref = torch.softmax(logits + causal, dim=-1).sum(0).numpy()
    np.testing.assert_allclose(oracle.scores(q, k), ref, rtol=1e-12)


def harmonic_tail(L):
    """A_s[j] = sum_{i=j}^{L-1} 1/(i+1) for uniform causal attention."""
    inv = 1.0 / np.arange(1, L + 1, dtype=np.float64)
    return np.cumsum(inv[::-1])[::-1]


def test_zero_queries_give_harmonic_numbers():
    L, d = 200, 16
    k = np.random.default_rng(7).standard_normal((L, d)).astype(np.float32)
    s = oracle.scores(np.zeros((L, d), np.float32), k)
    np.testing.assert_allclose(s, harmonic_tail(L), rtol=1e-13)
    assert np.all(np.diff(s) < 0)


def test_equal_keys_give_harmonic_numbers():
    L, d = 77, 8
    rng = np.random.default_rng(8)
    q = rng.standard_normal((L, d)).astype(np.float32)
    k = np.tile(rng.standard_normal((1, d)).astype(np.float32), (L, 1))
    np.testing.assert_allclose(oracle.scores(q, k), harmonic_tail(L), rtol=1e-12)


def test_two_token_closed_form_pins_the_scale():
    # row 1 sees logits [a*b/sqrt(d), 0]; with a*b = 4 and d = 16 the logit is exactly 1.
    d = 16
    q = np.zeros((2, d), np.float32)
    k = np.zeros((2, d), np.float32)
    q[1, 0], k[0, 0] = 2.0, 2.0
    sig = 1.0 / (1.0 + math.exp(-1.0))
    np.testing.assert_allclose(oracle.scores(q, k), [1.0 + sig, 1.0 - sig], rtol=1e-15)
    # a query / key mix-up (k q^T instead of q k^T) would give logits 0 here
    q2, k2 = k.copy(), q.copy()
    np.testing.assert_allclose(oracle.scores(q2, k2), [1.5, 0.5], rtol=1e-15)


def test_three_token_closed_form():
    # d = 1: logits are products q_i k_j; checked against a hand-expanded softmax
    q = np.array([[0.5], [1.0], [-2.0]], np.float32)
    k = np.array([[1.0], [-1.0], [0.5]], np.float32)
    r1 = np.exp([1.0, -1.0]); r1 /= r1.sum()
    r2 = np.exp([-2.0, 2.0, -1.0]); r2 /= r2.sum()
    ref = [1.0 + r1[0] + r2[0], r1[1] + r2[1], r2[2]]
    np.testing.assert_allclose(oracle.scores(q, k), ref, rtol=1e-14)


def test_row_stochastic_invariants():
    L, d = 150, 32
    rng = np.random.default_rng(9)
    q = (3.0 * rng.standard_normal((L, d))).astype(np.float32)
    k = (3.0 * rng.standard_normal((L, d))).astype(np.float32)
    s = oracle.scores(q, k)
    assert abs(s.sum() - L) < 1e-9          # every softmax row sums to one
    assert s[0] >= 1.0                      # row 0 puts all its mass on column 0
    assert 0.0 < s[-1] <= 1.0               # only the last row reaches the last column
    assert np.all(s > 0.0)


def test_large_logits_are_stable():
    L, d = 20, 4
    rng = np.random.default_rng(10)
    q = (200.0 * rng.standard_normal((L, d))).astype(np.float32)
    k = (200.0 * rng.standard_normal((L, d))).astype(np.float32)
    s = oracle.scores(q, k)
    assert np.all(np.isfinite(s)) and abs(s.sum() - L) < 1e-9
    np.testing.assert_allclose(s, dense_scores_numpy(q, k), rtol=1e-10, atol=1e-300)


def test_prefix_rows_are_causal():
    # rows < n never look at keys >= n: the first n rows' contribution is the score of the prefix
    L, n, d = 40, 25, 8
    rng = np.random.default_rng(11)
    q = rng.standard_normal((L, d)).astype(np.float32)
    k = rng.standard_normal((L, d)).astype(np.float32)
    k_changed = k.copy()
    k_changed[n:] += 5.0
    full = dense_scores_numpy(q, k)
    # oracle on the prefix alone must equal the dense prefix rows' column sums
    pref = oracle.scores(q[:n], k[:n])
    np.testing.assert_allclose(pref, dense_scores_numpy(q[:n], k[:n]), rtol=1e-12)
    # and changing later keys cannot change what the prefix rows contribute
    diff = oracle.scores(q, k_changed)[:n] - oracle.scores(q, k)[:n]
    later_only = dense_scores_numpy(q, k_changed)[:n] - full[:n]
    np.testing.assert_allclose(diff, later_only, rtol=1e-9, atol=1e-13)


def test_heads_are_independent_and_batched_call_matches():
    H, L, d = 3, 33, 16
    rng = np.random.default_rng(12)
    q = rng.standard_normal((H, L, d)).astype(np.float32)
    k = rng.standard_normal((H, L, d)).astype(np.float32)
    s = oracle.scores(q, k)
    for h in range(H):
        np.testing.assert_array_equal(s[h], oracle.scores(q[h], k[h]))
    np.testing.assert_array_equal(oracle.scores(q[::-1].copy(), k[::-1].copy()), s[::-1])


def test_bf16_inputs_are_widened_exactly():
    L, d = 31, 16
    g = torch.Generator().manual_seed(5)
    q = torch.randn(L, d, generator=g).to(torch.bfloat16)
    k = torch.randn(L, d, generator=g).to(torch.bfloat16)
    np.testing.assert_allclose(oracle.scores(q, k), dense_scores_numpy(q.double().numpy(), k.double().numpy()),
                               rtol=1e-12)


def test_row_lse_matches_library_logsumexp_and_rebuilds_the_scores():
    L, d = 70, 32
    g = torch.Generator().manual_seed(77)
    q = torch.randn(L, d, generator=g) * 1.5
    k = torch.randn(L, d, generator=g)
    logits = (q.double() @ k.double().T) / math.sqrt(d)
    causal = torch.full((L, L), float("-inf"), dtype=torch.float64).triu(1)
    ref = torch.logsumexp(logits + causal, dim=-1).numpy()
    lse = oracle.row_lse(q, k)
    np.testing.assert_allclose(lse, ref, rtol=1e-13, atol=1e-13)
    assert abs(lse[0] - float(logits[0, 0])) < 1e-14        # row 0 has a single term
    # A_p[i, j] = exp(s_ij - lse_i): its column sums are the accumulated scores
    A_p = torch.exp(logits + causal - torch.from_numpy(lse)[:, None]).numpy()
    np.testing.assert_allclose(A_p.sum(0), oracle.scores(q, k), rtol=1e-12)


def test_row_lse_closed_form_for_zero_queries():
    L, d = 50, 8
    k = np.random.default_rng(3).standard_normal((L, d)).astype(np.float32)
    np.testing.assert_allclose(oracle.row_lse(np.zeros((L, d), np.float32), k), np.log(np.arange(1, L + 1)), rtol=1e-14)


# ---- observation window: only the last w query rows are summed -------------------------------------------------

@pytest.mark.parametrize("L,d,w,seed", [(40, 16, 1, 0), (40, 16, 7, 1), (96, 64, 32, 2), (130, 32, 129, 3)])
def test_window_scores_match_library_softmax_rows(L, d, w, seed):
    g = torch.Generator().manual_seed(900 + seed)
    q = torch.randn(L, d, generator=g)
    k = torch.randn(L, d, generator=g) * 1.5
    logits = (q.double() @ k.double().T) / math.sqrt(d)
    causal = torch.full((L, L), float("-inf"), dtype=torch.float64).triu(1)
    ref = torch.softmax(logits + causal, dim=-1)[L - w:].sum(0).numpy()
    got = oracle.scores_window(q, k, w)
    np.testing.assert_allclose(got, ref, rtol=1e-12, atol=1e-300)
    assert abs(got.sum() - w) < 1e-10                      # w rows of a softmax


def test_window_scores_special_cases():
    rng = np.random.default_rng(11)
    L, d = 70, 32
    q = rng.standard_normal((2, L, d)).astype(np.float32)
    k = rng.standard_normal((2, L, d)).astype(np.float32)
    np.testing.assert_array_equal(oracle.scores_window(q, k, L), oracle.scores(q, k))      # the whole prompt
    # w = 1: the last row's attention; w rows are additive
    last = oracle.scores_window(q[0], k[0], 1)
    z = (q[0, -1].astype(np.float64) @ k[0].astype(np.float64).T) / math.sqrt(d)
    np.testing.assert_allclose(last, np.exp(z - z.max()) / np.exp(z - z.max()).sum(), rtol=1e-12)
    # zero queries: uniform rows, a closed form; columns after the window's first row see fewer rows
    w = 9
    got = oracle.scores_window(np.zeros((L, d), np.float32), k[0], w)
    inv = 1.0 / np.arange(1, L + 1)
    ref = np.array([inv[max(j, L - w):].sum() for j in range(L)])
    np.testing.assert_allclose(got, ref, rtol=1e-13)
    with pytest.raises(oracle.OracleError):
        oracle.scores_window(q, k, 0)


# ---- grouped query heads: a key head's score is the sum over the query heads that read it ------------------------

def test_grouped_scores():
    rng = np.random.default_rng(21)
    H, kvh, L, d = 6, 2, 45, 16
    q = rng.standard_normal((H, L, d)).astype(np.float32)
    k = rng.standard_normal((kvh, L, d)).astype(np.float32)
    got = oracle.scores_grouped(q, k)
    ref = np.stack([sum(dense_scores_numpy(q[kh * 3 + m], k[kh]) for m in range(3)) for kh in range(kvh)])
    np.testing.assert_allclose(got, ref, rtol=1e-12)
    np.testing.assert_allclose(got.sum(1), 3 * L, rtol=1e-12)                  # three softmax rows per position
    np.testing.assert_array_equal(oracle.scores_grouped(q[:2], k), oracle.scores(q[:2], k))   # groups of one
    twin = np.concatenate([q[:1], q[:1], q[1:2], q[1:2]])                      # identical query heads: twice the score
    np.testing.assert_allclose(oracle.scores_grouped(twin, k), 2 * oracle.scores(q[:2], k), rtol=1e-14)
    with pytest.raises(oracle.OracleError):
        oracle.scores_grouped(q[:5], k)                                        # 5 heads do not split into 2 groups
