"""Pins for the oracle's decoding-step attention over a cache (Eq. 3 of the paper, cache of Eq. 2 / Eq. 6-7)."""
import math

import numpy as np
import pytest
import torch

import oracle


@pytest.mark.parametrize("H,S,d,seed", [(1, 1, 8, 0), (2, 5, 16, 1), (3, 257, 64, 2), (2, 1000, 128, 3)])
def test_matches_library_softmax(H, S, d, seed):
    g = torch.Generator().manual_seed(seed)
    q = torch.randn(H, d, generator=g)
    k = torch.randn(H, S, d, generator=g) * 1.5
    v = torch.randn(H, S, d, generator=g)
    w = torch.softmax(torch.einsum("hd,hsd->hs", q.double(), k.double()) / math.sqrt(d), dim=-1)
    ref = torch.einsum("hs,hsd->hd", w, v.double()).numpy()
    np.testing.assert_allclose(oracle.decode(q, k, v), ref, rtol=1e-12, atol=1e-14)


def test_closed_forms_and_invariants():
    rng = np.random.default_rng(4)
    H, S, d = 2, 40, 32
    q = rng.standard_normal((H, d)).astype(np.float32)
    k = rng.standard_normal((H, S, d)).astype(np.float32)
    v = rng.standard_normal((H, S, d)).astype(np.float32)
    # a zero query attends uniformly: the mean value row
    np.testing.assert_allclose(oracle.decode(np.zeros_like(q), k, v), v.astype(np.float64).mean(1), rtol=1e-13)
    # one row: that row's value, whatever the key
    np.testing.assert_allclose(oracle.decode(q, k, v, S=1), v[:, 0].astype(np.float64), rtol=1e-15)
    # two rows with logits a, b: weights sigmoid(a - b) and its complement - pins scale and operand order
    a = (q[0].astype(np.float64) @ k[0, 0].astype(np.float64)) / math.sqrt(d)
    b = (q[0].astype(np.float64) @ k[0, 1].astype(np.float64)) / math.sqrt(d)
    w0 = 1.0 / (1.0 + math.exp(b - a))
    v64 = v.astype(np.float64)
    np.testing.assert_allclose(oracle.decode(q, k, v, S=2)[0], w0 * v64[0, 0] + (1 - w0) * v64[0, 1], rtol=1e-12)
    # the order of the cache rows does not matter (why the compact cache may be written in position order)
    perm = rng.permutation(S)
    np.testing.assert_allclose(oracle.decode(q, k[:, perm], v[:, perm]), oracle.decode(q, k, v), rtol=1e-12)
    # only the first S rows are read
    np.testing.assert_array_equal(oracle.decode(q, k, v, S=17), oracle.decode(q, k[:, :17].copy(), v[:, :17].copy()))
    # the output lies in the hull of the value rows
    o = oracle.decode(q, k, v)
    assert np.all(o <= v.max(1) + 1e-12) and np.all(o >= v.min(1) - 1e-12)
    # large logits do not overflow
    big = oracle.decode(q * 100, k * 100, v)
    assert np.all(np.isfinite(big))
