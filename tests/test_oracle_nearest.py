"""Pins for the oracle's cosine nearest-kept matching (Eq. 9 of the paper)."""
import math

import numpy as np
import pytest

import oracle


def dense_nearest(k, kept, evicted):
    k = np.asarray(k, np.float64)
    n = np.linalg.norm(k, axis=1)
    kn = np.divide(k, n[:, None], out=np.zeros_like(k), where=n[:, None] > 0)
    S = kn[evicted] @ kn[kept].T                   # L^e x L^c similarity matrix
    return S.argmax(axis=1), S.max(axis=1), S


def split(L, B, seed):
    rng = np.random.default_rng(seed)
    kept = np.sort(rng.choice(L, B, replace=False)).astype(np.int32)
    evicted = np.setdiff1d(np.arange(L), kept).astype(np.int32)
    return kept, evicted


@pytest.mark.parametrize("L,B,d,seed", [(12, 4, 3, 0), (60, 17, 16, 1), (150, 40, 64, 2), (90, 89, 8, 3), (40, 1, 8, 4)])
def test_matches_dense_similarity_matrix(L, B, d, seed):
    k = np.random.default_rng(seed).standard_normal((L, d)).astype(np.float32)
    kept, ev = split(L, B, seed + 50)
    a, s = oracle.nearest(k, kept, ev)
    ra, rs, _ = dense_nearest(k, kept, ev)
    assert a.tolist() == ra.tolist()
    np.testing.assert_allclose(s, rs, rtol=1e-12, atol=1e-15)


def test_planar_angles():
    # unit vectors at known angles: cos of the angle difference
    ang = np.deg2rad([0.0, 90.0, 180.0, 30.0, 100.0, 200.0])
    k = np.stack([np.cos(ang), np.sin(ang)], 1).astype(np.float32) * np.array([[1], [3], [0.5], [2], [7], [0.1]], np.float32)
    kept, ev = np.array([0, 1, 2], np.int32), np.array([3, 4, 5], np.int32)
    a, s = oracle.nearest(k, kept, ev)
    assert a.tolist() == [0, 1, 2]
    np.testing.assert_allclose(s, [math.cos(math.radians(30)), math.cos(math.radians(10)), math.cos(math.radians(20))], rtol=1e-6)


def test_scaled_copy_of_a_kept_key_has_cosine_one():
    L, d = 50, 16
    rng = np.random.default_rng(5)
    k = rng.standard_normal((L, d)).astype(np.float32)
    kept, ev = split(L, 12, 6)
    for n, e in enumerate(ev[:10]):
        k[e] = k[kept[n % 12]] * np.float32(2.0 ** (n - 3))     # exact power-of-two multiple
    a, s = oracle.nearest(k, kept, ev)
    assert a[:10].tolist() == [n % 12 for n in range(10)]
    np.testing.assert_allclose(s[:10], 1.0, rtol=1e-15)


def test_invariant_under_positive_row_scaling():
    L, d = 80, 32
    rng = np.random.default_rng(7)
    k = rng.standard_normal((L, d)).astype(np.float32)
    kept, ev = split(L, 20, 8)
    a0, s0 = oracle.nearest(k, kept, ev)
    scale = (2.0 ** rng.integers(-3, 4, L)).astype(np.float32)[:, None]
    a1, s1 = oracle.nearest(k * scale, kept, ev)
    assert a0.tolist() == a1.tolist()
    np.testing.assert_allclose(s0, s1, rtol=1e-14)


def test_negative_scaling_flips_sign():
    k = np.array([[1.0, 0.0], [0.0, 1.0], [-2.0, -0.1]], np.float32)
    a, s = oracle.nearest(k, np.array([0, 1], np.int32), np.array([2], np.int32))
    # cos with key 0 is about -0.9988, with key 1 about -0.05: the larger (less negative) one wins
    assert a.tolist() == [1] and s[0] < 0


def test_identical_kept_keys_tie_to_lower_position():
    k = np.array([[1, 2, 3], [9, 9, 9], [1, 2, 3], [2, 4, 6], [1, 2, 3.5]], np.float32)
    a, s = oracle.nearest(k, np.array([0, 2, 3], np.int32), np.array([1, 4], np.int32))
    assert a.tolist() == [0, 0]                    # slots 0, 1, 2 are parallel: the first wins


def test_zero_norm_key_has_cosine_zero():
    k = np.array([[0, 0], [1, 0], [-1, 0], [0, 0]], np.float32)
    # evicted zero key: all cosines 0 -> first kept slot; sim 0
    a, s = oracle.nearest(k, np.array([1, 2], np.int32), np.array([0], np.int32))
    assert a.tolist() == [0] and s[0] == 0.0
    # kept zero key scores 0, which beats a negative cosine
    a, s = oracle.nearest(k, np.array([1, 3], np.int32), np.array([2], np.int32))
    assert a.tolist() == [1] and s[0] == 0.0


def test_assignment_uses_slot_indices_not_positions():
    k = np.eye(6, dtype=np.float32)
    k[5] = k[4] * 3
    a, _ = oracle.nearest(k, np.array([1, 4], np.int32), np.array([5], np.int32))
    assert a.tolist() == [1]                       # slot 1 of kept == position 4
