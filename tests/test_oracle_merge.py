"""Pins for the oracle's merging rules (Eq. 10-12 of the paper) and the compact layout."""
from pathlib import Path

import numpy as np
import pytest

import oracle

GOLDEN = Path(__file__).parent / "golden"


def random_case(L, B, d, seed):
    rng = np.random.default_rng(seed)
    x = rng.standard_normal((L, d)).astype(np.float32)
    kept = np.sort(rng.choice(L, B, replace=False)).astype(np.int32)
    ev = np.setdiff1d(np.arange(L), kept).astype(np.int32)
    assign = rng.integers(0, B, ev.size).astype(np.int32)
    sim = rng.uniform(0.05, 1.0, ev.size)
    return x, kept, ev, assign, sim


def read_prose_example():
    """tests/golden/merge_prose_example.txt: 'target' and 'members' token ids from Section 3.3."""
    vals = {}
    for line in (GOLDEN / "merge_prose_example.txt").read_text().splitlines():
        if line.strip() and not line.startswith("#"):
            key, v = line.split("=")
            vals[key.strip()] = [int(t) for t in v.split()]
    return vals["target"][0], vals["members"]


def test_prose_example_of_section_3_3():
    # the similarity set of token 1 holds tokens 4 and 8 -> token 1 becomes the mean of the three
    target, members = read_prose_example()
    L, d = 10, 5
    x = np.random.default_rng(0).standard_normal((L, d)).astype(np.float32)
    kept = np.array([target, 9], np.int32)
    ev = np.array(sorted(members), np.int32)
    out = oracle.merge(x, kept, ev, np.zeros(len(members), np.int32), np.ones(len(members)), "averaged")
    ref = (x[target].astype(np.float64) + sum(x[m].astype(np.float64) for m in members)) / (len(members) + 1)
    np.testing.assert_allclose(out[0], ref, rtol=1e-15)
    np.testing.assert_array_equal(out[1], x[9].astype(np.float64))


def test_single_member_weights():
    x = np.array([[8.0, -4.0], [2.0, 6.0]], np.float32)     # kept row 0, evicted row 1
    kept, ev, a = np.array([0], np.int32), np.array([1], np.int32), np.array([0], np.int32)
    s = np.array([0.25])
    np.testing.assert_array_equal(oracle.merge(x, kept, ev, a, s, "averaged")[0], [5.0, 1.0])       # 1/2, 1/2
    np.testing.assert_array_equal(oracle.merge(x, kept, ev, a, s, "pivotal")[0], [6.5, -1.5])       # 3/4, 1/4
    np.testing.assert_array_equal(oracle.merge(x, kept, ev, a, s, "weighted")[0], [4.25, -1.25])    # (x_c + s x_e)/2
    np.testing.assert_array_equal(oracle.merge(x, kept, ev, a, s, "none")[0], [8.0, -4.0])


def weights_via_identity(L, kept, ev, assign, sim, mode):
    """Merging the identity matrix returns, row by row, the weight each source token receives."""
    return oracle.merge(np.eye(L, dtype=np.float32), kept, ev, assign, sim, mode)


@pytest.mark.parametrize("seed", range(4))
def test_explicit_weight_vectors(seed):
    L, B = 60, 13
    _, kept, ev, assign, sim = random_case(L, B, 4, seed)
    n = np.bincount(assign, minlength=B)
    for mode in ("averaged", "pivotal", "weighted"):
        W = weights_via_identity(L, kept, ev, assign, sim, mode)
        assert W.shape == (B, L) and np.all(W >= 0)
        for r in range(B):
            members = ev[assign == r]
            support = set(np.flatnonzero(W[r]).tolist())
            assert support == set(members.tolist()) | {int(kept[r])}
            if mode == "averaged":
                np.testing.assert_allclose(W[r, kept[r]], 1.0 / (n[r] + 1), rtol=1e-15)
                np.testing.assert_allclose(W[r, members], 1.0 / (n[r] + 1), rtol=1e-15)
                np.testing.assert_allclose(W[r].sum(), 1.0, rtol=1e-14)
            elif mode == "pivotal":
                np.testing.assert_allclose(W[r, kept[r]], (2.0 + n[r]) / (2.0 * (n[r] + 1)), rtol=1e-15)
                np.testing.assert_allclose(W[r, members], 0.5 / (n[r] + 1), rtol=1e-15)
                np.testing.assert_allclose(W[r].sum(), 1.0, rtol=1e-14)
            else:
                np.testing.assert_allclose(W[r, kept[r]], 1.0 / (n[r] + 1), rtol=1e-15)
                np.testing.assert_allclose(W[r, members], sim[assign == r] / (n[r] + 1), rtol=1e-15)
                np.testing.assert_allclose(W[r].sum(), (1.0 + sim[assign == r].sum()) / (n[r] + 1), rtol=1e-14)


@pytest.mark.parametrize("seed", range(3))
def test_mass_conservation(seed):
    L, B, d = 90, 21, 7
    x, kept, ev, assign, sim = random_case(L, B, d, 10 + seed)
    n = np.bincount(assign, minlength=B)[:, None].astype(np.float64)
    x64 = x.astype(np.float64)
    avg = oracle.merge(x, kept, ev, assign, sim, "averaged")
    np.testing.assert_allclose(((n + 1) * avg).sum(0), x64.sum(0), rtol=1e-12, atol=1e-12)
    piv = oracle.merge(x, kept, ev, assign, sim, "pivotal")
    lhs = (2 * (n + 1) * piv - n * x64[kept]).sum(0)
    np.testing.assert_allclose(lhs, 2 * x64[kept].sum(0) + x64[ev].sum(0), rtol=1e-12, atol=1e-12)


def test_weighted_with_unit_similarity_is_averaged():
    x, kept, ev, assign, _ = random_case(70, 15, 6, 20)
    np.testing.assert_array_equal(oracle.merge(x, kept, ev, assign, np.ones(ev.size), "weighted"),
                                  oracle.merge(x, kept, ev, assign, np.ones(ev.size), "averaged"))


def test_rows_without_members_are_exact_copies_and_none_is_a_gather():
    x, kept, ev, assign, sim = random_case(50, 20, 9, 21)
    assign[:] = 3                                       # everything goes to slot 3
    for mode in ("averaged", "pivotal", "weighted"):
        out = oracle.merge(x, kept, ev, assign, sim, mode)
        others = np.arange(20) != 3
        np.testing.assert_array_equal(out[others], x[kept][others].astype(np.float64))
        assert not np.array_equal(out[3], x[kept[3]].astype(np.float64))
    np.testing.assert_array_equal(oracle.merge(x, kept, ev, assign, sim, "none"), x[kept].astype(np.float64))


def test_results_stay_in_the_bounding_box_of_their_sources():
    x, kept, ev, assign, sim = random_case(120, 25, 11, 22)
    x64 = x.astype(np.float64)
    for mode in ("averaged", "pivotal", "weighted"):
        out = oracle.merge(x, kept, ev, assign, sim, mode)
        for r in range(25):
            src = np.vstack([x64[kept[r]][None], x64[ev[assign == r]]])
            if mode == "weighted":                      # total weight <= 1: hull of sources and the origin
                src = np.vstack([src, np.zeros((1, x.shape[1]))])
            assert np.all(out[r] <= src.max(0) + 1e-12) and np.all(out[r] >= src.min(0) - 1e-12)


def test_pivotal_is_the_average_with_the_pairwise_midpoints():
    # Section 3.3: first average each evicted token with its target (the pivotal tokens),
    # then average the target with its pivotal tokens
    x, kept, ev, assign, sim = random_case(40, 8, 5, 23)
    x64 = x.astype(np.float64)
    out = oracle.merge(x, kept, ev, assign, sim, "pivotal")
    for r in range(8):
        piv = [(x64[e] + x64[kept[r]]) / 2 for e in ev[assign == r]]
        ref = (x64[kept[r]] + sum(piv)) / (len(piv) + 1) if piv else x64[kept[r]]
        np.testing.assert_allclose(out[r], ref, rtol=1e-14, atol=1e-15)


def test_bad_mode():
    x, kept, ev, assign, sim = random_case(10, 3, 2, 24)
    with pytest.raises(oracle.OracleError):
        oracle.merge(x, kept, ev, assign, sim, 7)
