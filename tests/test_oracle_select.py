"""Pins for the oracle's text-prior selection (Eq. 5-8 of the paper).

The reference here is a separately written Python statement of the rule: text tokens and
the last M positions always survive, the remaining budget goes to the highest-scoring image
tokens, equal scores go to the lower position.
"""
import itertools

import numpy as np
import pytest

import oracle


def lexicographic_select(scores, mask, B, M):
    L = len(scores)
    protected = [j for j in range(L) if mask[j] == 0 or j >= L - M]
    cand = [j for j in range(L) if j not in set(protected)]
    cand.sort(key=lambda j: (-scores[j], j))
    k_img = B - len(protected)
    assert k_img >= 0
    kept = sorted(protected + cand[:k_img])
    evicted = sorted(cand[k_img:])
    return np.array(kept, np.int32), np.array(evicted, np.int32)


def literal_eq5_select(scores, mask, B, M):
    """Eq. 5 and Eq. 8 spelled with NumPy: boost text by max(A_s), take top N = B - M of A_s[:-M]."""
    s = np.array(scores, np.float64)
    L = len(s)
    s[np.asarray(mask) == 0] += s.max()
    head = s[: L - M]
    order = np.lexsort((np.arange(L - M), -head))   # primary: -score, secondary: position
    top = order[: B - M]
    kept = np.sort(np.concatenate([top, np.arange(L - M, L)])).astype(np.int32)
    return kept


def test_hand_made_ties_go_to_lower_position():
    #            0    1    2    3    4    5    6    7
    scores = [0.5, 2.0, 2.0, 1.0, 2.0, 3.0, 1.0, 0.1]
    mask = [1, 1, 1, 1, 1, 1, 1, 1]
    kept, ev = oracle.select(scores, mask, budget=3, recent_window=0)
    assert kept.tolist() == [1, 2, 5]          # 5 (3.0) then the two earliest of the 2.0 tie
    assert ev.tolist() == [0, 3, 4, 6, 7]
    kept, _ = oracle.select(scores, mask, budget=5, recent_window=0)
    assert kept.tolist() == [1, 2, 3, 4, 5]    # 1.0 tie: position 3 beats 6
    kept, _ = oracle.select(scores, mask, budget=4, recent_window=2)
    assert kept.tolist() == [1, 5, 6, 7]       # last two always in; two best of the rest


def test_text_outranks_any_image_score():
    scores = [9.0, 0.01, 8.0, 0.02, 7.0, 6.0]
    mask = [1, 0, 1, 0, 1, 1]
    kept, ev = oracle.select(scores, mask, budget=3, recent_window=0)
    assert kept.tolist() == [0, 1, 3]
    assert ev.tolist() == [2, 4, 5]


def test_budget_equal_to_length_keeps_everything():
    rng = np.random.default_rng(0)
    L = 37
    kept, ev = oracle.select(rng.random(L), rng.integers(0, 2, L), budget=L, recent_window=5)
    assert kept.tolist() == list(range(L)) and ev.size == 0


def test_all_image_no_window_is_plain_top_b():
    rng = np.random.default_rng(1)
    L, B = 200, 41
    s = rng.random(L)
    kept, _ = oracle.select(s, np.ones(L, np.uint8), budget=B, recent_window=0)
    ref = np.sort(np.argsort(-s, kind="stable")[:B])
    assert kept.tolist() == ref.tolist()


@pytest.mark.parametrize("seed", range(6))
def test_random_cases_match_both_readings(seed):
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(20, 300))
    M = int(rng.integers(0, 12))
    mask = (rng.random(L) < 0.7).astype(np.uint8)
    # coarse scores: many exact ties
    s = rng.integers(1, 12, L).astype(np.float64) / 4.0
    P = oracle.protected_count(mask, M)
    for B in {P, min(L, P + 1), (P + L) // 2, L}:
        kept, ev = oracle.select(s, mask, B, M)
        rk, re_ = lexicographic_select(s, mask, B, M)
        assert kept.tolist() == rk.tolist() and ev.tolist() == re_.tolist()
        assert kept.tolist() == literal_eq5_select(s, mask, B, M).tolist()
        # structural invariants
        assert len(kept) == B and np.all(np.diff(kept) > 0) and kept.min() >= 0 and kept.max() < L
        assert set(np.flatnonzero(mask == 0)) <= set(kept.tolist())
        assert set(range(L - M, L)) <= set(kept.tolist())
        assert sorted(kept.tolist() + ev.tolist()) == list(range(L))


def test_exhaustive_small_inputs():
    # every mask and a grid of tied scores on L = 6: no evicted image token may beat a kept one
    L = 6
    for mask in itertools.product([0, 1], repeat=L):
        for s in [(1, 1, 1, 1, 1, 1), (1, 2, 3, 1, 2, 3), (3, 2, 1, 3, 2, 1), (2, 2, 1, 1, 3, 3)]:
            for M in (0, 2):
                P = oracle.protected_count(np.array(mask, np.uint8), M)
                for B in range(P, L + 1):
                    kept, ev = oracle.select(np.array(s, float), np.array(mask, np.uint8), B, M)
                    prot = {j for j in range(L) if mask[j] == 0 or j >= L - M}
                    assert prot <= set(kept.tolist())
                    kept_img = [j for j in kept if j not in prot]
                    for e in ev:
                        for c in kept_img:
                            assert (s[c], -c) > (s[e], -e)


def test_protected_count():
    mask = np.array([0, 1, 1, 0, 1, 1, 0, 1], np.uint8)
    assert oracle.protected_count(mask, 0) == 3
    assert oracle.protected_count(mask, 2) == 4      # positions 6 (text, counted once) and 7
    assert oracle.protected_count(mask, 8) == 8


def test_error_codes():
    s = np.ones(8)
    mask = np.array([0, 0, 0, 1, 1, 1, 1, 1], np.uint8)
    with pytest.raises(oracle.OracleError) as e:
        oracle.select(s, mask, budget=9, recent_window=0)
    assert e.value.code == oracle.ERR_BUDGET_RANGE
    with pytest.raises(oracle.OracleError) as e:
        oracle.select(s, mask, budget=2, recent_window=3)
    assert e.value.code == oracle.ERR_BUDGET_RANGE
    with pytest.raises(oracle.OracleError) as e:
        oracle.select(s, mask, budget=4, recent_window=2)   # 3 text + 2 recent = 5 > 4
    assert e.value.code == oracle.ERR_BUDGET_BELOW_PROTECTED


# ---- Eq. 8 taken literally (any budget), and the ratio form of the budget ------------------------------

def top_text_only(scores, mask, B, M):
    """Below |T u R|: the window, and the N = B - M best text tokens outside it; no image token."""
    L = len(scores)
    text = [j for j in range(L - M) if mask[j] == 0]
    text.sort(key=lambda j: (-scores[j], j))
    return np.array(sorted(text[: B - M] + list(range(L - M, L))), np.int32)


@pytest.mark.parametrize("seed", range(6))
def test_literal_rule_equals_the_protecting_rule_when_text_fits(seed):
    rng = np.random.default_rng(100 + seed)
    L = int(rng.integers(5, 200))
    M = int(rng.integers(0, L // 3 + 1))
    mask = (rng.random(L) < 0.6).astype(np.uint8)
    scores = rng.random(L) + 1e-3
    P = oracle.protected_count(mask, M)
    for B in sorted({P, (P + L) // 2, L}):
        a = oracle.select(scores, mask, B, M, "protect_text")
        b = oracle.select(scores, mask, B, M, "literal")
        assert a[0].tolist() == b[0].tolist() and a[1].tolist() == b[1].tolist()


@pytest.mark.parametrize("seed", range(6))
def test_literal_rule_below_the_protected_count(seed):
    rng = np.random.default_rng(200 + seed)
    L = int(rng.integers(8, 300))
    M = int(rng.integers(0, L // 4 + 1))
    mask = (rng.random(L) < 0.5).astype(np.uint8)
    scores = np.round(rng.random(L) * 8) / 8 + 0.125 if seed % 2 else rng.random(L) + 1e-3   # odd seeds: many ties
    P = oracle.protected_count(mask, M)
    prev = None
    for B in range(M, L + 1):
        kept, ev = oracle.select(scores, mask, B, M, "literal")
        assert len(kept) == B and sorted(set(kept.tolist()) | set(ev.tolist())) == list(range(L))
        assert set(range(L - M, L)) <= set(kept.tolist())
        if B < P:
            assert kept.tolist() == top_text_only(scores, mask, B, M).tolist()
            assert all(mask[j] == 0 or j >= L - M for j in kept)
            with pytest.raises(oracle.OracleError):
                oracle.select(scores, mask, B, M, "protect_text")
        if prev is not None:
            assert set(prev) < set(kept.tolist())            # one more place never drops a token
        prev = kept.tolist()


def test_literal_rule_hand_example():
    #                 0    1    2    3    4    5     6     7
    s = np.array([5.0, 1.0, 4.0, 2.0, 3.0, 0.5, 0.25, 9.0])
    m = np.array([0, 1, 0, 1, 0, 1, 1, 1], np.uint8)       # text at 0, 2, 4; window = position 7
    assert oracle.select(s, m, 3, 1, "literal")[0].tolist() == [0, 2, 7]     # N = 2 of three text tokens
    assert oracle.select(s, m, 4, 1, "literal")[0].tolist() == [0, 2, 4, 7]
    assert oracle.select(s, m, 5, 1, "literal")[0].tolist() == [0, 2, 3, 4, 7]   # then the best image token
    assert oracle.select(s, m, 1, 1, "literal")[0].tolist() == [7]


def test_budget_from_ratios():
    assert oracle.budget_from_ratios(1000, 0.1, 0.1) == (100, 200)
    assert oracle.budget_from_ratios(12644, 0.0, 0.05) == (0, 632)
    with pytest.raises(oracle.OracleError):
        oracle.budget_from_ratios(7, 0.5, 0.5)              # 4 + 4 > 7
    with pytest.raises(oracle.OracleError):
        oracle.budget_from_ratios(100, 1.5, 0.0)
    for L in (1, 17, 4096, 12644):
        for a1, a2 in ((0.01, 0.04), (0.1, 0.1), (0.0, 0.99), (0.3, 0.5)):
            M, S = oracle.budget_from_ratios(L, a1, a2)
            assert abs(M - a1 * L) <= 0.5 and abs((S - M) - a2 * L) <= 0.5 and 0 <= M <= S <= L
