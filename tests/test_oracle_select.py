"""Pins for the two-stage selection oracle (Sec. 3.2, Stage I / Stage II,
Eq. 6-7): NumPy brute force (stable lexsort), closed forms and invariants."""
import numpy as np
import pytest

import oracle
from paper_2508_16201_amd import synth


def brute(scores, k, B):
    """Independent brute force with NumPy sorting primitives."""
    s = np.asarray(scores, np.float32).copy()
    V = s.shape[0]
    key = np.where(np.isnan(s), -np.inf, s + np.float32(0.0))      # -0.0 + 0.0 = +0.0
    nan_last = np.isnan(s).astype(np.int8)
    order = np.lexsort((np.arange(V), -key.astype(np.float64), nan_last))
    top = np.zeros(V, bool); top[order[:k]] = True
    rem = np.flatnonzero(~top)
    R, U = V - k, B - k
    ranks = [(t * R) // U for t in range(U)]
    uni = rem[ranks] if U else np.zeros(0, np.int64)
    keep = np.sort(np.concatenate([np.flatnonzero(top), uni]))
    return keep.astype(np.int32), top[keep].astype(np.uint8)


@pytest.mark.parametrize("V,k,B,seed", [(1568, 78, 157, 0), (200, 0, 20, 1), (200, 20, 20, 2),
                                         (97, 13, 41, 3), (6272, 313, 627, 4), (64, 5, 64, 5),
                                         (33, 1, 2, 6), (1, 1, 1, 7), (32768, 1638, 3277, 8)])
def test_matches_brute_force(V, k, B, seed):
    s = synth.make_scores(V, seed)
    keep, flag = oracle.select(s, k, B)
    bk, bf = brute(s, k, B)
    np.testing.assert_array_equal(keep, bk)
    np.testing.assert_array_equal(flag, bf)


@pytest.mark.parametrize("levels", [2, 8])
def test_duplicate_scores_break_ties_toward_lower_index(levels):
    s = synth.make_scores(3000, 11, levels=levels)
    keep, flag = oracle.select(s, 300, 600)
    bk, bf = brute(s, 300, 600)
    np.testing.assert_array_equal(keep, bk)
    np.testing.assert_array_equal(flag, bf)


def test_invariants():
    V, k, B = 5000, 250, 500
    s = synth.make_scores(V, 12)
    keep, flag = oracle.select(s, k, B)
    assert keep.shape == (B,) and np.all(np.diff(keep) > 0)
    assert keep.min() >= 0 and keep.max() < V
    assert flag.sum() == k                                   # |V_R| + |V_U| = B
    top = keep[flag == 1]
    rest = np.setdiff1d(np.arange(V), top)
    assert s[top].min() >= s[rest].max()                      # V_R dominates everything else
    # Stage II gaps (in remainder rank) are floor(I) or ceil(I), first remaining token kept
    rank_of = np.full(V, -1); rank_of[rest] = np.arange(rest.size)
    uni_ranks = rank_of[keep[flag == 0]]
    assert uni_ranks[0] == 0
    I = (V - k) / (B - k)
    gaps = np.diff(uni_ranks)
    assert set(np.unique(gaps)) <= {int(np.floor(I)), int(np.ceil(I))}


def test_closed_forms():
    V = 120
    s = synth.make_scores(V, 13)
    keep, flag = oracle.select(s, 0, 30)                      # pure uniform, I = 4
    np.testing.assert_array_equal(keep, np.arange(0, V, 4)); assert flag.sum() == 0
    keep, flag = oracle.select(s, 17, V)                      # B = V: identity
    np.testing.assert_array_equal(keep, np.arange(V)); assert flag.sum() == 17
    keep, _ = oracle.select(np.full(V, 0.25, np.float32), 10, 10)   # constant: lowest indices
    np.testing.assert_array_equal(keep, np.arange(10))
    ramp = np.linspace(1.0, 0.0, V).astype(np.float32)
    keep, flag = oracle.select(ramp, 10, 10)
    np.testing.assert_array_equal(keep, np.arange(10))
    keep, flag = oracle.select(ramp[::-1].copy(), 10, 10)     # increasing ramp: the last ten
    np.testing.assert_array_equal(keep, np.arange(V - 10, V))
    keep, flag = oracle.select(s, 0, 0)                       # 100 % pruning is legal
    assert keep.size == 0


def test_hand_worked_example():
    # V = 10, k = 2, B = 5.  Scores: tokens 7 and 3 are the two largest.
    s = np.array([.1, .2, .1, .9, .1, .3, .1, .95, .1, .1], np.float32)
    # remainder (ascending) = 0 1 2 4 5 6 8 9, R = 8, U = 3: ranks floor(t*8/3) = 0, 2, 5
    # -> tokens 0, 2, 6.  Union sorted: 0 2 3 6 7.
    keep, flag = oracle.select(s, 2, 5)
    np.testing.assert_array_equal(keep, [0, 2, 3, 6, 7])
    np.testing.assert_array_equal(flag, [0, 0, 1, 0, 1])


def test_signed_zero_and_nan_ordering():
    s = np.array([0.0, -0.0, 0.0, np.nan, -1.0, -0.0], np.float32)
    keep, flag = oracle.select(s, 3, 3)
    np.testing.assert_array_equal(keep, [0, 1, 2])            # -0.0 ties with +0.0, lower index wins
    keep, flag = oracle.select(s, 5, 5)
    np.testing.assert_array_equal(keep, [0, 1, 2, 4, 5])      # NaN is last of all


def test_rejects_bad_budgets():
    s = synth.make_scores(10, 14)
    for k, B in ((3, 2), (0, 11), (-1, 4)):
        with pytest.raises(ValueError):
            oracle.select(s, k, B)


def test_top_p_count_is_minimal_prefix():
    # Eq. 6: smallest c whose c largest scores reach lambda of the total.
    s = np.array([.05, .4, .05, .3, .1, .1], np.float32)      # sorted: .4 .3 .1 .1 .05 .05
    assert oracle.top_p_count(s, 0.0) == 0
    assert oracle.top_p_count(s, 0.39) == 1
    assert oracle.top_p_count(s, 0.5) == 2
    assert oracle.top_p_count(s, 0.75) == 3
    assert oracle.top_p_count(s, 1.0) == 6
    # margin: distance of lambda*total to the nearer deciding prefix sum, over the total
    c, m = oracle.top_p_count(np.array([.4, .3, .2, .1], np.float32), 0.5, want_margin=True)
    assert c == 2 and abs(m - 0.1) < 1e-6                     # prefix sums .4 | .7 around the goal .5
    s = synth.make_scores(4000, 15)
    for lam in (0.1, 0.4, 0.5, 0.9):
        c = oracle.top_p_count(s, lam)
        srt = np.sort(s.astype(np.float64))[::-1]
        cs = np.cumsum(srt)
        assert cs[c - 1] >= lam * cs[-1] * (1 - 1e-12) and (c == 1 or cs[c - 2] < lam * cs[-1] * (1 + 1e-12))


def test_top_p_count_values_without_mass():
    """Eq. 6 sums attention masses: a score that is not a finite positive number (negative, zero,
    NaN, infinite) adds nothing but keeps its place in the descending order.  Worked by hand."""
    s = np.array([0.5, -1.0, 0.25, np.nan, 0.25, 0.0, -0.0], np.float32)
    # descending: .5 .25 .25 0 -0 -1 NaN ; masses .5 .25 .25 0 0 0 0 ; total 1
    assert oracle.top_p_count(s, 0.0) == 0
    assert oracle.top_p_count(s, 0.5) == 1             # .5 >= .5
    assert oracle.top_p_count(s, 0.6) == 2             # .75 >= .6
    assert oracle.top_p_count(s, 0.75) == 2
    assert oracle.top_p_count(s, 0.76) == 3
    assert oracle.top_p_count(s, 1.0) == 3             # the mass ends at the third token
    c, m = oracle.top_p_count(s, 0.6, want_margin=True)
    assert c == 2 and abs(m - 0.1) < 1e-12             # prefix sums .5 | .75 around the goal .6
    # the raw sum of this vector is 0 (the -1 cancels the mass): a rule that summed raw values would return 0
    assert float(np.nansum(s.astype(np.float64))) == 0.0
    # an infinite score ranks first and carries no mass: it is counted on the way to the first unit score
    s = np.array([1.0, np.inf, 1.0], np.float32)
    assert oracle.top_p_count(s, 0.5) == 2 and oracle.top_p_count(s, 1.0) == 3
    # nothing with mass at all
    assert oracle.top_p_count(np.array([-1.0, np.nan, 0.0], np.float32), 0.7) == 0
    # lambda = 1 stops exactly at the last positive score, whatever the order of the input
    s = synth.make_scores(5000, 21)
    s[::7] = 0.0
    s[3::11] = -s[3::11]
    assert oracle.top_p_count(s, 1.0) == int((s > 0).sum())
