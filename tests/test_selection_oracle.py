"""Pins for the block-selection oracle (oracle/selection.py): each selector against what the
paper and the mathematics fix, never against itself.

  * every valid selection enumerated for b <= 16: the optimal selector's total is the best one,
    its index set is the unique best set when the scores are generic; greedy and expansion +
    division return valid selections that are never better;
  * the two examples the text walks through (Section 3.2: N = 2, eight weights, three blocks;
    Section 4.1: w0 and w3 merged into (w1, w2)), with scores chosen to produce the described
    order -- the figures' own numbers are not in the text;
  * closed forms: N = 1 is top-m for all three; back-to-back blocks are all selectable; a layer
    two blocks tile exactly;
  * invariant of Algorithm 1: the scores it records add up to the l1 norm that the divided blocks
    keep, so a wrong sign, a dropped term or a shifted index in its update shows;
  * Eq. 1's -inf cases and Eq. 5's end points (0 for the aligned selection itself, 1 when blocks
    can hold exactly the largest magnitudes).
"""
import itertools

import numpy as np
import pytest

from oracle import selection as sel

NEG = -np.inf


def _valid(I, S, N, m=None):
    I = sorted(I)
    assert len(set(I)) == len(I)
    assert all(0 <= k < len(S) and S[k] > NEG for k in I), "a candidate with score -inf was kept"
    assert all(b - a >= N for a, b in zip(I, I[1:])), "kept blocks overlap"
    if m is not None:
        assert len(I) == m


def _enumerate(S, N, m):
    """Best total and all index sets reaching it, over every valid choice of m candidates."""
    cand = [k for k in range(len(S)) if S[k] > NEG]
    best, sets = NEG, []
    for I in itertools.combinations(cand, m):
        if all(b - a >= N for a, b in zip(I, I[1:])):
            t = sum(S[k] for k in I)
            if t > best:
                best, sets = t, [I]
            elif t == best:
                sets.append(I)
    return best, sets


def _layer(rng, c_out, c_in, N, integer=True):
    W = rng.integers(-9, 10, size=(c_out, c_in)).astype(np.float64) if integer else rng.standard_normal((c_out, c_in))
    return W, sel.block_scores(W, N)


# ------------------------------------------------------------------ Eq. 1
def test_scores_follow_eq1_on_a_hand_example():
    W = np.array([[1., -2.], [3., 4.], [-5., 6.], [7., -8.]])          # c_out = 4, c_in = 2
    S = sel.block_scores(W, 2)
    assert S.tolist() == [4., 8., 12., NEG, 6., 10., 14., NEG]          # k = i + 4 j
    S = sel.block_scores(W, 2, aligned=True)
    assert S.tolist() == [4., NEG, 12., NEG, 6., NEG, 14., NEG]
    S = sel.block_scores(W, 3)
    assert S.tolist() == [9., 15., NEG, NEG, 12., 18., NEG, NEG]
    S = sel.block_scores(W, 2, bw=2)                                     # one input channel of two columns
    assert S.tolist() == [10., 18., 26., NEG]


# ------------------------------------------------------------------ the paper's two examples
def test_greedy_example_of_section_3_2():
    e = np.array([4., 9., 8., 5., 2., 7., 6., 1.])                      # w0 .. w7, N = 2, keep 3 blocks
    S = sel.block_scores(e.reshape(-1, 1), 2)
    assert sel.select_greedy(S, 2, 3) == [1, 5, 3]                       # (w1,w2), (w5,w6), (w3,w4): w0, w7 dropped
    assert sel.select_optimal(S, 2, 3) == [0, 2, 5]                      # keeps w0 in place of w4
    assert e[0] > e[4]
    assert sel.select_bed(S, 2, 3) == [0, 2, 5]


def test_expansion_example_of_section_4_1():
    e = np.array([5., 9., 9., 4., 1., 0.5])
    S = sel.block_scores(e.reshape(-1, 1), 2)
    I_bar, picked = sel.block_expansion(S, 2, 2)
    assert I_bar == [1, 0]                                                # (w1,w2) first, then the block joined from w0 and w3
    assert picked == [18., e[0] + e[3]] and e[0] + e[3] > e[3] + e[4]
    assert sel.block_division(I_bar, 2) == [0, 2]                        # (w0,w1), (w2,w3)
    assert sel.select_greedy(S, 2, 2) == [1, 3]                          # greedy is left with (w3,w4)


# ------------------------------------------------------------------ closed forms
@pytest.mark.parametrize("m", [0, 1, 5, 12])
def test_block_size_one_is_top_m(m):
    rng = np.random.default_rng(5)
    S = rng.permutation(12).astype(np.float64)
    top = sorted(np.argsort(-S)[:m].tolist())
    assert sorted(sel.select_greedy(S, 1, m)) == top
    assert sorted(sel.select_bed(S, 1, m)) == top
    assert sel.select_optimal(S, 1, m) == top


def test_back_to_back_blocks_are_all_selectable():
    S = np.array([3., 0., 2., 0., 1., NEG])
    assert sel.select_greedy(S, 2, 3) == [0, 2, 4]                       # k and k+N do not overlap
    assert sel.select_optimal(S, 2, 3) == [0, 2, 4]
    assert sorted(sel.select_bed(S, 2, 3)) == [0, 2, 4]
    S = np.array([1., 5., 1., NEG, NEG])                                 # k-N+1 .. k+N-1 are shut out
    assert sel.select_greedy(S, 3, 2) == [1]
    assert sel.select_optimal(S, 3, 2) is None


def test_two_blocks_tile_the_layer():
    W = np.array([[1.], [2.], [3.], [4.], [5.], [6.]])
    S = sel.block_scores(W, 3)
    for f in (sel.select_greedy, sel.select_bed):
        assert sorted(f(S, 3, 2)) in ([0, 3], [3])                       # greedy may block itself: (w3..w5) first, then (w0..w2)
    assert sel.select_optimal(S, 3, 2) == [0, 3]
    assert sorted(sel.select_bed(S, 3, 2)) == [0, 3]


def test_selectors_stop_when_nothing_is_left():
    S = np.array([1., 2., NEG, NEG, 4., NEG])
    assert sel.select_greedy(S, 2, 5) == [4, 1]
    assert sorted(sel.select_bed(S, 2, 5)) == [1, 4]
    assert sel.select_optimal(S, 2, 5) is None
    assert sel.select_greedy([], 2, 1) == [] and sel.select_bed([], 2, 1) == []


# ------------------------------------------------------------------ exhaustive enumeration
@pytest.mark.parametrize("seed", range(40))
def test_against_every_valid_selection(seed):
    rng = np.random.default_rng(seed)
    N = int(rng.integers(2, 5))
    c_in = int(rng.integers(1, 4))
    c_out = int(rng.integers(N, max(N + 1, 16 // c_in + 1)))
    W, S = _layer(rng, c_out, c_in, N, integer=bool(seed % 2))
    cap = sum(c_out // N for _ in range(c_in))
    for m in range(0, cap + 1):
        best, sets = _enumerate(S, N, m)
        I = sel.select_optimal(S, N, m)
        assert I is not None and I == sorted(I)
        _valid(I, S, N, m)
        total = sum(S[k] for k in I)
        assert total == pytest.approx(best, rel=1e-12, abs=1e-12)
        if len(sets) == 1:
            assert tuple(I) == sets[0]
        for f in (sel.select_greedy, sel.select_bed):
            J = f(S, N, m)
            _valid(J, S, N)
            assert len(J) <= m
            if len(J) == m:
                assert sum(S[k] for k in J) <= best + 1e-9
    assert sel.select_optimal(S, N, cap + 1) is None


def test_optimal_prefers_not_taking_on_ties():
    # Eq. 4 takes candidate k only if that is strictly better, so of equal totals the one whose
    # last difference from the other lies at a lower index wins
    S = np.array([2., 2., 2., NEG])
    assert sel.select_optimal(S, 2, 1) == [0]
    S = np.array([1., 3., 1., 3., 1., NEG])
    assert sel.select_optimal(S, 2, 2) == [1, 3]


# ------------------------------------------------------------------ Algorithm 1 + 2
@pytest.mark.parametrize("seed", range(30))
def test_expansion_scores_add_up_to_what_division_keeps(seed):
    rng = np.random.default_rng(100 + seed)
    N = int(rng.integers(2, 7))
    c_out, c_in = int(rng.integers(N, 40)), int(rng.integers(1, 6))
    W, S = _layer(rng, c_out, c_in, N)                                  # integer weights: sums are exact
    cap = c_in * (c_out // N)
    for m in sorted({1, cap // 3, cap // 2, cap}):
        I_bar, picked = sel.block_expansion(S, N, m)
        I = sel.block_division(I_bar, N)
        _valid(I, S, N, len(I_bar))
        assert sum(picked) == sel.kept_l1(W, I, N)
        assert sum(S[k] for k in I) == sum(picked)
        assert not picked or picked[0] == S.max()
        if len(I) == m:                                                   # never above the optimum
            assert sum(picked) <= sum(S[k] for k in sel.select_optimal(S, N, m))


def test_expansion_reaches_every_block_when_asked_for_all():
    rng = np.random.default_rng(3)
    W = np.abs(rng.standard_normal((12, 3))) + 0.1                       # c_out a multiple of N: the layer can be tiled
    S = sel.block_scores(W, 4)
    I = sel.select_bed(S, 4, 9)
    assert sorted(I) == [0, 4, 8, 12, 16, 20, 24, 28, 32]
    assert len(sel.select_greedy(S, 4, 9)) <= 9


def test_division_cuts_runs_into_blocks_of_n():
    assert sel.block_division([], 3) == []
    assert sel.block_division([7], 3) == [7]
    assert sel.block_division([5, 4, 9], 3) == [4, 7, 10]                # one run of three blocks starting at 4
    assert sel.block_division([0, 3, 6], 3) == [0, 3, 6]                 # touching blocks stay where they are
    assert sel.block_division([2, 0, 12, 11], 2) == [0, 2, 11, 13]


def test_bed_is_no_worse_than_greedy_on_average():
    # the method's claim (Section 5.1) in its weakest checkable form, on synthetic Gaussian weights
    rng = np.random.default_rng(11)
    g = b = 0.0
    for _ in range(20):
        W = rng.standard_normal((64, 8))
        S = sel.block_scores(W, 4)
        m = int(64 * 8 * 0.3 / 4)
        g += sum(S[k] for k in sel.select_greedy(S, 4, m))
        b += sum(S[k] for k in sel.select_bed(S, 4, m))
    assert b > g


# ------------------------------------------------------------------ Eq. 5
def test_efficacy_end_points():
    W = np.zeros((8, 2))
    W[1:3, 0] = [5., 6.]                                                 # the four largest magnitudes form two unaligned blocks
    W[5:7, 1] = [7., 8.]
    W[0, 0], W[3, 0], W[4, 1], W[7, 1] = 1., 2., 3., 4.
    S, Sa = sel.block_scores(W, 2), sel.block_scores(W, 2, aligned=True)
    I_abp = sel.select_greedy(Sa, 2, 2)
    I_opt = sel.select_optimal(S, 2, 2)
    assert sorted(I_abp) == [8 + 4, 8 + 6] and I_opt == [1, 8 + 5]
    assert sel.efficacy(W, 2, I_abp, I_abp) == 0.0
    assert sel.efficacy(W, 2, I_opt, I_abp) == 1.0
    # hand value: UBP keeps 26, ABP keeps (3+7)+(8+4) = 22, EP keeps 26
    assert sel.kept_l1(W, I_abp, 2) == 22.0 and sel.kept_l1(W, I_opt, 2) == 26.0
    I_mid = [1, 8 + 4]                                                    # 11 + 10 = 21 -> below the aligned choice
    assert sel.efficacy(W, 2, I_mid, I_abp) == pytest.approx((21. - 22.) / (26. - 22.))


def test_indices_to_blocks():
    assert sel.indices_to_blocks([0, 5, 13], 6, bw=3).tolist() == [[0, 0], [5, 0], [1, 6]]
    assert sel.indices_to_blocks([], 6).shape == (0, 2)
