"""Pins for the oracle's variance-optimal level search (Sec. 3)."""
import itertools

import numpy as np
import pytest

import oracle


def total_variance(points, endpoints):
    """sum_x (b - x)(x - a) for x in [a, b], straight from the definition of err(x, I)."""
    e = np.asarray(endpoints, np.float64)
    tot = 0.0
    for x in points:
        k = np.searchsorted(e, x, side="right") - 1
        k = min(max(k, 0), len(e) - 2)
        tot += (e[k + 1] - x) * (x - e[k])
    return tot


def brute_force(points, cand, s):
    """Best total variance over every choice of s-1 interior endpoints among cand[1:-1]."""
    best, arg = np.inf, None
    M = len(cand) - 1
    for interior in itertools.combinations(range(1, M), s - 1):
        idx = (0,) + interior + (M,)
        v = total_variance(points, [cand[i] for i in idx])
        if v < best - 1e-15:
            best, arg = v, idx
    return best, arg


def test_interval_cost_from_moments_equals_definition():
    rng = np.random.default_rng(0)
    t = np.sort(rng.uniform(0, 1, 300))
    M = 10
    cand = np.arange(M + 1) / M
    mom = oracle.bin_moments(t, cand)
    assert mom[:, 0].sum() == 300
    # one interval [0,1]: T(1, M)
    tot, idx = oracle.dp_levels(mom, cand, 1)
    assert list(idx) == [0, M]
    assert np.isclose(tot, total_variance(t, [0.0, 1.0]), rtol=1e-12)


@pytest.mark.parametrize("M,s,seed", [(8, 2, 0), (12, 3, 1), (16, 4, 2), (16, 5, 3), (10, 7, 4)])
def test_dp_equals_brute_force_on_candidate_grid(M, s, seed):
    rng = np.random.default_rng(seed)
    # skewed data, so the optimum is far from uniform
    t = np.clip(rng.beta(0.6, 3.0, size=200), 0, 1)
    cand = np.arange(M + 1) / M
    mom = oracle.bin_moments(t, cand)
    tot, idx = oracle.dp_levels(mom, cand, s)
    bf, arg = brute_force(t, cand, s)
    assert np.isclose(tot, bf, rtol=1e-10, atol=1e-12)
    assert idx[0] == 0 and idx[-1] == M and np.all(np.diff(idx) > 0)
    assert np.isclose(total_variance(t, cand[idx]), tot, rtol=1e-10, atol=1e-12)


def test_exact_dp_with_data_points_as_candidates():
    """Lemma 3: an optimal partition has its endpoints at data points (or 0, 1).  The DP on
    candidates = data points must therefore be as good as a fine brute force over an
    independent dense grid of endpoints."""
    rng = np.random.default_rng(5)
    t = np.sort(np.round(rng.beta(2, 5, size=10), 3))
    t = np.unique(t)
    cand = np.concatenate([[0.0], t[(t > 0) & (t < 1)], [1.0]])
    mom = oracle.bin_moments(t, cand)
    s = 3
    tot, idx = oracle.dp_levels(mom, cand, s)
    bf, _ = brute_force(t, cand, s)
    assert np.isclose(tot, bf, rtol=1e-10, atol=1e-13)
    fine = np.arange(0, 1001) / 1000.0           # contains every data point (3 decimals)
    best = np.inf
    for a, b in itertools.combinations(range(1, 1000, 7), 2):
        best = min(best, total_variance(t, [0.0, fine[a], fine[b], 1.0]))
    assert tot <= best + 1e-12


def test_monotone_in_levels_and_refinement_and_beats_uniform():
    rng = np.random.default_rng(6)
    t = np.clip(rng.lognormal(-2.0, 1.0, size=2000), 0, 1)
    M = 63                                       # divisible by 2^b - 1 for b = 1, 2, 3
    cand = np.arange(M + 1) / M
    mom = oracle.bin_moments(t, cand)
    prev = np.inf
    for bits in (1, 2, 3):
        s = (1 << bits) - 1
        tot, idx = oracle.dp_levels(mom, cand, s)
        assert tot <= prev + 1e-12
        prev = tot
        uniform = np.arange(s + 1) / s           # a subset of the candidates
        assert tot <= total_variance(t, uniform) + 1e-10
    # the skew makes the gain large (Sec. 5.2: optimal levels save bits)
    assert prev < 0.7 * total_variance(t, np.arange(8) / 7)
    # refining the candidate grid cannot hurt
    cand2 = np.arange(2 * M + 1) / (2 * M)
    tot2, _ = oracle.dp_levels(oracle.bin_moments(t, cand2), cand2, 7)
    assert tot2 <= prev + 1e-12


def test_discretisation_error_shrinks_with_M():
    """Theorem 2: the gap to the optimum decays like 1/(M k); here against the exact DP."""
    rng = np.random.default_rng(7)
    t = np.sort(rng.uniform(0, 1, 120))
    cand_exact = np.concatenate([[0.0], t, [1.0]])
    s = 3
    opt, _ = oracle.dp_levels(oracle.bin_moments(t, cand_exact), cand_exact, s)
    gaps = []
    for M in (8, 32, 128):
        cand = np.arange(M + 1) / M
        tot, _ = oracle.dp_levels(oracle.bin_moments(t, cand), cand, s)
        assert tot >= opt - 1e-12
        gaps.append((tot - opt) / len(t))
        # a = 1 (equal small intervals); b, c from the data
        bmax = oracle.bin_moments(t, cand)[:, 0].max() * M / len(t)
        c = 1.0 * s          # a large interval crosses at most M = c M / k small ones
        assert gaps[-1] <= bmax * s / (4 * M ** 3) + bmax * c ** 2 / (M * s) + 1e-12
    assert gaps[2] < gaps[0]


def test_hist_moments_and_levels_optimal_end_to_end():
    rng = np.random.default_rng(8)
    n, d, M, bits = 3000, 3, 64, 2
    A = np.exp(rng.standard_normal((n, d))).astype(np.float32)
    A[:, 2] = 0.25                               # a flat column
    lo, hi = oracle.col_range(A)
    hist = oracle.hist_moments(A, lo, hi, M)
    assert np.all(hist[:, :, 0].sum(axis=1) == n)
    t0 = (A[:, 0].astype(np.float64) - lo[0]) / (float(hi[0]) - float(lo[0]))
    ref = oracle.bin_moments(t0, np.arange(M + 1) / M)
    assert np.allclose(hist[0], ref, rtol=1e-12, atol=1e-12)
    L, G, mv = oracle.levels_optimal(hist, lo, hi, bits)
    assert np.array_equal(L[:, 0], lo) and np.array_equal(L[:, -1], hi)
    assert np.all(G[:, 0] == 0) and np.all(G[:, -1] == M)
    assert np.all(np.diff(G[:2].astype(int), axis=1) > 0)
    assert np.all(L[2] == 0.25)
    for j in range(2):
        expect = lo[j].astype(np.float64) + (float(hi[j]) - float(lo[j])) * G[j] / M
        assert np.allclose(L[j], expect, rtol=1e-7)
    # reported objective is the mean over features of total/N in normalised units
    per = []
    for j in range(3):
        tot, _ = oracle.dp_levels(hist[j], np.arange(M + 1) / M, 3)
        per.append(tot / n)
    assert np.isclose(mv, np.mean(per), rtol=1e-12)
    # optimal levels give a lower quantisation variance than uniform levels on this data
    tj = t0
    var_opt = total_variance(tj, G[0] / M)
    var_uni = total_variance(tj, np.arange(4) / 3)
    assert var_opt < 0.6 * var_uni


# ------------------------------------------------------------------ greedy intervals (supplement, Algorithm 1)
def test_greedy_intervals_worked_by_hand():
    """M = 8 bins, k = 1 (2 pairs stay split, at most 5 intervals).  Errors of the merged pairs, by
    the definition err = sum (b - t)(t - a):
      pass 1:  [0,.25): .2*.05 + .15*.1 = .025   [.25,.5): .2*.05 = .010
               [.5,.75): .2*.05 + .15*.1 + .05*.2 = .035   [.75,1]: .05*.2 = .010
               -> first and third stay split: edges 0 1 2 4 5 6 8 (6 intervals)
      pass 2:  [0,.25): .025   [.25,.625): .325*.05 + .075*.3 + .025*.35 = .0475
               [.625,1]: .3*.075 + .05*.325 = .03875
               -> second and third stay split: edges 0 2 4 5 6 8 (5 intervals, done)."""
    t = np.array([0.05, 0.10, 0.30, 0.55, 0.60, 0.70, 0.95])
    M = 8
    mom = oracle.bin_moments(t, np.arange(M + 1) / M)
    edge, out = oracle.greedy_intervals(mom, 1)
    assert edge.tolist() == [0, 2, 4, 5, 6, 8]
    assert out[:, 0].tolist() == [2, 1, 2, 1, 1]
    assert np.allclose(out, oracle.bin_moments(t, edge / M), rtol=0, atol=1e-15)


def test_greedy_intervals_ties_go_left():
    """One point in the middle of each of 16 bins, k = 1: every number is a short dyadic fraction, so
    equal errors are equal to the last bit and the rule for ties decides.
      pass 1:  8 equal pairs, the two on the left stay split: 0 1 2 3 4 6 8 10 12 14 16
      pass 2:  pairs [0,2) [2,4) (2 points) [4,8) [8,12) [12,16) (4 points, larger): the first two
               of the three large ones stay split: 0 2 4 6 8 10 12 16
      pass 3:  [0,4) [4,8) [8,12) equal (the odd interval [12,16) is left alone): 0 2 4 6 8 12 16
      pass 4:  [0,4) [4,8) (4 points) [8,16) (8 points): 0 2 4 8 12 16."""
    M = 16
    t = (np.arange(M) + 0.5) / M
    edge, out = oracle.greedy_intervals(oracle.bin_moments(t, np.arange(M + 1) / M), 1)
    assert edge.tolist() == [0, 2, 4, 8, 12, 16]
    assert out[:, 0].tolist() == [2, 2, 4, 4, 4]


@pytest.mark.parametrize("M,k,seed", [(64, 3, 0), (128, 7, 1), (256, 7, 2), (100, 4, 3), (512, 15, 4)])
def test_greedy_intervals_within_twice_the_optimum(M, k, seed):
    """The supplement's theorem with gamma = 1: at most 4k + 1 intervals whose error, taken from the
    points by the definition, is at most 2 OPT_k (OPT_k from the dynamic program over all bin edges)."""
    rng = np.random.default_rng(seed)
    t = np.concatenate([rng.beta(0.6, 2.5, 4000), rng.uniform(0.7, 0.9, 500), [0.0, 1.0]])
    cand = np.arange(M + 1) / M
    mom = oracle.bin_moments(t, cand)
    edge, out = oracle.greedy_intervals(mom, k)
    P = len(edge) - 1
    assert k <= P <= 4 * k + 1
    assert edge[0] == 0 and edge[-1] == M and np.all(np.diff(edge) > 0)
    assert np.allclose(out, oracle.bin_moments(t, edge / M), rtol=1e-12, atol=1e-12)
    opt, _ = oracle.dp_levels(mom, cand, k)
    assert opt > 0
    assert total_variance(t, edge / M) <= 2.0 * opt * (1 + 1e-12)


def test_levels_greedy_against_the_full_dynamic_program():
    rng = np.random.default_rng(11)
    n, d, M, bits = 4000, 4, 256, 3
    A = np.exp(rng.standard_normal((n, d))).astype(np.float32)
    # column 3: eight clusters on bin edges -> the optimum is zero and the greedy search must keep it
    pos = np.array([0, 16, 40, 64, 100, 160, 200, 256]) / M
    A[:, 3] = pos[rng.integers(0, 8, n)]
    A[:8, 3] = pos
    lo, hi = oracle.col_range(A)
    hist = oracle.hist_moments(A, lo, hi, M)
    Lg, Gg, mvg = oracle.levels_greedy(hist, lo, hi, bits)
    Lo, Go, mvo = oracle.levels_optimal(hist, lo, hi, bits)
    assert np.array_equal(Gg[3], (pos * M).astype(np.uint16)) and np.array_equal(Gg[3], Go[3])
    assert np.all(Gg[:, 0] == 0) and np.all(Gg[:, -1] == M) and np.all(np.diff(Gg.astype(int), axis=1) > 0)
    for j in range(d):
        tg, _ = oracle.dp_levels(hist[j], np.arange(M + 1) / M, 7)
        tj = (A[:, j].astype(np.float64) - lo[j]) / (float(hi[j]) - float(lo[j]))
        vg = total_variance(tj, Gg[j] / M)
        assert vg >= tg * (1 - 1e-9) - 1e-9            # k intervals cannot beat the optimum ...
        assert vg <= 2.0 * tg * (1 + 1e-9) + 1e-9      # ... and stay within the factor the paper gives
    assert mvo <= mvg * (1 + 1e-12) <= 2 * mvo * (1 + 1e-9) + 1e-12
    # with no more than 4k + 1 bins nothing is merged: the plain dynamic program
    hist2 = oracle.hist_moments(A, lo, hi, 29)
    L1, G1, mv1 = oracle.levels_greedy(hist2, lo, hi, bits)
    L2, G2, mv2 = oracle.levels_optimal(hist2, lo, hi, bits)
    assert np.array_equal(G1, G2) and np.array_equal(L1, L2) and mv1 == mv2
