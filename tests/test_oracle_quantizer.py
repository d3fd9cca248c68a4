"""Pins for the oracle's random numbers, level tables and stochastic quantiser.

Each test checks the oracle against something the paper or the mathematics fixes,
never against the oracle's own formula.
"""
import itertools
import os

import numpy as np
import pytest

import oracle

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _read_rows(name):
    rows = []
    with open(os.path.join(GOLDEN, name)) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                rows.append(line.split())
    return rows


# ------------------------------------------------------------------ Philox
def test_philox_known_answers():
    for row in _read_rows("philox4x32_10_kat.txt"):
        v = [int(t, 16) for t in row]
        out = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(o) for o in out] == v[6:10]


def test_uniform24_keying_and_range():
    # word (col % 4) of the block keyed by (row, col // 4, epoch*256 + stream)
    seed, epoch, row = 0x0123456789ABCDEF, 7, (5 << 32) | 11
    for col in range(12):
        for stream in (1, 2, 3, 4):
            blk = oracle.philox4x32_10([row & 0xFFFFFFFF, row >> 32, col // 4,
                                        (epoch << 8) | stream],
                                       [seed & 0xFFFFFFFF, seed >> 32])
            expect = (int(blk[col % 4]) >> 8) / 2.0 ** 24
            got = oracle.uniform24(seed, epoch, row, col, stream)
            assert got == expect and 0.0 <= got < 1.0


def test_uniform24_moments_and_stream_independence():
    n = 40000
    u1 = np.array([oracle.uniform24(3, 0, i, 5, 1) for i in range(n)])
    u2 = np.array([oracle.uniform24(3, 0, i, 5, 2) for i in range(n)])
    assert abs(u1.mean() - 0.5) < 5 * np.sqrt(1 / 12 / n)
    assert abs(u1.var() - 1 / 12) < 5 * np.sqrt(1 / 180 / n)
    corr = np.corrcoef(u1, u2)[0, 1]
    assert abs(corr) < 5 / np.sqrt(n)
    # neighbouring columns and rows are uncorrelated too
    u3 = np.array([oracle.uniform24(3, 0, i, 6, 1) for i in range(n)])
    assert abs(np.corrcoef(u1, u3)[0, 1]) < 5 / np.sqrt(n)
    assert abs(np.corrcoef(u1[:-1], u1[1:])[0, 1]) < 5 / np.sqrt(n)


# ------------------------------------------------------------------ levels
@pytest.mark.parametrize("bits", [1, 2, 3, 4, 8])
def test_uniform_levels_closed_form(bits):
    lo = np.array([-1.0, 0.0, -0.05, 2.5], np.float32)
    hi = np.array([1.0, 1.0, 0.05, 2.5], np.float32)
    L = oracle.levels_uniform(lo, hi, bits)
    K = 1 << bits
    assert L.shape == (4, K)
    assert np.array_equal(L[:, 0], lo) and np.array_equal(L[:, -1], hi)
    assert np.all(np.diff(L, axis=1) >= 0)
    # evenly spaced: equal to numpy's linspace within one fp32 ulp of the range
    for j in range(4):
        ref = np.linspace(float(lo[j]), float(hi[j]), K)
        assert np.max(np.abs(L[j] - ref)) <= 1.2e-7 * max(1.0, abs(float(hi[j])))


def test_col_range_matches_numpy():
    rng = np.random.default_rng(0)
    A = rng.standard_normal((333, 17)).astype(np.float32)
    lo, hi = oracle.col_range(A)
    assert np.array_equal(lo, A.min(0)) and np.array_equal(hi, A.max(0))
    lo, hi = oracle.col_range(A, symmetric=True)
    M = np.abs(A).max(0)
    assert np.array_equal(hi, M) and np.array_equal(lo, -M)


# ------------------------------------------------------------------ quantiser
def test_paper_example_point_seven():
    (row,) = _read_rows("paper_quantize_example.txt")
    v, a, b, p = (float(t) for t in row)
    L = np.array([a, b], np.float32)
    l, frac = oracle.bracket(L, 1, v)
    assert l == 0
    assert abs(frac - p) < 1e-7
    # drawn frequency of the upper level
    n = 200000
    A = np.full((n, 1), v, np.float32)
    c1, c2 = oracle.quantize(A, L[None, :], 1, seed=1, epoch=0)
    for c in (c1, c2):
        f = c.mean()
        assert abs(f - p) < 5 * np.sqrt(p * (1 - p) / n)


def test_two_outcome_expectation_is_the_value():
    """E[Q(v)] = v (Sec. 2.1): with P(up) = frac the mean of the two outcomes is v."""
    rng = np.random.default_rng(1)
    for bits in (1, 2, 3, 5, 8):
        K = 1 << bits
        lo, hi = np.float32(-0.7), np.float32(1.3)
        L = oracle.levels_uniform([lo], [hi], bits)[0]
        for v in rng.uniform(lo, hi, size=200).astype(np.float32):
            l, frac = oracle.bracket(L, bits, float(v))
            assert 0 <= l <= K - 2 and 0.0 <= frac <= 1.0
            assert L[l] <= v <= L[l + 1]
            mean = (1 - frac) * float(L[l]) + frac * float(L[l + 1])
            w = float(L[l + 1]) - float(L[l])
            assert abs(mean - float(v)) <= 2e-7 * w + 1e-12


def test_values_on_a_level_outside_the_range_and_flat_columns():
    L = oracle.levels_uniform([-1.0], [1.0], 2)[0]           # -1, -1/3, 1/3, 1
    for c in range(4):
        l, frac = oracle.bracket(L, 2, float(L[c]))
        assert frac == 0.0 or (frac == 1.0 and l + 1 == c) or l == c
        # decoded value is the level itself with certainty
        assert (frac == 0.0 and L[l] == L[c]) or (frac == 1.0 and L[l + 1] == L[c])
    assert oracle.bracket(L, 2, -5.0) == (0, 0.0)
    l, frac = oracle.bracket(L, 2, 5.0)
    assert (l, frac) == (2, 1.0)
    flat = np.full(4, 2.5, np.float32)
    A = np.full((50, 1), 2.5, np.float32)
    c1, c2 = oracle.quantize(A, flat[None, :], 2, 0, 0)
    assert np.all(flat[c1] == 2.5) and np.all(flat[c2] == 2.5)


@pytest.mark.parametrize("bits", [2, 4])
def test_empirical_mean_and_variance(bits):
    """Unbiasedness and the per-point variance (b - x)(x - a) of Sec. 3, by sampling."""
    n = 120000
    lo, hi = -1.0, 1.0
    L = oracle.levels_uniform([lo] * 6, [hi] * 6, bits)
    vals = np.array([-0.93, -0.41, 0.0, 0.123, 0.5, 0.99], np.float32)
    A = np.tile(vals, (n, 1))
    c1, c2 = oracle.quantize(A, L, bits, seed=42, epoch=3)
    for j, v in enumerate(vals):
        l, _ = oracle.bracket(L[j], bits, float(v))
        a, b = float(L[j, l]), float(L[j, l + 1])
        var = (b - float(v)) * (float(v) - a)
        for c in (c1, c2):
            assert set(np.unique(c[:, j])) <= {l, l + 1}
            q = L[j][c[:, j]].astype(np.float64)
            assert abs(q.mean() - float(v)) < 5 * np.sqrt(var / n) + 1e-7
            # variance of the sample variance of a two-point distribution
            m4 = np.mean((q - q.mean()) ** 4)
            assert abs(q.var() - var) < 5 * np.sqrt(max(m4 - var ** 2, 0) / n) + 1e-9
        # the two copies differ by at most one level and are independent
        assert np.max(np.abs(c1[:, j].astype(int) - c2[:, j].astype(int))) <= 1
        if var > 0:
            corr = np.corrcoef(c1[:, j], c2[:, j])[0, 1]
            assert abs(corr) < 5 / np.sqrt(n)


def test_quantize_row_offset_and_epoch_key_the_draw():
    rng = np.random.default_rng(5)
    A = rng.uniform(-1, 1, (64, 8)).astype(np.float32)
    L = oracle.levels_uniform([-1] * 8, [1] * 8, 3)
    full1, full2 = oracle.quantize(A, L, 3, 9, 1)
    part1, part2 = oracle.quantize(A[32:], L, 3, 9, 1, row0=32)
    assert np.array_equal(full1[32:], part1) and np.array_equal(full2[32:], part2)
    other1, _ = oracle.quantize(A, L, 3, 9, 2)
    assert not np.array_equal(full1, other1)


# ------------------------------------------------------------------ estimators (Sec. 2.2)
def _outcomes(L, bits, a):
    """Per coordinate: (lower code, P(up))."""
    return [oracle.bracket(L[j], bits, float(a[j])) for j in range(len(a))]


def test_naive_estimator_bias_is_D_x_and_double_sampling_removes_it():
    """Exact enumeration of every quantisation outcome for one sample (d = 5).

    Naive: E[g] = a(a.x - b) + D x with D_jj = E[Q(a_j)^2] - a_j^2 = (hi - a_j)(a_j - lo)
    (Sec. 2.2).  Double sampling (eq. (5)): E[g] = a(a.x - b).
    """
    rng = np.random.default_rng(11)
    d, bits = 5, 2
    L = oracle.levels_uniform([-1] * d, [1] * d, bits)
    a = rng.uniform(-1, 1, d).astype(np.float32)
    x = rng.standard_normal(d)
    b = 0.37
    oc = _outcomes(L, bits, a)
    g_full = a.astype(np.float64) * (a.astype(np.float64) @ x - b)
    err = np.array([(float(L[j, l + 1]) - float(a[j])) * (float(a[j]) - float(L[j, l]))
                    for j, (l, _) in enumerate(oc)])

    def prob(ups):
        p = 1.0
        for (l, f), up in zip(oc, ups):
            p *= f if up else 1.0 - f
        return p

    def codes(ups):
        return np.array([l + up for (l, _), up in zip(oc, ups)], np.uint8)

    e_naive = np.zeros(d)
    for ups in itertools.product((0, 1), repeat=d):
        e_naive += prob(ups) * oracle.grad_naive(codes(ups), L, bits, x, b)
    assert np.allclose(e_naive - g_full, err * x, atol=2e-6)
    assert np.linalg.norm(err * x) > 1e-2          # the bias is not small

    e_double = np.zeros(d)
    for u1 in itertools.product((0, 1), repeat=d):
        p1, c1 = prob(u1), codes(u1)
        for u2 in itertools.product((0, 1), repeat=d):
            e_double += p1 * prob(u2) * oracle.grad_double(c1, codes(u2), L, bits, x, b)
    assert np.allclose(e_double, g_full, atol=2e-6)


def test_double_sampled_gradient_monte_carlo_d64():
    """Same statement at the shape of the tiny workload, with the oracle's own draws."""
    rng = np.random.default_rng(2)
    d, bits, reps = 64, 4, 6000
    L = oracle.levels_uniform([-1] * d, [1] * d, bits)
    a = rng.uniform(-1, 1, d).astype(np.float32)
    x = rng.standard_normal(d)
    b = 0.5
    A = np.tile(a, (reps, 1))
    c1, c2 = oracle.quantize(A, L, bits, seed=77, epoch=0)
    G = np.stack([oracle.grad_double(c1[i], c2[i], L, bits, x, b) for i in range(reps)])
    g_full = a.astype(np.float64) * (a.astype(np.float64) @ x - b)
    se = G.std(axis=0) / np.sqrt(reps)
    assert np.all(np.abs(G.mean(axis=0) - g_full) < 5 * se + 1e-9)
    # and the naive estimator (same copy twice) is visibly off along x
    Gn = np.stack([oracle.grad_naive(c1[i], L, bits, x, b) for i in range(reps)])
    bias = Gn.mean(axis=0) - g_full
    err = np.array([(float(L[j, l + 1]) - float(a[j])) * (float(a[j]) - float(L[j, l]))
                    for j, (l, _) in enumerate(_outcomes(L, bits, a))])
    sen = Gn.std(axis=0) / np.sqrt(reps)
    assert np.all(np.abs(bias - err * x) < 5 * sen + 1e-9)


# ------------------------------------------------------------------ compact storage of the two samples
def test_compact_storage_of_two_samples():
    """Sec. 2.2, "Overhead of Storing Samples": the two samples of a value differ by at most one
    level, so a base level plus one bit per sample (b + 2 bits instead of 2 b) stores both."""
    # the paper's example: 0.7 between the levels 0 and 1 -- base 0, one bit per sample
    L = np.array([[0.0, 1.0]], np.float32)
    seen = set()
    for seed in range(40):
        c1, c2 = oracle.quantize(np.array([[0.7]], np.float32), L, 1, seed, 0)
        base, u1, u2 = oracle.compact_encode(c1, c2)
        assert base.shape == (1, 1) and base[0, 0] == min(c1[0, 0], c2[0, 0])
        assert (int(base[0, 0]) + int(u1[0, 0]), int(base[0, 0]) + int(u2[0, 0])) == (int(c1[0, 0]), int(c2[0, 0]))
        seen.add((int(c1[0, 0]), int(c2[0, 0])))
    assert seen == {(0, 0), (0, 1), (1, 0), (1, 1)}          # all four outcomes occur, all are stored
    # every pair that can occur round-trips; pairs further apart cannot occur and are refused
    for bits in (1, 2, 3, 8):
        K = 1 << bits
        a = np.array([(c, c) for c in range(K)] + [(c, c + 1) for c in range(K - 1)] +
                     [(c + 1, c) for c in range(K - 1)], np.uint8)
        base, u1, u2 = oracle.compact_encode(a[:, 0], a[:, 1])
        assert set(np.unique(u1)) <= {0, 1} and set(np.unique(u2)) <= {0, 1} and base.max() <= K - 1
        d1, d2 = oracle.compact_decode(base, u1, u2)
        assert np.array_equal(d1, a[:, 0]) and np.array_equal(d2, a[:, 1])
        assert oracle.compact_bits_per_value(bits) == bits + 2
    with pytest.raises(ValueError):
        oracle.compact_encode(np.array([0], np.uint8), np.array([2], np.uint8))
    # the premise, on quantised data: the two copies never differ by more than one level, and do
    # differ somewhere (per-feature levels, values inside, outside and on the levels)
    rng = np.random.default_rng(3)
    A = rng.uniform(-1.3, 1.3, (500, 37)).astype(np.float32)
    A[::9] = 0.5
    for bits in (1, 3, 8):
        Lv = oracle.levels_uniform(np.full(37, -1, np.float32), np.full(37, 1, np.float32), bits)
        c1, c2 = oracle.quantize(A, Lv, bits, 11, 2)
        diff = c1.astype(np.int64) - c2.astype(np.int64)
        assert np.abs(diff).max() == 1
        base, u1, u2 = oracle.compact_encode(c1, c2)
        d1, d2 = oracle.compact_decode(base, u1, u2)
        assert np.array_equal(d1, c1) and np.array_equal(d2, c2)
