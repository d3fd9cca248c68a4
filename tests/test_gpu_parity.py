"""GPU parity: every step of the hot path, through the C ABI, against the CPU oracle.

Integer results (quantised codes, model/gradient codes, int32 dot products) must be
bit-exact; the fp32 model and the loss must agree within a relative L2 of 1e-5.
"""
import numpy as np
import pytest
import torch

import oracle
from gpu_harness import (DEV, E2E_EPOCH_BAND, GpuProblem, check_level_sets, dev, e2e_step_check,
                         max_abs_ok, rel_l2)
from paper_1611_05402_amd import synth, zipml

pytestmark = pytest.mark.gpu

# Relative L2 on model and loss.  The oracle evaluates a step in fp64 and stores the model in fp32; the
# kernels sum in fp32 in another order (about sqrt(d) 2^-24 per dot product) or exactly on fixed-point
# digits (2^-29 of the largest element); SGD contracts these errors, the observed figure is 1e-7.
TOL = 1e-5


def say(*a):
    print(*a, flush=True)


def uniform_levels_np(d, bits, lo, hi):
    return oracle.levels_uniform(np.full(d, lo, np.float32), np.full(d, hi, np.float32), bits)


# ------------------------------------------------------------------ levels
@pytest.mark.parametrize("flags", [0, zipml.SYMMETRIC])
def test_uniform_levels_and_ranges(flags):
    say("levels uniform flags", flags)
    rng = np.random.default_rng(0)
    A = (rng.standard_normal((3000, 70)) * rng.uniform(0.1, 3, 70)).astype(np.float32)
    p = GpuProblem(A, np.zeros(3000, np.float32), 5, 32)
    p.make_levels(zipml.UNIFORM, flags)
    lo, hi = oracle.col_range(A, symmetric=bool(flags & zipml.SYMMETRIC))
    assert np.array_equal(p.lo.cpu().numpy(), lo) and np.array_equal(p.hi.cpu().numpy(), hi)
    assert np.array_equal(p.levels.cpu().numpy(), oracle.levels_uniform(lo, hi, 5))
    assert np.array_equal(p.grid.cpu().numpy(), np.tile(np.arange(32, dtype=np.int16), (70, 1)))
    # a given range is used as is
    p.make_levels(zipml.UNIFORM, 0, lo=np.full(70, -4.0), hi=np.full(70, 4.0))
    assert np.array_equal(p.levels.cpu().numpy(), uniform_levels_np(70, 5, -4.0, 4.0))


@pytest.mark.parametrize("n,d,M", [(6000, 40, 256), (20000, 288, 1024)], ids=["M256", "M1024"])
def test_optimal_levels_match_oracle_dp(n, d, M):
    """3-bit variance-optimal levels (Sec. 3.1-3.2) on M candidates -- 1024 is the value of the
    end-to-end workload -- against the oracle's dynamic program: objective, levels and grid
    indices; where the indices differ the two level sets must cost the same (ties)."""
    say("levels optimal", n, d, M)
    w = synth.e2e(n=n, d=d, n_candidates=M)
    A, b = w.full()
    p = GpuProblem(A, b, 3, 32, n_candidates=M)
    mv = p.make_levels(zipml.OPTIMAL, 0, n_candidates=M, want_mv=True)
    lo, hi = oracle.col_range(A)
    assert np.array_equal(p.lo.cpu().numpy(), lo) and np.array_equal(p.hi.cpu().numpy(), hi)
    hist = oracle.hist_moments(A, lo, hi, M)
    L, G, mv_ref = oracle.levels_optimal(hist, lo, hi, 3)
    assert np.isclose(mv, mv_ref, rtol=1e-9)
    Gg = p.grid.cpu().numpy().view(np.uint16)
    Lg = p.levels.cpu().numpy()
    frac = check_level_sets(oracle, A, lo, hi, M, Gg, G, 0.9)
    say(f"  identical level sets on {frac:.4f} of the features")
    for j in range(d):
        expect = (lo[j].astype(np.float64) + (float(hi[j]) - float(lo[j])) * Gg[j] / M)
        assert np.array_equal(Lg[j], expect.astype(np.float32))


def test_device_and_host_level_search_agree(knobs):
    """The dynamic program runs on the device when its tables fit in LDS and on the host cores
    otherwise; both must give the same levels, index by index."""
    say("levels optimal: device vs host dynamic program")
    w = synth.e2e(n=4096, d=70, n_candidates=512)
    A, b = w.full()
    for bits in (2, 3, 5):
        res = []
        for host in (False, True):
            if host:
                knobs(zipml.KNOB_HOST_DP, 1)
            else:
                knobs(zipml.KNOB_HOST_DP, -1)
            p = GpuProblem(A, b, bits, 32, n_candidates=512)
            mv = p.make_levels(zipml.OPTIMAL, 0, n_candidates=512, want_mv=True)
            res.append((p.grid.cpu().numpy().copy(), p.levels.cpu().numpy().copy(), mv))
        knobs(zipml.KNOB_HOST_DP, -1)
        assert np.array_equal(res[0][0], res[1][0])
        assert np.array_equal(res[0][1], res[1][1])
        # (the bin moments are accumulated with atomics, so two runs may differ in the last bits)
        assert np.isclose(res[0][2], res[1][2], rtol=1e-12, atol=0)
        G = res[0][0].view(np.uint16)
        assert np.all(G[:, 0] == 0) and np.all(G[:, -1] == 512) and np.all(np.diff(G.astype(np.int32), axis=1) > 0)


def test_greedy_levels_bit_exact_on_dyadic_data():
    """Greedy merging of the bins, then the dynamic program over the end points that are left
    (Sec. 3.2; supplement, Algorithm 1).  The values are multiples of 2^-10 on a given range [0, 1],
    so the bin moments are exact whatever the order of their sums, and every later step has a fixed
    order: levels, grid indices and objective must be those of the oracle, bit for bit."""
    say("levels greedy: dyadic data")
    rng = np.random.default_rng(5)
    n, d = 6000, 40
    t = np.concatenate([rng.beta(0.5, 3.0, (n // 2, d)), rng.beta(4.0, 1.5, (n - n // 2, d))])
    t[:, 7] = rng.integers(0, 5, n) / 4.0                   # a column with five values
    t[:, 8] = 0.375                                         # a constant column
    A = (np.round(t * 1024) / 1024).astype(np.float32)
    b = np.zeros(n, np.float32)
    for bits, M in ((2, 256), (3, 512), (4, 1024), (5, 2000), (3, 4096), (1, 77)):
        p = GpuProblem(A, b, bits, 32, n_candidates=M)
        mv = p.make_levels(zipml.GREEDY, 0, lo=np.zeros(d), hi=np.ones(d), n_candidates=M, want_mv=True)
        hist = oracle.hist_moments(A, np.zeros(d, np.float32), np.ones(d, np.float32), M)
        L, G, mv_ref = oracle.levels_greedy(hist, np.zeros(d, np.float32), np.ones(d, np.float32), bits)
        say(f"  bits {bits}, {M} bins: objective {mv:.6e} (oracle {mv_ref:.6e})")
        assert np.array_equal(p.grid.cpu().numpy().view(np.uint16), G)
        assert np.array_equal(p.levels.cpu().numpy(), L)
        assert mv == mv_ref
        # not the plain search: on some feature the greedy candidates miss the optimum
        Lo, Go, mvo = oracle.levels_optimal(hist, np.zeros(d, np.float32), np.ones(d, np.float32), bits)
        assert mvo <= mv <= 2 * mvo
    # more features than the launch has workgroups (each then takes several)
    n2, d2, M2 = 512, 2100, 512
    A2 = (rng.integers(0, 1025, (n2, d2)) ** 2 / 1024 ** 2 * 1024).round().astype(np.float32) / 1024
    z2, o2 = np.zeros(d2, np.float32), np.ones(d2, np.float32)
    p = GpuProblem(A2, np.zeros(n2, np.float32), 2, 32, n_candidates=M2)
    mv = p.make_levels(zipml.GREEDY, 0, lo=z2, hi=o2, n_candidates=M2, want_mv=True)
    L, G, mv_ref = oracle.levels_greedy(oracle.hist_moments(A2, z2, o2, M2), z2, o2, 2)
    assert np.array_equal(p.grid.cpu().numpy().view(np.uint16), G)
    assert np.array_equal(p.levels.cpu().numpy(), L)
    assert np.isclose(mv, mv_ref, rtol=1e-12)      # (the mean over 2100 features is summed on the host)
    # The bin moments are gathered in one of two ways: many features -> a workgroup has all rows of
    # its features and stores its bins; few features -> slabs of rows, each with its own copy of the
    # bins, added up afterwards.  On this data both give the same moments exactly, so 300 features at
    # once (first way: at 4096 bins two features per workgroup) must get the levels that slices of
    # 40 of them get (second way, the one compared with the oracle above).
    n3, d3, M3 = 2048, 300, 4096
    A3 = (rng.beta(0.7, 2.0, (n3, d3)) * 1024).round().astype(np.float32) / 1024
    z3, o3 = np.zeros(d3, np.float32), np.ones(d3, np.float32)
    p = GpuProblem(A3, np.zeros(n3, np.float32), 3, 32, n_candidates=M3)
    p.make_levels(zipml.GREEDY, 0, lo=z3, hi=o3, n_candidates=M3)
    G_all = p.grid.cpu().numpy().view(np.uint16).copy()
    for c0 in range(0, d3, 40):
        sl = slice(c0, min(c0 + 40, d3))
        q = GpuProblem(np.ascontiguousarray(A3[:, sl]), np.zeros(n3, np.float32), 3, 32, n_candidates=M3)
        q.make_levels(zipml.GREEDY, 0, lo=z3[sl], hi=o3[sl], n_candidates=M3)
        assert np.array_equal(q.grid.cpu().numpy().view(np.uint16), G_all[sl])
    L, G, _ = oracle.levels_greedy(oracle.hist_moments(A3[:, :8], z3[:8], o3[:8], M3), z3[:8], o3[:8], 3)
    assert np.array_equal(G_all[:8], G)
    # with few bins nothing is merged: the plain search, on the device or on the host
    p = GpuProblem(A, b, 3, 32, n_candidates=29)
    p.make_levels(zipml.GREEDY, 0, lo=np.zeros(d), hi=np.ones(d), n_candidates=29)
    g1 = p.grid.cpu().numpy().copy()
    p.make_levels(zipml.OPTIMAL, 0, lo=np.zeros(d), hi=np.ones(d), n_candidates=29)
    assert np.array_equal(g1, p.grid.cpu().numpy())
    # tables that do not fit on the chip are refused
    p = GpuProblem(A, b, 8, 32, n_candidates=2048)
    with pytest.raises(zipml.ZipmlError) as e:
        p.make_levels(zipml.GREEDY, 0, lo=np.zeros(d), hi=np.ones(d), n_candidates=2048)
    assert e.value.code == zipml.EUNSUPPORTED


@pytest.mark.parametrize("n,d,pad,M", [(5000, 40, 0, 256), (5000, 42, 0, 256), (9000, 24, 3, 1024),
                                        (3000, 132, 4, 64), (70000, 8, 0, 128), (1500, 1, 0, 2048)],
                         ids=["d40", "d42_scalar_loads", "unaligned_rows", "padded_rows", "tall", "one_feature"])
def test_column_statistics_in_every_decomposition(n, d, pad, M, knobs):
    """Ranges (Supp. A.3) and bin moments (Sec. 3.2) are gathered by blocks of features x slabs of
    rows, with 16-byte or 4-byte loads depending on alignment, the number of features per
    workgroup depending on the bins that fit in LDS.  On values that are multiples of 2^-10 inside
    a range of width 1 the moments are exact in any order -- and every value sits exactly on a bin
    edge or at a fixed place inside a bin -- so ranges, levels, grid indices and objective must be
    the oracle's bit for bit, whatever the decomposition (features per workgroup forced to 1, 2,
    4 and the default; rows with and without padding)."""
    say("column statistics", n, d, pad, M)
    rng = np.random.default_rng(11)
    t = rng.beta(0.6, 2.5, (n, d))
    t[0, :] = 0.0
    t[1, :] = 1.0                                          # every column spans [0, 1] exactly
    A = (np.round(t * 1024) / 1024).astype(np.float32) + np.float32(0.25)    # ranges [0.25, 1.25]
    lda = d + pad
    Ap = np.full((n, lda), np.float32(99.0), np.float32)
    Ap[:, :d] = A
    A_dev = dev(Ap)
    bits = 3
    lo_ref, hi_ref = oracle.col_range(A)
    assert np.all(lo_ref == np.float32(0.25)) and np.all(hi_ref == np.float32(1.25))
    hist = oracle.hist_moments(A, lo_ref, hi_ref, M)
    L, G, mv_ref = oracle.levels_optimal(hist, lo_ref, hi_ref, bits)
    ws = torch.zeros(zipml.workspace_bytes(n, d, bits, 32, M), dtype=torch.uint8, device=DEV)
    for feats in (-1, 1, 2, 4):
        knobs(zipml.KNOB_HIST_FEATURES, feats)
        lo = torch.zeros(d, device=DEV)
        hi = torch.zeros(d, device=DEV)
        lev = torch.zeros(d, 1 << bits, device=DEV)
        grid = torch.zeros(d, 1 << bits, dtype=torch.int16, device=DEV)
        mv = zipml.levels(A_dev, n, d, lda, bits, zipml.OPTIMAL, 0, M, lo, hi, lev, grid, ws, True)
        assert np.array_equal(lo.cpu().numpy(), lo_ref) and np.array_equal(hi.cpu().numpy(), hi_ref)
        assert np.array_equal(grid.cpu().numpy().view(np.uint16), G), feats
        assert np.array_equal(lev.cpu().numpy(), L), feats
        assert np.isclose(mv, mv_ref, rtol=1e-12), feats
    knobs(zipml.KNOB_HIST_FEATURES, -1)


def test_greedy_levels_on_float_data():
    """Ordinary data: the device accumulates the bin moments with atomics, so their last bits --
    and with them a near-tie in the greedy search -- may differ from the oracle's.  What must hold
    either way: valid levels on the grid, an objective between the optimum and twice the optimum,
    and the oracle's choice on nearly every feature."""
    say("levels greedy: float data")
    w = synth.e2e(n=6000, d=40, n_candidates=512)
    A, b = w.full()
    M, bits = 512, 3
    p = GpuProblem(A, b, bits, 32, n_candidates=M)
    mv = p.make_levels(zipml.GREEDY, 0, n_candidates=M, want_mv=True)
    lo, hi = oracle.col_range(A)
    hist = oracle.hist_moments(A, lo, hi, M)
    L, G, mv_ref = oracle.levels_greedy(hist, lo, hi, bits)
    _, _, mv_opt = oracle.levels_optimal(hist, lo, hi, bits)
    Gg = p.grid.cpu().numpy().view(np.uint16)
    Lg = p.levels.cpu().numpy()
    assert np.all(Gg[:, 0] == 0) and np.all(Gg[:, -1] == M) and np.all(np.diff(Gg.astype(int), axis=1) > 0)
    for j in range(w.d):
        expect = (lo[j].astype(np.float64) + (float(hi[j]) - float(lo[j])) * Gg[j] / M)
        assert np.array_equal(Lg[j], expect.astype(np.float32))
    same = np.mean([np.array_equal(Gg[j], G[j]) for j in range(w.d)])
    say(f"  objective {mv:.6e}, oracle {mv_ref:.6e}, optimum {mv_opt:.6e}; same levels on {same:.0%} of the features")
    assert same > 0.9
    assert mv_opt * (1 - 1e-9) <= mv <= 2 * mv_opt
    if same == 1.0:
        assert np.isclose(mv, mv_ref, rtol=1e-9)


# ------------------------------------------------------------------ quantise
QCASES = [
    # name, n, d, bits, level spec
    ("tiny", 4096, 64, 4, "fixed"),
    ("ragged1", 1000, 70, 1, "fixed"),
    ("ragged3", 1000, 70, 3, "minmax"),
    ("b5", 512, 33, 5, "symmetric"),
    ("b6", 480, 160, 6, "fixed"),
    ("b7", 96, 224, 7, "fixed"),
    ("dense8", 2048, 288, 8, "fixed"),
    ("lowbit", 4096, 96, 2, "symmetric"),
]


@pytest.mark.parametrize("name,n,d,bits,spec", QCASES)
def test_quantized_codes_bit_exact(name, n, d, bits, spec):
    say("quantize", name, n, d, bits, spec)
    w = synth.lowbit(n=n, d=d) if spec == "symmetric" else synth.tiny(n=n, d=d)
    A, b = w.full()
    if name == "ragged3":
        A = (A * 1.7 + 0.3).astype(np.float32)
    p = GpuProblem(A, b, bits, 32)
    if spec == "fixed":
        A[::7, ::5] = 1.5          # values outside the level range are clamped
        A[1::7, ::3] = -1.0        # and values exactly on a level stay there
        p = GpuProblem(A, b, bits, 32)
        L = uniform_levels_np(d, bits, -1.0, 1.0)
        p.set_levels(L)
    else:
        lo, hi = oracle.col_range(A, symmetric=(spec == "symmetric"))
        L = oracle.levels_uniform(lo, hi, bits)
        p.make_levels(zipml.UNIFORM, zipml.SYMMETRIC if spec == "symmetric" else 0)
        assert np.array_equal(p.levels.cpu().numpy(), L)
    seed, epoch = 0x1234567887654321, 5
    p.quantize(seed, epoch)
    c1, c2 = oracle.quantize(A, L, bits, seed, epoch)
    assert np.array_equal(p.codes(1), c1)
    assert np.array_equal(p.codes(2), c2)
    # chunk-wise quantisation fills the same buffers
    q = GpuProblem(A, b, bits, 32)
    q.set_levels(L)
    q.quantize(seed, epoch, chunks=3)
    assert torch.equal(q.p1, p.p1) and torch.equal(q.p2, p.p2)


def test_quantize_optimal_levels_and_epoch_key():
    say("quantize optimal levels")
    w = synth.e2e(n=2048, d=64, n_candidates=128)
    A, b = w.full()
    lo, hi = oracle.col_range(A)
    L, G, _ = oracle.levels_optimal(oracle.hist_moments(A, lo, hi, 128), lo, hi, 3)
    p = GpuProblem(A, b, 3, 32)
    p.set_levels(L, G)
    for epoch in (0, 1):
        p.quantize(9, epoch)
        c1, c2 = oracle.quantize(A, L, 3, 9, epoch)
        assert np.array_equal(p.codes(1), c1) and np.array_equal(p.codes(2), c2)


# ------------------------------------------------------------------ compact storage
@pytest.mark.parametrize("n,d,bits", [(4096, 64, 4), (1000, 70, 3), (2048, 288, 8), (333, 5, 1), (96, 224, 7)])
def test_compact_storage_roundtrip_and_layout(n, d, bits):
    """Base level + one bit per sample (Sec. 2.2, "Overhead of Storing Samples"): what the device
    stores is the oracle's (min of the codes, bit, bit), it is (bits + 2) / (2 bits) of the two
    packed copies, and decoding restores both copies bit for bit -- in both layouts."""
    say("compact", n, d, bits)
    w = synth.tiny(n=n, d=d)
    A, b = w.full()
    L = uniform_levels_np(d, bits, -1.0, 1.0)
    p = GpuProblem(A, b, bits, 32)
    p.set_levels(L)
    p.quantize(17, 1)
    p1s, p2s = torch.zeros_like(p.p1), torch.zeros_like(p.p2)
    zipml.quantize_swapped(p.A, n, d, d, 0, n, p.levels, bits, 17, 1, p1s, p2s)
    c1, c2 = oracle.quantize(A, L, bits, 17, 1)
    base, u1, u2 = oracle.compact_encode(c1, c2)
    nbytes = zipml.compact_bytes(n, d, bits)
    assert nbytes * 2 * bits == 2 * zipml.packed_bytes(n, d, bits) * (bits + 2)
    out = torch.zeros(n, d, dtype=torch.uint8, device=DEV)
    # (a, b) = (copy 1, copy 2): sample-major pair (packed2s, packed2), feature-major pair (packed1, packed1s)
    for copy, pa, pb in ((2, p2s, p.p2), (1, p.p1, p1s)):
        comp = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
        zipml.compact_encode(pa, pb, n, d, bits, comp, p.ws)
        # the base plane is a packed array of its own, then come pairs of dwords: two 1-bit packed arrays
        nbase = zipml.packed_bytes(n, d, bits)
        zipml.unpack_codes(comp[:nbase], copy, n, d, bits, out)
        assert np.array_equal(out.cpu().numpy(), base)
        pairs = comp[nbase:].view(torch.int32).view(-1, 2)
        for plane, want in ((0, u1), (1, u2)):
            zipml.unpack_codes(pairs[:, plane].contiguous().view(torch.uint8), copy, n, d, 1, out)
            assert np.array_equal(out.cpu().numpy(), want)
        qa, qb = torch.zeros_like(pa), torch.zeros_like(pb)
        zipml.compact_decode(comp, n, d, bits, qa, qb)
        assert torch.equal(qa, pa) and torch.equal(qb, pb)
    # two arrays that are not samples of the same values are refused
    if bits >= 2:
        far = GpuProblem(-A, b, bits, 32)
        far.set_levels(L)
        far.quantize(17, 1)
        comp = torch.zeros(nbytes, dtype=torch.uint8, device=DEV)
        with pytest.raises(zipml.ZipmlError) as e:
            zipml.compact_encode(far.p2, p.p2, n, d, bits, comp, p.ws)
        assert e.value.code == zipml.EINVAL


# ------------------------------------------------------------------ loss
def test_loss_fp32_and_packed():
    """fp32 rows and both packed copies; copy 2 at 2, 4 and 8 bits runs on the matrix cores when the
    levels are evenly spaced (ragged n and d, an odd number of feature groups, many tiles per
    workgroup) and on the table path when one feature's levels are not."""
    say("loss")
    for (n, d, bits, uneven) in [(4096, 64, 4, False), (1000, 70, 3, False), (2048, 288, 8, False),
                                 (333, 5, 2, False), (70000, 1100, 8, False), (4096, 288, 4, True)]:
        w = synth.tiny(n=n, d=d)
        A, b = w.full()
        L = uniform_levels_np(d, bits, -1.0, 1.0)
        if uneven:
            L = L.copy()
            L[7] = np.sort(np.random.default_rng(1).uniform(-1, 1, 1 << bits)).astype(np.float32)
            L[7, 0], L[7, -1] = -1.0, 1.0
        p = GpuProblem(A, b, bits, 32)
        p.set_levels(L)
        p.quantize(3, 0)
        rng = np.random.default_rng(n)
        for x in (np.zeros(d, np.float32), w.x_star, rng.standard_normal(d).astype(np.float32)):
            xd = dev(x)
            ref = oracle.loss(A, b, x)
            assert abs(p.loss(xd) - ref) <= TOL * ref + 1e-12
            c1, c2 = oracle.quantize(A, L, bits, 3, 0)
            for copy, c in ((1, c1), (2, c2)):
                ref = oracle.loss_codes(c, L, bits, b, x)
                assert abs(p.loss(xd, packed_copy=copy) - ref) <= TOL * ref + 1e-12


# ------------------------------------------------------------------ SGD, fp32 model
SGD_CASES = [
    # name, workload factory, kwargs, epochs, lr
    ("tiny", synth.tiny, dict(), 5, 0.01),
    ("tiny_b4", synth.tiny, dict(n=512, d=64, batch=4), 2, 0.01),
    ("tiny_b8_ragged_d", synth.tiny, dict(n=512, d=70, batch=8, bits=3), 2, 0.01),
    ("dense8_small", synth.dense8, dict(n=4096, d=288, batch=256), 3, 1e-3),
    ("lowbit_small", synth.lowbit, dict(n=8192, d=96, batch=1024), 2, 0.05),
    ("b1", synth.tiny, dict(n=1024, d=96, batch=32, bits=1), 2, 0.01),
    ("b5", synth.tiny, dict(n=1024, d=160, batch=64, bits=5), 2, 0.01),
    ("b6", synth.tiny, dict(n=1024, d=32, batch=128, bits=6), 2, 0.01),
    ("b7", synth.tiny, dict(n=1024, d=64, batch=32, bits=7), 2, 0.01),
    ("tomo_small", synth.tomo, dict(n=2048, d=1024, batch=512), 2, 0.5),
]


def _levels_for(w, A):
    if w.range_mode == "symmetric":
        lo, hi = oracle.col_range(A, symmetric=True)
    else:
        lo, hi = np.full(w.d, w.lo, np.float32), np.full(w.d, w.hi, np.float32)
    return oracle.levels_uniform(lo, hi, w.bits)


@pytest.mark.parametrize("flags", [0, zipml.SGD_STEPWISE], ids=["persistent", "stepwise"])
@pytest.mark.parametrize("name,factory,kw,epochs,lr", SGD_CASES, ids=[c[0] for c in SGD_CASES])
def test_sgd_epochs_match_oracle(name, factory, kw, epochs, lr, flags):
    say("sgd", name, "flags", flags)
    w = factory(**kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L)
    p.quantize(7, 0)
    c1, c2 = oracle.quantize(A, L, w.bits, 7, 0)
    assert np.array_equal(p.codes(1), c1) and np.array_equal(p.codes(2), c2)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(epochs):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, lr)
        p.epoch(x, lr, flags=flags)
        xg = x.cpu().numpy()
        err = rel_l2(xg, x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}")
        assert err <= TOL and max_abs_ok(xg, x_ref, TOL)
        l_ref = oracle.loss(A, b, x_ref)
        assert abs(p.loss(x) - l_ref) <= TOL * l_ref + 1e-12
    assert np.linalg.norm(x_ref) > 0


@pytest.mark.parametrize("name,factory,kw,lr", [
    ("dense8_small", synth.dense8, dict(n=8192, d=288, batch=256), 1e-3),     # matrix-core loop
    ("lowbit_small", synth.lowbit, dict(n=8192, d=96, batch=1024), 0.05),     # 2-bit, per-column ranges
    ("b5", synth.tiny, dict(n=2048, d=160, batch=64, bits=5), 0.01),          # vector loop
    ("dense8_replicas", synth.dense8, dict(n=16384, d=288, batch=8192), 0.05),  # chunks on four replicas
])
def test_fp32_epochs_are_bit_reproducible(name, factory, kw, lr):
    """Sums across workgroups are integer sums: the order of arrival must not show in the result."""
    say("reproducible", name)
    w = factory(**kw)
    A, b = w.full()
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(_levels_for(w, A))
    p.quantize(3, 0)
    runs = []
    for _ in range(3):
        x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
        for _ep in range(3):
            p.epoch(x, lr)
        runs.append(x.cpu().numpy().view(np.uint32).copy())
    assert np.array_equal(runs[0], runs[1]) and np.array_equal(runs[0], runs[2])
    assert np.isfinite(runs[0].view(np.float32)).all() and np.any(runs[0] != 0)


@pytest.mark.parametrize("name,factory,kw,lr,exact", [
    ("dense8_small", synth.dense8, dict(n=8192, d=288, batch=256), 1e-3, True),          # feature owners
    ("dense8_replicas", synth.dense8, dict(n=16384, d=288, batch=8192), 0.05, True),     # replicas of them
    ("dense8_rows", synth.dense8, dict(n=32768, d=288, batch=16384), 0.05, False),       # sample owners
])
def test_ordinary_and_cooperative_launch_agree(name, factory, kw, lr, exact, knobs):
    """The epoch kernels are launched as ordinary kernels after the library's own check that the
    grid can be resident; the runtime's cooperative launch stays available behind a knob.  Same
    kernels, same arguments: the models must agree (bit for bit where the sums are integer sums)."""
    say("launch kinds", name)
    w = factory(**kw)
    A, b = w.full()
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(_levels_for(w, A))
    p.quantize(3, 0)
    res = []
    for coop in (-1, 1):
        knobs(zipml.KNOB_COOPERATIVE_LAUNCH, coop)
        x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
        for _ep in range(2):
            p.epoch(x, lr)
        res.append(x.cpu().numpy().copy())
    knobs(zipml.KNOB_COOPERATIVE_LAUNCH, -1)
    assert np.isfinite(res[0]).all() and np.any(res[0] != 0)
    if exact:
        assert np.array_equal(res[0].view(np.uint32), res[1].view(np.uint32))
    else:
        assert np.max(np.abs(res[0] - res[1])) <= 1e-6 * np.max(np.abs(res[0]))


@pytest.mark.parametrize("name,factory,kw,batch,lr,l2", [
    ("dense8_b16384", synth.dense8, dict(n=32768, d=288), 16384, 0.05, 0.0),     # odd number of feature groups
    ("dense8_wide_full_batch", synth.dense8, dict(n=16384, d=1100), 16384, 0.02, 0.0),
    ("lowbit_full_batch", synth.lowbit, dict(n=32768, d=96), 32768, 0.2, 0.0),   # 2-bit, per-column ranges
    ("tomo4_b16384", synth.tomo, dict(n=32768, d=256), 16384, 0.5, 0.0),         # 4-bit, sparse rows
    ("lssvm_b16384", synth.lssvm, dict(n=16384, d=288, bits=8), 16384, 0.05, 0.05),
])
def test_very_large_minibatches_on_sample_owners(name, factory, kw, batch, lr, l2, knobs):
    """Very large minibatches (by default from two tiles of 64 samples per compute unit on; here
    from 16,384 samples, the smallest the workspace provides for) go to workgroups that own samples
    instead of features: same estimator, same oracle."""
    say("sample owners", name)
    knobs(zipml.KNOB_ROWS_MIN_BATCH, 16384)
    w = factory(batch=batch, **kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, batch)
    p.set_levels(L)
    p.quantize(8, 0)
    c1, c2 = oracle.quantize(A, L, w.bits, 8, 0)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    runs = []
    for ep in range(4):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, batch, lr, l2=l2)
        zipml.sgd_epoch_l2(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, batch, lr, l2, p.ws)
        assert zipml.sgd_status(p.ws) == 0
        err = rel_l2(x.cpu().numpy(), x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}")
        assert err <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)
    assert np.linalg.norm(x_ref) > 0
    # the sums are taken in a fixed order: a second run gives the same bits
    y = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(4):
        zipml.sgd_epoch_l2(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, y, batch, lr, l2, p.ws)
    assert torch.equal(x, y)
    # levels that are not evenly spaced are refused through the status word
    L2 = L.copy()
    L2[1] = np.sort(np.random.default_rng(0).uniform(L[1, 0], L[1, -1], L.shape[1])).astype(np.float32)
    L2[1, 0], L2[1, -1] = L[1, 0], L[1, -1]
    p.set_levels(L2)
    x0 = x.clone()
    zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, batch, lr, p.ws)
    assert zipml.sgd_status(p.ws) == zipml.EUNSUPPORTED
    assert torch.equal(x, x0)


@pytest.mark.parametrize("name,factory,kw,batch,lr", [
    ("dense8_b4096", synth.dense8, dict(n=8192, d=288), 4096, 0.05),       # two chunks of 2048
    ("dense8_full_batch", synth.dense8, dict(n=8192, d=288), 8192, 0.05),  # gradient descent
    ("lowbit_b8192", synth.lowbit, dict(n=16384, d=96), 8192, 0.2),        # 2-bit, per-column ranges
    ("dense8_b6144", synth.dense8, dict(n=12288, d=288), 6144, 0.05),      # three chunks: one replica
    ("dense8_wide_b8192", synth.dense8, dict(n=16384, d=1100), 8192, 0.02),  # 8 chunks on 4 replicas of 35
    ("tomo4_b4096", synth.tomo, dict(n=8192, d=256), 4096, 0.5),           # 4-bit, sparse rows
])
def test_large_minibatches_taken_in_chunks(name, factory, kw, batch, lr):
    """A minibatch that does not fit one exchange is taken in chunks, and the chunks are shared
    out over replicas of the workgroups that exchange their gradient shares once per step."""
    say("large batch", name)
    w = factory(batch=batch, **kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, batch)
    p.set_levels(L)
    p.quantize(6, 0)
    c1, c2 = oracle.quantize(A, L, w.bits, 6, 0)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(4):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, batch, lr)
        p.epoch(x, lr)
        err = rel_l2(x.cpu().numpy(), x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}")
        assert err <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)
    assert np.linalg.norm(x_ref) > 0
    # with levels that are not evenly spaced such a batch is refused through the status word
    L2 = L.copy()
    L2[1] = np.sort(np.random.default_rng(0).uniform(L[1, 0], L[1, -1], L.shape[1])).astype(np.float32)
    L2[1, 0], L2[1, -1] = L[1, 0], L[1, -1]
    p.set_levels(L2)
    x0 = x.clone()
    zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, batch, lr, p.ws)
    assert zipml.sgd_status(p.ws) == zipml.EUNSUPPORTED
    assert torch.equal(x, x0)


@pytest.mark.parametrize("name,factory,kw,lr,avg", [
    ("dense8_wide_b512", synth.dense8, dict(n=4096, d=1100, batch=512), 1e-2, False),
    ("lowbit_b1024", synth.lowbit, dict(n=8192, d=640, batch=1024), 0.05, False),
    ("tomo4_b512", synth.tomo, dict(n=4096, d=1024, batch=512), 0.05, False),
    ("dense4_chunks_b4096", synth.dense8, dict(n=8192, d=1100, bits=4, batch=4096), 0.05, False),
    ("dense8_wide_b512_avg", synth.dense8, dict(n=4096, d=1100, batch=512), 1e-2, True),
    ("dense8_b4096_replicas", synth.dense8, dict(n=8192, d=288, batch=4096), 0.1, False),   # rows and results per replica
    ("tomo4_b2048_replicas", synth.tomo, dict(n=4096, d=2304, batch=2048), 0.05, False),
])
def test_exchange_through_tagged_stores(name, factory, kw, lr, avg, knobs):
    """The matrix-core loop with the sums of a step exchanged through tagged stores and reducer
    workgroups (forced here on small shapes; by default only hundreds of workgroups x samples take
    it): the sums are exact integers either way, so the epochs must equal those of the exchange
    through atomics bit for bit, and the oracle's within the tolerance."""
    say("tagged-store exchange", name)
    w = factory(**kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L)
    p.quantize(8, 0)
    p1s = p2s = None
    if avg:
        p1s, p2s = torch.zeros_like(p.p1), torch.zeros_like(p.p2)
        zipml.quantize_swapped(p.A, w.n, w.d, w.d, 0, w.n, p.levels, w.bits, 8, 0, p1s, p2s)
    c1, c2 = oracle.quantize(A, L, w.bits, 8, 0)
    res = []
    # (exchange through atomics; through tagged stores with the workgroups the library adds to do the
    # reducing on idle compute units -- a launch of the plain estimator without replicas gets them --;
    # with the owners of the features reducing themselves; with three such workgroups, which take
    # their pieces one after the other; with pieces of four words)
    # (and with none or five of the workgroups that read the next chunks' codes ahead on what is idle then)
    for xmin, reducers, readers in ((1 << 40, -1, -1), (0, -1, -1), (0, 0, -1), (0, 3, 5), (0, 104, 0), (0, -1, 0)):
        knobs(zipml.KNOB_STORE_EXCHANGE_MIN, xmin)
        knobs(zipml.KNOB_REDUCER_WORKGROUPS, reducers)
        knobs(zipml.KNOB_PREFETCH_WORKGROUPS, readers)
        x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
        for ep in range(2):
            if avg:
                zipml.sgd_epoch_avg(p.p1, p.p2, p1s, p2s, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, lr, p.ws)
                assert zipml.sgd_status(p.ws) == 0
            else:
                p.epoch(x, lr)
        res.append(x.cpu().numpy())
    knobs(zipml.KNOB_REDUCER_WORKGROUPS, -1)
    knobs(zipml.KNOB_PREFETCH_WORKGROUPS, -1)
    x_ref = np.zeros(w.d, np.float32)
    for ep in range(2):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, lr, symmetric=avg)
    for r in res[1:]:
        assert np.array_equal(res[0].view(np.uint32), r.view(np.uint32))
    assert rel_l2(res[1], x_ref) <= TOL and max_abs_ok(res[1], x_ref, TOL)


def test_sgd_fp32_one_feature_not_evenly_spaced():
    """Evenly spaced levels take the matrix-core loop; a single feature with other levels must
    send every workgroup down the table path (workgroups on different loops would scale their
    contributions to the exchange differently)."""
    say("sgd fp32, 8-bit, one feature with uneven levels")
    w = synth.dense8(n=4096, d=288, batch=256)
    A, b = w.full()
    L = _levels_for(w, A).copy()
    rng = np.random.default_rng(3)
    L[200] = np.sort(rng.uniform(-1, 1, 256)).astype(np.float32)
    L[200, 0], L[200, -1] = -1.0, 1.0
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L)
    p.quantize(2, 0)
    c1, c2 = oracle.quantize(A, L, w.bits, 2, 0)
    assert np.array_equal(p.codes(1), c1) and np.array_equal(p.codes(2), c2)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(2):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, 1e-3)
        p.epoch(x, 1e-3)
        assert rel_l2(x.cpu().numpy(), x_ref) <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)


def test_sgd_fp32_with_non_uniform_levels():
    say("sgd fp32, optimal levels (table look-up path)")
    w = synth.e2e(n=2048, d=96, batch=64, n_candidates=128)
    A, b = w.full()
    lo, hi = oracle.col_range(A)
    L, G, _ = oracle.levels_optimal(oracle.hist_moments(A, lo, hi, 128), lo, hi, 3)
    p = GpuProblem(A, b, 3, 64)
    p.set_levels(L, G)
    p.quantize(1, 0)
    c1, c2 = oracle.quantize(A, L, 3, 1, 0)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(2):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, 3, x_ref, 64, 0.2)
        p.epoch(x, 0.2)
        assert rel_l2(x.cpu().numpy(), x_ref) <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)


# ------------------------------------------------------------------ the production step, element by element
@pytest.mark.parametrize("bits", [8, 4, 2])
def test_production_step_residuals_and_gradient_element_by_element(bits):
    """One step of the headline shape's width (batch 256, d = 2048) in the launch and on the
    matrix-core loop that zipml_sgd_epoch takes, residuals and gradient compared element by
    element with the definition (eq. (5), Sec. 2.2) in fp64 on the oracle's codes; d + 13 covers
    a ragged last block of features."""
    for d in (2048, 2048 + 13):
        say("production step: bits", bits, "d", d)
        B, n = 256, 1024
        w = synth.dense8(n=n, d=d, bits=bits, batch=B)
        A, b = w.full()
        L = uniform_levels_np(d, bits, -1.0, 1.0)
        p = GpuProblem(A, b, bits, B)
        p.set_levels(L)
        p.quantize(3, 0)
        c1, c2 = oracle.quantize(A, L, bits, 3, 0)
        rng = np.random.default_rng(2)
        x0 = (rng.standard_normal(d) / np.sqrt(d)).astype(np.float32)
        for t in (0, 3):
            rows = slice(t * B, (t + 1) * B)
            Q2 = np.take_along_axis(L.T, c2[rows].astype(np.int64), axis=0).astype(np.float64)
            Q1 = np.take_along_axis(L.T, c1[rows].astype(np.int64), axis=0).astype(np.float64)
            r_ref = Q2 @ x0.astype(np.float64) - b[rows]
            g_ref = Q1.T @ r_ref / B
            x_ref = oracle.sgd_epoch(c1[rows], c2[rows], L, b[rows], bits, x0, B, 0.05)
            x = dev(x0)
            r = torch.zeros(B, dtype=torch.float32, device=DEV)
            g = torch.zeros(d, dtype=torch.float32, device=DEV)
            zipml.debug_step(p.p1, p.p2, p.levels, p.b, n, d, bits, x, B, 0.05, t, p.ws, r=r, g=g,
                             flags=zipml.SGD_PRODUCTION)
            assert zipml.sgd_status(p.ws) == 0
            rg, gg, xg = r.cpu().numpy(), g.cpu().numpy(), x.cpu().numpy()
            say(f"  step {t}: max|dr|/max|r| {np.max(np.abs(rg - r_ref)) / np.max(np.abs(r_ref)):.1e}, "
                f"max|dg|/max|g| {np.max(np.abs(gg - g_ref)) / np.max(np.abs(g_ref)):.1e}")
            assert rel_l2(rg, r_ref) <= TOL and max_abs_ok(rg, r_ref, TOL)
            assert rel_l2(gg, g_ref) <= TOL and max_abs_ok(gg, g_ref, TOL)
            assert rel_l2(xg, x_ref) <= TOL and max_abs_ok(xg, x_ref, TOL)
            # and the vector loop of the plain debug launch gives the same step
            x2 = dev(x0)
            r2 = torch.zeros_like(r)
            g2 = torch.zeros_like(g)
            zipml.debug_step(p.p1, p.p2, p.levels, p.b, n, d, bits, x2, B, 0.05, t, p.ws, r=r2, g=g2)
            assert max_abs_ok(r2.cpu().numpy(), r_ref, TOL) and max_abs_ok(g2.cpu().numpy(), g_ref, TOL)


def test_production_step_refusals():
    w = synth.tiny(n=1024, d=64, batch=64, bits=3)
    A, b = w.full()
    p = GpuProblem(A, b, 3, 64)
    p.set_levels(uniform_levels_np(64, 3, -1.0, 1.0))
    p.quantize(0, 0)
    x = torch.zeros(64, dtype=torch.float32, device=DEV)
    r = torch.zeros(64, dtype=torch.float32, device=DEV)
    mo = torch.zeros(64, dtype=torch.int32, device=DEV)
    with pytest.raises(zipml.ZipmlError) as e:      # 3-bit codes never take the matrix-core loop
        zipml.debug_step(p.p1, p.p2, p.levels, p.b, w.n, 64, 3, x, 64, 0.1, 0, p.ws, r=r,
                         flags=zipml.SGD_PRODUCTION)
    assert e.value.code == zipml.EUNSUPPORTED
    with pytest.raises(zipml.ZipmlError) as e:      # integer outputs belong to the end-to-end mode
        zipml.debug_step(p.p1, p.p2, p.levels, p.b, w.n, 64, 3, x, 64, 0.1, 0, p.ws, r=r, model_codes=mo,
                         flags=zipml.SGD_PRODUCTION)
    assert e.value.code == zipml.EINVAL
    with pytest.raises(zipml.ZipmlError) as e:      # nothing asked for
        zipml.debug_step(p.p1, p.p2, p.levels, p.b, w.n, 64, 3, x, 64, 0.1, 0, p.ws,
                         flags=zipml.SGD_PRODUCTION)
    assert e.value.code == zipml.EINVAL


# ------------------------------------------------------------------ end-to-end low precision
def _grid_uniform(bits, lo, hi):
    K = 1 << bits
    return np.float32(lo), np.float32((np.float64(hi) - np.float64(lo)) / (K - 1)), K - 1


E2E_CASES = [
    ("tiny_u4", dict(n=1024, d=64, batch=16, bits=4), 8, 8),
    ("tiny_u8_b256", dict(n=2048, d=288, batch=256, bits=8), 8, 8),
    ("tiny_u2_ragged", dict(n=512, d=70, batch=32, bits=2), 4, 6),
    ("model_only", dict(n=1024, d=96, batch=64, bits=4), 0, 8),
    # more than 256 features: several workgroups (the production launch takes the end-to-end loop)
    ("wide_u4_ragged", dict(n=2048, d=300, batch=64, bits=4), 8, 8),
    ("wide_u2", dict(n=1024, d=520, batch=32, bits=2), 4, 6),
    ("wide_model_only", dict(n=1024, d=352, batch=128, bits=4), 0, 8),
    ("wide_u4_b16", dict(n=512, d=288, batch=16, bits=4), 8, 8),
    ("wide_u3_b512", dict(n=2048, d=1100, batch=512, bits=3), 8, 8),
]


def e2e_epochs_check(p, c1, c2, L, G, glo, gstep, gmax, b, bits, batch, x0, lr, gb, mb, seed, epochs,
                     flags=0):
    """Whole end-to-end epochs against the oracle (band: see gpu_harness); returns the models."""
    x_ref = x0.copy()
    xd = dev(x0)
    for ep in range(epochs):
        x_ref = oracle.sgd_epoch_e2e(c1, c2, L, G, glo, gstep, b, bits, x_ref, batch, lr, gb, mb,
                                     seed, ep)
        p.epoch(xd, lr, seed=seed, epoch=ep, flags=flags, grad_bits=gb, model_bits=mb, grid_lo=glo,
                grid_step=gstep, grid_max=gmax)
        got = xd.cpu().numpy()
        same = np.array_equal(got.view(np.uint32), x_ref.view(np.uint32))
        say(f"    epoch {ep}: models {'identical' if same else 'differ'}, rel L2 {rel_l2(got, x_ref):.1e}")
        assert rel_l2(got, x_ref) <= E2E_EPOCH_BAND
    return xd, x_ref


@pytest.mark.parametrize("flags", [0, zipml.SGD_STEPWISE, zipml.SGD_PRODUCTION],
                         ids=["persistent", "stepwise", "production"])
@pytest.mark.parametrize("name,kw,gb,mb", E2E_CASES, ids=[c[0] for c in E2E_CASES])
def test_end_to_end_uniform_grid_steps_and_epochs(name, kw, gb, mb, flags):
    """flags = 0: single steps in the debug launch, epochs in the production launch; stepwise:
    both in one launch per segment; production: single steps in the production launch as well
    (shapes of more than 256 features, which several workgroups share)."""
    say("e2e", name, "flags", flags)
    if flags == zipml.SGD_PRODUCTION and kw["d"] <= 256:
        pytest.skip("one workgroup: no production step loop of its own")
    w = synth.tiny(**kw)
    A, b = w.full()
    L = uniform_levels_np(w.d, w.bits, -1.0, 1.0)
    G = np.tile(np.arange(1 << w.bits, dtype=np.uint16), (w.d, 1))
    glo, gstep, gmax = _grid_uniform(w.bits, -1.0, 1.0)
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L, G)
    p.quantize(11, 2)
    c1, c2 = oracle.quantize(A, L, w.bits, 11, 2)
    rng = np.random.default_rng(5)
    x0 = (rng.standard_normal(w.d) * 0.3).astype(np.float32)
    # single steps from a given model: every intermediate
    for step in (0, 3):
        e2e_step_check(p, oracle, c1, c2, L, G, glo, gstep, gmax, b, x0, 0.05, gb, mb, 11, 2, step, flags)
    eflags = flags & zipml.SGD_STEPWISE
    xd, _ = e2e_epochs_check(p, c1, c2, L, G, glo, gstep, gmax, b, w.bits, w.batch, x0, 0.05, gb, mb, 11, 2,
                             eflags)
    # and the run is reproducible
    xd2 = dev(x0)
    for ep in range(2):
        p.epoch(xd2, 0.05, seed=11, epoch=ep, flags=eflags, grad_bits=gb, model_bits=mb, grid_lo=glo,
                grid_step=gstep, grid_max=gmax)
    assert torch.equal(xd, xd2)


@pytest.mark.parametrize("d", [160, 416])
@pytest.mark.parametrize("batch", [64, 96, 512])
def test_end_to_end_optimal_levels_steps_and_epochs(batch, d):
    say("e2e optimal 3-bit levels, 8-bit model and gradient, batch", batch, "d", d)
    M = 256
    w = synth.e2e(n=batch * 24, d=d, batch=batch, n_candidates=M)
    A, b = w.full()
    lo, hi = np.zeros(w.d, np.float32), np.ones(w.d, np.float32)
    L, G, _ = oracle.levels_optimal(oracle.hist_moments(A, lo, hi, M), lo, hi, 3)
    glo, gstep, gmax = np.float32(0.0), np.float32(1.0 / M), M
    p = GpuProblem(A, b, 3, batch)
    p.set_levels(L, G)
    p.quantize(4, 0)
    c1, c2 = oracle.quantize(A, L, 3, 4, 0)
    assert np.array_equal(p.codes(1), c1) and np.array_equal(p.codes(2), c2)
    rng = np.random.default_rng(6)
    x0 = (rng.standard_normal(w.d) * 0.1).astype(np.float32)
    for step in (0, 7, 23):
        e2e_step_check(p, oracle, c1, c2, L, G, glo, gstep, gmax, b, x0, 0.3, 8, 8, 4, 0, step)
        if d > 256:
            e2e_step_check(p, oracle, c1, c2, L, G, glo, gstep, gmax, b, x0, 0.3, 8, 8, 4, 0, step,
                           zipml.SGD_PRODUCTION)
    _, x_ref = e2e_epochs_check(p, c1, c2, L, G, glo, gstep, gmax, b, 3, batch, np.zeros(w.d, np.float32),
                                0.3, 8, 8, 4, 2)
    assert np.linalg.norm(x_ref) > 0


# ------------------------------------------------------------------ symmetrised estimator
@pytest.mark.parametrize("name,factory,kw,lr,l2", [
    ("dense8_small", synth.dense8, dict(n=4096, d=288, batch=256), 1e-3, 0.0),
    ("dense8_wide_b512", synth.dense8, dict(n=4096, d=1100, batch=512), 1e-3, 0.0),
    ("lowbit_small", synth.lowbit, dict(n=8192, d=640, batch=1024), 0.05, 0.0),
    ("lssvm_4bit", synth.lssvm, dict(n=4096, d=288, bits=4, batch=128), 0.05, 0.05),
    ("dense8_b4096_chunks", synth.dense8, dict(n=8192, d=288, batch=4096), 0.05, 0.0),
    # sample owners (two tiles per sample block, one per code pair)
    ("dense8_b16384_rows", synth.dense8, dict(n=32768, d=288, batch=16384), 0.05, 0.0),
    ("lowbit_full_batch_rows", synth.lowbit, dict(n=32768, d=96, batch=32768), 0.2, 0.0),
    ("tomo4_b16384_rows", synth.tomo, dict(n=16384, d=1024, batch=16384), 0.5, 0.01),
])
def test_symmetrised_estimator_matches_oracle(name, factory, kw, lr, l2, knobs):
    """g = 1/2 mean_i [Q1 (Q2^T x - b) + Q2 (Q1^T x - b)] (Supp. B.2, footnote)."""
    say("averaged", name)
    knobs(zipml.KNOB_ROWS_MIN_BATCH, 16384)
    w = factory(**kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L)
    p.quantize(21, 0)
    p1s, p2s = torch.zeros_like(p.p1), torch.zeros_like(p.p2)
    zipml.quantize_swapped(p.A, w.n, w.d, w.d, 0, w.n, p.levels, w.bits, 21, 0, p1s, p2s)
    c1, c2 = oracle.quantize(A, L, w.bits, 21, 0)
    # the swapped arrays hold the other copy in the same layout
    out = torch.zeros(w.n, w.d, dtype=torch.uint8, device=DEV)
    zipml.unpack_codes(p1s, 1, w.n, w.d, w.bits, out)
    assert np.array_equal(out.cpu().numpy(), c2)
    zipml.unpack_codes(p2s, 2, w.n, w.d, w.bits, out)
    assert np.array_equal(out.cpu().numpy(), c1)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(3):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, lr, symmetric=True, l2=l2)
        zipml.sgd_epoch_avg(p.p1, p.p2, p1s, p2s, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, lr,
                            p.ws, l2=l2)
        assert zipml.sgd_status(p.ws) == 0
        err = rel_l2(x.cpu().numpy(), x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}")
        assert err <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)
    # it is a different estimator from eq. (5)
    x_plain = oracle.sgd_epoch(c1, c2, L, b, w.bits, np.zeros(w.d, np.float32), w.batch, lr, l2=l2)
    x_sym = oracle.sgd_epoch(c1, c2, L, b, w.bits, np.zeros(w.d, np.float32), w.batch, lr, symmetric=True, l2=l2)
    assert rel_l2(x_sym, x_plain) > 1e-5


def test_symmetrised_estimator_refusals():
    w = synth.tiny(n=1024, d=64, batch=64, bits=4)             # fits one workgroup: not on the matrix cores
    A, b = w.full()
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(_levels_for(w, A))
    p.quantize(1, 0)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    with pytest.raises(zipml.ZipmlError) as e:
        zipml.sgd_epoch_avg(p.p1, p.p2, p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, 0.01, p.ws)
    assert e.value.code == zipml.EUNSUPPORTED
    with pytest.raises(zipml.ZipmlError) as e:      # the flag of the plain entry point has no arrays to work on
        zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, 0.01, p.ws,
                        flags=zipml.SGD_AVERAGED)
    assert e.value.code == zipml.EUNSUPPORTED


@pytest.mark.parametrize("name,kw,batch,lr", [
    ("d96_full_batch", dict(n=32768, d=96), 32768, 0.2),        # one block of 128 features, a quarter of it padding
    ("d1100_b16384", dict(n=32768, d=1100), 16384, 0.1),        # 9 blocks: some waves have two; 35 feature groups
    ("d2100_b16384", dict(n=16384, d=2100), 16384, 0.05),       # 33 blocks of 64: the last block of 128 is half empty
])
def test_two_bit_sample_owners_with_the_dot_pass_in_fp4(name, kw, batch, lr, knobs):
    """2-bit codes at very large minibatches: the dot pass on the 4-bit floating-point matrix
    instruction (codes as E2M1 numbers, y in base-4 digits).  Same integers as the integer kernel:
    the same model bit for bit, and both match the oracle."""
    say("fp4 dot pass", name)
    knobs(zipml.KNOB_ROWS_MIN_BATCH, 16384)
    w = synth.lowbit(batch=batch, **kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, batch)
    p.set_levels(L)
    p.quantize(19, 0)
    c1, c2 = oracle.quantize(A, L, w.bits, 19, 0)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    x_int = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    x128 = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(4):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, batch, lr)
        knobs(zipml.KNOB_ROWS_ITEM_BLOCKS, -1)                # automatic: here tiles of 64 samples
        p.epoch(x, lr)
        knobs(zipml.KNOB_ROWS_ITEM_BLOCKS, 2)                 # an explicit item size: the integer kernel
        p.epoch(x_int, lr)
        knobs(zipml.KNOB_ROWS_ITEM_BLOCKS, 102)               # tiles of 128 samples (automatic from 32,768 x CUs / 128 samples on)
        p.epoch(x128, lr)
        err = rel_l2(x.cpu().numpy(), x_ref)
        err128 = rel_l2(x128.cpu().numpy(), x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}, with tiles of 128 samples {err128:.2e}")
        assert err <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)
        assert err128 <= TOL and max_abs_ok(x128.cpu().numpy(), x_ref, TOL)
        assert torch.equal(x, x_int)      # (same tiles, same sums; larger tiles add in another order)
    assert float(x.abs().max()) > 0.0


# ------------------------------------------------------------------ epoch on the compact record
@pytest.mark.parametrize("name,kw,lr", [
    ("d1000_b16384", dict(n=32768, d=1000, batch=16384), 0.05),    # 16 blocks of 64 features: two per wave
    ("d600_b16384", dict(n=16384, d=600, batch=16384), 0.05),      # 10 blocks, the last one half padding
    ("d1990_b16384", dict(n=32768, d=1990, batch=16384), 0.02),    # 32 blocks: four per wave, last half padding
    ("d2048_full_batch", dict(n=32768, d=2048, batch=32768), 0.02),
])
def test_epoch_on_the_compact_record(name, kw, lr, knobs):
    """Sec. 2.2, "Overhead of Storing Samples": the sample-owner epoch reading base + 1 bit per copy.
    Same integers as on the two packed copies, so the model is bit-identical to zipml_sgd_epoch's,
    and both match the oracle."""
    say("compact epoch", name)
    knobs(zipml.KNOB_ROWS_MIN_BATCH, 16384)       # zipml_sgd_epoch on the packed copies: sample owners too
    w = synth.dense8(**kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L)
    p.quantize(33, 0)
    p1s, p2s = torch.zeros_like(p.p1), torch.zeros_like(p.p2)
    zipml.quantize_swapped(p.A, w.n, w.d, w.d, 0, w.n, p.levels, w.bits, 33, 0, p1s, p2s)
    comp = torch.zeros(zipml.compact_bytes(w.n, w.d, w.bits), dtype=torch.uint8, device=DEV)
    zipml.compact_encode(p2s, p.p2, w.n, w.d, w.bits, comp, p.ws)      # (copy 1, copy 2), sample-major
    assert comp.numel() * 16 == p.p2.numel() * 2 * 10                 # 10 bits per value instead of 16
    del p1s, p2s
    c1, c2 = oracle.quantize(A, L, w.bits, 33, 0)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    xc = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(3):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, lr)
        p.epoch(x, lr)
        zipml.sgd_epoch_compact(comp, p.levels, p.b, w.n, w.d, w.bits, xc, w.batch, lr, p.ws)
        assert zipml.sgd_status(p.ws) == 0
        err = rel_l2(xc.cpu().numpy(), x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}")
        assert err <= TOL and max_abs_ok(xc.cpu().numpy(), x_ref, TOL)
        assert torch.equal(x, xc)
    assert float(xc.abs().max()) > 0.0


def test_epoch_on_the_compact_record_refusals():
    def refused(w, levels=None):
        A, b = w.full()
        p = GpuProblem(A, b, w.bits, w.batch)
        p.set_levels(_levels_for(w, A) if levels is None else levels(w, A))
        comp = torch.zeros(max(zipml.compact_bytes(w.n, w.d, w.bits), 16), dtype=torch.uint8, device=DEV)
        x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
        try:
            zipml.sgd_epoch_compact(comp, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, 0.01, p.ws)
        except zipml.ZipmlError as e:
            return e.code
        return zipml.sgd_status(p.ws)
    assert refused(synth.tiny(n=16384, d=1024, batch=16384, bits=4)) == zipml.EUNSUPPORTED     # 8 bits only
    assert refused(synth.dense8(n=8192, d=1024, batch=4096)) == zipml.EUNSUPPORTED             # small minibatch
    assert refused(synth.dense8(n=16384, d=512, batch=16384)) == zipml.EUNSUPPORTED            # 8 blocks: too few
    assert refused(synth.dense8(n=16384, d=2049, batch=16384)) == zipml.EUNSUPPORTED           # 33 blocks: too many

    def uneven(w, A):   # a level table that is not evenly spaced: refused through the status word
        L = _levels_for(w, A).copy()
        L[5, 100] += 0.25 * (L[5, 101] - L[5, 100])
        return L
    assert refused(synth.dense8(n=16384, d=576, batch=16384), levels=uneven) == zipml.EUNSUPPORTED


# ------------------------------------------------------------------ least-squares SVM
@pytest.mark.parametrize("name,kw", [
    ("lssvm_8bit", dict()),                                   # matrix-core loop
    ("lssvm_5bit_wide", dict(n=2048, d=1056, bits=5, batch=64)),   # vector loop, many workgroups
    ("lssvm_small", dict(n=1024, d=96, bits=4, batch=32)),    # single workgroup
])
def test_least_squares_svm_epochs_match_oracle(name, kw):
    say("ls-svm", name)
    w = synth.lssvm(**kw)
    A, b = w.full()
    assert set(np.unique(b)) == {-1.0, 1.0}
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L)
    p.quantize(12, 0)
    c1, c2 = oracle.quantize(A, L, w.bits, 12, 0)
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(3):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, w.lr, l2=w.l2)
        zipml.sgd_epoch_l2(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, w.lr, w.l2, p.ws)
        assert zipml.sgd_status(p.ws) == 0
        err = rel_l2(x.cpu().numpy(), x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}")
        assert err <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)
    # the term matters, and the classifier it trains is better than chance
    x_plain = oracle.sgd_epoch(c1, c2, L, b, w.bits, np.zeros(w.d, np.float32), w.batch, w.lr)
    x_one = oracle.sgd_epoch(c1, c2, L, b, w.bits, np.zeros(w.d, np.float32), w.batch, w.lr, l2=w.l2)
    assert rel_l2(x_one, x_plain) > 1e-4
    acc = np.mean(np.sign(A @ x.cpu().numpy()) == b)
    assert acc > 0.7
    with pytest.raises(zipml.ZipmlError) as e:
        zipml.sgd_epoch_l2(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, w.lr, -1.0, p.ws)
    assert e.value.code == zipml.EINVAL


# ------------------------------------------------------------------ proximal step
@pytest.mark.parametrize("name,factory,kw,lr", [
    ("dense8_small", synth.dense8, dict(n=4096, d=288, batch=256), 0.02),          # matrix-core loop
    ("b5_wide", synth.tiny, dict(n=2048, d=1056, batch=64, bits=5), 0.01),          # vector loop
    ("tiny_one_workgroup", synth.tiny, dict(n=2048, d=64, batch=16, bits=4), 0.01),  # no exchange
    ("dense8_replicas", synth.dense8, dict(n=8192, d=288, batch=4096), 0.1),        # chunks on replicas
    ("dense8_sample_owners", synth.dense8, dict(n=16384, d=288, batch=16384), 0.2),
])
@pytest.mark.parametrize("kind,coef", [(zipml.PROX_L1, 0.05), (zipml.PROX_L2SQ, 0.5), (zipml.PROX_BOX, 0.04)])
def test_proximal_step_matches_oracle(name, factory, kw, lr, kind, coef, knobs):
    """x <- prox_{lr R}(x - lr g) (Sec. 2) on every step loop, for the three regularisers."""
    say("prox", name, kind)
    knobs(zipml.KNOB_ROWS_MIN_BATCH, 16384)
    w = factory(**kw)
    A, b = w.full()
    L = _levels_for(w, A)
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(L)
    p.quantize(13, 0)
    c1, c2 = oracle.quantize(A, L, w.bits, 13, 0)
    plain = np.zeros(w.d, np.float32)
    for ep in range(3):
        plain = oracle.sgd_epoch(c1, c2, L, b, w.bits, plain, w.batch, lr)
    if kind == zipml.PROX_BOX:
        coef = float(np.float32(0.5 * np.abs(plain).max()))     # a box that the run does hit
    x_ref = np.zeros(w.d, np.float32)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for ep in range(3):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, lr, prox_kind=kind, prox_coef=coef)
        zipml.sgd_epoch_prox(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, lr, kind, coef, p.ws)
        assert zipml.sgd_status(p.ws) == 0
        err = rel_l2(x.cpu().numpy(), x_ref)
        say(f"  epoch {ep}: rel L2 {err:.2e}")
        assert err <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)
    xg = x.cpu().numpy()
    assert rel_l2(x_ref, plain) > 1e-4      # the step matters
    if kind == zipml.PROX_L1:
        # the soft threshold leaves exact zeros, the same ones on both sides up to coordinates
        # that sit at the threshold
        z_ref, z_gpu = x_ref == 0, xg == 0
        assert np.mean(z_ref != z_gpu) <= 0.01
        if name.startswith("dense8"):            # small true weights: many are thresholded away
            assert z_ref.sum() > 0
    if kind == zipml.PROX_BOX:
        assert np.abs(xg).max() <= np.float32(coef) and (np.abs(xg) == np.float32(coef)).sum() > 0


def test_proximal_step_refusals():
    w = synth.tiny(n=1024, d=64, batch=16, bits=4)
    A, b = w.full()
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(_levels_for(w, A))
    p.quantize(1, 0)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    for kind, coef in ((7, 0.1), (zipml.PROX_L1, -0.1)):
        with pytest.raises(zipml.ZipmlError) as e:
            zipml.sgd_epoch_prox(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, 0.01, kind, coef, p.ws)
        assert e.value.code == zipml.EINVAL
    # no regulariser: the same bits as the plain entry point
    y = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    zipml.sgd_epoch_prox(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, 0.01, zipml.PROX_NONE, 0.0, p.ws)
    p.epoch(y, 0.01)
    assert torch.equal(x, y)


# ------------------------------------------------------------------ failure handling
@pytest.mark.parametrize("name,factory,kw", [
    ("dense8_small", synth.dense8, dict(n=4096, d=288, batch=256)),          # matrix-core loop
    ("b5_wide", synth.tiny, dict(n=2048, d=1056, batch=64, bits=5)),         # vector loop, 33 groups
    ("dense8_replicas", synth.dense8, dict(n=8192, d=288, batch=4096)),      # chunks on two replicas
    ("dense8_sample_owners", synth.dense8, dict(n=16384, d=288, batch=16384)),
    ("dense8_tagged_stores", synth.dense8, dict(n=2048, d=1100, batch=512)),
    ("e2e_like_wide", synth.dense8, dict(n=2048, d=1100, bits=4, batch=512)),
])
def test_wait_that_gives_up_is_reported_not_hung(name, factory, kw, knobs):
    """Every device-wide wait is bounded.  With the bound forced to zero polls from the host, each
    wait gives up at once: the kernel must still run to its end and leave ZIPML_ETIMEOUT."""
    say("timeout path", name)
    knobs(zipml.KNOB_ROWS_MIN_BATCH, 16384)    # (for the sample-owner case)
    if name == "dense8_tagged_stores":
        knobs(zipml.KNOB_STORE_EXCHANGE_MIN, 0)
    w = factory(**kw)
    A, b = w.full()
    p = GpuProblem(A, b, w.bits, w.batch)
    p.set_levels(_levels_for(w, A))
    p.quantize(3, 0)
    x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
    knobs(zipml.KNOB_SPIN_LIMIT, 0)
    if name == "e2e_like_wide":
        # the end-to-end production loop: its three exchanges give up as well
        K = 1 << w.bits
        p.grid.copy_(dev(np.tile(np.arange(K, dtype=np.int16), (w.d, 1))))
        zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, 1e-3, p.ws, grid_idx=p.grid,
                        grid_lo=-1.0, grid_step=2.0 / (K - 1), grid_max=K - 1, grad_bits=8, model_bits=8)
    else:
        zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, x, w.batch, 1e-3, p.ws)
    st = zipml.sgd_status(p.ws)
    knobs(zipml.KNOB_SPIN_LIMIT, -1)
    assert st == zipml.ETIMEOUT, zipml.strerror(st)
    # the next call on the same workspace is sound again
    x.zero_()
    p.epoch(x, 1e-3)
    c1, c2 = oracle.quantize(A, _levels_for(w, A), w.bits, 3, 0)
    x_ref = oracle.sgd_epoch(c1, c2, _levels_for(w, A), b, w.bits, np.zeros(w.d, np.float32), w.batch, 1e-3)
    assert rel_l2(x.cpu().numpy(), x_ref) <= TOL and max_abs_ok(x.cpu().numpy(), x_ref, TOL)


# ------------------------------------------------------------------ caller's stream
def test_stream_probe_reads_and_copies_every_byte():
    """The plain streaming kernel used for the read ceiling and the counter calibration: the XOR of
    all 32-bit words it read, and the copy it wrote, against NumPy; sizes around its unrolling."""
    rng = np.random.default_rng(0)
    for nbytes in (16, 16 * 1023, 16 * 4096 * 5 + 48, 1 << 24):
        a = rng.integers(0, 2 ** 32, nbytes // 4, dtype=np.uint32)
        src = dev(a.view(np.int32))
        sink = torch.zeros(4, dtype=torch.int32, device=DEV)
        zipml.debug_stream(src, sink)
        assert np.uint32(sink[0].item() & 0xFFFFFFFF) == np.bitwise_xor.reduce(a)
        dst = torch.zeros_like(src)
        sink.zero_()
        zipml.debug_stream(src, sink, dst=dst)
        assert torch.equal(src, dst) and np.uint32(sink[0].item() & 0xFFFFFFFF) == np.bitwise_xor.reduce(a)
    with pytest.raises(zipml.ZipmlError) as e:
        zipml.debug_stream(src, sink, nbytes=24)
    assert e.value.code == zipml.EINVAL


def test_everything_runs_on_the_callers_stream():
    """All device work is enqueued on the stream the caller passes: the same calls on a stream of
    the caller's own (default priority) give the same bits as on the default stream."""
    say("caller's stream")
    w = synth.dense8(n=8192, d=288, batch=256)
    A, b = w.full()
    L = _levels_for(w, A)
    res = []
    for own in (False, True):
        st = torch.cuda.Stream() if own else torch.cuda.current_stream()
        with torch.cuda.stream(st):
            p = GpuProblem(A, b, w.bits, w.batch)
            p.set_levels(L)
            p.quantize(2, 0)
            x = torch.zeros(w.d, dtype=torch.float32, device=DEV)
            for _ in range(2):
                p.epoch(x, 1e-3)
            ws_big = torch.zeros(zipml.workspace_bytes(w.n, w.d, w.bits, 4096), dtype=torch.uint8, device=DEV)
            y = torch.zeros(w.d, dtype=torch.float32, device=DEV)
            zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, w.n, w.d, w.bits, y, 4096, 0.05, ws_big)   # replicas
            assert zipml.sgd_status(ws_big) == 0
            loss = p.loss(x, packed_copy=2)
            st.synchronize()
            res.append((p.p1.clone(), p.p2.clone(), x.clone(), y.clone(), loss))
    torch.cuda.synchronize()
    for u, v in zip(res[0][:4], res[1][:4]):
        assert torch.equal(u, v)
    assert res[0][4] == res[1][4]
    c1, c2 = oracle.quantize(A, L, w.bits, 2, 0)
    x_ref = np.zeros(w.d, np.float32)
    for _ in range(2):
        x_ref = oracle.sgd_epoch(c1, c2, L, b, w.bits, x_ref, w.batch, 1e-3)
    assert rel_l2(res[1][2].cpu().numpy(), x_ref) <= TOL and max_abs_ok(res[1][2].cpu().numpy(), x_ref, TOL)


# ------------------------------------------------------------------ edge cases
def test_degenerate_inputs():
    say("edge cases")
    # a single step per epoch, one feature group, flat column, zero model in integer mode
    w = synth.tiny(n=32, d=5, batch=32, bits=2)
    A, b = w.full()
    A[:, 2] = 0.5
    lo, hi = oracle.col_range(A)
    L = oracle.levels_uniform(lo, hi, 2)
    p = GpuProblem(A, b, 2, 32)
    p.make_levels(zipml.UNIFORM, 0)
    assert np.array_equal(p.levels.cpu().numpy(), L)
    p.quantize(1, 0)
    c1, c2 = oracle.quantize(A, L, 2, 1, 0)
    assert np.array_equal(p.codes(1), c1) and np.array_equal(p.codes(2), c2)
    x = torch.zeros(5, dtype=torch.float32, device=DEV)
    p.epoch(x, 0.1)
    assert rel_l2(x.cpu().numpy(), oracle.sgd_epoch(c1, c2, L, b, 2, np.zeros(5), 32, 0.1)) <= TOL and max_abs_ok(x.cpu().numpy(), oracle.sgd_epoch(c1, c2, L, b, 2, np.zeros(5), 32, 0.1), TOL)
    # zero-length work and rejected shapes return codes
    with pytest.raises(zipml.ZipmlError) as e:
        zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, 32, 5, 2, x, 24, 0.1, p.ws)
    assert e.value.code == zipml.EINVAL
    # one feature group and a minibatch of 32,768: no feature owners to share the work, the
    # sample-owner kernel takes it
    big = synth.tiny(n=1 << 15, d=32, batch=1 << 15, bits=8)
    Ab, bb = big.full()
    Lb = uniform_levels_np(32, 8, -1.0, 1.0)
    pb = GpuProblem(Ab, bb, 8, 1 << 15)
    pb.set_levels(Lb)
    pb.quantize(4, 0)
    cb1, cb2 = oracle.quantize(Ab, Lb, 8, 4, 0)
    xb = torch.zeros(32, dtype=torch.float32, device=DEV)
    pb.epoch(xb, 0.1)
    assert rel_l2(xb.cpu().numpy(), oracle.sgd_epoch(cb1, cb2, Lb, bb, 8, np.zeros(32), 1 << 15, 0.1)) <= TOL and max_abs_ok(xb.cpu().numpy(), oracle.sgd_epoch(cb1, cb2, Lb, bb, 8, np.zeros(32), 1 << 15, 0.1), TOL)
    # a batch too large for one exchange at a code width the matrix cores do not take is refused,
    # not mis-executed
    odd = synth.tiny(n=1 << 13, d=32, batch=1 << 13, bits=5)
    Ao, bo = odd.full()
    po = GpuProblem(Ao, bo, 5, 1 << 13)
    po.set_levels(uniform_levels_np(32, 5, -1.0, 1.0))
    po.quantize(4, 0)
    xo = torch.zeros(32, dtype=torch.float32, device=DEV)
    with pytest.raises(zipml.ZipmlError) as e:
        zipml.sgd_epoch(po.p1, po.p2, po.levels, po.b, 1 << 13, 32, 5, xo, 1 << 13, 0.1, po.ws)
    assert e.value.code == zipml.EUNSUPPORTED
