"""Helpers for the GPU parity tests: device buffers + calls through the C ABI binding."""
from __future__ import annotations

import numpy as np
import torch

from paper_1611_05402_amd import zipml

DEV = "cuda"


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).to(DEV)


class GpuProblem:
    """One least-squares problem resident on the GPU, quantised with the library."""

    def __init__(self, A: np.ndarray, b: np.ndarray, bits: int, batch: int, n_candidates: int = 0):
        self.n, self.d = A.shape
        self.bits, self.batch = bits, batch
        self.K = 1 << bits
        self.A = dev(A.astype(np.float32))
        self.b = dev(b.astype(np.float32))
        self.ws = torch.zeros(zipml.workspace_bytes(self.n, self.d, bits, batch, n_candidates),
                              dtype=torch.uint8, device=DEV)
        self.lo = torch.zeros(self.d, dtype=torch.float32, device=DEV)
        self.hi = torch.zeros(self.d, dtype=torch.float32, device=DEV)
        self.levels = torch.zeros(self.d, self.K, dtype=torch.float32, device=DEV)
        self.grid = torch.zeros(self.d, self.K, dtype=torch.int16, device=DEV)
        nb = zipml.packed_bytes(self.n, self.d, bits)
        self.p1 = torch.zeros(nb, dtype=torch.uint8, device=DEV)
        self.p2 = torch.zeros(nb, dtype=torch.uint8, device=DEV)

    # ---- levels
    def set_levels(self, L: np.ndarray, G: np.ndarray = None):
        self.levels.copy_(dev(L.astype(np.float32)))
        if G is not None:
            self.grid.copy_(dev(G.astype(np.uint16).view(np.int16)))

    def make_levels(self, mode=zipml.UNIFORM, flags=0, lo=None, hi=None, n_candidates=0,
                    want_mv=False):
        if lo is not None:
            self.lo.copy_(dev(np.asarray(lo, np.float32)))
            self.hi.copy_(dev(np.asarray(hi, np.float32)))
            flags |= zipml.RANGE_GIVEN
        return zipml.levels(self.A, self.n, self.d, self.d, self.bits, mode, flags, n_candidates,
                            self.lo, self.hi, self.levels, self.grid, self.ws, want_mv)

    # ---- quantise
    def quantize(self, seed, epoch, chunks=1):
        rows = self.n if chunks == 1 else ((self.n // chunks + 31) // 32) * 32
        r0 = 0
        while r0 < self.n:
            cnt = min(rows, self.n - r0)
            zipml.quantize(self.A[r0:], cnt, self.d, self.d, r0, self.n, self.levels, self.bits,
                           seed, epoch, self.p1, self.p2)
            r0 += cnt

    def codes(self, copy):
        out = torch.zeros(self.n, self.d, dtype=torch.uint8, device=DEV)
        zipml.unpack_codes(self.p1 if copy == 1 else self.p2, copy, self.n, self.d, self.bits, out)
        torch.cuda.synchronize()
        return out.cpu().numpy()

    # ---- SGD
    def epoch(self, x: torch.Tensor, lr, seed=0, epoch=0, flags=0, grad_bits=0, model_bits=0,
              grid_lo=0.0, grid_step=0.0, grid_max=0):
        zipml.sgd_epoch(self.p1, self.p2, self.levels, self.b, self.n, self.d, self.bits, x,
                        self.batch, lr, self.ws, grid_idx=self.grid if model_bits else None,
                        grid_lo=grid_lo, grid_step=grid_step, grid_max=grid_max,
                        grad_bits=grad_bits, model_bits=model_bits, seed=seed, epoch=epoch,
                        flags=flags)
        st = zipml.sgd_status(self.ws)
        assert st == 0, zipml.strerror(st)

    def loss(self, x, packed_copy=0):
        if packed_copy:
            return zipml.loss(self.b, x, self.n, self.d, self.ws,
                              packed=self.p1 if packed_copy == 1 else self.p2, copy=packed_copy,
                              levels_t=self.levels, bits=self.bits)
        return zipml.loss(self.b, x, self.n, self.d, self.ws, A=self.A, lda=self.d)


def max_abs_ok(a, b, tol):
    """max |a - b| <= tol * max |b|: the element-wise companion of a relative-L2 bound (one wrong
    element of a long vector can hide under a norm, not under this)."""
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.max(np.abs(a - b))) <= tol * max(float(np.max(np.abs(b))), 1e-30)


def ulp_diff(a, b):
    """Element-wise distance of two fp32 arrays in units of the last place."""
    ai = np.asarray(a, np.float32).view(np.int32).astype(np.int64)
    bi = np.asarray(b, np.float32).view(np.int32).astype(np.int64)
    ai = np.where(ai < 0, -(ai & 0x7FFFFFFF), ai)
    bi = np.where(bi < 0, -(bi & 0x7FFFFFFF), bi)
    return np.abs(ai - bi)


# End-to-end mode (Supp. C-E).  The paper fixes no order for the sum over a minibatch, so the
# contract is per step, from identical model bits:
#   - what does not depend on any order is bit-equal: the Q3 model codes, the int32 dot products,
#     the residual bits;
#   - the mean gradient before Q4 equals the oracle's (the exact mean rounded to fp32) to
#     E2E_G_ULP units in the last place (both sides sum in fp64, in different orders: a
#     difference of one unit has probability about 2^-29 per element);
#   - Q4's codes and the updated model are bit-equal to the oracle's quantiser and update formula
#     applied to the library's OWN gradient.
# Whole epochs: identical models follow from identical steps as long as no gradient element
# falls on a rounding boundary (2^-29 per element and step); then ONE Q4 code may differ, which
# moves one coordinate by lr * ||g|| / s.  E2E_EPOCH_BAND bounds the relative L2 distance of the
# models after an epoch for a handful of such events; the tests print whether the models were
# identical (they are on every case here).
E2E_G_ULP = 1
E2E_EPOCH_BAND = 1e-3


def e2e_step_check(p, oracle, c1, c2, L, G, glo, gstep, gmax, b, x0, lr, gb, mb, seed, epoch, step,
                   flags=0):
    """One end-to-end step of `p` from the model x0 against the oracle, to the contract above
    (c1, c2: the oracle's codes of at least the rows up to the end of that minibatch).  Returns
    the largest distance of a gradient element from the oracle's, in units of the last place."""
    n_rows = c1.shape[0]
    B, d = p.batch, p.d
    assert n_rows >= (step + 1) * B
    _, dbg = oracle.sgd_epoch_e2e(c1, c2, L, G, glo, gstep, b[:n_rows], p.bits, x0, B, lr, gb, mb,
                                  seed, epoch, first_step=step, num_steps=1, debug=True)
    xd = dev(x0)
    mo = torch.zeros(d, dtype=torch.int32, device=DEV)
    ac = torch.zeros(B, dtype=torch.int32, device=DEV)
    rr = torch.zeros(B, dtype=torch.float32, device=DEV)
    gg = torch.zeros(d, dtype=torch.float32, device=DEV)
    gq = torch.zeros(d, dtype=torch.int32, device=DEV)
    zipml.debug_step(p.p1, p.p2, p.levels, p.b, p.n, d, p.bits, xd, B, lr, step, p.ws,
                     grid_idx=p.grid, grid_lo=glo, grid_step=gstep, grid_max=gmax, grad_bits=gb,
                     model_bits=mb, seed=seed, epoch=epoch, flags=flags, model_codes=mo, acc=ac, r=rr,
                     g=gg, grad_codes=gq)
    assert zipml.sgd_status(p.ws) == 0
    assert np.array_equal(mo.cpu().numpy(), dbg["m"])
    assert np.array_equal(ac.cpu().numpy(), dbg["acc"])
    assert np.array_equal(rr.cpu().numpy().view(np.uint32), dbg["r"].view(np.uint32))
    g_gpu = gg.cpu().numpy()
    ud = ulp_diff(g_gpu, dbg["g"])
    assert ud.max() <= E2E_G_ULP, f"gradient differs by {ud.max()} ulp at {int(ud.argmax())}"
    lr32 = np.float32(lr)
    if gb:
        codes, sg = oracle.quantize_vec(g_gpu, gb, seed, epoch, step, 4)
        assert np.array_equal(gq.cpu().numpy(), codes)
        x_new = x0 - lr32 * (np.float32(sg) * codes.astype(np.float32))
    else:
        x_new = x0 - lr32 * g_gpu
    assert np.array_equal(xd.cpu().numpy().view(np.uint32), x_new.astype(np.float32).view(np.uint32))
    return int(ud.max())


def level_set_cost(oracle, col, lo, hi, M, idx):
    """Objective of eq. (6) (Sec. 3) of one feature for the level set at the candidate indices
    `idx`, from the oracle's bin moments of that column: sum over the intervals of
    sum_t (d_b - t)(t - d_a)."""
    cand = np.arange(M + 1) / M
    t = (col.astype(np.float64) - float(lo)) / (float(hi) - float(lo))
    mom = oracle.bin_moments(t, cand)
    C = np.concatenate([[0], np.cumsum(mom[:, 0])])
    S1 = np.concatenate([[0], np.cumsum(mom[:, 1])])
    S2 = np.concatenate([[0], np.cumsum(mom[:, 2])])
    tot = 0.0
    for a_, b_ in zip(idx[:-1], idx[1:]):
        tot += (-(S2[b_] - S2[a_]) + (cand[a_] + cand[b_]) * (S1[b_] - S1[a_])
                - cand[a_] * cand[b_] * (C[b_] - C[a_]))
    return tot


def check_level_sets(oracle, A, lo, hi, M, G_gpu, G_ref, min_same):
    """The library's level sets against the oracle's: identical grid indices, or -- where the
    dynamic program has several optima -- a level set of the same cost.  Returns the fraction of
    features with identical indices (at least min_same)."""
    G_gpu = np.asarray(G_gpu).astype(np.int64)
    G_ref = np.asarray(G_ref).astype(np.int64)
    d = G_ref.shape[0]
    same = np.all(G_gpu == G_ref, axis=1)
    for j in np.nonzero(~same)[0]:
        assert G_gpu[j, 0] == 0 and G_gpu[j, -1] == M and np.all(np.diff(G_gpu[j]) > 0)
        cg = level_set_cost(oracle, A[:, j], lo[j], hi[j], M, G_gpu[j])
        cr = level_set_cost(oracle, A[:, j], lo[j], hi[j], M, G_ref[j])
        assert np.isclose(cg, cr, rtol=1e-9, atol=1e-12), (j, cg, cr)
    assert same.mean() >= min_same
    return float(same.mean())


def rel_l2(a, b):
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-30))


def oracle_quantize_rows(A, L, bits, seed, epoch, workers=16, rows_per_task=2048):
    """The oracle's quantiser over all rows of A, row ranges spread over host threads.

    Every code is a pure function of (seed, epoch, row, column), so splitting by rows changes
    nothing; the oracle call releases the interpreter lock while it runs.
    """
    from concurrent.futures import ThreadPoolExecutor

    import oracle

    n = A.shape[0]
    starts = list(range(0, n, rows_per_task))

    def part(r0):
        return oracle.quantize(A[r0:r0 + rows_per_task], L, bits, seed, epoch, row0=r0)

    with ThreadPoolExecutor(workers) as ex:
        res = list(ex.map(part, starts))
    return (np.concatenate([r[0] for r in res]), np.concatenate([r[1] for r in res]))
