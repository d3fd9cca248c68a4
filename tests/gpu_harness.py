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
