"""Seeded synthetic least-squares problems shaped like the paper's workloads.

This module only *generates inputs* (feature matrix, labels, ground-truth model and
the hyper-parameters of each workload).  It contains none of the method's
arithmetic (no quantisation, no gradient, no level search), so the CPU oracle's
tests and the GPU path's tests can both draw their inputs from it.

The paper's datasets (Table 1: Synthetic 10/100/1000, YearPrediction, cadata,
cpusmall, cod-rna, gisette, the 128-projection tomography volume) are not
available; each workload below stands in for one of them with the same shape and
value structure.  Rows are produced in fixed chunks of ``CHUNK`` rows, each from
its own seed, so any row range of a large problem can be regenerated without
materialising the rest.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

CHUNK = 4096


@dataclass
class Workload:
    name: str
    n: int
    d: int
    bits: int
    batch: int
    lr: float
    epochs: int
    levels: str = "uniform"          # "uniform" | "optimal"
    range_mode: str = "fixed"        # "fixed" (lo, hi given) | "minmax" | "symmetric"
    lo: float = -1.0
    hi: float = 1.0
    n_candidates: int = 0
    grad_bits: int = 0
    model_bits: int = 0
    noise: float = 0.0
    seed: int = 0
    kind: str = "uniform"
    sign_labels: bool = False        # two-class labels b = sign(a.x* + noise) in {-1, +1}
    l2: float = 0.0                  # coefficient of the (c/2)||x||^2 term
    x_star: np.ndarray = field(default=None, repr=False)
    _col_scale: np.ndarray = field(default=None, repr=False)
    _col_min: np.ndarray = field(default=None, repr=False)
    _col_max: np.ndarray = field(default=None, repr=False)

    # ---------------------------------------------------------------- rows
    def _chunk_rng(self, chunk: int, what: int) -> np.random.Generator:
        return np.random.default_rng([self.seed, _KIND_ID[self.kind], what, chunk])

    def _raw_chunk(self, chunk: int) -> np.ndarray:
        rng = self._chunk_rng(chunk, 0)
        rows = min(CHUNK, self.n - chunk * CHUNK)
        d = self.d
        if self.kind in ("uniform", "hetero"):
            A = rng.uniform(-1.0, 1.0, size=(rows, d)).astype(np.float32)
            if self.kind == "hetero":
                A *= self._col_scale[None, :]
        elif self.kind == "gauss":
            A = np.clip(rng.standard_normal(size=(rows, d), dtype=np.float32), -3.0, 3.0)
        elif self.kind == "lognormal":
            A = np.exp(rng.standard_normal(size=(rows, d), dtype=np.float32))
        elif self.kind == "tomo":
            A = _tomo_rows(rng, rows, d)
        elif self.kind == "ongrid":
            K = 1 << self.bits
            c = rng.integers(0, K, size=(rows, d))
            A = (self.lo + (self.hi - self.lo) * c / (K - 1)).astype(np.float32)
        else:
            raise ValueError(self.kind)
        return A

    def rows(self, i0: int, i1: int) -> np.ndarray:
        """Feature rows [i0, i1) as fp32, row-major."""
        out = np.empty((i1 - i0, self.d), np.float32)
        for chunk in range(i0 // CHUNK, (i1 - 1) // CHUNK + 1):
            A = self._raw_chunk(chunk)
            if self.kind == "lognormal":
                A = (A - self._col_min[None, :]) / (self._col_max - self._col_min)[None, :]
                A = np.clip(A, 0.0, 1.0).astype(np.float32)
            elif self.kind == "gauss":
                A = A / self._col_max[None, :]      # every column scaled by its own max-abs to [-1, 1]
            c0 = chunk * CHUNK
            a, b = max(i0, c0), min(i1, c0 + A.shape[0])
            out[a - i0:b - i0] = A[a - c0:b - c0]
        return out

    def labels(self, i0: int, i1: int, A: np.ndarray = None) -> np.ndarray:
        """b = A x* + noise for rows [i0, i1) (fp32)."""
        if A is None:
            A = self.rows(i0, i1)
        out = (A.astype(np.float64) @ self.x_star.astype(np.float64))
        if self.noise > 0.0:
            for chunk in range(i0 // CHUNK, (i1 - 1) // CHUNK + 1):
                rng = self._chunk_rng(chunk, 1)
                rows = min(CHUNK, self.n - chunk * CHUNK)
                e = rng.standard_normal(rows) * self.noise
                c0 = chunk * CHUNK
                a, b = max(i0, c0), min(i1, c0 + rows)
                out[a - i0:b - i0] += e[a - c0:b - c0]
        if self.sign_labels:
            out = np.where(out >= 0.0, 1.0, -1.0)
        return out.astype(np.float32)

    def full(self):
        """(A, b) for the whole problem; only for sizes that fit in host memory."""
        A = self.rows(0, self.n)
        return A, self.labels(0, self.n, A)


_KIND_ID = {"uniform": 1, "gauss": 2, "hetero": 3, "tomo": 4, "lognormal": 5, "ongrid": 6}


def _tomo_rows(rng: np.random.Generator, rows: int, d: int) -> np.ndarray:
    """Dense rows of line-integral weights through a side x side image.

    Each row is one ray (angle U[0, pi), signed offset U over the image diagonal);
    the pixels it crosses (0 to about 1.4*side, never more than 256 for side 128)
    get weights U[0,1], every other entry is an exact zero.
    """
    side = int(round(np.sqrt(d)))
    assert side * side == d, "tomography workload needs a square image"
    theta = rng.uniform(0.0, np.pi, size=rows)
    half = side / 2.0
    off = rng.uniform(-half * np.sqrt(2.0), half * np.sqrt(2.0), size=rows)
    steps = 2 * side
    t = np.linspace(-half * np.sqrt(2.0), half * np.sqrt(2.0), steps)
    cx = half + off[:, None] * (-np.sin(theta))[:, None] + t[None, :] * np.cos(theta)[:, None]
    cy = half + off[:, None] * (np.cos(theta))[:, None] + t[None, :] * np.sin(theta)[:, None]
    px = np.floor(cx).astype(np.int64)
    py = np.floor(cy).astype(np.int64)
    ok = (px >= 0) & (px < side) & (py >= 0) & (py < side)
    w = rng.uniform(0.0, 1.0, size=(rows, steps)).astype(np.float32)
    A = np.zeros((rows, d), np.float32)
    ri = np.broadcast_to(np.arange(rows)[:, None], (rows, steps))
    A[ri[ok], (py * side + px)[ok]] = w[ok]
    return A


def _smooth_field(rng: np.random.Generator, side: int) -> np.ndarray:
    """A smooth random image: a few low-frequency cosines with random phases."""
    yy, xx = np.meshgrid(np.arange(side) / side, np.arange(side) / side, indexing="ij")
    img = np.zeros((side, side))
    for _ in range(6):
        fx, fy = rng.integers(0, 4, size=2)
        ph = rng.uniform(0, 2 * np.pi)
        img += rng.uniform(0.2, 1.0) * np.cos(2 * np.pi * (fx * xx + fy * yy) + ph)
    img -= img.min()
    img /= max(img.max(), 1e-12)
    return img.reshape(-1).astype(np.float32)


def _finish(w: Workload, x_scale: float) -> Workload:
    rng = np.random.default_rng([w.seed, _KIND_ID[w.kind], 99])
    if w.kind == "tomo":
        w.x_star = _smooth_field(rng, int(round(np.sqrt(w.d))))
    else:
        w.x_star = (rng.standard_normal(w.d) * x_scale).astype(np.float32)
    if w.kind == "hetero":
        scale = np.ones(w.d, np.float32)
        small = rng.permutation(w.d)[: w.d // 5]      # a fixed random 20 % of the columns
        scale[small] = 0.05
        w._col_scale = scale
    if w.kind == "gauss":
        # column max-abs over all rows (with 65,536 rows every column holds clipped values, so it
        # is the clip bound 3 for all of them; shorter test problems get their own maxima)
        mx = np.zeros(w.d, np.float32)
        for chunk in range((w.n + CHUNK - 1) // CHUNK):
            mx = np.maximum(mx, np.abs(w._raw_chunk(chunk)).max(axis=0))
        w._col_max = np.maximum(mx, np.float32(1e-30))
    if w.kind == "lognormal":
        mn = np.full(w.d, np.inf, np.float32)
        mx = np.full(w.d, -np.inf, np.float32)
        for chunk in range((w.n + CHUNK - 1) // CHUNK):
            A = w._raw_chunk(chunk)
            mn = np.minimum(mn, A.min(axis=0))
            mx = np.maximum(mx, A.max(axis=0))
        w._col_min, w._col_max = mn, mx
    return w


def tiny(n=4096, d=64, seed=0, bits=4, batch=16) -> Workload:
    """Workload 1: U[-1,1] features, x* ~ N(0,1), noise 0.01, uniform 4-bit on [-1,1]."""
    return _finish(Workload("tiny", n, d, bits, batch, 0.01, 5, kind="uniform", noise=0.01,
                            seed=seed), 1.0)


def dense8(n=65536, d=2048, seed=0, bits=8, batch=256) -> Workload:
    """Workload 2: clipped N(0,1) scaled per column to [-1,1], x* ~ N(0,1/d), noise 0.1."""
    return _finish(Workload("dense8", n, d, bits, batch, 1e-3, 10, kind="gauss", noise=0.1,
                            seed=seed), 1.0 / np.sqrt(d))


def lssvm(n=8192, d=288, seed=0, bits=8, batch=256, l2=0.05) -> Workload:
    """Two-class least-squares SVM: clipped-normal features scaled to [-1,1], labels +-1 from a
    random hyperplane with label noise, (c/2)||x||^2 regularisation."""
    return _finish(Workload("lssvm", n, d, bits, batch, 0.05, 5, kind="gauss", noise=0.05,
                            seed=seed, sign_labels=True, l2=l2), 1.0 / np.sqrt(d))


def lowbit(n=1048576, d=512, seed=0, bits=2, batch=1024) -> Workload:
    """Workload 3: U[-1,1] with 20 % of the columns scaled by 0.05; per-column ranges."""
    return _finish(Workload("lowbit", n, d, bits, batch, 0.2, 5, kind="hetero", noise=0.1,
                            range_mode="symmetric", seed=seed), 1.0 / np.sqrt(d))


def tomo(n=262144, d=16384, seed=0, bits=4, batch=512) -> Workload:
    """Workload 4: tomography-shaped rows (sparse nonnegative weights stored dense)."""
    return _finish(Workload("tomo", n, d, bits, batch, 1.0, 3, kind="tomo", noise=0.0, lo=0.0,
                            hi=1.0, seed=seed), 1.0)


def e2e(n=524288, d=4096, seed=0, bits=3, batch=512, n_candidates=1024) -> Workload:
    """Workload 5: lognormal features min-max scaled to [0,1]; optimal 3-bit levels;
    gradient and model quantised to 8 bits every step."""
    return _finish(Workload("e2e", n, d, bits, batch, 0.5, 5, levels="optimal", kind="lognormal",
                            noise=0.1, lo=0.0, hi=1.0, n_candidates=n_candidates, grad_bits=8,
                            model_bits=8, seed=seed), 1.0 / np.sqrt(d))


def ongrid(n=1024, d=32, seed=0, bits=3, batch=32, lo=-1.0, hi=1.0) -> Workload:
    """Every feature value sits exactly on a uniform level, so quantisation is
    deterministic and the method reduces to ordinary minibatch SGD."""
    return _finish(Workload("ongrid", n, d, bits, batch, 0.05, 1, kind="ongrid", noise=0.01,
                            lo=lo, hi=hi, seed=seed), 1.0)


WORKLOADS = {"lssvm": lssvm, "tiny": tiny, "dense8": dense8, "lowbit": lowbit, "tomo": tomo, "e2e": e2e}


# ---------------------------------------------------------------------------------------------
# The same recipes generated on the GPU with torch, for the full-size problems of bench.py (16 GiB
# of fp32 rows for the tomography shape would take minutes through NumPy and the host link).  The
# random streams differ from the NumPy ones above -- these are other samples of the same
# distributions -- and are seeded per chunk as well.  Input generation only: no method arithmetic.
# ---------------------------------------------------------------------------------------------
def _device_gen(w: Workload, chunk: int, what: int, device):
    import torch
    g = torch.Generator(device=device)
    g.manual_seed((((w.seed * 8 + _KIND_ID[w.kind]) * 4 + what) << 24) + chunk)
    return g


def _device_raw_chunk(w: Workload, chunk: int, rows: int, device):
    import torch
    g = _device_gen(w, chunk, 0, device)
    d = w.d
    if w.kind in ("uniform", "hetero"):
        A = torch.rand(rows, d, generator=g, device=device, dtype=torch.float32) * 2.0 - 1.0
        if w.kind == "hetero":
            A *= torch.from_numpy(w._col_scale).to(device)[None, :]
    elif w.kind == "gauss":
        A = torch.randn(rows, d, generator=g, device=device, dtype=torch.float32).clamp_(-3.0, 3.0)
    elif w.kind == "lognormal":
        A = torch.randn(rows, d, generator=g, device=device, dtype=torch.float32).exp_()
    elif w.kind == "tomo":
        # rays as in _tomo_rows; a crossed pixel gets a U[0,1] weight of its own (a ray visits a
        # pixel in several steps, and which duplicate write wins is not defined on a GPU)
        side = int(round(np.sqrt(d)))
        half = side / 2.0
        diag = half * np.sqrt(2.0)
        theta = torch.rand(rows, generator=g, device=device, dtype=torch.float64) * np.pi
        off = (torch.rand(rows, generator=g, device=device, dtype=torch.float64) * 2.0 - 1.0) * diag
        steps = 2 * side
        t = torch.linspace(-diag, diag, steps, device=device, dtype=torch.float64)
        cx = half + off[:, None] * (-torch.sin(theta))[:, None] + t[None, :] * torch.cos(theta)[:, None]
        cy = half + off[:, None] * torch.cos(theta)[:, None] + t[None, :] * torch.sin(theta)[:, None]
        px, py = torch.floor(cx).long(), torch.floor(cy).long()
        ok = (px >= 0) & (px < side) & (py >= 0) & (py < side)
        idx = (py * side + px).clamp_(0, d - 1)
        mask = torch.zeros(rows, d, device=device, dtype=torch.float32)
        mask.scatter_add_(1, idx, ok.to(torch.float32))
        A = torch.rand(rows, d, generator=g, device=device, dtype=torch.float32)
        A *= (mask > 0).to(torch.float32)
    else:
        raise ValueError(w.kind)
    return A


def device_chunks(w: Workload, device, chunk_rows: int = CHUNK):
    """Yields (first row, A [rows, d] fp32 on `device`, b [rows] fp32) for consecutive row chunks of
    the whole problem, generated on the device.  Kinds normalised per column (gauss, lognormal)
    take a first pass over the raw chunks for the column statistics."""
    import torch
    n, d = w.n, w.d
    nchunks = (n + chunk_rows - 1) // chunk_rows
    rows_of = lambda c: min(chunk_rows, n - c * chunk_rows)
    col_min = col_max = None
    if w.kind in ("gauss", "lognormal"):
        col_min = torch.full((d,), float("inf"), device=device)
        col_max = torch.full((d,), float("-inf"), device=device)
        for c in range(nchunks):
            A = _device_raw_chunk(w, c, rows_of(c), device)
            if w.kind == "gauss":
                A = A.abs_()
            col_min = torch.minimum(col_min, A.min(dim=0).values)
            col_max = torch.maximum(col_max, A.max(dim=0).values)
            del A
    xs = torch.from_numpy(np.asarray(w.x_star, np.float32)).to(device)
    for c in range(nchunks):
        rows = rows_of(c)
        A = _device_raw_chunk(w, c, rows, device)
        if w.kind == "gauss":
            A /= col_max[None, :]
        elif w.kind == "lognormal":
            A = ((A - col_min[None, :]) / (col_max - col_min)[None, :]).clamp_(0.0, 1.0)
        b = A @ xs
        if w.noise > 0.0:
            b += torch.randn(rows, generator=_device_gen(w, c, 1, device), device=device) * w.noise
        if w.sign_labels:
            b = torch.where(b >= 0, 1.0, -1.0)
        yield c * chunk_rows, A, b.to(torch.float32)


def light(factory, n: int, **kw) -> Workload:
    """The description of an n-row workload without the host-side column statistics (for
    device_chunks, which takes its own): the full-size lognormal problem would otherwise be
    generated once on the host just for them."""
    w = factory(n=min(n, CHUNK), **kw)
    w.n = n
    return w
