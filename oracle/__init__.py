"""ctypes front end of the CPU oracle (test infrastructure, not product code).

Holds no arithmetic: it compiles ``zipml_oracle.c`` with gcc and marshals numpy
arrays.  Only ``tests/``, ``__graft_entry__.smoke()`` and the ``cpu_baseline`` leg
of ``bench.py`` may import this package; the GPU library never does.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "zipml_oracle.c")
_SO = os.path.join(_HERE, "libzipml_oracle.so")

# -ffp-contract=off: the oracle's fp32 decision sequences must stay single IEEE ops.
# -fopenmp: only zo_sgd_epoch_threads (the all-cores leg of the benchmark's baseline) has a
# parallel region; every other function runs on the calling thread.
_CFLAGS = ["-O1", "-ffp-contract=off", "-fno-fast-math", "-fPIC", "-shared", "-std=c11", "-fopenmp"]


def build(force: bool = False) -> str:
    """Compile the oracle; returns the path of the shared object."""
    if force or not os.path.exists(_SO) or os.path.getmtime(_SO) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", *_CFLAGS, _SRC, "-o", _SO, "-lm"])
    return _SO


_lib = None


def lib():
    global _lib
    if _lib is None:
        _lib = C.CDLL(build())
        _lib.zo_uniform24.restype = C.c_float
        _lib.zo_norm2.restype = C.c_float
        _lib.zo_quantize_vec.restype = C.c_float
        _lib.zo_quantize_vec_u.restype = C.c_float
        _lib.zo_dp_levels.restype = C.c_double
        _lib.zo_loss.restype = C.c_double
        _lib.zo_loss_codes.restype = C.c_double
    return _lib


def _p(a):
    return a.ctypes.data_as(C.c_void_p) if a is not None else None


def _f32(a):
    return np.ascontiguousarray(a, dtype=np.float32)


def philox4x32_10(ctr, key):
    c = np.asarray(ctr, dtype=np.uint32)
    k = np.asarray(key, dtype=np.uint32)
    out = np.zeros(4, dtype=np.uint32)
    lib().zo_philox4x32_10(_p(c), _p(k), _p(out))
    return out


def uniform24(seed, epoch, row, col, stream):
    return float(lib().zo_uniform24(C.c_uint64(seed), C.c_uint32(epoch), C.c_uint64(row),
                                    C.c_uint32(col), C.c_uint32(stream)))


def col_range(A, symmetric=False):
    A = _f32(A)
    n, d = A.shape
    lo = np.empty(d, np.float32)
    hi = np.empty(d, np.float32)
    lib().zo_col_range(_p(A), C.c_int64(n), C.c_int64(d), C.c_int64(d), C.c_int(int(symmetric)),
                       _p(lo), _p(hi))
    return lo, hi


def levels_uniform(lo, hi, bits):
    lo, hi = _f32(lo), _f32(hi)
    d = lo.shape[0]
    L = np.empty((d, 1 << bits), np.float32)
    lib().zo_levels_uniform(_p(lo), _p(hi), C.c_int64(d), C.c_int(bits), _p(L))
    return L


def hist_moments(A, lo, hi, M):
    A, lo, hi = _f32(A), _f32(lo), _f32(hi)
    n, d = A.shape
    hist = np.empty((d, M, 3), np.float64)
    lib().zo_hist_moments(_p(A), C.c_int64(n), C.c_int64(d), C.c_int64(d), _p(lo), _p(hi),
                          C.c_int(M), _p(hist))
    return hist


def bin_moments(t, cand):
    t = np.ascontiguousarray(t, np.float64)
    cand = np.ascontiguousarray(cand, np.float64)
    M = cand.shape[0] - 1
    mom = np.empty((M, 3), np.float64)
    lib().zo_bin_moments(_p(t), C.c_int64(t.shape[0]), _p(cand), C.c_int(M), _p(mom))
    return mom


def dp_levels(mom, cand, s):
    mom = np.ascontiguousarray(mom, np.float64)
    cand = np.ascontiguousarray(cand, np.float64)
    M = cand.shape[0] - 1
    idx = np.empty(s + 1, np.int32)
    total = lib().zo_dp_levels(_p(mom), _p(cand), C.c_int(M), C.c_int(s), _p(idx))
    return float(total), idx


def levels_optimal(hist, lo, hi, bits):
    hist = np.ascontiguousarray(hist, np.float64)
    lo, hi = _f32(lo), _f32(hi)
    d, M, _ = hist.shape
    K = 1 << bits
    L = np.empty((d, K), np.float32)
    G = np.empty((d, K), np.uint16)
    mv = C.c_double(0.0)
    lib().zo_levels_optimal(_p(hist), _p(lo), _p(hi), C.c_int64(d), C.c_int(bits), C.c_int(M),
                            _p(L), _p(G), C.byref(mv))
    return L, G, mv.value


def greedy_intervals(mom, k):
    """Greedy merging of the M bins into at most 4k + 1 intervals (supplement, Algorithm 1, with
    gamma = 1, delta = 1): (edge indices [P+1], moments [P, 3])."""
    mom = np.ascontiguousarray(mom, np.float64)
    M = mom.shape[0]
    edge = np.empty(M + 1, np.int32)
    out = np.empty((M, 3), np.float64)
    lib().zo_greedy_intervals.restype = C.c_int
    P = lib().zo_greedy_intervals(_p(mom), C.c_int(M), C.c_int(k), _p(edge), _p(out))
    return edge[:P + 1].copy(), out[:P].copy()


def levels_greedy(hist, lo, hi, bits):
    """Dynamic program over the end points of the greedy intervals (Sec. 3.2)."""
    hist = np.ascontiguousarray(hist, np.float64)
    lo, hi = _f32(lo), _f32(hi)
    d, M = hist.shape[0], hist.shape[1]
    K = 1 << bits
    L = np.empty((d, K), np.float32)
    G = np.empty((d, K), np.uint16)
    mv = C.c_double(0.0)
    lib().zo_levels_greedy(_p(hist), _p(lo), _p(hi), C.c_int64(d), C.c_int(bits), C.c_int(M),
                           _p(L), _p(G), C.byref(mv))
    return L, G, mv.value


def bracket(L_row, bits, v):
    L_row = _f32(L_row)
    frac = C.c_float(0.0)
    l = lib().zo_bracket(_p(L_row), C.c_int(bits), C.c_float(v), C.byref(frac))
    return int(l), float(frac.value)


def quantize(A, levels, bits, seed, epoch, row0=0):
    A, levels = _f32(A), _f32(levels)
    n, d = A.shape
    c1 = np.empty((n, d), np.uint8)
    c2 = np.empty((n, d), np.uint8)
    lib().zo_quantize(_p(A), C.c_int64(n), C.c_int64(d), C.c_int64(d), C.c_int64(row0),
                      _p(levels), C.c_int(bits), C.c_uint64(seed), C.c_uint32(epoch), _p(c1),
                      _p(c2))
    return c1, c2


def norm2(v):
    v = _f32(v)
    return float(lib().zo_norm2(_p(v), C.c_int64(v.shape[0])))


def quantize_vec(v, bits, seed, epoch, step, stream):
    v = _f32(v)
    codes = np.empty(v.shape[0], np.int32)
    sigma = lib().zo_quantize_vec(_p(v), C.c_int64(v.shape[0]), C.c_int(bits), C.c_uint64(seed),
                                  C.c_uint32(epoch), C.c_uint64(step), C.c_uint32(stream),
                                  _p(codes))
    return codes, float(sigma)


def quantize_vec_u(v, bits, u):
    v, u = _f32(v), _f32(u)
    codes = np.empty(v.shape[0], np.int32)
    sigma = lib().zo_quantize_vec_u(_p(v), C.c_int64(v.shape[0]), C.c_int(bits), _p(u), _p(codes))
    return codes, float(sigma)


def grad_naive(code, levels, bits, x, b):
    code = np.ascontiguousarray(code, np.uint8)
    levels = _f32(levels)
    x = np.ascontiguousarray(x, np.float64)
    g = np.empty(x.shape[0], np.float64)
    lib().zo_grad_naive(_p(code), _p(levels), C.c_int64(x.shape[0]), C.c_int(bits), _p(x),
                        C.c_double(b), _p(g))
    return g


def grad_double(code1, code2, levels, bits, x, b):
    code1 = np.ascontiguousarray(code1, np.uint8)
    code2 = np.ascontiguousarray(code2, np.uint8)
    levels = _f32(levels)
    x = np.ascontiguousarray(x, np.float64)
    g = np.empty(x.shape[0], np.float64)
    lib().zo_grad_double(_p(code1), _p(code2), _p(levels), C.c_int64(x.shape[0]), C.c_int(bits),
                         _p(x), C.c_double(b), _p(g))
    return g


PROX_NONE, PROX_L1, PROX_L2SQ, PROX_BOX = 0, 1, 2, 3


def prox(v, kind, gamma, coef):
    """Proximal operator of gamma * R at the scalar v (Sec. 2)."""
    f = lib().zo_prox
    f.restype = C.c_double
    return float(f(C.c_double(v), C.c_int(kind), C.c_double(gamma), C.c_double(coef)))


def sgd_epoch(codes1, codes2, levels, b, bits, x, batch, lr, symmetric=False, l2=0.0,
              prox_kind=PROX_NONE, prox_coef=0.0):
    """One epoch in full-precision-model mode; returns the new fp32 model."""
    codes1 = np.ascontiguousarray(codes1, np.uint8)
    codes2 = np.ascontiguousarray(codes2, np.uint8)
    levels, b = _f32(levels), _f32(b)
    x = _f32(x).copy()
    n, d = codes1.shape
    lib().zo_sgd_epoch(_p(codes1), _p(codes2), _p(levels), _p(b), C.c_int64(n), C.c_int64(d),
                       C.c_int(bits), _p(x), C.c_int64(batch), C.c_float(lr),
                       C.c_int(int(symmetric)), C.c_float(l2), C.c_int(prox_kind),
                       C.c_float(prox_coef))
    return x


def sgd_epoch_threads(codes1, codes2, levels, b, bits, x, batch, lr, threads):
    """The plain epoch of sgd_epoch with the rows of a minibatch shared out over host threads
    (partial gradients added in thread order); returns (new fp32 model, threads used)."""
    codes1 = np.ascontiguousarray(codes1, np.uint8)
    codes2 = np.ascontiguousarray(codes2, np.uint8)
    levels, b = _f32(levels), _f32(b)
    x = _f32(x).copy()
    n, d = codes1.shape
    f = lib().zo_sgd_epoch_threads
    f.restype = C.c_int
    used = f(_p(codes1), _p(codes2), _p(levels), _p(b), C.c_int64(n), C.c_int64(d), C.c_int(bits),
             _p(x), C.c_int64(batch), C.c_float(lr), C.c_int(threads))
    return x, int(used)


def sgd_epoch_e2e(codes1, codes2, levels, grid_idx, grid_lo, grid_step, b, bits, x, batch, lr,
                  grad_bits, model_bits, seed, epoch, first_step=0, num_steps=-1, debug=False):
    """End-to-end low-precision epoch (or a range of its steps).

    Returns the new fp32 model, plus a dict of the last step's intermediates if
    ``debug``.
    """
    codes1 = np.ascontiguousarray(codes1, np.uint8)
    codes2 = np.ascontiguousarray(codes2, np.uint8)
    levels, b = _f32(levels), _f32(b)
    grid_idx = np.ascontiguousarray(grid_idx, np.uint16)
    x = _f32(x).copy()
    n, d = codes1.shape
    dbg = None
    args = [None] * 5
    if debug:
        dbg = dict(m=np.zeros(d, np.int32), acc=np.zeros(batch, np.int32),
                   r=np.zeros(batch, np.float32), g=np.zeros(d, np.float32),
                   gq=np.zeros(d, np.int32))
        args = [_p(dbg[k]) for k in ("m", "acc", "r", "g", "gq")]
    rc = lib().zo_sgd_epoch_e2e(_p(codes1), _p(codes2), _p(levels), _p(grid_idx),
                                C.c_float(grid_lo), C.c_float(grid_step), _p(b), C.c_int64(n),
                                C.c_int64(d), C.c_int(bits), _p(x), C.c_int64(batch),
                                C.c_float(lr), C.c_int(grad_bits), C.c_int(model_bits),
                                C.c_uint64(seed), C.c_uint32(epoch), C.c_int64(first_step),
                                C.c_int64(num_steps), *args)
    if rc != 0:
        raise OverflowError("integer dot product left the int32 range")
    return (x, dbg) if debug else x


# ---------------------------------------------------------------------------------------------
# Compact storage of the two samples (Sec. 2.2, "Overhead of Storing Samples"): the two
# quantisations of a value lie on the two ends of ONE interval of the level grid, so they differ
# by at most one level.  Stored: a base level (b bits) and, per sample, one bit saying whether the
# sample sits on the base level or on the next one: b + 2 bits instead of 2 b.
# Reading taken here: the base is the smaller of the two codes (when both samples rounded up the
# paper's "smallest number of the interval" would be one lower with both bits set; the decoded
# samples and the size are the same, and this form needs the codes only).
# ---------------------------------------------------------------------------------------------
def compact_encode(codes1, codes2):
    """(base, bit1, bit2) with codes_k = base + bit_k; ValueError if a pair differs by more than one."""
    c1 = np.asarray(codes1).astype(np.int64)
    c2 = np.asarray(codes2).astype(np.int64)
    base = np.minimum(c1, c2)
    u1, u2 = c1 - base, c2 - base
    if u1.max(initial=0) > 1 or u2.max(initial=0) > 1:
        raise ValueError("the two samples of a value differ by more than one level")
    return base.astype(np.uint8), u1.astype(np.uint8), u2.astype(np.uint8)


def compact_decode(base, bit1, bit2):
    base = np.asarray(base).astype(np.int64)
    return (base + np.asarray(bit1)).astype(np.uint8), (base + np.asarray(bit2)).astype(np.uint8)


def compact_bits_per_value(bits, samples=2):
    """Bits per value for `samples` ordered samples: the base level and one bit each."""
    return bits + samples


def loss(A, b, x):
    A, b, x = _f32(A), _f32(b), _f32(x)
    n, d = A.shape
    return float(lib().zo_loss(_p(A), C.c_int64(n), C.c_int64(d), C.c_int64(d), _p(b), _p(x)))


def loss_codes(codes, levels, bits, b, x):
    codes = np.ascontiguousarray(codes, np.uint8)
    levels, b, x = _f32(levels), _f32(b), _f32(x)
    n, d = codes.shape
    return float(lib().zo_loss_codes(_p(codes), _p(levels), C.c_int(bits), C.c_int64(n),
                                     C.c_int64(d), _p(b), _p(x)))
