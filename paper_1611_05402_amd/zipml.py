"""Thin ctypes binding of libzipml.so: argument marshalling only.

Every function takes torch tensors that already live on the GPU (PyTorch is used for
device memory and streams, nothing else), passes their raw pointers through the C ABI
declared in ``include/zipml.h`` and raises ``ZipmlError`` on a non-zero status.  There is
no CPU fallback: if the library has not been built, ``lib()`` raises.
"""
from __future__ import annotations

import ctypes as C
import os

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(HERE, "libzipml.so")

UNIFORM, OPTIMAL, GREEDY = 0, 1, 2
RANGE_GIVEN, SYMMETRIC = 1, 2
SGD_STEPWISE, SGD_AVERAGED, SGD_PRODUCTION = 1, 2, 4
STATIC_WORKSPACE_BYTES = 8 << 20
PROX_NONE, PROX_L1, PROX_L2SQ, PROX_BOX = 0, 1, 2, 3

OK, EINVAL, EALIGN, ERANGE, EWORKSPACE, ELAUNCH, EUNSUPPORTED, ETIMEOUT = 0, -1, -2, -3, -4, -5, -6, -7

EXPORTS = ["zipml_strerror", "zipml_packed_bytes", "zipml_workspace_bytes", "zipml_levels",
           "zipml_quantize", "zipml_quantize_swapped", "zipml_compact_bytes", "zipml_compact_encode",
           "zipml_compact_decode", "zipml_sgd_epoch", "zipml_sgd_epoch_l2",
           "zipml_sgd_epoch_prox", "zipml_sgd_epoch_avg", "zipml_sgd_epoch_static", "zipml_sgd_status",
           "zipml_loss", "zipml_debug_stream", "zipml_debug_set", "zipml_sgd_epoch_compact",
           "zipml_unpack_codes", "zipml_debug_step"]


class ZipmlError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        super().__init__(f"{where}: {strerror(code)} ({code})")


_lib = None


def lib() -> C.CDLL:
    """Loads libzipml.so; raises if it has not been built (no fallback path exists)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_1611_05402_amd.build` "
                               "(or __graft_entry__.build()) first")
        # PyTorch ships its own HIP runtime; it has to be the one already loaded when libzipml.so
        # resolves libamdhip64, otherwise the process ends up with two runtimes and the tensors'
        # device pointers belong to the other one.
        import torch  # noqa: F401
        L = C.CDLL(LIB_PATH)
        L.zipml_strerror.restype = C.c_char_p
        L.zipml_strerror.argtypes = [C.c_int]
        L.zipml_packed_bytes.restype = C.c_size_t
        L.zipml_packed_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int]
        L.zipml_compact_bytes.restype = C.c_size_t
        L.zipml_compact_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int]
        L.zipml_compact_encode.restype = C.c_int
        L.zipml_compact_encode.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int,
                                           C.c_void_p, C.c_void_p, C.c_size_t]
        L.zipml_compact_decode.restype = C.c_int
        L.zipml_compact_decode.argtypes = [C.c_void_p, C.c_void_p, C.c_int64, C.c_int64, C.c_int, C.c_void_p,
                                           C.c_void_p]
        L.zipml_workspace_bytes.restype = C.c_size_t
        L.zipml_workspace_bytes.argtypes = [C.c_int64, C.c_int64, C.c_int, C.c_int64, C.c_int]
        vp, i64, i32, f32, u64, u32, sz = (C.c_void_p, C.c_int64, C.c_int, C.c_float, C.c_uint64,
                                           C.c_uint32, C.c_size_t)
        L.zipml_levels.restype = i32
        L.zipml_levels.argtypes = [vp, vp, i64, i64, i64, i32, i32, i32, i32, vp, vp, vp, vp,
                                   C.POINTER(C.c_double), vp, sz]
        L.zipml_quantize.restype = i32
        L.zipml_quantize.argtypes = [vp, vp, i64, i64, i64, i64, i64, vp, i32, u64, u32, vp, vp]
        L.zipml_quantize_swapped.restype = i32
        L.zipml_quantize_swapped.argtypes = L.zipml_quantize.argtypes
        L.zipml_sgd_epoch_avg.restype = i32
        L.zipml_sgd_epoch_avg.argtypes = [vp, vp, vp, vp, vp, vp, vp, i64, i64, i32, vp, i64, f32, f32, i32, vp, sz]
        sgd = [vp, vp, vp, vp, vp, f32, f32, i32, vp, i64, i64, i32, vp, i64, f32, i32, i32, u64, u32]
        L.zipml_sgd_epoch.restype = i32
        L.zipml_sgd_epoch.argtypes = sgd + [i32, vp, sz]
        L.zipml_sgd_epoch_compact.restype = i32
        L.zipml_sgd_epoch_compact.argtypes = [vp, vp, vp, vp, i64, i64, i32, vp, i64, f32, vp, sz]
        L.zipml_sgd_epoch_static.restype = i32
        L.zipml_sgd_epoch_static.argtypes = sgd + [i32, vp]
        L.zipml_sgd_epoch_l2.restype = i32
        L.zipml_sgd_epoch_l2.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, vp, i64, f32, f32, i32, vp, sz]
        L.zipml_sgd_epoch_prox.restype = i32
        L.zipml_sgd_epoch_prox.argtypes = [vp, vp, vp, vp, vp, i64, i64, i32, vp, i64, f32, f32, i32, f32,
                                           i32, vp, sz]
        L.zipml_debug_step.restype = i32
        L.zipml_debug_step.argtypes = sgd + [i64, i32, vp, vp, vp, vp, vp, vp, sz]
        L.zipml_sgd_status.restype = i32
        L.zipml_sgd_status.argtypes = [vp, vp, sz]
        L.zipml_loss.restype = i32
        L.zipml_loss.argtypes = [vp, vp, i64, vp, i32, vp, i32, vp, vp, i64, i64,
                                 C.POINTER(C.c_double), vp, sz]
        L.zipml_debug_stream.restype = i32
        L.zipml_debug_stream.argtypes = [vp, vp, vp, sz, vp]
        L.zipml_debug_set.restype = i32
        L.zipml_debug_set.argtypes = [i32, i64]
        L.zipml_unpack_codes.restype = i32
        L.zipml_unpack_codes.argtypes = [vp, vp, i32, i64, i64, i32, vp]
        _lib = L
    return _lib


def strerror(code: int) -> str:
    return lib().zipml_strerror(code).decode()


def _check(code: int, where: str) -> None:
    if code != 0:
        raise ZipmlError(code, where)


def _ptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream(stream=None):
    import torch
    s = stream if stream is not None else torch.cuda.current_stream()
    return C.c_void_p(s.cuda_stream)


(KNOB_TARGET_WORKGROUPS, KNOB_NO_MATRIX_CORES, KNOB_CHUNK_SAMPLES, KNOB_MAX_REPLICAS, KNOB_ROWS_MIN_BATCH,
 KNOB_ROWS_ITEM_BLOCKS, KNOB_ROWS_WORKGROUPS, KNOB_SPIN_LIMIT, KNOB_HOST_DP, KNOB_HIST_FEATURES,
 KNOB_STORE_EXCHANGE_MIN, KNOB_COOPERATIVE_LAUNCH, KNOB_REDUCER_WORKGROUPS, KNOB_PREFETCH_WORKGROUPS) = range(14)


def debug_set(knob: int, value: int) -> None:
    """Development knob (see include/zipml.h); value -1 restores the automatic choice."""
    _check(lib().zipml_debug_set(knob, value), "zipml_debug_set")


def debug_stream(src, sink, dst=None, nbytes=None, stream=None) -> None:
    """Plain streaming read (or copy, with dst) of known size; XOR of all dwords into sink[0]."""
    nb = src.numel() * src.element_size() if nbytes is None else nbytes
    _check(lib().zipml_debug_stream(_stream(stream), _ptr(src), _ptr(dst), nb, _ptr(sink)),
           "zipml_debug_stream")


def packed_bytes(n: int, d: int, bits: int) -> int:
    return int(lib().zipml_packed_bytes(n, d, bits))


def workspace_bytes(n: int, d: int, bits: int, batch: int, n_candidates: int = 0) -> int:
    return int(lib().zipml_workspace_bytes(n, d, bits, batch, n_candidates))


def levels(A, n, d, lda, bits, mode, flags, n_candidates, lo, hi, levels_out, grid_idx, workspace,
           want_mean_variance=False, stream=None):
    mv = C.c_double(0.0)
    code = lib().zipml_levels(_stream(stream), _ptr(A), n, d, lda, bits, mode, flags, n_candidates,
                              _ptr(lo), _ptr(hi), _ptr(levels_out), _ptr(grid_idx),
                              C.byref(mv) if want_mean_variance else None, _ptr(workspace),
                              0 if workspace is None else workspace.numel() * workspace.element_size())
    _check(code, "zipml_levels")
    return mv.value if want_mean_variance else None


def quantize(A, n_rows, d, lda, row0, n_total, levels_t, bits, seed, epoch, packed1, packed2,
             stream=None):
    _check(lib().zipml_quantize(_stream(stream), _ptr(A), n_rows, d, lda, row0, n_total,
                                _ptr(levels_t), bits, seed, epoch, _ptr(packed1), _ptr(packed2)),
           "zipml_quantize")


def quantize_swapped(A, n_rows, d, lda, row0, n_total, levels_t, bits, seed, epoch, packed1s,
                     packed2s, stream=None):
    _check(lib().zipml_quantize_swapped(_stream(stream), _ptr(A), n_rows, d, lda, row0, n_total,
                                        _ptr(levels_t), bits, seed, epoch, _ptr(packed1s),
                                        _ptr(packed2s)), "zipml_quantize_swapped")


def _sgd_args(packed1, packed2, levels_t, grid_idx, grid_lo, grid_step, grid_max, b, n, d, bits, x,
              batch, lr, grad_bits, model_bits, seed, epoch, stream):
    return [_stream(stream), _ptr(packed1), _ptr(packed2), _ptr(levels_t), _ptr(grid_idx),
            float(grid_lo), float(grid_step), int(grid_max), _ptr(b), n, d, bits, _ptr(x), batch,
            float(lr), grad_bits, model_bits, seed, epoch]


def sgd_epoch(packed1, packed2, levels_t, b, n, d, bits, x, batch, lr, workspace, *, grid_idx=None,
              grid_lo=0.0, grid_step=0.0, grid_max=0, grad_bits=0, model_bits=0, seed=0, epoch=0,
              flags=0, stream=None):
    args = _sgd_args(packed1, packed2, levels_t, grid_idx, grid_lo, grid_step, grid_max, b, n, d,
                     bits, x, batch, lr, grad_bits, model_bits, seed, epoch, stream)
    _check(lib().zipml_sgd_epoch(*args, flags, _ptr(workspace),
                                 workspace.numel() * workspace.element_size()), "zipml_sgd_epoch")


def sgd_epoch_static(packed1, packed2, levels_t, b, n, d, bits, x, batch, lr, status, *, grid_idx=None,
                     grid_lo=0.0, grid_step=0.0, grid_max=0, grad_bits=0, model_bits=0, seed=0, epoch=0,
                     flags=0, stream=None):
    """zipml_sgd_epoch on the library's built-in workspace (no allocation); `status`: int32 tensor."""
    args = _sgd_args(packed1, packed2, levels_t, grid_idx, grid_lo, grid_step, grid_max, b, n, d,
                     bits, x, batch, lr, grad_bits, model_bits, seed, epoch, stream)
    _check(lib().zipml_sgd_epoch_static(*args, flags, _ptr(status)), "zipml_sgd_epoch_static")


def sgd_epoch_compact(compact, levels_t, b, n, d, bits, x, batch, lr, workspace, stream=None):
    """The epoch on the compact record of (packed2s, packed2) alone (very large minibatches, 8 bits)."""
    _check(lib().zipml_sgd_epoch_compact(_stream(stream), _ptr(compact), _ptr(levels_t), _ptr(b), n, d,
                                         bits, _ptr(x), batch, lr, _ptr(workspace),
                                         workspace.numel() * workspace.element_size()),
           "zipml_sgd_epoch_compact")


def sgd_epoch_l2(packed1, packed2, levels_t, b, n, d, bits, x, batch, lr, l2, workspace, *, flags=0,
                 stream=None):
    _check(lib().zipml_sgd_epoch_l2(_stream(stream), _ptr(packed1), _ptr(packed2), _ptr(levels_t),
                                    _ptr(b), n, d, bits, _ptr(x), batch, lr, l2, flags,
                                    _ptr(workspace), workspace.numel() * workspace.element_size()),
           "zipml_sgd_epoch_l2")


def compact_bytes(n, d, bits):
    return int(lib().zipml_compact_bytes(n, d, bits))


def compact_encode(packed_a, packed_b, n, d, bits, compact, workspace, *, stream=None):
    _check(lib().zipml_compact_encode(_stream(stream), _ptr(packed_a), _ptr(packed_b), n, d, bits,
                                      _ptr(compact), _ptr(workspace),
                                      workspace.numel() * workspace.element_size()),
           "zipml_compact_encode")


def compact_decode(compact, n, d, bits, packed_a, packed_b, *, stream=None):
    _check(lib().zipml_compact_decode(_stream(stream), _ptr(compact), n, d, bits, _ptr(packed_a),
                                      _ptr(packed_b)), "zipml_compact_decode")


def sgd_epoch_prox(packed1, packed2, levels_t, b, n, d, bits, x, batch, lr, prox, prox_coef,
                   workspace, *, l2=0.0, flags=0, stream=None):
    _check(lib().zipml_sgd_epoch_prox(_stream(stream), _ptr(packed1), _ptr(packed2), _ptr(levels_t),
                                      _ptr(b), n, d, bits, _ptr(x), batch, lr, l2, prox, prox_coef,
                                      flags, _ptr(workspace),
                                      workspace.numel() * workspace.element_size()),
           "zipml_sgd_epoch_prox")


def sgd_epoch_avg(packed1, packed2, packed1s, packed2s, levels_t, b, n, d, bits, x, batch, lr,
                  workspace, *, l2=0.0, flags=0, stream=None):
    _check(lib().zipml_sgd_epoch_avg(_stream(stream), _ptr(packed1), _ptr(packed2), _ptr(packed1s),
                                     _ptr(packed2s), _ptr(levels_t), _ptr(b), n, d, bits, _ptr(x),
                                     batch, lr, l2, flags, _ptr(workspace),
                                     workspace.numel() * workspace.element_size()),
           "zipml_sgd_epoch_avg")


def debug_step(packed1, packed2, levels_t, b, n, d, bits, x, batch, lr, step, workspace, *,
               grid_idx=None, grid_lo=0.0, grid_step=0.0, grid_max=0, grad_bits=0, model_bits=0,
               seed=0, epoch=0, flags=0, model_codes=None, acc=None, r=None, g=None,
               grad_codes=None, stream=None):
    args = _sgd_args(packed1, packed2, levels_t, grid_idx, grid_lo, grid_step, grid_max, b, n, d,
                     bits, x, batch, lr, grad_bits, model_bits, seed, epoch, stream)
    _check(lib().zipml_debug_step(*args, step, flags, _ptr(model_codes), _ptr(acc), _ptr(r), _ptr(g),
                                  _ptr(grad_codes), _ptr(workspace),
                                  workspace.numel() * workspace.element_size()), "zipml_debug_step")


def sgd_status(workspace, stream=None) -> int:
    return int(lib().zipml_sgd_status(_stream(stream), _ptr(workspace),
                                      workspace.numel() * workspace.element_size()))


def loss(b, x, n, d, workspace, *, A=None, lda=0, packed=None, copy=2, levels_t=None, bits=0,
         stream=None) -> float:
    out = C.c_double(0.0)
    _check(lib().zipml_loss(_stream(stream), _ptr(A), lda, _ptr(packed), copy, _ptr(levels_t), bits,
                            _ptr(b), _ptr(x), n, d, C.byref(out), _ptr(workspace),
                            workspace.numel() * workspace.element_size()), "zipml_loss")
    return out.value


def unpack_codes(packed, copy, n, d, bits, codes_out, stream=None):
    _check(lib().zipml_unpack_codes(_stream(stream), _ptr(packed), copy, n, d, bits,
                                    _ptr(codes_out)), "zipml_unpack_codes")
