"""The C-ABI library loads, exports every symbol its header declares, and rejects bad
arguments with error codes before touching the GPU (runs without a GPU)."""
import ctypes as C
import os
import re

import pytest

from paper_1611_05402_amd import zipml

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(zipml.LIB_PATH):
        from paper_1611_05402_amd import build
        build.build()
    return zipml.lib()


def declared_functions():
    text = open(os.path.join(ROOT, "include", "zipml.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(zipml_[a-z0-9_]+)\s*\(", text)))


def test_exports_match_header(lib):
    names = declared_functions()
    assert len(names) >= 10
    for name in names:
        assert hasattr(lib, name), f"{name} declared in include/zipml.h but not exported"
    assert sorted(zipml.EXPORTS) == names


def test_strerror_and_sizes(lib):
    assert zipml.strerror(0) == "ok"
    for code in range(-7, 0):
        assert zipml.strerror(code) not in ("ok", "unknown error")
    assert zipml.strerror(-99) == "unknown error"
    # n, d padded to multiples of 32; bits/8 bytes per value
    assert zipml.packed_bytes(4096, 64, 4) == 4096 * 64 // 2
    assert zipml.packed_bytes(65536, 2048, 8) == 128 << 20
    assert zipml.packed_bytes(1000, 70, 3) == 1024 * 96 * 3 // 8
    assert zipml.packed_bytes(0, 64, 4) == 0 and zipml.packed_bytes(10, 64, 9) == 0
    assert zipml.workspace_bytes(4096, 64, 4, 16) >= 4096
    assert zipml.workspace_bytes(4096, 64, 4, 16, 1024) >= 64 * 1024 * 24
    assert zipml.workspace_bytes(4096, 64, 0, 16) == 0


def test_argument_errors_are_codes_not_crashes(lib):
    null = None
    fake = C.c_void_p(0x1000)          # aligned, never dereferenced: validation fails first
    odd = C.c_void_p(0x1004)
    # quantize
    assert lib.zipml_quantize(null, null, 32, 8, 8, 0, 32, fake, 4, 0, 0, fake, fake) == zipml.EINVAL
    assert lib.zipml_quantize(null, fake, 32, 8, 4, 0, 32, fake, 4, 0, 0, fake, fake) == zipml.EINVAL   # lda < d
    assert lib.zipml_quantize(null, fake, 32, 8, 8, 0, 32, fake, 9, 0, 0, fake, fake) == zipml.EINVAL   # bits
    assert lib.zipml_quantize(null, fake, 32, 8, 8, 16, 64, fake, 4, 0, 0, fake, fake) == zipml.EINVAL  # row0 % 32
    assert lib.zipml_quantize(null, fake, 20, 8, 8, 0, 64, fake, 4, 0, 0, fake, fake) == zipml.EINVAL   # ragged middle chunk
    assert lib.zipml_quantize(null, fake, 32, 8, 8, 0, 32, fake, 4, 0, 1 << 24, fake, fake) == zipml.EINVAL
    assert lib.zipml_quantize(null, fake, 32, 8, 8, 0, 32, fake, 4, 0, 0, odd, fake) == zipml.EALIGN
    # unpack
    assert lib.zipml_unpack_codes(null, fake, 3, 32, 8, 4, fake) == zipml.EINVAL
    assert lib.zipml_unpack_codes(null, odd, 1, 32, 8, 4, fake) == zipml.EALIGN
    # sgd
    def sgd(n=64, d=8, bits=4, batch=16, gb=0, mb=0, grid=null, gmax=0, flags=0, ws=fake, wsb=1 << 20,
            x=fake, epoch=0):
        return lib.zipml_sgd_epoch(null, fake, fake, fake, grid, 0.0, 0.0, gmax, fake, n, d, bits, x,
                                   batch, 0.1, gb, mb, 0, epoch, flags, ws, wsb)
    assert sgd(batch=24) == zipml.EINVAL            # not 4/8/16 or a multiple of 32
    assert sgd(n=100, batch=32) == zipml.EINVAL     # batch does not divide n
    assert sgd(bits=0) == zipml.EINVAL
    assert sgd(mb=1) == zipml.EINVAL and sgd(mb=9) == zipml.EINVAL
    assert sgd(mb=8) == zipml.EINVAL                # integer mode needs grid indices
    assert sgd(gb=8) == zipml.EUNSUPPORTED          # gradient quantisation needs model quantisation
    assert sgd(flags=zipml.SGD_AVERAGED) == zipml.EUNSUPPORTED
    assert sgd(flags=64) == zipml.EINVAL
    assert sgd(x=odd) == zipml.EALIGN
    assert sgd(ws=null) in (zipml.EWORKSPACE, zipml.EALIGN)
    assert sgd(wsb=16) == zipml.EWORKSPACE
    assert sgd(n=1 << 20, d=1 << 20, bits=8, batch=32, mb=8, grid=fake, gmax=255) == zipml.ERANGE
    assert sgd(epoch=1 << 24) == zipml.EINVAL
    # levels
    assert lib.zipml_levels(null, fake, 64, 8, 8, 4, 7, 0, 0, fake, fake, fake, null, None, fake, 1 << 20) == zipml.EINVAL   # no such mode
    assert lib.zipml_levels(null, fake, 64, 8, 8, 4, zipml.GREEDY, 0, 8, fake, fake, fake, null, None, fake, 1 << 20) == zipml.EINVAL   # M < 2^bits - 1
    assert lib.zipml_levels(null, fake, 64, 8, 8, 4, zipml.GREEDY, 0, 5000, fake, fake, fake, null, None, fake, 1 << 30) == zipml.EINVAL  # M > 4096
    assert lib.zipml_levels(null, fake, 64, 8, 8, 4, zipml.GREEDY, 0, 512, fake, fake, fake, null, None, fake, 1024) == zipml.EWORKSPACE
    # the workspace covers the candidates the greedy search leaves: edges [d][M + 1] uint16 and their number [d]
    assert zipml.workspace_bytes(64, 8, 4, 16, 512) >= 8 * 512 * 24 + 8 * 8 + 8 * 513 * 2 + 8 * 4
    assert lib.zipml_levels(null, fake, 64, 8, 8, 4, zipml.OPTIMAL, 0, 8, fake, fake, fake, null, None, fake, 1 << 20) == zipml.EINVAL  # M < 2^bits - 1
    assert lib.zipml_levels(null, fake, 64, 8, 8, 4, zipml.UNIFORM, 0, 0, fake, fake, fake, null, None, fake, 8) == zipml.EWORKSPACE
    # proximal step, symmetrised estimator
    def prox(kind=zipml.PROX_L1, coef=0.1, n=64, batch=16, x=fake):
        return lib.zipml_sgd_epoch_prox(null, fake, fake, fake, fake, n, 8, 4, x, batch, 0.1, 0.0, kind, coef,
                                        0, fake, 1 << 20)
    assert prox(kind=9) == zipml.EINVAL
    assert prox(coef=-1.0) == zipml.EINVAL
    assert prox(coef=float("nan")) == zipml.EINVAL
    assert prox(batch=24) == zipml.EINVAL
    assert prox(x=odd) == zipml.EALIGN

    def compact(rec=fake, n=32768, d=1024, bits=8, batch=16384, ws=1 << 30):
        return lib.zipml_sgd_epoch_compact(null, rec, fake, fake, n, d, bits, fake, batch, 0.1, fake, ws)
    assert compact(rec=null) == zipml.EINVAL
    assert compact(rec=odd) == zipml.EALIGN
    assert compact(n=1000) == zipml.EINVAL            # whole minibatches
    assert compact(ws=1024) == zipml.EWORKSPACE
    assert compact(bits=4) == zipml.EUNSUPPORTED      # built for 8-bit codes,
    assert compact(batch=4096) == zipml.EUNSUPPORTED  # very large minibatches
    assert compact(d=512) == zipml.EUNSUPPORTED       # and 513 .. 2048 features
    assert compact(d=2049) == zipml.EUNSUPPORTED

    def avg(p1s=fake, p2s=fake, bits=4, batch=64, flags=0):
        return lib.zipml_sgd_epoch_avg(null, fake, fake, p1s, p2s, fake, fake, 128, 8, bits, fake, batch, 0.1,
                                       0.0, flags, fake, 1 << 20)
    assert avg(p1s=null) == zipml.EINVAL
    assert avg(p2s=odd) == zipml.EALIGN
    assert avg(bits=3) == zipml.EUNSUPPORTED        # 2-, 4- or 8-bit codes only
    assert avg(batch=32) == zipml.EUNSUPPORTED      # whole blocks of 64 samples
    assert avg(flags=zipml.SGD_STEPWISE) == zipml.EUNSUPPORTED
    # compact storage
    assert zipml.compact_bytes(4096, 64, 4) == 4096 * 64 * 6 // 8
    assert zipml.compact_bytes(1000, 70, 3) == 1024 * 96 * 5 // 8
    assert zipml.compact_bytes(0, 64, 4) == 0 and zipml.compact_bytes(64, 64, 9) == 0
    assert lib.zipml_compact_encode(null, fake, null, 64, 8, 4, fake, fake, 256) == zipml.EINVAL
    assert lib.zipml_compact_encode(null, fake, fake, 64, 8, 4, fake, fake, 8) == zipml.EWORKSPACE
    assert lib.zipml_compact_encode(null, fake, odd, 64, 8, 4, fake, fake, 256) == zipml.EALIGN
    assert lib.zipml_compact_decode(null, fake, 64, 8, 0, fake, fake) == zipml.EINVAL
    assert lib.zipml_compact_decode(null, odd, 64, 8, 4, fake, fake) == zipml.EALIGN
    # loss
    out = C.c_double(0)
    assert lib.zipml_loss(null, fake, 8, null, 2, null, 0, fake, fake, 0, 8, C.byref(out), fake, 1 << 20) == zipml.EINVAL
    assert lib.zipml_loss(null, null, 0, null, 2, null, 0, fake, fake, 64, 8, C.byref(out), fake, 1 << 20) == zipml.EINVAL
    assert lib.zipml_loss(null, fake, 8, null, 2, null, 0, fake, fake, 64, 8, C.byref(out), fake, 8) == zipml.EWORKSPACE
    assert lib.zipml_sgd_status(null, null, 0) == zipml.EWORKSPACE


def test_static_workspace_entry_point_argument_errors(lib):
    """zipml_sgd_epoch_static validates before it touches the GPU: a missing or misaligned status
    word, an invalid shape, and a shape whose workspace exceeds the built-in array are codes."""
    null = None
    fake = C.c_void_p(0x1000)
    odd = C.c_void_p(0x1002)

    def call(n=64, d=8, bits=4, batch=16, status=fake):
        return lib.zipml_sgd_epoch_static(null, fake, fake, fake, null, 0.0, 0.0, 0, fake, n, d, bits,
                                          fake, batch, 0.1, 0, 0, 0, 0, 0, status)
    assert call(status=null) == zipml.EINVAL
    assert call(status=odd) == zipml.EINVAL
    assert call(bits=9) == zipml.EINVAL
    assert call(n=0) == zipml.EINVAL
    n_big = 1 << 20
    assert lib.zipml_workspace_bytes(n_big, 16384, 4, n_big, 0) > zipml.STATIC_WORKSPACE_BYTES
    assert call(n=n_big, d=16384, batch=n_big) == zipml.EWORKSPACE


def test_development_knobs_are_validated(lib):
    assert lib.zipml_debug_set(zipml.KNOB_SPIN_LIMIT, 5) == zipml.OK
    assert lib.zipml_debug_set(zipml.KNOB_SPIN_LIMIT, -1) == zipml.OK
    assert lib.zipml_debug_set(-1, 0) == zipml.EINVAL
    assert lib.zipml_debug_set(14, 0) == zipml.EINVAL
    assert lib.zipml_debug_set(zipml.KNOB_HOST_DP, -2) == zipml.EINVAL
    # and the product reads no environment variable
    import glob
    for path in glob.glob(os.path.join(ROOT, "paper_1611_05402_amd", "csrc", "*")):
        assert "getenv" not in open(path).read(), path


def test_bench_refuses_more_than_one_gpu():
    """This build runs on one GPU; bench.py says so instead of starting ranks."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode != 0
    assert "ONE GPU" in (r.stdout + r.stderr)
