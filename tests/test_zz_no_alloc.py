"""The entry point that allocates nothing: zipml_sgd_epoch_static (workspace = a fixed array inside
the library) must give what zipml_sgd_epoch gives on a workspace of the caller's, bit for bit, on
two calls in a row of which the second is the smaller problem (the array keeps what the first call
left in it)."""
import numpy as np
import pytest
import torch

from gpu_harness import DEV, GpuProblem, dev
from paper_1611_05402_amd import synth, zipml

pytestmark = pytest.mark.gpu


def say(*a):
    print(*a, flush=True)


def _problem(factory, kw, bits, lo, hi, seed):
    w = factory(**kw)
    A, b = w.full()
    p = GpuProblem(A, b, bits, w.batch)
    p.make_levels(zipml.UNIFORM, 0, lo=np.full(w.d, lo, np.float32), hi=np.full(w.d, hi, np.float32))
    p.quantize(seed, 0)
    return w, p


def _both(w, p, lr, epochs, **kw):
    """(model from zipml_sgd_epoch, model from zipml_sgd_epoch_static) after `epochs` epochs."""
    rng = np.random.default_rng(1)
    x0 = (rng.standard_normal(w.d) * 0.1).astype(np.float32)
    xa, xb = dev(x0), dev(x0)
    status = torch.full((4,), -99, dtype=torch.int32, device=DEV)
    for ep in range(epochs):
        zipml.sgd_epoch(p.p1, p.p2, p.levels, p.b, w.n, w.d, p.bits, xa, w.batch, lr, p.ws, epoch=ep,
                        grid_idx=p.grid if kw.get("model_bits") else None, **kw)
        assert zipml.sgd_status(p.ws) == 0
        zipml.sgd_epoch_static(p.p1, p.p2, p.levels, p.b, w.n, w.d, p.bits, xb, w.batch, lr, status,
                               epoch=ep, grid_idx=p.grid if kw.get("model_bits") else None, **kw)
        torch.cuda.synchronize()
        assert int(status[0].item()) == 0
    return xa.cpu().numpy(), xb.cpu().numpy()


def test_static_workspace_epochs_equal_caller_workspace_epochs():
    # first the larger problem: the matrix-core loop on 9 workgroups ...
    say("static workspace: dense8 n=4096 d=288 batch=256")
    w1, p1 = _problem(synth.dense8, dict(n=4096, d=288, batch=256), 8, -1.0, 1.0, 3)
    a, b = _both(w1, p1, 1e-2, 2)
    assert np.linalg.norm(a) > 0 and np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # ... then, on what it left behind, a smaller one in the end-to-end mode (three exchanges per step)
    say("static workspace: tiny n=1024 d=96 batch=64, 8-bit model and gradient")
    w2, p2 = _problem(synth.tiny, dict(n=1024, d=96, batch=64, bits=4), 4, -1.0, 1.0, 4)
    K = 16
    a, b = _both(w2, p2, 0.05, 2, grad_bits=8, model_bits=8, grid_lo=-1.0, grid_step=2.0 / (K - 1),
                 grid_max=K - 1, seed=4)
    assert np.linalg.norm(a) > 0 and np.array_equal(a.view(np.uint32), b.view(np.uint32))
    # ... and a still smaller fp32 one on the vector loop (3-bit codes)
    say("static workspace: tiny n=512 d=70 batch=32, 3 bits")
    w3, p3 = _problem(synth.tiny, dict(n=512, d=70, batch=32, bits=3), 3, -1.0, 1.0, 5)
    a, b = _both(w3, p3, 0.05, 1)
    assert np.linalg.norm(a) > 0 and np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_static_workspace_refuses_what_does_not_fit():
    w, p = _problem(synth.tiny, dict(n=1024, d=64, batch=16), 4, -1.0, 1.0, 0)
    x = torch.zeros(64, dtype=torch.float32, device=DEV)
    status = torch.zeros(4, dtype=torch.int32, device=DEV)
    # a shape whose workspace exceeds the built-in array: nothing is enqueued, the code says why
    n_big, d_big, B_big = 1 << 20, 16384, 1 << 20
    assert zipml.workspace_bytes(n_big, d_big, 4, B_big) > zipml.STATIC_WORKSPACE_BYTES
    with pytest.raises(zipml.ZipmlError) as e:
        zipml.sgd_epoch_static(p.p1, p.p2, p.levels, p.b, n_big, d_big, 4, x, B_big, 0.1, status)
    assert e.value.code == zipml.EWORKSPACE
    with pytest.raises(zipml.ZipmlError) as e:      # the status word is required
        zipml.sgd_epoch_static(p.p1, p.p2, p.levels, p.b, w.n, w.d, 4, x, 16, 0.1, None)
    assert e.value.code == zipml.EINVAL
