#!/usr/bin/env python3
"""Benchmark: double-sampled low-precision SGD epochs on one MI355X.

One timed "step" is one full pass of the SGD hot path over the resident quantised data set
(one zipml_sgd_epoch call = n / batch sequential minibatch steps: dot pass over copy 2,
residuals, gradient pass over copy 1, model update).  The workload is the dense 8-bit
least-squares problem (n = 65,536, d = 2,048, batch 256) with both packed copies already in
HBM.  Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0   # MI355X HBM3E, published


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="timed epochs")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="dense8", choices=["tiny", "dense8", "lowbit"])
    ap.add_argument("--batch", type=int, default=0, help="override the minibatch size")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-seconds", type=float, default=10.0)
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch plain device copies of known size (untimed), so that a "
                         "rocprofv3 --pmc run of this command yields the HBM counter scale")
    return ap.parse_args()


def recorded_traffic(workload, batch):
    """HBM bytes per epoch launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), as
    recorded in the text summary under profiles/ for this workload; None if there is none."""
    path = os.path.join(ROOT, "profiles", f"sgd_epoch_{workload}_hbm_traffic.txt")
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    fields = line.split()
                    if len(fields) >= 4 and fields[2] == "batch" and int(fields[3]) != batch:
                        return None
                    return float(fields[1])
    except OSError:
        pass
    return None


def cpu_baseline(w, A_rows, b_rows, L, seconds):
    """The oracle's epoch loop, as it stands, timed on one host core on the first rows of
    the same workload."""
    import numpy as np
    import oracle
    c1, c2 = oracle.quantize(A_rows, L, w.bits, 0, 0)
    x = np.zeros(w.d, np.float32)
    n_s = A_rows.shape[0]
    t0 = time.perf_counter()
    passes = 0
    while True:
        x = oracle.sgd_epoch(c1, c2, L, b_rows, w.bits, x, w.batch, w.lr)
        passes += 1
        el = time.perf_counter() - t0
        if el >= seconds:
            break
    return {"value": passes * n_s / el, "unit": "samples/s", "cores": 1, "kind": "oracle",
            "sample": f"first {n_s} of {w.n} samples (d={w.d}, batch {w.batch}), {passes} passes "
                      f"of the oracle epoch loop in {el:.1f} s, single thread"}


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no multi-GPU path exists); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    import oracle  # only for the cpu_baseline leg and the level table check
    from paper_1611_05402_amd import synth, zipml

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    zipml.lib()   # fails loudly if the HIP library is missing
    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = synth.WORKLOADS[args.workload]()
    if args.batch:
        w.batch = args.batch
    n, d, bits, B = w.n, w.d, w.bits, w.batch
    K = 1 << bits

    # ---- synthetic data, resident in HBM before anything is timed
    t0 = time.perf_counter()
    ws = torch.zeros(zipml.workspace_bytes(n, d, bits, B), dtype=torch.uint8, device=dev)
    lev = torch.zeros(d, K, dtype=torch.float32, device=dev)
    lo = torch.zeros(d, dtype=torch.float32, device=dev)
    hi = torch.zeros(d, dtype=torch.float32, device=dev)
    p1 = torch.zeros(zipml.packed_bytes(n, d, bits), dtype=torch.uint8, device=dev)
    p2 = torch.zeros_like(p1)
    bd = torch.zeros(n, dtype=torch.float32, device=dev)
    chunk = 8192
    A_head = b_head = None
    Ad_full = torch.empty(n, d, dtype=torch.float32, device=dev)
    for r0 in range(0, n, chunk):
        r1 = min(n, r0 + chunk)
        A = w.rows(r0, r1)
        b = w.labels(r0, r1, A)
        if r0 == 0:
            A_head, b_head = A, b
        Ad_full[r0:r1].copy_(torch.from_numpy(A))
        bd[r0:r1].copy_(torch.from_numpy(b))
    gen_s = time.perf_counter() - t0

    def timed(fn, reps=3):
        fn()                      # first call: code object load, not what is being timed
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        for _ in range(reps):
            fn()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) / reps   # ms

    if w.range_mode == "fixed":
        lo.fill_(w.lo)
        hi.fill_(w.hi)
        flags = zipml.RANGE_GIVEN
    else:
        flags = zipml.SYMMETRIC if w.range_mode == "symmetric" else 0
    levels_ms = timed(lambda: zipml.levels(Ad_full, n, d, d, bits, zipml.UNIFORM, flags, 0, lo, hi,
                                           lev, None, ws))
    quant_ms = timed(lambda: zipml.quantize(Ad_full, n, d, d, 0, n, lev, bits, 0, 0, p1, p2))

    x = torch.zeros(d, dtype=torch.float32, device=dev)

    def epoch():
        zipml.sgd_epoch(p1, p2, lev, bd, n, d, bits, x, B, w.lr, ws)

    for _ in range(args.warmup):
        epoch()
    assert zipml.sgd_status(ws) == 0
    torch.cuda.synchronize()
    # K epochs, bracketed by synchronize; HIP events on the launch stream give the device time
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for k in range(args.steps):
        epoch()
        ev[k + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    assert zipml.sgd_status(ws) == 0
    per_epoch_ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(args.steps)]
    kern_ms = sum(per_epoch_ms) / len(per_epoch_ms)

    if args.copy_calibration:
        # a copy of known size on the same stream: 256 MiB read + 256 MiB written per launch
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()

    # ---- what a plain streaming read reaches on this machine: the library's fp32 loss kernel (reads
    # 4 n d bytes once, nothing else) over 2 GiB
    n_c = (2 << 30) // (4 * d)
    A_c = torch.empty(n_c, d, dtype=torch.float32, device=dev).normal_()
    b_c = torch.zeros(n_c, dtype=torch.float32, device=dev)
    ws_c = torch.zeros(zipml.workspace_bytes(n_c, d, bits, B), dtype=torch.uint8, device=dev)
    ceil_ms = timed(lambda: zipml.loss(b_c, x, n_c, d, ws_c, A=A_c, lda=d), reps=5)
    read_ceiling = 4.0 * n_c * d / (ceil_ms * 1e-3) / 1e9
    del A_c, b_c, ws_c

    # ---- the same epoch at larger minibatches (same resident data; not part of `value`):
    # 4x, 16x and the whole data set per step, and the whole-data-set step on 8x the samples
    # (random codes: only the rate matters there)
    sweep = []

    def sweep_point(nn, p1s, p2s, bs, batch, reps=5):
        xs = torch.zeros(d, dtype=torch.float32, device=dev)
        wss = torch.zeros(zipml.workspace_bytes(nn, d, bits, batch), dtype=torch.uint8, device=dev)
        try:
            ms = timed(lambda: zipml.sgd_epoch(p1s, p2s, lev, bs, nn, d, bits, xs, batch, w.lr, wss), reps)
        except zipml.ZipmlError as e:       # e.g. a shape whose large minibatches no kernel takes
            sweep.append({"n": nn, "batch": batch, "error": str(e)})
            return
        if zipml.sgd_status(wss) != 0:
            sweep.append({"n": nn, "batch": batch, "error": zipml.strerror(zipml.sgd_status(wss))})
            return
        nbytes = nn * (2 * d * bits / 8 + 4)
        sweep.append({"n": nn, "batch": batch, "ms_per_epoch": ms, "us_per_step": ms * 1e3 / (nn // batch),
                      "GBps": nbytes / (ms * 1e-3) / 1e9, "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                      "frac_of_measured_read_ceiling": nbytes / (ms * 1e-3) / 1e9 / read_ceiling})

    if not args.batch:
        for mult in (4, 16):
            if n % (B * mult) == 0:
                sweep_point(n, p1, p2, bd, B * mult)
        sweep_point(n, p1, p2, bd, n)
        n8 = 8 * n
        q1 = torch.randint(0, 256, (zipml.packed_bytes(n8, d, bits),), dtype=torch.uint8, device=dev)
        q2 = torch.randint(0, 256, (zipml.packed_bytes(n8, d, bits),), dtype=torch.uint8, device=dev)
        sweep_point(n8, q1, q2, torch.randn(n8, device=dev), n8)
        del q1, q2

    loss_ms = timed(lambda: zipml.loss(bd, x, n, d, ws, A=Ad_full, lda=d))
    final_loss = zipml.loss(bd, x, n, d, ws, A=Ad_full, lda=d)
    loss_p_ms = timed(lambda: zipml.loss(bd, x, n, d, ws, packed=p2, copy=2, levels_t=lev, bits=bits))

    # the data-dependent level computations on the same matrix (their results are not used by the
    # timed epochs): column ranges + uniform levels, and the 3-bit level search over 1024 bins,
    # plain dynamic program and greedy candidates
    level_ms = {}
    try:
        lo2, hi2 = torch.zeros_like(lo), torch.zeros_like(hi)
        lev3 = torch.zeros(d, 8, dtype=torch.float32, device=dev)
        ws3 = torch.zeros(zipml.workspace_bytes(n, d, 3, B, 1024), dtype=torch.uint8, device=dev)
        lev2 = torch.zeros_like(lev)
        level_ms["levels_with_range_scan"] = timed(
            lambda: zipml.levels(Ad_full, n, d, d, bits, zipml.UNIFORM, 0, 0, lo2, hi2, lev2, None, ws3))
        level_ms["levels_optimal_3bit_1024bins"] = timed(
            lambda: zipml.levels(Ad_full, n, d, d, 3, zipml.OPTIMAL, 0, 1024, lo2, hi2, lev3, None, ws3))
        level_ms["levels_greedy_3bit_1024bins"] = timed(
            lambda: zipml.levels(Ad_full, n, d, d, 3, zipml.GREEDY, 0, 1024, lo2, hi2, lev3, None, ws3))
        del ws3, lev3
    except zipml.ZipmlError as e:
        level_ms["error"] = str(e)

    samples_per_s = args.steps * n / wall
    alg_bytes = n * (2 * d * bits / 8 + 4)            # both packed copies once + labels
    achieved = alg_bytes / (kern_ms * 1e-3) / 1e9
    out = {
        "metric": "double-sampled SGD samples/sec (packed-data GB/s and % of HBM peak in roofline)",
        "value": samples_per_s,
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": wall / args.steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32 (model, residuals; sums taken exactly on i8 digits)",
        "data": "synthetic",
        "config": {"workload": f"{w.name}: n={n}, d={d}, {bits}-bit uniform levels, batch {B}, "
                               f"lr {w.lr}, fp32 model", "minibatch_steps_per_epoch": n // B,
                   "packed_bytes_per_epoch": int(alg_bytes)},
        "packed_GBps": alg_bytes * args.steps / wall / 1e9,
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBS, "traffic": recorded_traffic(w.name, B),
                     "kernel": f"k_sgd<{bits}> (persistent epoch kernel)",
                     "kernel_ms": kern_ms, "us_per_minibatch_step": kern_ms * 1e3 / (n // B),
                     "measured_read_ceiling_GBps": read_ceiling,
                     "frac_of_measured_read_ceiling": achieved / read_ceiling},
        "other_ms": {"levels": levels_ms, "quantize": quant_ms, "loss_fp32": loss_ms,
                     "loss_packed": loss_p_ms, **level_ms, "generate_and_upload_s": gen_s},
        "batch_sweep": sweep,
        "final_loss": final_loss,
        "paper_context": "paper reports ratios only: up to 6.5x over a 32-bit FPGA implementation "
                         "or 10-core Hogwild! (other hardware; not a target)",
    }
    if not args.no_cpu_baseline:
        n_s = min(n, 4096 if d >= 1024 else 16384)
        n_s -= n_s % B
        L = oracle.levels_uniform(lo.cpu().numpy(), hi.cpu().numpy(), bits)
        out["cpu_baseline"] = cpu_baseline(w, A_head[:n_s], b_head[:n_s], L, args.cpu_seconds)
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
