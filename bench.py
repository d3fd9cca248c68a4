#!/usr/bin/env python3
"""Benchmark: double-sampled low-precision SGD epochs on one MI355X.

One timed "step" is one full pass of the SGD hot path over the resident quantised data set (one
zipml_sgd_epoch call = n / batch sequential minibatch steps: [model quantisation,] dot pass over
copy 2, residuals, gradient pass over copy 1, [gradient quantisation,] model update).  Every
workload of the benchmark spec beyond the tiny one is generated on the device at its full size,
quantised by the library, and timed with both packed copies resident in HBM:

  dense8  n=65,536   d=2,048   8-bit uniform levels             batch 256
  lowbit  n=1,048,576 d=512    2-bit, per-column ranges         batch 1,024
  tomo    n=262,144  d=16,384  4-bit uniform levels on [0,1]    batch 512   (4 GiB of codes)
  e2e     n=524,288  d=4,096   3-bit variance-optimal levels from 1,024 candidates,
                               8-bit model and gradient         batch 512

The headline (`value`, `roofline`, `config.workload`) is the largest of them, the tomography
shape; `configs` carries the same figures for all four.  Prints ONE JSON line.
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
HEADLINE = "tomo"
ALL = ["dense8", "lowbit", "tomo", "e2e"]


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20, help="timed epochs per workload")
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="all", choices=["all", "tiny"] + ALL,
                    help="all: the four full-size workloads, headline = tomo; else only that one")
    ap.add_argument("--batch", type=int, default=0, help="override the minibatch size")
    ap.add_argument("--rows", type=int, default=0, help="override the number of samples (development)")
    ap.add_argument("--dim", type=int, default=0, help="override the number of features (development)")
    ap.add_argument("--bits", type=int, default=0, help="override the code width (development)")
    ap.add_argument("--no-matrix-cores", action="store_true",
                    help="keep evenly spaced levels on the vector-ALU step loop (A/B measurement)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true",
                    help="skip the batch sweep and the timings of the other entry points")
    ap.add_argument("--cpu-seconds", type=float, default=8.0, help="per leg of the oracle baseline")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also launch plain streaming reads and copies of known size (untimed), so "
                         "that a rocprofv3 --pmc run of this command yields the HBM counter scale")
    return ap.parse_args()


def recorded_traffic(workload, batch, note=False):
    """HBM bytes per epoch launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE), as
    recorded in the text summary under profiles/ for this workload; None if there is none.
    note=True: the remark recorded with it (what the counters include), or None."""
    path = os.path.join(ROOT, "profiles", f"sgd_epoch_{workload}_hbm_traffic.txt")
    value, remark = None, None
    try:
        with open(path) as f:
            for line in f:
                if line.startswith("traffic_bytes_per_launch:"):
                    fields = line.split()
                    if len(fields) >= 4 and fields[2] == "batch" and int(fields[3]) != batch:
                        return None
                    value = float(fields[1])
                elif line.startswith("traffic_note:"):
                    remark = line[len("traffic_note:"):].strip()
    except OSError:
        pass
    return remark if note else value


class Problem:
    """One workload resident on the GPU: packed copies, levels, labels, workspace."""


def prepare(name, args, torch, zipml, synth, dev):
    """Generates the workload on the device chunk by chunk, computes its levels and quantises it
    with the library.  The fp32 rows are kept only where a later call needs them."""
    factory = synth.WORKLOADS[name]
    n_full = args.rows or {"tiny": 4096, "dense8": 65536, "lowbit": 1048576, "tomo": 262144, "e2e": 524288}[name]
    kw = {}
    if args.dim:
        kw["d"] = args.dim
    if args.bits:
        kw["bits"] = args.bits
    w = synth.light(factory, n_full, **kw)
    if args.batch:
        w.batch = args.batch
    n, d, bits, B = w.n, w.d, w.bits, w.batch
    K = 1 << bits
    P = Problem()
    P.w, P.name = w, name
    t0 = time.perf_counter()
    n_cand = w.n_candidates if w.levels == "optimal" else 0
    P.ws = torch.zeros(zipml.workspace_bytes(n, d, bits, B, n_cand), dtype=torch.uint8, device=dev)
    P.lev = torch.zeros(d, K, dtype=torch.float32, device=dev)
    P.grid = torch.zeros(d, K, dtype=torch.int16, device=dev)
    P.lo = torch.zeros(d, dtype=torch.float32, device=dev)
    P.hi = torch.zeros(d, dtype=torch.float32, device=dev)
    P.p1 = torch.zeros(zipml.packed_bytes(n, d, bits), dtype=torch.uint8, device=dev)
    P.p2 = torch.zeros_like(P.p1)
    P.b = torch.zeros(n, dtype=torch.float32, device=dev)
    # levels that need the data (per-column ranges, level search) keep the fp32 rows resident;
    # fixed ranges are quantised chunk by chunk as the rows are generated
    keep = w.range_mode != "fixed" or w.levels == "optimal" or name == "dense8"
    P.A = torch.empty(n, d, dtype=torch.float32, device=dev) if keep else None
    P.A_head = P.b_head = None
    fixed = w.range_mode == "fixed" and w.levels == "uniform"
    if fixed:
        P.lo.fill_(w.lo)
        P.hi.fill_(w.hi)
        zipml.levels(None, n, d, d, bits, zipml.UNIFORM, zipml.RANGE_GIVEN, 0, P.lo, P.hi, P.lev, P.grid, P.ws)
    chunk = 8192 if d <= 4096 else 4096
    head_rows = min(n, 4096)
    for r0, A, b in synth.device_chunks(w, dev, chunk):
        rows = A.shape[0]
        P.b[r0:r0 + rows] = b
        if r0 == 0:
            P.A_head, P.b_head = A[:head_rows].cpu().numpy(), b[:head_rows].cpu().numpy()
        if keep:
            P.A[r0:r0 + rows] = A
        if fixed:
            zipml.quantize(A, rows, d, d, r0, n, P.lev, bits, 0, 0, P.p1, P.p2)
        del A, b
    torch.cuda.synchronize()
    P.gen_s = time.perf_counter() - t0
    P.grid_lo = P.grid_step = 0.0
    P.grid_max = 0
    t0 = time.perf_counter()
    if not fixed:
        if w.levels == "optimal":
            # per-feature variance-optimal levels on the common grid [lo, hi] / n_candidates
            P.lo.fill_(w.lo)
            P.hi.fill_(w.hi)
            zipml.levels(P.A, n, d, d, bits, zipml.OPTIMAL, zipml.RANGE_GIVEN, w.n_candidates, P.lo, P.hi,
                         P.lev, P.grid, P.ws)
            P.grid_lo, P.grid_step, P.grid_max = w.lo, (w.hi - w.lo) / w.n_candidates, w.n_candidates
        else:
            flags = zipml.SYMMETRIC if w.range_mode == "symmetric" else 0
            zipml.levels(P.A, n, d, d, bits, zipml.UNIFORM, flags, 0, P.lo, P.hi, P.lev, P.grid, P.ws)
        zipml.quantize(P.A, n, d, d, 0, n, P.lev, bits, 0, 0, P.p1, P.p2)
    elif w.model_bits:
        P.grid_lo, P.grid_step, P.grid_max = w.lo, (w.hi - w.lo) / (K - 1), K - 1
    torch.cuda.synchronize()
    P.levels_quantize_s = time.perf_counter() - t0
    if keep and name != "dense8":
        P.A = None          # only the dense workload times the fp32 entry points afterwards
    return P


def run_epochs(P, args, torch, zipml):
    """Warm-up epochs, then K timed epochs with a HIP event after each; returns the figures."""
    w = P.w
    n, d, bits, B = w.n, w.d, w.bits, w.batch
    x = torch.zeros(d, dtype=torch.float32, device=P.b.device)
    kw = {}
    if w.model_bits:
        kw = dict(grid_idx=P.grid, grid_lo=P.grid_lo, grid_step=P.grid_step, grid_max=P.grid_max,
                  grad_bits=w.grad_bits, model_bits=w.model_bits)
    epoch_no = [0]

    def epoch():
        zipml.sgd_epoch(P.p1, P.p2, P.lev, P.b, n, d, bits, x, B, w.lr, P.ws, seed=0, epoch=epoch_no[0], **kw)
        epoch_no[0] += 1

    for _ in range(args.warmup):
        epoch()
    st = zipml.sgd_status(P.ws)
    assert st == 0, zipml.strerror(st)
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    t0 = time.perf_counter()
    ev[0].record()
    for k in range(args.steps):
        epoch()
        ev[k + 1].record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    st = zipml.sgd_status(P.ws)
    assert st == 0, zipml.strerror(st)
    per_epoch_ms = [ev[k].elapsed_time(ev[k + 1]) for k in range(args.steps)]
    kern_ms = sum(per_epoch_ms) / len(per_epoch_ms)
    alg_bytes = n * (2 * d * bits / 8 + 4)            # both packed copies once + labels
    gbps = alg_bytes / (kern_ms * 1e-3) / 1e9
    loss = zipml.loss(P.b, x, n, d, P.ws, packed=P.p2, copy=2, levels_t=P.lev, bits=bits)
    mode = (f"{w.model_bits}-bit model and {w.grad_bits}-bit gradient" if w.model_bits else "fp32 model")
    lv = (f"{bits}-bit variance-optimal levels from {w.n_candidates} candidates" if w.levels == "optimal"
          else f"{bits}-bit uniform levels" + (" on per-column ranges" if w.range_mode != "fixed" else ""))
    P.x = x
    return {
        "name": P.name,
        "workload": f"{P.name}: n={n}, d={d}, {lv}, batch {B}, lr {w.lr}, {mode}",
        "n": n, "d": d, "bits": bits, "batch": B,
        "minibatch_steps_per_epoch": n // B,
        "packed_bytes_per_epoch": int(alg_bytes),
        "ms_per_epoch": kern_ms,
        "ms_per_epoch_wall": wall / args.steps * 1e3,
        "us_per_minibatch_step": kern_ms * 1e3 / (n // B),
        "samples_per_s": args.steps * n / wall,
        "packed_GBps": gbps,
        "frac_hbm_peak": gbps / HBM_PEAK_GBS,
        "loss_on_copy2_after_run": loss,
        "generate_s": P.gen_s, "levels_and_quantize_s": P.levels_quantize_s,
    }


def cpu_baseline(P, seconds, threads):
    """The oracle's epoch loop, as it stands, on the first rows of the workload: one thread, and
    (plain estimator only) the rows of a minibatch over all host threads."""
    import numpy as np
    import oracle
    w = P.w
    B = w.batch
    n_s = min(P.A_head.shape[0], max(B, (4096 if w.d <= 4096 else 1024)))
    n_s -= n_s % B
    A, b = P.A_head[:n_s], P.b_head[:n_s]
    L = P.lev.cpu().numpy()
    c1, c2 = oracle.quantize(A, L, w.bits, 0, 0)
    x = np.zeros(w.d, np.float32)
    G = P.grid.cpu().numpy().view(np.uint16)

    def one(x, ep):
        if w.model_bits:
            return oracle.sgd_epoch_e2e(c1, c2, L, G, P.grid_lo, P.grid_step, b, w.bits, x, B, w.lr,
                                        w.grad_bits, w.model_bits, 0, ep)
        return oracle.sgd_epoch(c1, c2, L, b, w.bits, x, B, w.lr)

    t0 = time.perf_counter()
    passes = 0
    while True:
        x = one(x, passes)
        passes += 1
        el = time.perf_counter() - t0
        if el >= seconds:
            break
    what = f"first {n_s} of {w.n} samples of {P.name} (d={w.d}, batch {B})"
    single = {"value": passes * n_s / el, "unit": "samples/s", "cores": 1, "kind": "oracle",
              "sample": f"{what}, {passes} passes of the oracle epoch loop in {el:.1f} s, one thread"}
    many = None
    if not w.model_bits:
        x = np.zeros(w.d, np.float32)
        t0 = time.perf_counter()
        passes, used = 0, 1
        while True:
            x, used = oracle.sgd_epoch_threads(c1, c2, L, b, w.bits, x, B, w.lr, threads)
            passes += 1
            el = time.perf_counter() - t0
            if el >= seconds:
                break
        many = {"value": passes * n_s / el, "unit": "samples/s", "cores": used, "kind": "oracle",
                "sample": f"{what}, {passes} passes in {el:.1f} s, rows of each minibatch over {used} "
                          f"threads, partial gradients added in thread order"}
    return single, many


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU only (no multi-GPU path exists); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)
    import numpy as np
    import torch

    from paper_1611_05402_amd import synth, zipml

    assert torch.cuda.is_available(), "bench.py needs a GPU"
    zipml.lib()   # fails loudly if the HIP library is missing
    if args.no_matrix_cores:
        zipml.debug_set(zipml.KNOB_NO_MATRIX_CORES, 1)
    dev = "cuda:0"
    torch.cuda.set_device(0)
    names = ALL if args.workload == "all" else [args.workload]
    headline = HEADLINE if HEADLINE in names else names[0]

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

    # ---- what a plain streaming read reaches on this machine: back-to-back launches of the library's
    # streaming kernel over 4 GiB, timed by events only (no host synchronisation in between)
    probe = torch.empty(4 << 30, dtype=torch.uint8, device=dev)
    probe.view(torch.int32).random_(0, 1 << 30)
    sink = torch.zeros(64, dtype=torch.int32, device=dev)
    read_ms = timed(lambda: zipml.debug_stream(probe, sink), reps=8)
    read_ceiling = probe.numel() / (read_ms * 1e-3) / 1e9
    if args.copy_calibration:
        # launches of known traffic for the counter scale: 1 GiB read; 1 GiB read + 1 GiB written
        dst = torch.empty(1 << 30, dtype=torch.uint8, device=dev)
        for _ in range(3):
            zipml.debug_stream(probe, sink, nbytes=1 << 30)
            zipml.debug_stream(probe, sink, dst=dst, nbytes=1 << 30)
        torch.cuda.synchronize()
        del dst
    del probe

    results, extras, baseline = [], {}, None
    threads = min(os.cpu_count() or 1, int(os.environ.get("OMP_NUM_THREADS", "16") or 16))
    for name in names:
        P = prepare(name, args, torch, zipml, synth, dev)
        res = run_epochs(P, args, torch, zipml)
        res["frac_of_measured_stream_read"] = res["packed_GBps"] / read_ceiling
        res["hbm_traffic_bytes_per_epoch"] = recorded_traffic(name, P.w.batch)
        res["hbm_traffic_note"] = recorded_traffic(name, P.w.batch, note=True)
        results.append(res)
        if name == headline and not args.no_cpu_baseline:
            baseline = cpu_baseline(P, args.cpu_seconds, threads)
        if name == "dense8" and not args.no_extras:
            extras.update(dense_extras(P, args, torch, zipml, timed))
        if name == headline and name != "dense8" and not args.no_extras and not args.batch:
            extras["batch_sweep_headline"] = headline_sweep(P, torch, zipml, timed)
        del P
        torch.cuda.empty_cache()

    head = [r for r in results if r["name"] == headline][0]
    model_dtype = ("i32 dot products on 8-bit model codes, f64 gradient sums, f32 master model"
                   if headline == "e2e" else "f32 (model, residuals; sums taken exactly on i8 digits)")
    out = {
        "metric": "double-sampled SGD samples/sec (packed-data GB/s and % of HBM peak in roofline)",
        "value": head["samples_per_s"],
        "unit": "samples/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": head["ms_per_epoch_wall"],
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": model_dtype,
        "data": "synthetic",
        "config": {"workload": head["workload"],
                   "minibatch_steps_per_epoch": head["minibatch_steps_per_epoch"],
                   "packed_bytes_per_epoch": head["packed_bytes_per_epoch"]},
        "packed_GBps": head["packed_GBps"],
        "roofline": {"bound": "hbm", "achieved": head["packed_GBps"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": head["frac_hbm_peak"], "traffic": head["hbm_traffic_bytes_per_epoch"],
                     "traffic_note": head.get("hbm_traffic_note"),
                     "kernel": f"k_sgd<{head['bits']}> (persistent epoch kernel, one launch per epoch)",
                     "kernel_ms": head["ms_per_epoch"],
                     "us_per_minibatch_step": head["us_per_minibatch_step"],
                     "measured_stream_read_GBps": read_ceiling,
                     "frac_of_measured_stream_read": head["packed_GBps"] / read_ceiling},
        "configs": results,
        "paper_context": "paper reports ratios only: up to 6.5x over a 32-bit FPGA implementation "
                         "or 10-core Hogwild! (other hardware; not a target)",
    }
    out.update(extras)
    if baseline:
        out["cpu_baseline"] = baseline[0]
        if baseline[1]:
            out["cpu_baseline_all_cores"] = baseline[1]
    print(json.dumps(out), flush=True)
    # release everything and drain the device before the interpreter starts tearing modules down
    del results, out
    torch.cuda.synchronize()


def headline_sweep(P, torch, zipml, timed):
    """The headline workload's epoch at larger minibatches (not part of `value`): where the packed-data
    rate approaches the HBM peak on this shape."""
    w = P.w
    n, d, bits = w.n, w.d, w.bits
    dev = P.b.device
    out = []
    for batch in (4 * w.batch, 16 * w.batch, 64 * w.batch, n):
        if batch > n or n % batch:
            continue
        x = torch.zeros(d, dtype=torch.float32, device=dev)
        ws = torch.zeros(zipml.workspace_bytes(n, d, bits, batch), dtype=torch.uint8, device=dev)
        try:
            ms = timed(lambda: zipml.sgd_epoch(P.p1, P.p2, P.lev, P.b, n, d, bits, x, batch, w.lr, ws), 3)
        except zipml.ZipmlError as e:
            out.append({"batch": batch, "error": str(e)})
            continue
        st = zipml.sgd_status(ws)
        gbps = n * (2 * d * bits / 8 + 4) / (ms * 1e-3) / 1e9
        out.append({"batch": batch, "status": zipml.strerror(st) if st else "ok", "ms_per_epoch": ms,
                    "us_per_step": ms * 1e3 / (n // batch), "GBps": gbps, "frac_hbm_peak": gbps / HBM_PEAK_GBS})
        del ws
    return out


def dense_extras(P, args, torch, zipml, timed):
    """On the dense 8-bit workload: the other entry points, and the same epoch at larger
    minibatches (not part of `value`)."""
    w = P.w
    n, d, bits, B = w.n, w.d, w.bits, w.batch
    dev = P.b.device
    x = P.x
    other = {}
    other["levels_uniform"] = timed(lambda: zipml.levels(P.A, n, d, d, bits, zipml.UNIFORM, zipml.RANGE_GIVEN, 0,
                                                         P.lo, P.hi, P.lev, None, P.ws))
    q1, q2 = torch.zeros_like(P.p1), torch.zeros_like(P.p2)
    other["quantize"] = timed(lambda: zipml.quantize(P.A, n, d, d, 0, n, P.lev, bits, 0, 0, q1, q2))
    del q1, q2
    other["loss_fp32"] = timed(lambda: zipml.loss(P.b, x, n, d, P.ws, A=P.A, lda=d))
    other["loss_packed"] = timed(lambda: zipml.loss(P.b, x, n, d, P.ws, packed=P.p2, copy=2, levels_t=P.lev, bits=bits))
    try:
        lo2, hi2 = torch.zeros_like(P.lo), torch.zeros_like(P.hi)
        lev3 = torch.zeros(d, 8, dtype=torch.float32, device=dev)
        ws3 = torch.zeros(zipml.workspace_bytes(n, d, 3, B, 1024), dtype=torch.uint8, device=dev)
        lev2 = torch.zeros_like(P.lev)
        other["levels_with_range_scan"] = timed(
            lambda: zipml.levels(P.A, n, d, d, bits, zipml.UNIFORM, 0, 0, lo2, hi2, lev2, None, ws3))
        other["levels_optimal_3bit_1024bins"] = timed(
            lambda: zipml.levels(P.A, n, d, d, 3, zipml.OPTIMAL, 0, 1024, lo2, hi2, lev3, None, ws3))
        other["levels_greedy_3bit_1024bins"] = timed(
            lambda: zipml.levels(P.A, n, d, d, 3, zipml.GREEDY, 0, 1024, lo2, hi2, lev3, None, ws3))
        del ws3, lev3
    except zipml.ZipmlError as e:
        other["error"] = str(e)

    sweep = []

    def sweep_point(nn, p1s, p2s, bs, batch, reps=5):
        xs = torch.zeros(d, dtype=torch.float32, device=dev)
        wss = torch.zeros(zipml.workspace_bytes(nn, d, bits, batch), dtype=torch.uint8, device=dev)
        try:
            ms = timed(lambda: zipml.sgd_epoch(p1s, p2s, P.lev, bs, nn, d, bits, xs, batch, w.lr, wss), reps)
        except zipml.ZipmlError as e:       # e.g. a shape whose large minibatches no kernel takes
            sweep.append({"n": nn, "batch": batch, "error": str(e)})
            return
        if zipml.sgd_status(wss) != 0:
            sweep.append({"n": nn, "batch": batch, "error": zipml.strerror(zipml.sgd_status(wss))})
            return
        nbytes = nn * (2 * d * bits / 8 + 4)
        sweep.append({"n": nn, "batch": batch, "ms_per_epoch": ms, "us_per_step": ms * 1e3 / (nn // batch),
                      "GBps": nbytes / (ms * 1e-3) / 1e9, "frac_hbm_peak": nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBS})

    if not args.batch:
        for mult in (4, 16):
            if n % (B * mult) == 0:
                sweep_point(n, P.p1, P.p2, P.b, B * mult)
        sweep_point(n, P.p1, P.p2, P.b, n)
        n8 = 8 * n
        q1 = torch.randint(0, 256, (zipml.packed_bytes(n8, d, bits),), dtype=torch.uint8, device=dev)
        q2 = torch.randint(0, 256, (zipml.packed_bytes(n8, d, bits),), dtype=torch.uint8, device=dev)
        sweep_point(n8, q1, q2, torch.randn(n8, device=dev), n8)
        del q1, q2
    # What a device-wide exchange costs: the same epoch with minibatches of 4 and 32 samples -- a
    # step then moves 16 or 128 KiB of codes, and what is left of it is one exchange of the partial
    # sums between the workgroups (an atomic add, a wait, a poll) plus the fixed work around it.
    exchange = []
    if not args.batch:
        for bsmall in (4, 32):
            xs = torch.zeros(d, dtype=torch.float32, device=dev)
            wss = torch.zeros(zipml.workspace_bytes(n, d, bits, bsmall), dtype=torch.uint8, device=dev)
            try:
                ms = timed(lambda: zipml.sgd_epoch(P.p1, P.p2, P.lev, P.b, n, d, bits, xs, bsmall, w.lr, wss), 3)
                st = zipml.sgd_status(wss)
                exchange.append({"batch": bsmall, "steps_per_epoch": n // bsmall, "us_per_step": ms * 1e3 / (n // bsmall),
                                 "status": zipml.strerror(st) if st else "ok"})
            except zipml.ZipmlError as e:
                exchange.append({"batch": bsmall, "error": str(e)})
            del wss
    compact = []
    if not args.batch and bits == 8 and 512 < d <= 2048 and n >= 16384:
        # Sec. 2.2, compact storage: the full-batch epoch reading base + 1 bit per copy (10 bits per
        # value) instead of the two packed copies (16 bits), on the same codes -- the real ones, and
        # the same rows eight times over (each feature group of an array is contiguous in the samples)
        p1s, p2s = torch.zeros_like(P.p1), torch.zeros_like(P.p2)
        zipml.quantize_swapped(P.A, n, d, d, 0, n, P.lev, bits, 0, 0, p1s, p2s)
        comp = torch.zeros(zipml.compact_bytes(n, d, bits), dtype=torch.uint8, device=dev)
        zipml.compact_encode(p2s, P.p2, n, d, bits, comp, P.ws)
        del p1s, p2s
        d32 = (d + 31) // 32
        for rep in (1, 8):
            nn = n * rep
            tile = lambda t: t.view(d32, -1).repeat(1, rep).reshape(-1) if rep > 1 else t
            nbase = zipml.packed_bytes(n, d, bits)      # the record is two planes: base levels, pairs of bit words
            q1, q2, bs = tile(P.p1), tile(P.p2), P.b.repeat(rep)
            qc = torch.cat([tile(comp[:nbase]), tile(comp[nbase:])])
            xs = torch.zeros(d, dtype=torch.float32, device=dev)
            xc = torch.zeros(d, dtype=torch.float32, device=dev)
            wss = torch.zeros(zipml.workspace_bytes(nn, d, bits, nn), dtype=torch.uint8, device=dev)
            try:
                ms_p = timed(lambda: zipml.sgd_epoch(q1, q2, P.lev, bs, nn, d, bits, xs, nn, w.lr, wss), 5)
                ms_c = timed(lambda: zipml.sgd_epoch_compact(qc, P.lev, bs, nn, d, bits, xc, nn, w.lr, wss), 5)
            except zipml.ZipmlError as e:
                compact.append({"n": nn, "batch": nn, "error": str(e)})
                continue
            st = zipml.sgd_status(wss)
            read_c = nn * (d32 * 32 * (bits + 2) / 8 + 4)
            compact.append({"n": nn, "batch": nn, "status": zipml.strerror(st) if st else "ok",
                            "ms_per_epoch_two_packed_copies": ms_p, "ms_per_epoch_compact_record": ms_c,
                            "speedup": ms_p / ms_c, "same_model_bits": bool(torch.equal(xs, xc)),
                            "compact_GBps": read_c / (ms_c * 1e-3) / 1e9,
                            "packed_equivalent_GBps": nn * (2 * d * bits / 8 + 4) / (ms_c * 1e-3) / 1e9})
            del q1, q2, qc, bs, wss
    # 2-bit codes at very large minibatches (random codes, evenly spaced levels, d=4096): the
    # sample-owner kernel with its dot pass on the 4-bit floating-point matrix instruction against
    # the integer kernel, at 1 and 4 GiB of codes per step
    two_bit = []
    if not args.batch:
        d2 = 4096
        lev2 = torch.zeros(d2, 4, dtype=torch.float32, device=dev)
        lo2 = torch.full((d2,), -1.0, dtype=torch.float32, device=dev)
        hi2 = torch.full((d2,), 1.0, dtype=torch.float32, device=dev)
        zipml.levels(None, 64, d2, d2, 2, zipml.UNIFORM, zipml.RANGE_GIVEN, 0, lo2, hi2, lev2, None, P.ws)
        for nn in (524288, 2097152):
            q1 = torch.randint(0, 256, (zipml.packed_bytes(nn, d2, 2),), dtype=torch.uint8, device=dev)
            q2 = torch.randint(0, 256, (zipml.packed_bytes(nn, d2, 2),), dtype=torch.uint8, device=dev)
            bs = torch.randn(nn, device=dev)
            wss = torch.zeros(zipml.workspace_bytes(nn, d2, 2, nn), dtype=torch.uint8, device=dev)
            row = {"n": nn, "d": d2, "batch": nn}
            try:
                for tag, kn in (("integer_kernel", 2), ("fp4_dot_pass", -1)):
                    zipml.debug_set(zipml.KNOB_ROWS_ITEM_BLOCKS, kn)
                    xs = torch.zeros(d2, dtype=torch.float32, device=dev)
                    ms = timed(lambda: zipml.sgd_epoch(q1, q2, lev2, bs, nn, d2, 2, xs, nn, 1e-6, wss), 5)
                    gb = nn * (2 * d2 * 2 / 8 + 4) / (ms * 1e-3) / 1e9
                    row[tag] = {"ms_per_epoch": ms, "GBps": gb, "frac_hbm_peak": gb / HBM_PEAK_GBS,
                                "status": zipml.strerror(zipml.sgd_status(wss)) if zipml.sgd_status(wss) else "ok"}
            except zipml.ZipmlError as e:
                row["error"] = str(e)
            finally:
                zipml.debug_set(zipml.KNOB_ROWS_ITEM_BLOCKS, -1)
            two_bit.append(row)
            del q1, q2, bs, wss
    return {"other_ms": other, "batch_sweep": sweep, "step_with_next_to_no_data": exchange,
            "compact_record_epoch": compact, "two_bit_large_minibatch": two_bit}


if __name__ == "__main__":
    main()
