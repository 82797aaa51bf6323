#!/usr/bin/env python3
"""Throughput of index-batched snapshot construction on one MI355X.

A "step" is one pass of the hot path over one batch: the fused gather+standardise launch
(pgti_build_batch); at every epoch boundary inside the timed region the epoch's shuffled index
list is generated first (pgti_epoch_indices), so the timed region holds all per-epoch and
per-batch work.  The resident series is loaded before timing starts (it is loaded once per run).

Prints ONE JSON line: whole-job snapshots/s, the roofline of the dominant kernel (measured live
with HIP events on the launch stream) and the CPU oracle timed on this host as a baseline.
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

HBM_PEAK_GBS = 8000.0  # MI355X HBM3E published peak


def parse_args():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=0, help="batches to time (0 = one full epoch)")
    ap.add_argument("--warmup", type=int, default=64)
    ap.add_argument("--workload", default="statewide")
    ap.add_argument("--out-pairs", type=int, default=0,
                    help="output buffer pairs rotated (0 = enough to exceed the 256 MB last-level cache)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--cpu-batches", type=int, default=0, help="oracle batches on one core (0 = auto)")
    ap.add_argument("--roofline-launches", type=int, default=4096,
                    help="upper bound on back-to-back launches in the kernel-duration measurement")
    ap.add_argument("--copy-calibration", type=int, default=3,
                    help="plain device copies of one x buffer issued after the measurements: a kernel of "
                         "known traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def traffic_from_profiles(workload: str):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, scaled by a
    copy kernel of known size); recorded in profiles/ by hand after a counter run, else null."""
    path = os.path.join(ROOT, "profiles", f"gather_{workload}_pmc.md")
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch:"):
                return float(line.split(":", 1)[1].split()[0])
    except OSError:
        pass
    return None


def cpu_baseline(w, series, mean, std, n_batches_1core: int):
    """The oracle as it stands, on this host, on a bounded sample of the same workload."""
    import concurrent.futures as cf

    import numpy as np

    import oracle

    storage = oracle.F32 if w.storage == "f32" else oracle.BF16
    ser = series if storage == oracle.F32 else oracle.store_bf16(series)
    share = oracle.epoch_indices(w.seed, w.epochs[0], w.rank, w.world, w.n_windows)
    nb = -(-len(share) // w.B)
    per_batch = lambda b: oracle.build_batch(ser, storage, w.P, w.Q, mean, std, share[b * w.B:(b + 1) * w.B])
    per_batch(0)  # touch code and pages once
    if n_batches_1core <= 0:
        t0 = time.perf_counter()
        per_batch(1 % nb)
        one = time.perf_counter() - t0
        n_batches_1core = max(4, min(nb, int(12.0 / max(one, 1e-6))))
    picks = [int(i * nb / n_batches_1core) for i in range(n_batches_1core)]
    snaps = sum(min(w.B, len(share) - b * w.B) for b in picks)
    t0 = time.perf_counter()
    for b in picks:
        per_batch(b)
    t1 = time.perf_counter() - t0
    # the same loop spread over the host's cores (ctypes releases the GIL around the C call)
    cores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    cores = min(cores, int(os.environ.get("OMP_NUM_THREADS", cores)) or cores)
    picks_all = [int(i * nb / (cores * 6)) for i in range(cores * 6)] if nb >= cores * 6 else list(range(nb))
    snaps_all = sum(min(w.B, len(share) - b * w.B) for b in picks_all)
    t0 = time.perf_counter()
    with cf.ThreadPoolExecutor(max_workers=cores) as ex:
        list(ex.map(per_batch, picks_all))
    tall = time.perf_counter() - t0
    bps = w.bytes_per_snapshot()
    return {
        "value": snaps / t1, "unit": "snapshots/s", "cores": 1, "kind": "oracle",
        "sample": f"{len(picks)} of {nb} batches of epoch {w.epochs[0]} ({snaps} snapshots), evenly spaced, "
                  f"single thread, {t1:.1f} s",
        "gb_per_s": snaps * bps / t1 / 1e9,
        "all_cores": {"value": snaps_all / tall, "unit": "snapshots/s", "cores": cores,
                      "gb_per_s": snaps_all * bps / tall / 1e9,
                      "sample": f"{len(picks_all)} batches over a {cores}-thread pool, {tall:.1f} s"},
    }


def main():
    args = parse_args()
    if args.gpus != 1:
        print(f"bench.py: this build runs on one GPU; --gpus {args.gpus} is not supported (every rank would "
              "hold the full series and build its own contiguous share of the same shuffle; see DESIGN.md)",
              file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    from paper_2507_11683_amd import pgti, workloads

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    w = workloads.WORKLOADS[args.workload]
    storage = pgti.PGTI_F32 if w.storage == "f32" else pgti.PGTI_BF16
    torch.cuda.set_device(0)

    # ---- input: generated straight into pinned host memory, loaded once ----------------------
    t0 = time.perf_counter()
    host = torch.empty((w.T, w.N, w.F), dtype=torch.float32, pin_memory=True)
    series = host.numpy()
    workloads.make_series(w, out=series)
    t_gen = time.perf_counter() - t0

    ctx = pgti.Context(0)
    t0 = time.perf_counter()
    ctx.load_series(host, w.P, w.Q, w.B, storage, None, None)  # statistics computed on the device
    t_load = time.perf_counter() - t0
    mean, std = ctx.get_stats()
    # Channel 0 keeps the statistics the device computed; the time-of-day channel passes through
    # unchanged.  Statistics are fixed by the load call, so load once more with the final values.
    mean[1:], std[1:] = 0.0, 1.0
    t0 = time.perf_counter()
    ctx.load_series(host, w.P, w.Q, w.B, storage, mean, std)
    t_load2 = time.perf_counter() - t0

    # ---- output buffers: rotate enough pairs that writes cannot sit in the last-level cache ----
    out_bytes = w.B * (w.P + w.Q) * w.N * w.F * 4
    pairs = args.out_pairs or max(4, -(-(512 << 20) // out_bytes))
    pairs = min(pairs, 256)
    xs = [torch.empty((w.B, w.P, w.N, w.F), dtype=torch.float32, device="cuda") for _ in range(pairs)]
    ys = [torch.empty((w.B, w.Q, w.N, w.F), dtype=torch.float32, device="cuda") for _ in range(pairs)]
    xp, yp = [t.data_ptr() for t in xs], [t.data_ptr() for t in ys]
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream

    n_share = ctx.epoch_indices(w.seed, w.epochs[0], w.rank, w.world)
    nb = ctx.num_batches()
    steps = args.steps or nb * len(w.epochs)

    def run(n_steps: int, first_step: int = 0) -> int:
        """Enqueues n_steps batches, generating indices at each epoch boundary.  Returns snapshots."""
        snaps = 0
        for i in range(first_step, first_step + n_steps):
            e, b = divmod(i, nb)
            if b == 0:
                ctx.epoch_indices(w.seed, w.epochs[0] + e, w.rank, w.world)  # consecutive epochs
            rc = ctx.build_batch_raw(b, xp[i % pairs], yp[i % pairs], sh)
            if rc < 0:
                raise RuntimeError(pgti.last_error())
            snaps += rc
        return snaps

    # ---- warm-up, then the timed region --------------------------------------------------------
    run(args.warmup)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    snaps = run(steps)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t0

    # ---- dominant kernel: batch builds back to back between two events on the launch stream -----
    ctx.epoch_indices(w.seed, w.epochs[0], w.rank, w.world)
    ctx.get_indices()  # waits for the sort so that only gather launches sit between the events
    full = nb - 1 if n_share % w.B else nb  # full batches only: every launch moves the same bytes
    full = max(1, min(full, args.roofline_launches))
    reps = max(1, min(8, args.roofline_launches // full))
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for b in range(min(full, 32)):
        ctx.build_batch_raw(b, xp[b % pairs], yp[b % pairs], sh)
    torch.cuda.synchronize()
    ev0.record(stream)
    k = 0
    for _ in range(reps):
        for b in range(full):
            ctx.build_batch_raw(b, xp[k % pairs], yp[k % pairs], sh)
            k += 1
    ev1.record(stream)
    torch.cuda.synchronize()
    launches = reps * full
    bsz = min(w.B, n_share)
    avg_launch_s = ev0.elapsed_time(ev1) * 1e-3 / launches
    bytes_per_launch = bsz * w.bytes_per_snapshot()
    achieved = bytes_per_launch / avg_launch_s / 1e9

    # ---- calibration copies for the counter runs (known size: reads and writes one x buffer) ----
    for _ in range(args.copy_calibration):
        xs[1].copy_(xs[0])
    torch.cuda.synchronize()

    # ---- index generation alone ----------------------------------------------------------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e in range(10):
        ctx.epoch_indices(w.seed, 100 + e, w.rank, w.world)
    ctx.get_indices()
    t_idx = (time.perf_counter() - t0) / 10

    result = {
        "metric": "snapshots/sec and achieved HBM GB/s (% of peak) for index-batched window build",
        "value": snaps / elapsed,
        "unit": "snapshots/s",
        "n_gpus": 1,
        "steps": steps,
        "warmup": args.warmup,
        "ms_per_step": elapsed / steps * 1e3,
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "T": w.T, "N": w.N, "F": w.F, "P": w.P, "Q": w.Q, "B": w.B,
                   "storage": w.storage, "world": w.world, "rank": w.rank, "seed": w.seed,
                   "epochs": list(w.epochs), "batches_per_epoch": nb, "snapshots_timed": snaps,
                   "out_buffer_pairs": pairs},
        "gb_per_s": snaps * w.bytes_per_snapshot() / elapsed / 1e9,
        "pct_of_hbm_peak": snaps * w.bytes_per_snapshot() / elapsed / 1e9 / HBM_PEAK_GBS * 100,
        "roofline": {
            "bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": achieved / HBM_PEAK_GBS, "traffic": traffic_from_profiles(w.name),
            "kernel": "gather_quads_kernel", "launches": launches,
            "avg_launch_us": avg_launch_s * 1e6, "algorithmic_bytes_per_launch": bytes_per_launch,
        },
        "epoch_indices_ms": t_idx * 1e3,
        "copy_calibration": {"count": args.copy_calibration, "bytes_read": xs[0].numel() * 4,
                             "bytes_written": xs[0].numel() * 4},
        "setup": {"generate_s": t_gen, "load_with_device_stats_s": t_load, "load_s": t_load2,
                  "series_bytes": w.series_bytes_f32, "load_gb_per_s": w.series_bytes_f32 / t_load2 / 1e9},
    }
    ctx.destroy()
    del xs, ys
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, series, mean, std, args.cpu_batches)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
