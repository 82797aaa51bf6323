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
    ap.add_argument("--batches-per-launch", type=int, default=0,
                    help="batches built by one launch (0 = auto: about 512 MB of traffic per launch)")
    ap.add_argument("--out-pairs", type=int, default=0,
                    help="output buffer sets rotated (0 = enough to exceed the 256 MB last-level cache)")
    ap.add_argument("--order", default="shuffle", choices=["shuffle", "sequential", "batch_shuffle"],
                    help="epoch order (the headline metric is the global shuffle)")
    ap.add_argument("--out-dtype", default="f32", choices=["f32", "bf16"],
                    help="output element type (the headline metric uses fp32 outputs)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--repeats", type=int, default=5,
                    help="further timed passes of the same steps, reported as median / max / min beside value")
    ap.add_argument("--cpu-batches", type=int, default=0, help="oracle batches on one core (0 = auto)")
    ap.add_argument("--roofline-launches", type=int, default=4096,
                    help="upper bound on back-to-back launches in the kernel-duration measurement")
    ap.add_argument("--copy-calibration", type=int, default=3,
                    help="plain device copies of one x buffer issued after the measurements: a kernel of "
                         "known traffic for scaling rocprofv3's FETCH_SIZE / WRITE_SIZE counters")
    return ap.parse_args()


def traffic_from_profiles(workload: str, batches_per_launch: int):
    """HBM bytes per launch measured with rocprofv3 --pmc (FETCH_SIZE / WRITE_SIZE, scaled by a
    copy kernel of known size); recorded in profiles/ after a counter run of this same launch
    shape, else null."""
    path = os.path.join(ROOT, "profiles", f"gather_{workload}_pmc.md")
    try:
        found = {}
        for line in open(path):
            for key in ("traffic_bytes_per_launch", "batches_per_launch"):
                if line.startswith(key + ":"):
                    found[key] = float(line.split(":", 1)[1].split()[0])
        if found.get("batches_per_launch", 1) == batches_per_launch:
            return found.get("traffic_bytes_per_launch")
    except OSError:
        pass
    return None


def cpu_baseline(w, series, mean, std, n_batches_1core: int, order: int = 0):
    """The oracle as it stands, on this host, on a bounded sample of the same workload."""
    import concurrent.futures as cf

    import numpy as np

    import oracle

    storage = oracle.F32 if w.storage == "f32" else oracle.BF16
    ser = series if storage == oracle.F32 else oracle.store_bf16(series)
    share = oracle.epoch_indices_ex(order, w.n_windows, 0, w.n_windows, w.B, w.seed, w.epochs[0], w.rank, w.world)
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
              "hold the full series and build its own contiguous share of the same shuffle, with no exchange step)",
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
    # the paper's own rule (Algorithm 1: scalar statistics over the first 70 % of the windows), timed
    # as the on-device preprocessing figure; its result is not used for the batches below
    t0 = time.perf_counter()
    ctx.load_series_ex(host, w.P, w.Q, w.B, storage, stats_rule=pgti.PGTI_STATS_ALG1_TRAIN, train_fraction=0.70)
    t_load_alg1 = time.perf_counter() - t0
    alg1_mean, alg1_std = ctx.get_stats()
    # Channel 0 keeps the statistics the device computed; the time-of-day channel passes through
    # unchanged.  Statistics are fixed by the load call, so load once more with the final values.
    mean[1:], std[1:] = 0.0, 1.0
    t0 = time.perf_counter()
    ctx.load_series(host, w.P, w.Q, w.B, storage, mean, std)
    t_load2 = time.perf_counter() - t0

    # ---- launch shape: k batches per launch (pgti_build_batches) -----------------------------------
    order = {"shuffle": pgti.PGTI_ORDER_SHUFFLE, "sequential": pgti.PGTI_ORDER_SEQUENTIAL,
             "batch_shuffle": pgti.PGTI_ORDER_BATCH_SHUFFLE}[args.order]

    def gen_indices(epoch: int) -> int:
        return ctx.epoch_indices_ex(order, seed=w.seed, epoch=epoch, rank=w.rank, world=w.world)

    n_share = gen_indices(w.epochs[0])
    nb = ctx.num_batches()
    out_elem = 4 if args.out_dtype == "f32" else 2
    out_torch = torch.float32 if args.out_dtype == "f32" else torch.bfloat16
    bps = w.bytes_per_snapshot(out_elem)                  # algorithmic bytes per snapshot
    batch_bytes = w.B * bps                               # algorithmic read + write of a full batch
    out_bytes = w.B * (w.P + w.Q) * w.N * w.F * out_elem  # x + y of one batch
    build_raw = ctx.build_batches_raw if args.out_dtype == "f32" else ctx.build_batches_bf16_raw
    k = args.batches_per_launch or max(1, min(nb, -(-(512 << 20) // batch_bytes)))
    if not args.batches_per_launch and args.order != "shuffle" and w.series_bytes_f32 > (256 << 20):
        k = 1  # consecutive starts, write-bound row-centric kernel: measured fastest at one batch per launch
    k = min(k, nb, 65535 // w.B)

    # ---- output buffers: rotate enough sets that writes cannot sit in the 256 MB last-level cache --
    sets = args.out_pairs or min(64, max(3, -(-(768 << 20) // (k * out_bytes))))
    xs = [torch.empty((k, w.B, w.P, w.N, w.F), dtype=out_torch, device="cuda") for _ in range(sets)]
    ys = [torch.empty((k, w.B, w.Q, w.N, w.F), dtype=out_torch, device="cuda") for _ in range(sets)]
    xp, yp = [t.data_ptr() for t in xs], [t.data_ptr() for t in ys]
    stream = torch.cuda.current_stream()
    sh = stream.cuda_stream
    steps = args.steps or nb * len(w.epochs)

    x_batch_bytes, y_batch_bytes = w.B * w.P * w.N * w.F * out_elem, w.B * w.Q * w.N * w.F * out_elem

    def out_ptrs(launch: int, per_launch: int):
        """Rotates launches over every slot of every set (per_launch consecutive slots each)."""
        per_set = max(1, k // per_launch)
        idx = launch % (sets * per_set)
        st, slot = divmod(idx, per_set)
        return xp[st] + slot * per_launch * x_batch_bytes, yp[st] + slot * per_launch * y_batch_bytes

    def run(n_steps: int, per_launch: int) -> int:
        """Enqueues n_steps batches (per_launch of them per launch), generating the indices at each
        epoch boundary.  Returns the number of snapshots built."""
        snaps, i, launch = 0, 0, 0
        while i < n_steps:
            e, b = divmod(i, nb)
            if b == 0:
                gen_indices(w.epochs[0] + e)  # consecutive epochs
            kk = min(per_launch, nb - b, n_steps - i)
            rc = build_raw(b, kk, *out_ptrs(launch, per_launch), sh)
            if rc < 0:
                raise RuntimeError(pgti.last_error())
            snaps += rc
            i += kk
            launch += 1
        return snaps

    def timed(per_launch: int):
        run(args.warmup, per_launch)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        n = run(steps, per_launch)
        torch.cuda.synchronize()
        return n, time.perf_counter() - t0

    def kernel_rate(per_launch: int):
        """Average duration of back-to-back launches of per_launch FULL batches, from HIP events on
        the launch stream; only gather launches sit between the two events."""
        gen_indices(w.epochs[0])
        ctx.get_indices()  # waits for the sort
        full_batches = max(1, nb - 1 if n_share % w.B else nb)
        per_launch = min(per_launch, full_batches)
        per_epoch = max(1, full_batches // per_launch)
        per_epoch = min(per_epoch, args.roofline_launches)
        reps = max(1, min(64, args.roofline_launches // per_epoch))
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        for l in range(min(per_epoch, 16)):
            build_raw(l * per_launch, per_launch, *out_ptrs(l, per_launch), sh)
        torch.cuda.synchronize()
        ev0.record(stream)
        n = 0
        for _ in range(reps):
            for l in range(per_epoch):
                build_raw(l * per_launch, per_launch, *out_ptrs(n, per_launch), sh)
                n += 1
        ev1.record(stream)
        torch.cuda.synchronize()
        avg_s = ev0.elapsed_time(ev1) * 1e-3 / n
        nbytes = per_launch * min(w.B, n_share) * bps
        return {"launches": n, "avg_launch_us": avg_s * 1e6, "algorithmic_bytes_per_launch": nbytes,
                "achieved": nbytes / avg_s / 1e9, "batches_per_launch": per_launch}

    # ---- warm-up, timed region, kernel rate: k batches per launch, then one batch per launch -------
    snaps, elapsed = timed(k)
    repeat_values = []
    for _ in range(max(0, args.repeats)):
        n_r, t_r = timed(k)
        repeat_values.append(n_r / t_r)
    rate_k = kernel_rate(k)
    snaps1, elapsed1 = timed(1) if k > 1 else (snaps, elapsed)
    rate_1 = kernel_rate(1) if k > 1 else rate_k

    # ---- calibration copies for the counter runs (known size: reads and writes one x buffer) ----
    for _ in range(args.copy_calibration):
        xs[1][0].copy_(xs[0][0])
    torch.cuda.synchronize()

    # ---- index generation alone ----------------------------------------------------------------
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for e in range(10):
        gen_indices(100 + e)
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
        "dtype": "f32",  # arithmetic type: subtraction and division are binary32 whatever is stored or emitted
        "data": "synthetic",
        "config": {"workload": w.name, "T": w.T, "N": w.N, "F": w.F, "P": w.P, "Q": w.Q, "B": w.B,
                   "storage": w.storage, "world": w.world, "rank": w.rank, "seed": w.seed,
                   "epochs": list(w.epochs), "batches_per_epoch": nb, "snapshots_timed": snaps,
                   "batches_per_launch": k, "out_buffer_sets": sets, "order": args.order,
                   "out_dtype": args.out_dtype, "algorithmic_bytes_per_snapshot": bps},
        "gb_per_s": snaps * bps / elapsed / 1e9,
        "pct_of_hbm_peak": snaps * bps / elapsed / 1e9 / HBM_PEAK_GBS * 100,
        "roofline": {
            "bound": "hbm", "achieved": rate_k["achieved"], "peak": HBM_PEAK_GBS, "unit": "GB/s",
            "frac": rate_k["achieved"] / HBM_PEAK_GBS, "traffic": traffic_from_profiles(w.name, k),
            "kernel": "gather_quads_kernel", **{kk: v for kk, v in rate_k.items() if kk != "achieved"},
        },
        # bytes a launch must move if every distinct source row is fetched once: equals the algorithmic
        # bytes for the global shuffle (no shared rows), far fewer reads for consecutive starts
        "unique_bytes_ideal_per_launch": (
            rate_k["algorithmic_bytes_per_launch"] if args.order == "shuffle" else
            (rate_k["batches_per_launch"] * w.B + w.P + w.Q - 1) * w.N * w.F * (4 if w.storage == "f32" else 2)
            + rate_k["batches_per_launch"] * w.B * (w.P + w.Q) * w.N * w.F * out_elem),
        "one_batch_per_launch": {
            "value": snaps1 / elapsed1, "unit": "snapshots/s", "ms_per_step": elapsed1 / steps * 1e3,
            "gb_per_s": snaps1 * bps / elapsed1 / 1e9,
            "roofline": {"achieved": rate_1["achieved"], "frac": rate_1["achieved"] / HBM_PEAK_GBS,
                         **{kk: v for kk, v in rate_1.items() if kk != "achieved"}},
        },
        # the same K steps timed again (each pass with its own warm-up and synchronisation): run-to-run spread
        "repeats": {"count": len(repeat_values), "unit": "snapshots/s",
                    "median": float(sorted(repeat_values)[len(repeat_values) // 2]) if repeat_values else None,
                    "min": min(repeat_values) if repeat_values else None,
                    "max": max(repeat_values) if repeat_values else None},
        "epoch_indices_ms": t_idx * 1e3,
        "copy_calibration": {"count": args.copy_calibration, "bytes_read": xs[0][0].numel() * xs[0][0].element_size(),
                             "bytes_written": xs[0][0].numel() * xs[0][0].element_size()},
        "setup": {"generate_s": t_gen, "load_with_device_stats_s": t_load, "load_s": t_load2,
                  "load_with_alg1_train_stats_s": t_load_alg1,
                  "alg1_train_mean_std": [float(alg1_mean[0]), float(alg1_std[0])],
                  "series_bytes": w.series_bytes_f32, "load_gb_per_s": w.series_bytes_f32 / t_load2 / 1e9},
    }
    ctx.destroy()
    del xs, ys
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, series, mean, std, args.cpu_batches, order)
    print(json.dumps(result))


if __name__ == "__main__":
    main()
