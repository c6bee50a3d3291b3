#!/usr/bin/env python3
"""Benchmark of the TT-embedding hot path on one MI355X.

A step is one whole pass of the path over one synthetic minibatch that is already resident in HBM:
tt_emb_forward (index split, sort, dedup, prefix products, rows) followed by
tt_emb_backward_update (gradient sums, core gradients, SGD).  The metric is rows per second,
duplicates counted.  The default workload is the 2.5M-node rank-32 table with a 200,000-row Zipf
batch; `--config K` picks another of the synthetic workloads (6-8: the paper's own table shapes).

Repeated SGD steps on the same random gradients feed back through the three cores and overflow
within a few steps at the workloads' learning rate (the hottest id occurs 24,000 times in the default
batch), so the timed steps use a learning rate of 1e-8: the kernels execute exactly the same
instructions, and the cores stay where they are for hundreds of steps.  `--restore` times the other
protocol instead: the workload's own learning rate, with the cores put back from a snapshot by one
device-side copy per step inside the timed region (extra work, counted against the rate).

The loop is the one a training loop would run: tt_emb_wait_backward(1) (host-side flow control, at
most two steps in flight; `--free-running` leaves it out), tt_emb_prepare for the batch two steps
ahead (its index work overlaps this step's arithmetic; `--no-prepare` leaves it out), forward,
backward_update.

Prints ONE JSON line.  `roofline` describes the longest launch on the caller's stream, timed with HIP events
on its own stream by the library's profiling hook in a separate, untimed leg (an empty event pair
is timed too and taken off); `cpu_baseline` is the CPU oracle (fp32 build, OpenMP) on the same batch.
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

HBM_PEAK = 8.0e12        # bytes/s, MI355X HBM3E
FP32_PEAK = 157.3e12     # flop/s, MI355X fp32 (vector with packed ops, or fp32 MFMA)

# Bytes beyond L2 per launch (fetched + written), from two `rocprofv3 --pmc` runs (FETCH_SIZE,
# WRITE_SIZE) scaled by the readings for a plain 256 MiB device copy in the same process; the table
# and the commands are in profiles/step_config3_hbm_traffic.md.  Only the default workload was
# measured; for anything else `traffic` is null.
MEASURED_TRAFFIC = {3: {"row_fwd": 43.1e6 + 102.4e6, "gsum": 85.4e6 + 4.8e6, "u_bwd": 107.4e6 + 32.8e6,
                        "prefix_fwd": 6.5e6 + 34.8e6, "sgd": 35.3e6 + 2.4e6}}


def kernel_work(slot: str, w, B: int, U: int, Q: int, touched_bytes: int, passes: int):
    """Algorithmic (HBM bytes, fp32 flops) one step asks of a kernel slot.  Bytes are the slot's
    share of the path's compulsory traffic, 8 + 8*D per row plus touched core slices twice;
    intermediates that are meant to stay in cache count for nothing."""
    d1, d2, d3 = w.d
    r1, r2 = w.r
    D = w.D
    F1 = 2 * d1 * r1 * d2 * r2          # one prefix product
    F2 = 2 * d1 * d2 * r2 * d3          # one row product
    table = {
        "sort_hist": (8 * B, 0),        # reads the int64 ids (first pass)
        "sort_scatter": (0, 0),
        "seg_count": (0, 0),
        "seg_write": (0, 0),
        "group": (0, 0),
        "prefix_fwd": (0, Q * F1),
        "row_fwd": (4 * D * B, U * F2),
        "gsum": (4 * D * B, (B - U) * D),
        "gsum_fix": (0, 0),
        "u_bwd": (0, U * F2),
        "dg3": (0, U * F2),
        "prefix_bwd": (0, 2 * Q * F1),
        "sgd": (2 * touched_bytes, 0),
    }
    return table.get(slot, (0, 0))


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", type=int, default=3, choices=[1, 2, 3, 4, 5, 6, 7, 8])
    ap.add_argument("--seed", type=int, default=None)
    ap.add_argument("--profile-steps", type=int, default=20)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--restore", action="store_true",
                    help="workload learning rate, cores restored from a snapshot every step")
    ap.add_argument("--lr", type=float, default=1e-8,
                    help="learning rate of the timed steps (ignored with --restore)")
    ap.add_argument("--calib-copy-mib", type=int, default=0,
                    help="also run one plain device copy of this many MiB (known traffic, to scale "
                         "a profiler's HBM counters)")
    ap.add_argument("--free-running", action="store_true",
                    help="let the host run arbitrarily far ahead of the device (no tt_emb_wait_backward)")
    ap.add_argument("--no-prepare", action="store_true",
                    help="do not overlap the index work of coming steps with this step's arithmetic")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (the paper's scheme for more, replicated cores and "
              "an all-reduce of the core gradients, is not built); run with --gpus 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    import workloads as wl
    from paper_2206_10581_amd import TTEmbedding

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 3
    dev = torch.device("cuda:0")
    w = wl.CONFIGS[args.config]
    seed = args.config if args.seed is None else args.seed
    B, D = w.batch, w.D
    cores_np = wl.make_cores(w, seed)
    ids_np = wl.make_ids(w, seed)
    grad_np = wl.make_grads(w, seed)
    struct = wl.batch_structure(w, ids_np)

    # cores live in one flat buffer so that the per-step restore is a single device copy
    sizes = [c.size for c in cores_np]
    offs = [0]
    for s in sizes:
        offs.append(offs[-1] + ((s + 63) // 64) * 64)
    flat = torch.zeros(offs[-1], dtype=torch.float32, device=dev)
    cores = [flat[offs[k]:offs[k] + sizes[k]].view(cores_np[k].shape) for k in range(3)]
    for t, c in zip(cores, cores_np):
        t.copy_(torch.from_numpy(c))
    snapshot = flat.clone()
    ids = torch.from_numpy(ids_np).to(dev)
    grad = torch.from_numpy(grad_np).to(dev)
    out = torch.empty((B, D), dtype=torch.float32, device=dev)
    # the ids are resident before the timed region starts: TT_EMB_FLAG_IDS_READY (4)
    emb = TTEmbedding(w.n, w.d, w.r, B, cores, device=dev, flags=4)

    lr = w.lr if args.restore else args.lr

    waited = [0.0]                  # host seconds spent in the flow-control wait

    def step():
        if not args.free_running:
            # host-side flow control (enqueues nothing): at most two steps ahead of the device, so
            # that forward finds the pipeline of its prepared batch finished and need not wait for it
            w0 = time.perf_counter()
            emb.wait_backward(1)
            waited[0] += time.perf_counter() - w0
        if args.restore:
            flat.copy_(snapshot)
        if not args.no_prepare:
            emb.prepare(ids)        # index pipeline of the step after next, overlapped with this one
        emb.forward(ids, out)
        emb.backward_update(grad, lr)

    if args.calib_copy_mib > 0:
        src = torch.ones(args.calib_copy_mib << 18, dtype=torch.float32, device=dev)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)              # one copy kernel that reads and writes calib_copy_mib MiB
        torch.cuda.synchronize()
        del src, dst
    if not args.no_prepare:
        emb.prepare(ids)            # the first two steps' own index work
        emb.prepare(ids)
    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    stats = emb.stats()
    assert stats["U"] == struct["U"] and stats["Q"] == struct["Q"], (stats, struct)

    waited[0] = 0.0
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    t_enq = time.perf_counter()     # host side done: every launch of the timed steps is enqueued
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms_per_step = (t1 - t0) * 1e3 / args.steps
    host_ms_per_step = (t_enq - t0 - waited[0]) * 1e3 / args.steps   # enqueue work, waits taken off
    rows_per_s = B / (ms_per_step * 1e-3)
    # the same K steps with the host free to run any distance ahead (no host-side wait inside the
    # loop), reported beside the main figure
    other = None
    if not args.free_running and not args.no_prepare:
        args.free_running = True
        for _ in range(max(2, args.warmup // 2)):
            step()
        torch.cuda.synchronize()
        f0 = time.perf_counter()
        for _ in range(args.steps):
            step()
        torch.cuda.synchronize()
        f_ms = (time.perf_counter() - f0) * 1e3 / args.steps
        args.free_running = False
        other = {"ms_per_step": f_ms, "value": B / (f_ms * 1e-3), "host_steps_ahead": "unbounded"}
    if not bool(torch.isfinite(flat).all()) or not bool(torch.isfinite(out).all()):
        print("bench.py: cores or rows overflowed during the timed steps", file=sys.stderr)
        return 4

    # untimed leg: per-kernel durations from HIP events recorded on the launch stream
    prof = {}
    if args.profile_steps > 0:
        emb.profile(True)
        for _ in range(args.profile_steps):
            step()
        torch.cuda.synchronize()
        prof = emb.profile_read()
        emb.profile(False)

    U, Q = stats["U"], stats["Q"]
    ok = ids_np[(ids_np >= 0) & (ids_np < w.N)]
    n2, n3 = w.n[1], w.n[2]
    (d1, d2, d3), (r1, r2) = w.d, w.r
    touched_bytes = 4 * (np.unique(ok // (n2 * n3)).size * d1 * r1
                         + np.unique((ok // n3) % n2).size * r1 * d2 * r2
                         + np.unique(ok % n3).size * r2 * d3)
    kernels = {}
    # what a HIP event pair adds by itself (measured with nothing between the two events) is taken
    # off every launch, so that the durations are the kernels' own, as a profiler would report them
    ep = prof.pop("event_pair", {"launches": 0, "ms": 0.0})
    pair_us = ep["ms"] * 1e3 / ep["launches"] if ep["launches"] else 0.0
    for name, rec in prof.items():
        if rec["launches"] == 0:
            continue
        launches = rec["launches"] / max(args.profile_steps, 1)
        per_step_us = max(rec["ms"] * 1e3 / max(args.profile_steps, 1) - pair_us * launches, 0.0)
        by, fl = kernel_work(name, w, B, U, Q, touched_bytes, 0)
        if name == "u_bwd" and prof.get("dg3", {}).get("launches", 0) == 0:
            fl *= 2          # matrix-core shapes: dPsum and the dG3 partials share one launch
            if prof.get("prefix_bwd", {}).get("launches", 0) == 0:
                # ranks up to 32: the prefix-level gradients are formed in that launch too
                fl += kernel_work("prefix_bwd", w, B, U, Q, touched_bytes, 0)[1]
        kernels[name] = {"us_per_step": round(per_step_us, 2), "launches_per_step": launches,
                         "alg_bytes": int(by), "alg_flops": int(fl)}
    if not kernels:          # --profile-steps 0: no per-kernel leg (used under an external profiler)
        line = {"metric": "TT-embedding rows/s (fwd+bwd+update)", "value": rows_per_s,
                "unit": "rows/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
                "ms_per_step": ms_per_step, "higher_is_better": True, "scaling": "weak",
                "vs_baseline": None, "dtype": "f32", "data": "synthetic",
                "config": {"workload": w.name, "batch": B, "U": U, "Q": Q}}
        print(json.dumps(line))
        emb.close()
        return 0
    # the dominant kernel: the longest single launch on the caller's stream (the index kernels run
    # beside the arithmetic on the library's own streams and are not on the step's critical path)
    chain = [k for k in kernels if k in ("prefix_fwd", "row_fwd", "gsum", "gsum_fix", "u_bwd", "dg3",
                                         "prefix_bwd", "sgd")] or list(kernels)
    dom = max(chain, key=lambda k: kernels[k]["us_per_step"] / kernels[k]["launches_per_step"])
    kd = kernels[dom]
    launch_s = kd["us_per_step"] * 1e-6 / kd["launches_per_step"]
    by = kd["alg_bytes"] / kd["launches_per_step"]
    fl = kd["alg_flops"] / kd["launches_per_step"]
    if by / HBM_PEAK >= fl / FP32_PEAK:
        roofline = {"kernel": dom, "bound": "hbm", "achieved": by / launch_s / 1e9,
                    "peak": HBM_PEAK / 1e9, "unit": "GB/s", "frac": by / launch_s / HBM_PEAK,
                    "traffic": None}
    else:
        roofline = {"kernel": dom, "bound": "mfma", "achieved": fl / launch_s / 1e12,
                    "peak": FP32_PEAK / 1e12, "unit": "TFLOP/s", "frac": fl / launch_s / FP32_PEAK,
                    "traffic": None}
    roofline["avg_launch_us"] = round(launch_s * 1e6, 2)
    roofline["event_pair_us"] = round(pair_us, 2)     # already subtracted from avg_launch_us
    if args.seed is None:
        roofline["traffic"] = MEASURED_TRAFFIC.get(args.config, {}).get(dom)

    # the path as a whole against its binding bound
    F1, F2 = 2 * d1 * r1 * d2 * r2, 2 * d1 * d2 * r2 * d3
    alg_bytes = B * (8 + 8 * D) + 2 * touched_bytes
    alg_flops = 3 * (Q * F1 + U * F2) + (B - U) * D
    t_hbm, t_alu = alg_bytes / HBM_PEAK, alg_flops / FP32_PEAK
    path = {"alg_bytes": int(alg_bytes), "alg_flops": int(alg_flops),
            "t_hbm_us": round(t_hbm * 1e6, 2), "t_fp32_us": round(t_alu * 1e6, 2),
            "bound": "hbm" if t_hbm >= t_alu else "alu",
            "frac": max(t_hbm, t_alu) / (ms_per_step * 1e-3),
            "kernel_sum_us": round(sum(k["us_per_step"] for k in kernels.values()), 2)}

    cpu = None
    if not args.no_cpu_baseline:
        from oracle import tt_oracle as ora
        s = ora.Shape(w.n, w.d, w.r)

        def oracle_step(rows):
            ora.forward(s, *cores_np, ids_np[:rows], tag="f32")
            ora.backward_update(s, *cores_np, ids_np[:rows], grad_np[:rows], w.lr, tag="f32")

        oracle_step(256)                                   # loads the library
        probe = min(B, 20_000)
        c0 = time.perf_counter()
        oracle_step(probe)
        rate = probe / (time.perf_counter() - c0)          # rows/s, all host threads
        # about one second of wall time on all host threads, i.e. 10-30 s of CPU work
        want = max(int(rate * 1.2), probe)
        reps, rows = (max(1, round(want / B)), B) if want >= B else (1, want)
        c0 = time.perf_counter()
        for _ in range(reps):
            oracle_step(rows)
        c1 = time.perf_counter()
        what = (f"the whole batch, {reps} time(s)" if rows == B else f"first {rows} rows of the batch")
        cpu = {"value": reps * rows / (c1 - c0), "unit": "rows/s", "cores": ora.threads("f32"),
               "kind": "oracle",
               "sample": f"{what}: fp32 OpenMP build of the oracle, forward + backward + update, "
                         f"{c1 - c0:.2f} s wall on {ora.threads('f32')} threads"}

    line = {
        "metric": "TT-embedding rows/s (fwd+bwd+update)", "value": rows_per_s, "unit": "rows/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": ms_per_step,
        "host_enqueue_ms_per_step": host_ms_per_step, "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f32",
        "data": "synthetic",
        "config": {"workload": w.name, "N": w.N, "n": list(w.n), "d": list(w.d), "ranks": list(w.r),
                   "batch": B, "ids": w.ids, "zipf_s": w.zipf_s, "seed": seed, "lr": lr,
                   "protocol": "restore_each_step" if args.restore else "small_lr_no_restore",
                   "next_batch_index_overlap": not args.no_prepare,
                   "host_steps_ahead": "unbounded" if args.free_running else "at most 2",
                   "U": U, "Q": Q, "max_multiplicity": struct["max_multiplicity"]},
        "roofline": roofline, "cpu_baseline": cpu, "path_roofline": path,
        "free_running": other, "kernels": kernels,
    }
    print(json.dumps(line))
    emb.close()
    return 0


if __name__ == "__main__":
    sys.exit(main())
