#!/usr/bin/env python3
"""Benchmark of the ECRM update path on one MI355X.

A step is one call of ecrm_update: the whole hot path (grouping, load accounting, split-chain
path, optimizer + difference propagation) over one batch of synthetic updates that is already
resident in HBM.  The default workload is the largest one: 2^28 updates in 16 batches of 2^24 on
2^25 rows of 128 floats, even items uniform and odd items Zipf(0.99).

Prints ONE JSON line.  `value` is items/s over the timed steps (wall clock between two device
synchronisations); `roofline` is for the dominant kernel (apply_stripes), its duration measured
with HIP events recorded by the library on the stream it launches on; `cpu_baseline` is the CPU
oracle timed on this host on a bounded shard of the same workload.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="hbm_scale")
    ap.add_argument("--scale-shift", type=int, default=0, help="halve n and R this many times (debugging)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this build runs on ONE GPU (all servers' shards in one HBM); "
            "--gpus must be 1, no multi-GPU figure exists.")
        sys.exit(2)

    import numpy as np
    import torch

    import synth_inputs as si
    from paper_2104_01981_amd import binding

    if not os.path.exists(binding.library_path()):
        from paper_2104_01981_amd import build
        build.build()
    from paper_2104_01981_amd import Ecrm

    dev = "cuda:0"
    torch.cuda.set_device(0)
    w = si.WORKLOADS[args.workload]
    sh = args.scale_shift
    R, D, k, S = w["R"] >> sh, si.DEFAULT_D, si.DEFAULT_K, si.DEFAULT_S
    nb = w["batches"]
    per = (w["n"] >> sh) // nb
    seed = w["seed"]

    t_setup = time.perf_counter()
    E = si.table(seed, si.TAG_E0, R, D, dev)
    A = si.table(seed, si.TAG_A0, R, D, dev)
    PE = torch.empty(R // k, D, device=dev)
    PA = torch.empty(R // k, D, device=dev)
    ld = torch.zeros(S, dtype=torch.int64, device=dev)
    lp = torch.zeros(S, dtype=torch.int64, device=dev)
    ctx = Ecrm(R, D, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, per)
    scratch = torch.empty(ctx.scratch_bytes(), dtype=torch.uint8, device=dev)
    ctx.bind(E, A, PE, PA, ld, lp, scratch)
    ctx.encode()

    keys, grads, alg_path, alg_apply = [], [], [], []
    for b in range(nb):
        kt = si.workload_keys_t(args.workload, b, sh, dev)
        keys.append(kt)
        grads.append(si.grads(seed, b * per, per, D, dev))
        # measurement only: rows / stripes this batch touches, items on rows with long runs
        uk, cnt = torch.unique(kt, return_counts=True)
        U = int(uk.numel())
        Up = int(torch.unique(uk // k).numel())
        n_long = int(cnt[cnt > 256].sum())
        alg_path.append(per * (8 + 4 * D) + (U + Up) * 16 * D)
        alg_apply.append(per * 8 + (per - n_long) * 4 * D + (U + Up) * 16 * D)
        del uk, cnt
    torch.cuda.synchronize()
    log(f"setup {time.perf_counter() - t_setup:.1f}s: R={R} D={D} k={k} S={S} batches={nb}x{per}, "
        f"scratch {ctx.scratch_bytes() / 2**20:.0f} MiB, "
        f"alg bytes/item path {sum(alg_path) / (per * nb):.1f}")

    # host copy of the first 1/16 of the stripes for the CPU baseline (taken before any update)
    shard_rows = max(k, (R // 16) // k * k)
    if not args.no_cpu_baseline:
        hE, hA = E[:shard_rows].cpu().numpy(), A[:shard_rows].cpu().numpy()
        hPE, hPA = PE[:shard_rows // k].cpu().numpy(), PA[:shard_rows // k].cpu().numpy()

    for i in range(-args.warmup, 0):
        ctx.update(keys[i % nb], grads[i % nb])
    assert ctx.status() == 0
    ctx.profile(True)
    ctx.profile_read()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        ctx.update(keys[i % nb], grads[i % nb])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    ms, calls = ctx.profile_read()
    ctx.profile(False)
    assert ctx.status() == 0 and calls == min(args.steps, 256)

    elapsed = t1 - t0
    items = per * args.steps
    value = items / elapsed
    used = [i % nb for i in range(args.steps)]
    apply_ms = ms[2] / calls
    apply_bytes = sum(alg_apply[b] for b in used[:calls]) / calls
    achieved = apply_bytes / (apply_ms * 1e-3) / 1e9
    path_bytes = sum(alg_path[b] for b in used) / args.steps
    path_gbs = path_bytes * args.steps / elapsed / 1e9

    out = {
        "metric": "hot_path_items_per_sec", "value": value, "unit": "items/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": elapsed / args.steps * 1e3,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "f64",
        "data": "synthetic",
        "config": {"workload": f"{args.workload}" + (f">>{sh}" if sh else ""), "items_per_step": per,
                   "rows": R, "dim": D, "k": k, "servers": S, "storage": "f32", "optimizer": "adagrad",
                   "keys": w["kind"], "batches_resident": nb},
        "roofline": {"bound": "hbm", "kernel": "apply_stripes_kernel_d128", "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS, "traffic": None,
                     "algorithmic_bytes_per_launch": apply_bytes, "avg_launch_ms": apply_ms},
        "phases_ms_per_step": {"group": ms[0] / calls, "chains": ms[1] / calls, "apply": apply_ms},
        "path": {"algorithmic_bytes_per_step": path_bytes, "achieved_GBps": path_gbs,
                 "frac_of_hbm_peak": path_gbs / HBM_PEAK_GBS},
    }

    if not args.no_cpu_baseline:
        import oracle
        threads = min(16, oracle.max_threads())
        hld, hlp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
        cpu_items, cpu_s, nbatch = 0, 0.0, 0
        for b in range(nb):
            sel = torch.nonzero(keys[b] < shard_rows).squeeze(1)
            hk = keys[b][sel].cpu().numpy().view(np.uint64)
            hg = grads[b][sel].cpu().numpy()
            tc = time.perf_counter()
            oracle.update(hE, hA, hPE, hPA, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, hk, hg, hld, hlp, threads=threads)
            cpu_s += time.perf_counter() - tc
            cpu_items += len(hk)
            nbatch += 1
            if cpu_s * threads > 20.0 or nbatch == 4:
                break
        out["cpu_baseline"] = {"value": cpu_items / cpu_s, "unit": "items/s", "cores": threads, "kind": "oracle",
                               "sample": f"rows [0,{shard_rows}) (1/16 of the stripes) of the same tables and all "
                                         f"their updates from the first {nbatch} batches: {cpu_items} items, "
                                         f"{cpu_s:.2f}s wall"}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
