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
LONG_RUN = 1024          # ECRM_LONG_RUN of include/ecrm.h: longer runs leave the apply kernel for the split-chain path
# HBM bytes per launch of the apply kernel, from rocprofv3 FETCH_SIZE and WRITE_SIZE scaled by a plain copy of known
# size (profiles/update_path_<workload>_hbm_traffic.txt).  Reported only while the code of the kernel's sources is
# what the counters were taken on.
TRAFFIC_BYTES_PER_LAUNCH = {"hbm_scale": 37956210358, "large_uniform": 77511610801, "large_skewed": 42551350805}
TRAFFIC_SOURCES = ["paper_2104_01981_amd/csrc/update.hip", "paper_2104_01981_amd/csrc/rows.h",
                   "paper_2104_01981_amd/csrc/ecrm_internal.h"]
TRAFFIC_SOURCES_SHA256 = "0d2d60c869f179fb6dab8074dd53f02feb9a25a1b3a818c79621c76953355bf3"


def code_digest(paths):
    """sha256 of the sources' code: comments and white space do not count"""
    import hashlib
    import re
    h = hashlib.sha256()
    for rel in paths:
        text = open(os.path.join(ROOT, rel), "r").read()
        text = re.sub(r"/\*.*?\*/", " ", text, flags=re.S)
        text = re.sub(r"//[^\n]*", " ", text)
        h.update(" ".join(text.split()).encode())
    return h.hexdigest()


def measured_traffic(workload, scale_shift, variant=""):
    try:
        digest = code_digest(TRAFFIC_SOURCES)
    except OSError:
        return None
    if workload not in TRAFFIC_BYTES_PER_LAUNCH or scale_shift or variant or digest != TRAFFIC_SOURCES_SHA256:
        return None
    return TRAFFIC_BYTES_PER_LAUNCH[workload]


def log(*a):
    print(*a, file=sys.stderr, flush=True)


def _timed(torch, fn, reps=5):
    """seconds per call of fn (device time between two events on the current stream), after one untimed call"""
    fn()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) / reps * 1e-3


def memory_ceilings(torch, dev):
    """Rates of the plainest memory-bound kernels on this device, in GB/s of bytes read plus bytes written:
    an 8 GiB device-to-device copy; a gather of random 512-byte rows out of an 8 GiB table; and the
    read-modify-write of such rows (gather, then scatter back), which is the access pattern of the
    update path's tables."""
    def timed(fn, reps=5):
        return _timed(torch, fn, reps)
    rows, width = 1 << 24, 128                                    # 8 GiB of 512-byte rows
    src = torch.zeros(rows, width, device=dev)
    dst = torch.empty_like(src)
    copy_s = timed(lambda: dst.copy_(src))
    gen = torch.Generator(device=dev)
    gen.manual_seed(99)
    m = 1 << 22                                                   # 2 GiB worth of distinct random rows
    idx = torch.randperm(rows, device=dev, generator=gen)[:m]
    buf = torch.empty(m, width, device=dev)
    gather_s = timed(lambda: torch.index_select(src, 0, idx, out=buf))

    def rmw():
        torch.index_select(src, 0, idx, out=buf)
        src.index_copy_(0, idx, buf)
    rmw_s = timed(rmw)
    nbytes = rows * width * 4
    res = {"copy_ceiling_GBps": 2 * nbytes / copy_s / 1e9,
           "row_gather_ceiling_GBps": 2 * m * width * 4 / gather_s / 1e9,
           "row_rmw_ceiling_GBps": 4 * m * width * 4 / rmw_s / 1e9,
           "what": "8 GiB copy; gather of 2^22 random 512-byte rows of an 8 GiB table into a dense buffer; the same "
                   "rows gathered and scattered back (two kernels); bytes read + written per second"}
    del src, dst, buf, idx
    torch.cuda.empty_cache()
    return res


def row_traffic_by_distance(torch, dev):
    """The tables' own access pattern -- whole 512-byte rows at random row numbers, eight in flight per wavefront
    (the library's probe kernel) -- on two 8 GiB tables inside one allocation, as a function of how far apart they
    lie: read only, and read + written back.  GB/s of bytes read plus bytes written.  Meant for a process that holds
    no other device memory (bench.py runs it in a child process before it touches the device itself)."""
    from paper_2104_01981_amd import probe_row_traffic
    GiB, table_rows, n = 1 << 30, 1 << 24, 1 << 23
    arena = None
    for span in (200, 136, 72):                                   # GiB; the largest one the memory allows
        try:
            arena = torch.empty(span * GiB, dtype=torch.uint8, device=dev)
            break
        except RuntimeError:
            arena = None
    if arena is None:
        return None
    arena.zero_()
    gen = torch.Generator(device=dev)
    gen.manual_seed(7)
    rows = torch.randint(0, table_rows, (n,), device=dev, generator=gen, dtype=torch.int32)
    sink = torch.zeros(1, device=dev)
    out = {"what": "2^23 random rows of 128 floats, alternately from two 8 GiB tables that start this many GiB apart "
                   "inside one allocation (the first at its start), in a process that holds nothing else; read only / "
                   "read and written back; bytes read + written per second",
           "allocation_GiB": span,
           "read_GBps": {}, "read_write_GBps": {}}
    for dist in (8, 32, 56, 64, 72, 128):
        if dist + 8 > span:
            continue
        ta, tb = arena[:8 * GiB], arena[dist * GiB:(dist + 8) * GiB]
        for write, key in ((0, "read_GBps"), (1, "read_write_GBps")):
            secs = _timed(torch, lambda: probe_row_traffic(ta, tb, table_rows, rows, write, sink))
            out[key][str(dist)] = n * 512 * (2 if write else 1) / secs / 1e9
    del arena, rows, sink
    torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=16)
    ap.add_argument("--warmup", type=int, default=2)
    ap.add_argument("--workload", default="hbm_scale")
    ap.add_argument("--scale-shift", type=int, default=0, help="halve n and R this many times (debugging)")
    ap.add_argument("--dim", type=int, default=0, help="floats per entry (default: the workload's 128)")
    ap.add_argument("--k", type=int, default=0, help="entries per parity (default 4)")
    ap.add_argument("--servers", type=int, default=0, help="servers (default 5)")
    ap.add_argument("--optimizer", default="adagrad", choices=["adagrad", "momentum"])
    ap.add_argument("--combine", action="store_true", help="synchronous variant: one update per modified entry")
    ap.add_argument("--propagation", default="difference", choices=["difference", "gradient", "none"],
                    help="how the parities follow: the paper's difference propagation, the gradient-propagation "
                         "strawman (Sec. 3.3.1), or not at all (training without fault tolerance)")
    ap.add_argument("--resident", type=int, default=0, help="batches kept resident and cycled through (default: all)")
    ap.add_argument("--graph", action="store_true",
                    help="capture each resident batch's ecrm_update in a HIP graph and replay it (small, launch-bound "
                         "batches); phase timers are not available in this mode")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-recovery", action="store_true", help="skip the recovery-decode measurement")
    ap.add_argument("--no-ceilings", action="store_true",
                    help="skip the plain-copy and random-row ceilings of the device memory")
    ap.add_argument("--separate-figure", type=int, default=-1,
                    help="1: after the main measurement, measure the same update with one plain allocation per array "
                         "and report it beside the arena's figure (default: on for the large workloads)")
    ap.add_argument("--layout", default="auto", choices=["auto", "arena", "separate"],
                    help="auto: the built-in list of layouts, one per placement trial; arena: one arena in --order; "
                         "separate: one torch allocation per array as it comes")
    ap.add_argument("--placement-trials", type=int, default=4,
                    help="how many arenas to try at most when the placement probe is slow")
    ap.add_argument("--fresh-process-retry", type=int, default=1,
                    help="if every arena of this process probes slow, release the memory and run the benchmark "
                         "once more in a child process (0 disables)")
    ap.add_argument("--placement-accept-frac", type=float, default=None,
                    help="the probe accepts an arena when the apply kernel reaches this fraction of the HBM peak "
                         "(default: 0.70 for the default workload and configuration, whose usual rate is known; "
                         "0 = accept the first arena for every other one)")
    ap.add_argument("--order", default="",
                    help="arena only: order of the resident arrays (gN = batch N, padN = N GiB of padding); "
                         "default: the built-in list of geometries, one per placement trial")
    ap.add_argument("--first-geometry", type=int, default=0, help="index of the geometry the first trial uses")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="only run plain device-to-device copies of 8 GiB (to scale rocprof's HBM byte counters)")
    ap.add_argument("--row-traffic", type=int, default=1,
                    help="0: leave out the row-traffic-by-distance figures (a child process, run first)")
    ap.add_argument("--row-traffic-child", action="store_true", help="only measure those figures and print them")
    ap.add_argument("--per-step", action="store_true",
                    help="diagnostic: after the timed region, run the steps again one by one and log each one's phases")
    args = ap.parse_args()
    if args.gpus != 1:
        log("bench.py: this library runs on ONE GPU (all servers' shards in one HBM); "
            "--gpus must be 1, no multi-GPU figure exists.")
        sys.exit(2)

    # What the device's memory delivers for the tables' access pattern, by distance between two tables: measured
    # by a child process of its own BEFORE this one touches the device, so that it has the device memory to itself
    # and leaves nothing behind.
    row_traffic = json.loads(os.environ.get("ECRM_BENCH_ROW_TRAFFIC", "null"))
    if (args.row_traffic and not args.no_ceilings and not args.row_traffic_child and not args.calibrate_copy
            and row_traffic is None):
        import subprocess
        try:
            child = subprocess.run([sys.executable, os.path.abspath(__file__), "--row-traffic-child"],
                                   capture_output=True, text=True, timeout=300)
            row_traffic = json.loads(child.stdout.strip().splitlines()[-1]) if child.returncode == 0 else None
        except (subprocess.TimeoutExpired, ValueError, IndexError):
            row_traffic = None

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
    if args.row_traffic_child:
        print(json.dumps(row_traffic_by_distance(torch, dev)), flush=True)
        return
    if args.calibrate_copy:
        src = torch.zeros(1 << 31, dtype=torch.float32, device=dev)      # 8 GiB
        dst = torch.empty_like(src)
        for _ in range(5):
            dst.copy_(src)
        torch.cuda.synchronize()
        print(json.dumps({"calibrate_copy": {"bytes_read": src.numel() * 4, "bytes_written": src.numel() * 4,
                                             "copies": 5}}))
        return
    w = si.WORKLOADS[args.workload]
    sh = args.scale_shift
    D, k, S = args.dim or si.DEFAULT_D, args.k or si.DEFAULT_K, args.servers or si.DEFAULT_S
    R_gen = w["R"] >> sh                      # the key generators' row count (a power of two)
    R = R_gen // k * k                        # rows of the tables: the largest multiple of k below it
    per = (w["n"] >> sh) // w["batches"]
    nb = min(w["batches"], args.resident) if args.resident else w["batches"]
    seed = w["seed"]
    variant = "".join(f"/{n_}{v}" for n_, v, d in (("D", D, si.DEFAULT_D), ("k", k, si.DEFAULT_K), ("S", S, si.DEFAULT_S))
                      if v != d)
    if args.optimizer != "adagrad":
        variant += "/momentum0.9"
    if args.combine:
        variant += "/combined"
    if args.propagation != "difference":
        variant += f"/{args.propagation}-propagation"
    prop = {"difference": 0, "gradient": 1, "none": 2}[args.propagation]
    if args.separate_figure < 0:
        args.separate_figure = 1 if (w["n"] >> sh) >= (1 << 26) else 0
    if args.placement_accept_frac is None:
        args.placement_accept_frac = 0.70 if (args.workload == "hbm_scale" and not sh and not variant) else 0.0

    t_setup = time.perf_counter()
    ctx = Ecrm(R, D, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, per, optimizer=1 if args.optimizer == "momentum" else 0,
               momentum=0.9 if args.optimizer == "momentum" else 0.0, combine=1 if args.combine else 0, propagation=prop)
    # One arena for everything that stays resident (tables, scratch, all batches), carved at 2 MiB.
    # Order matters on this device (see the list of layouts below): batches are placed between the
    # tables.
    ALIGN = 2 << 20
    sizes = {"E": R * D * 4, "A": R * D * 4, "PE": R // k * D * 4, "PA": R // k * D * 4, "ld": S * 8, "lp": S * 8,
             "scratch": ctx.scratch_bytes()}
    for b in range(nb):
        sizes[f"keys{b}"] = per * 8
        sizes[f"grads{b}"] = per * D * 4
    # Layouts tried one after the other while the placement probe stays slow.  How fast the apply
    # kernel runs depends on where the four tables lie relative to each other AND on where the arena
    # starts in physical memory (measured: the first layout runs at 0.75 of the HBM peak with 0-48 GiB
    # of padding in front of it, at 0.68 with 56 GiB, at 0.75 again with 64 GiB; with the parity
    # tables moved from 64 to 80 GiB behind E it runs at 0.63).  All layouts below measured 0.75 on
    # an ordinary machine; they differ in both respects, so that a machine on which one of them lands
    # badly has others to offer.
    GEOMETRIES = ["E,g0,g1,A,g2,g3,PE,PA,scratch,keys,g*",
                  "pad16,E,g0,g1,A,g2,g3,PE,PA,scratch,keys,g*",
                  "E,g0,g1,g2,g3,A,g4,g5,g6,g7,PE,PA,scratch,keys,g*",
                  "separate"]

    def geometry(spec):
        """offsets of the resident arrays inside one arena, and its size"""
        sz, order, npad = dict(sizes), [], 0
        for tok in spec.split(","):
            if tok == "g*":
                order += [f"grads{b}" for b in range(nb) if f"grads{b}" not in order]
            elif tok == "keys":
                order += [f"keys{b}" for b in range(nb)]
            elif tok.startswith("pad"):
                sz[f"_pad{npad}"] = int(float(tok[3:]) * (1 << 30))
                order.append(f"_pad{npad}")
                npad += 1
            elif tok.startswith("g"):
                if int(tok[1:]) < nb:
                    order.append(f"grads{int(tok[1:])}")
            elif tok:
                order.append(tok)
        order += [n_ for n_ in sz if n_ not in order]
        offs, total = {}, 0
        for name in order:
            offs[name] = total
            total += (sz[name] + ALIGN - 1) // ALIGN * ALIGN
        return offs, total
    CH = 1 << 22                                  # rows generated per slice (2 GiB of fp32 at D = 128)

    def fill_tables():
        for r0 in range(0, R, CH):
            r1 = min(R, r0 + CH)
            E[r0:r1] = si.values(seed, si.TAG_E0, r0 * D, (r1 - r0) * D, dev).view(r1 - r0, D)
            A[r0:r1] = si.values(seed, si.TAG_A0, r0 * D, (r1 - r0) * D, dev).view(r1 - r0, D)
        ld.zero_()
        lp.zero_()
        ctx.encode()

    def fill_batch(b):
        kg = si.workload_keys_t(args.workload, b, sh, dev)
        keys[b].copy_(torch.where(kg >= R, kg - R, kg))      # only differs when k does not divide 2^m
        for i0 in range(0, per, CH):
            i1 = min(per, i0 + CH)
            grads[b][i0:i1] = si.grads(seed, b * per + i0, i1 - i0, D, dev)

    def batch_bytes(kt):
        """(whole-path, apply-kernel) algorithmic bytes of one batch -- measurement only, from the keys."""
        uk, cnt = torch.unique(kt, return_counts=True)
        U = int(uk.numel())
        Up = int(torch.unique(uk // k).numel())
        n_long = int(cnt[cnt > LONG_RUN].sum())
        if prop == 2:        # no parities
            return per * (8 + 4 * D) + U * 16 * D, (per - n_long) * (8 + 4 * D) + U * 16 * D
        if prop == 1:        # every gradient goes to two servers; the two apply launches together
            _, pcnt = torch.unique(kt // k, return_counts=True)
            n_long_p = int(pcnt[pcnt > LONG_RUN].sum())
            return (2 * per * (8 + 4 * D) + (U + Up) * 16 * D,
                    (2 * per - n_long - n_long_p) * (8 + 4 * D) + (U + Up) * 16 * D)
        return per * (8 + 4 * D) + (U + Up) * 16 * D, (per - n_long) * (8 + 4 * D) + (U + Up) * 16 * D

    # Physical placement is the driver's; the same kernel on the same data runs at 0.75 or at 0.63 of the
    # HBM peak depending on where the four tables lie relative to each other (rocprofv3 counters: same
    # request counts and hit rates, but 2.6x the DRAM-credit stalls and 11 % longer read latency at the
    # L2's memory interface in the slow case -- the loss is on the memory side).  Probe with three updates
    # of batch 0 and, if the apply kernel is clearly off its usual rate, release the memory and take the
    # next arrangement.
    placement, geometries = [], []
    for trial in range(max(1, args.placement_trials)):
        specs = [args.order] if args.order else GEOMETRIES if args.layout == "auto" else [g_ for g_ in GEOMETRIES if g_ != "separate"]
        spec = specs[(args.first_geometry + trial) % len(specs)]
        separate = args.layout == "separate" or spec == "separate"
        geometries.append("separate" if separate else spec)
        if separate:
            pieces = {name: torch.empty(sizes[name], dtype=torch.uint8, device=dev) for name in sizes}

            def carve(name, dtype, shape):
                return pieces[name].view(dtype).view(shape)
        else:
            offs, total = geometry(spec)
            arena = torch.empty(total, dtype=torch.uint8, device=dev)

            def carve(name, dtype, shape):
                return arena[offs[name]:offs[name] + sizes[name]].view(dtype).view(shape)

        E, A = carve("E", torch.float32, (R, D)), carve("A", torch.float32, (R, D))
        PE, PA = carve("PE", torch.float32, (R // k, D)), carve("PA", torch.float32, (R // k, D))
        ld, lp = carve("ld", torch.int64, (S,)), carve("lp", torch.int64, (S,))
        scratch = carve("scratch", torch.uint8, (sizes["scratch"],))
        keys = [carve(f"keys{b}", torch.int64, (per,)) for b in range(nb)]
        grads = [carve(f"grads{b}", torch.float32, (per, D)) for b in range(nb)]
        ctx.bind(E, A, PE, PA, ld, lp, scratch)
        fill_tables()
        fill_batch(0)
        ctx.update(keys[0], grads[0])
        ctx.profile(True)
        ctx.profile_read()
        for _ in range(3):
            ctx.update(keys[0], grads[0])
        pms, pcalls = ctx.profile_read()
        ctx.profile(False)
        assert ctx.status() == 0
        probe_frac = batch_bytes(keys[0])[1] / (pms[2] / pcalls * 1e-3) / 1e9 / HBM_PEAK_GBS
        placement.append(round(probe_frac, 4))
        if trial + 1 >= args.placement_trials or probe_frac >= args.placement_accept_frac:
            break
        log(f"placement trial {trial} ({geometries[-1]}): apply kernel at {probe_frac:.3f} of the HBM peak, "
            "trying the next geometry")
        ctx.drop_buffers()
        del E, A, PE, PA, ld, lp, scratch, keys, grads
        if separate:
            del pieces
        else:
            del arena
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
    if placement[-1] < args.placement_accept_frac and args.fresh_process_retry > 0:
        # every arena this process obtained is slow: hand over to a child process with fresh mappings
        import subprocess
        log(f"placement: {len(placement)} geometries at {placement} of the HBM peak; retrying in a fresh process")
        ctx.drop_buffers()
        del E, A, PE, PA, ld, lp, scratch, keys, grads
        if separate:
            del pieces
        else:
            del arena
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        argv = [a for a in sys.argv[1:]]
        rc = subprocess.call([sys.executable, os.path.abspath(__file__), *argv, "--fresh-process-retry", "0",
                              "--first-geometry", str(args.first_geometry + len(placement))],
                             env=dict(os.environ, ECRM_BENCH_PARENT_PROBES=json.dumps(placement),
                                      ECRM_BENCH_ROW_TRAFFIC=json.dumps(row_traffic)))
        sys.exit(rc)
    fill_tables()                                  # the probe's updates are undone: tables start from the recipe

    alg_path, alg_apply = [], []
    for b in range(nb):
        if b:
            fill_batch(b)
        bp, ba = batch_bytes(keys[b])
        alg_path.append(bp)
        alg_apply.append(ba)
    torch.cuda.synchronize()
    log(f"setup {time.perf_counter() - t_setup:.1f}s: R={R} D={D} k={k} S={S} batches={nb}x{per}, "
        f"scratch {ctx.scratch_bytes() / 2**20:.0f} MiB, "
        f"alg bytes/item path {sum(alg_path) / (per * nb):.1f}")

    # host copy of the first 1/16 of the stripes for the CPU baseline (taken before any update), and of
    # the updates of the first batches that fall on it
    shard_rows = max(k, (R // 16) // k * k)
    cpu_batches = []
    if not args.no_cpu_baseline:
        hE, hA = E[:shard_rows].cpu().numpy(), A[:shard_rows].cpu().numpy()
        hPE, hPA = PE[:shard_rows // k].cpu().numpy(), PA[:shard_rows // k].cpu().numpy()
        for b in range(min(nb, 4)):
            sel = torch.nonzero(keys[b] < shard_rows).squeeze(1)
            cpu_batches.append((keys[b][sel].cpu().numpy().view(np.uint64), grads[b][sel].cpu().numpy()))

    for i in range(-args.warmup, 0):
        ctx.update(keys[i % nb], grads[i % nb])
    assert ctx.status() == 0
    if args.graph:
        side = torch.cuda.Stream()
        graphs = []
        for b in range(nb):
            gph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(gph, stream=side):
                ctx.update(keys[b], grads[b], stream=side)
            graphs.append(gph)
        graphs[(-1) % nb].replay()                 # one untimed replay
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(args.steps):
            graphs[i % nb].replay()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ms, calls = [0.0, 0.0, (t1 - t0) * 1e3], args.steps      # no phase split: everything booked as one
        step_ms = None
    else:
        ctx.profile(True)
        ctx.profile_read()
        marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        marks[0].record()
        for i in range(args.steps):
            ctx.update(keys[i % nb], grads[i % nb])
            marks[i + 1].record()
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        step_ms = sorted(marks[i].elapsed_time(marks[i + 1]) for i in range(args.steps))
        ms, calls = ctx.profile_read()
        ctx.profile(False)
        assert calls == min(args.steps, 256)
    assert ctx.status() == 0

    if args.per_step:
        ctx.profile(True)
        for i in range(args.steps):
            ctx.update(keys[i % nb], grads[i % nb])
            pms, _ = ctx.profile_read()
            log(f"step {i:3d} batch {i % nb:2d}: group {pms[0]:.3f} chains {pms[1]:.3f} apply {pms[2]:.3f} ms")
        ctx.profile(False)

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
        "step_ms": None if not step_ms else {"median": step_ms[len(step_ms) // 2], "best": step_ms[0],
                                             "worst": step_ms[-1]},
        "config": {"workload": f"{args.workload}" + (f">>{sh}" if sh else "") + variant, "items_per_step": per,
                   "rows": R, "dim": D, "k": k, "servers": S, "storage": "f32", "optimizer": args.optimizer, "combine": bool(args.combine),
                   "keys": w["kind"], "batches_resident": nb, "hip_graph": bool(args.graph)},
        "roofline": {"bound": "hbm", "kernel": ("apply_stripes_kernel" if prop == 0 else "apply_rows_kernel") + ("_d128" if D <= 128 else "_d256")
                     + (" (two launches per step)" if prop == 1 else ""), "achieved": achieved,
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": achieved / HBM_PEAK_GBS,
                     "traffic": measured_traffic(args.workload, sh, variant),
                     "algorithmic_bytes_per_launch": apply_bytes, "avg_launch_ms": apply_ms},
        "phases_ms_per_step": {"group": ms[0] / calls, "chains": ms[1] / calls, "apply": apply_ms},
        "device": {"name": torch.cuda.get_device_properties(0).name,
                   "uuid": str(getattr(torch.cuda.get_device_properties(0), "uuid", "")),
                   "compute_units": torch.cuda.get_device_properties(0).multi_processor_count},
        "placement": {"arenas_tried": len(placement), "probe_apply_frac": placement, "geometry": geometries[-1],
                      "parent_process_probes": json.loads(os.environ.get("ECRM_BENCH_PARENT_PROBES", "null"))},
        "path": {"algorithmic_bytes_per_step": path_bytes, "achieved_GBps": path_gbs,
                 "frac_of_hbm_peak": path_gbs / HBM_PEAK_GBS},
    }

    # Updates per server over the warm-up and timed calls (Sec. 4.3, effect on load imbalance): entry
    # updates alone, and entry plus parity updates under the rotating placement.
    ldh, lph = ld.cpu().double(), lp.cpu().double()
    out["load_balance"] = {
        "entry_updates_per_server": [int(v) for v in ldh], "parity_updates_per_server": [int(v) for v in lph],
        "max_over_min_entries_only": float(ldh.max() / ldh.min()),
        "max_over_min_with_parities": float((ldh + lph).max() / (ldh + lph).min()),
    }

    if not args.no_recovery and prop == 0:
        # full recovery of one server and degraded reads (Sec. 3.4)
        def timed(fn, reps=3):
            fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            for _ in range(reps):
                fn()
            e1.record()
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / reps
        G = R // k
        held = sum(1 for g in range(S) for u in range(k + 1)
                   if (g % S == 0 if u == k else (g + 1 + u) % S == 0)) / S      # units of server 0 per stripe
        rec_ms = timed(lambda: ctx.recover_server(0))
        rec_bytes = G * held * (k + 1) * 2 * D * 4
        nread = min(per, 1 << 22)
        oe = torch.empty(nread, D, device=dev)
        oa = torch.empty(nread, D, device=dev)
        kread = keys[0][:nread]
        plain_ms = timed(lambda: ctx.degraded_read(kread, None, oe, oa))
        degr_ms = timed(lambda: ctx.degraded_read(kread, 1, oe, oa))
        lostfrac = float(((kread // k + 1 + kread % k) % S == 1).float().mean())
        plain_bytes = nread * 4 * D * 4
        degr_bytes = nread * (1 - lostfrac) * 4 * D * 4 + nread * lostfrac * (k + 1) * 2 * D * 4
        assert ctx.status() == 0
        out["recovery"] = {
            "recover_server": {"ms": rec_ms, "algorithmic_bytes": rec_bytes, "GBps": rec_bytes / rec_ms / 1e6,
                               "frac_of_hbm_peak": rec_bytes / rec_ms / 1e6 / HBM_PEAK_GBS,
                               "what": "rebuild every unit server 0 holds (k reads + 1 write per stripe, E and A)"},
            "degraded_read": {"keys": nread, "plain_ms": plain_ms, "plain_GBps": plain_bytes / plain_ms / 1e6,
                              "lost_server_ms": degr_ms, "lost_server_GBps": degr_bytes / degr_ms / 1e6,
                              "decoded_fraction": lostfrac},
        }
        del oe, oa

        # training while server 0 is rebuilt chunk by chunk: the decoder on a second stream, one update
        # batch enqueued while each chunk is locked, buffered updates replayed at every unlock
        buf_keys = torch.empty(2 * per, dtype=torch.int64, device=dev)
        buf_grads = torch.empty(2 * per, D, device=dev)
        side, main = torch.cuda.Stream(), torch.cuda.current_stream()
        under_load = {}
        def recover_under_load(chunks, watch):
            """one recovery of server 0 in `chunks` chunks, an update batch enqueued under every lock; with
            `watch` the number of waiting updates is read back at every chunk (which waits for the stream)"""
            ctx.recovery_begin(0, chunks, buf_keys, buf_grads, per)
            torch.cuda.synchronize()
            tr0 = time.perf_counter()
            waiting = 0
            for ch in range(chunks):
                ctx.recovery_lock()
                ev, done = torch.cuda.Event(), torch.cuda.Event()
                ev.record(main)
                side.wait_event(ev)
                ctx.recovery_decode(stream=side)
                done.record(side)
                ctx.update(keys[ch % nb], grads[ch % nb])
                main.wait_event(done)
                if watch:
                    waiting = max(waiting, ctx.recovery_state()["buffered"])
                ctx.recovery_unlock()
            torch.cuda.synchronize()
            return time.perf_counter() - tr0, waiting

        for chunks in (() if args.combine else (1, 10)):    # the protocol is defined for asynchronous training only
            secs, _ = recover_under_load(chunks, False)      # timed: nothing in the loop waits for the device
            rc_status = ctx.status()
            _, waiting = recover_under_load(chunks, True)    # once more, untimed, watching the buffer
            rc_status = rc_status or ctx.status()
            under_load[str(chunks)] = {
                "recovery_ms": secs * 1e3, "updates_applied_meanwhile": chunks * per,
                "items_per_s_during_recovery": chunks * per / secs,
                "relative_to_normal": chunks * per / secs / value,
                "max_updates_waiting": waiting, "status": rc_status}
            if rc_status != 0:
                ctx.clear_status()
        out["recovery"]["under_load"] = under_load
        del buf_keys, buf_grads

    # ---- what this device's memory delivers to the plainest kernels (context for the fractions above;
    #      measured after the timed region, on memory of its own)
    if not args.no_ceilings:
        out["ceilings"] = memory_ceilings(torch, dev)
        out["ceilings"]["row_traffic_by_distance"] = row_traffic

    # ---- the same update with one plain allocation per array, as a caller who does not arrange the tables
    #      would have it (the arena above is this benchmark's own arrangement)
    if args.separate_figure and not args.graph and geometries[-1] != "separate":
        ctx.drop_buffers()
        keep = min(nb, 2)
        hk = [keys[b].clone() for b in range(keep)]
        del E, A, PE, PA, ld, lp, scratch, keys, grads, arena
        torch.cuda.synchronize()
        torch.cuda.empty_cache()
        E, A = torch.empty(R, D, device=dev), torch.empty(R, D, device=dev)
        PE, PA = torch.empty(R // k, D, device=dev), torch.empty(R // k, D, device=dev)
        ld, lp = torch.zeros(S, dtype=torch.int64, device=dev), torch.zeros(S, dtype=torch.int64, device=dev)
        scratch = torch.empty(sizes["scratch"], dtype=torch.uint8, device=dev)
        keys = hk
        grads = [torch.empty(per, D, device=dev) for _ in range(keep)]
        ctx.bind(E, A, PE, PA, ld, lp, scratch)
        fill_tables()
        for b in range(keep):
            for i0 in range(0, per, CH):
                i1 = min(per, i0 + CH)
                grads[b][i0:i1] = si.grads(seed, b * per + i0, i1 - i0, D, dev)
        for b in range(keep):
            ctx.update(keys[b], grads[b])
        ctx.profile(True)
        ctx.profile_read()
        torch.cuda.synchronize()
        ts0 = time.perf_counter()
        reps = 6
        for i in range(reps):
            ctx.update(keys[i % keep], grads[i % keep])
        torch.cuda.synchronize()
        ts1 = time.perf_counter()
        sms, scalls = ctx.profile_read()
        ctx.profile(False)
        assert ctx.status() == 0
        sep_apply = sum(alg_apply[i % keep] for i in range(reps)) / (sms[2] * 1e-3) / 1e9
        sep_path = sum(alg_path[i % keep] for i in range(reps)) / (ts1 - ts0) / 1e9
        out["separate_allocations"] = {
            "what": "one torch allocation per array, as they come; same kernels, same batches",
            "ms_per_step": (ts1 - ts0) / reps * 1e3, "items_per_s": per * reps / (ts1 - ts0),
            "apply_frac_of_hbm_peak": sep_apply / HBM_PEAK_GBS, "path_frac_of_hbm_peak": sep_path / HBM_PEAK_GBS}

    if not args.no_cpu_baseline:
        import oracle
        threads = min(16, oracle.max_threads())
        hld, hlp = np.zeros(S, np.uint64), np.zeros(S, np.uint64)
        cpu_items, cpu_s, nbatch = 0, 0.0, 0
        for hk, hg in cpu_batches:
            tc = time.perf_counter()
            oracle.update(hE, hA, hPE, hPA, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, hk, hg, hld, hlp, threads=threads)
            cpu_s += time.perf_counter() - tc
            cpu_items += len(hk)
            nbatch += 1
            if cpu_s * threads > 20.0 or nbatch == 4:
                break
        # the same oracle on ONE thread, on the medium workload (2^22 updates on 2^20 rows): a 1/16 shard of
        # its stripes with all their updates
        wm = si.WORKLOADS["medium"]
        mR = wm["R"] // k * k
        m_rows = max(k, (mR // 16) // k * k)
        mk = si.workload_keys_t("medium", 0, 0, dev)
        mk = torch.where(mk >= mR, mk - mR, mk)
        msel = torch.nonzero(mk < m_rows).squeeze(1)
        mkeys = mk[msel].cpu().numpy().view(np.uint64)
        mg = np.ascontiguousarray(si.grad_rows(wm["seed"], msel.cpu().numpy(), D))
        mE = si.table(wm["seed"], si.TAG_E0, m_rows, D).numpy().copy()
        mA = si.table(wm["seed"], si.TAG_A0, m_rows, D).numpy().copy()
        mPE, mPA = oracle.encode(mE, k), oracle.encode(mA, k)
        tc = time.perf_counter()
        oracle.update(mE, mA, mPE, mPA, k, S, si.DEFAULT_LR, si.DEFAULT_EPS, mkeys, mg, threads=1)
        one_s = time.perf_counter() - tc
        out["cpu_baseline"] = {"value": cpu_items / cpu_s, "unit": "items/s", "cores": threads, "kind": "oracle",
                               "sample": f"rows [0,{shard_rows}) (1/16 of the stripes) of the same tables and all "
                                         f"their updates from the first {nbatch} batches: {cpu_items} items, "
                                         f"{cpu_s:.2f}s wall",
                               "single_thread_value": len(mkeys) / one_s,
                               "single_thread_sample": f"medium workload, rows [0,{m_rows}) (1/16 of its stripes) with all "
                                                       f"their updates: {len(mkeys)} items, {one_s:.2f}s wall",
                               "host_cpus": os.cpu_count()}
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
