#!/usr/bin/env python3
"""Benchmark of the fused W4A16 SplitK GEMM on one MI355X.

A step is one call of the whole hot path (zero-state handling, unpack, dequantise, product,
split-k reduction, fp16 store) on one batch of synthetic input.  The headline workload is
m = 16, n = k = 4096, group_size = 128 (the configuration the paper profiles); inputs are
resident in HBM before timing starts.  Weights rotate through enough distinct sets
(>= 512 MiB) that neither L2 nor the 256 MB Infinity Cache can serve them, which is what a
decoder does anyway: every layer has its own weights.

Prints ONE JSON line on stdout (progress and tables go to stderr):
  value        effective HBM GB/s = algorithmic bytes per call / wall time per call
  roofline     the same bytes over the HIP-event time per launch on the launch stream, vs 8 TB/s
  cpu_baseline the CPU oracle timed on this machine's host cores on the same workload
  extra        SplitK-vs-DP per shape, split_k sweep, warm (cache-resident) figures, non-square decoder shapes
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

HBM_PEAK_GBPS = 8000.0  # MI355X published HBM3E peak
ROTATE_BYTES = 512 << 20
ROOT = os.path.dirname(os.path.abspath(__file__))


def kernel_source_id():
    """What identifies the kernels that are being timed: a hash of the HIP sources and of the build
    script (which holds the compiler flags).  A counter summary under profiles/ carries the value
    it was taken with, so a number from it is only quoted while it still describes this build."""
    import hashlib

    h = hashlib.sha256()
    pkg = os.path.join(ROOT, "paper_2402_00025_amd")
    for rel in ("csrc/w4a16.hip", "csrc/w4a16_device.hpp", "csrc/w4a16_stream.hpp", "build.py"):
        with open(os.path.join(pkg, rel), "rb") as f:
            h.update(f.read())
    return h.hexdigest()[:16]


def measured_traffic(m, n, k, bits=4):
    """HBM bytes per launch of the timed kernel from the committed rocprofv3 counter summary
    (profiles/), or None when there is none for this shape or when it was taken with other kernel
    sources than the ones being timed (its `kernel_source_id=` line differs)."""
    tag = "splitk" if bits == 4 else f"splitk_w{bits}"
    path = os.path.join(ROOT, "profiles", f"hbm_traffic_{tag}_m{m}_n{n}_k{k}.txt")
    traffic, stamp = None, None
    try:
        for line in open(path):
            if line.startswith("traffic_bytes_per_launch="):
                traffic = float(line.split("=", 1)[1])
            if line.startswith("kernel_source_id="):
                stamp = line.split("=", 1)[1].strip()
    except OSError:
        return None
    return traffic if stamp == kernel_source_id() else None


def calibrate_copy(reps=6, mib=256):
    """A plain device-to-device copy of known size, so a counter run of this program can scale
    FETCH_SIZE / WRITE_SIZE by what they read for a known amount of traffic."""
    import torch

    src = torch.empty(mib << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
    dst = torch.empty_like(src)
    for _ in range(reps):
        dst.copy_(src)
    torch.cuda.synchronize()
    log(f"[bench] calibration: {reps} device copies of {mib} MiB (reads {mib} MiB, writes {mib} MiB each)")

PAPER_CONTEXT = {
    "note": "paper figures are for a Triton kernel on NVIDIA GPUs: context only, not a target",
    "avg_speedup_splitk_over_dp": {"A100": "+65%", "H100": "+124% (peak +295%)"},
    "nsight_m16_n4096_k4096_A100": {"splitk_us": 27.90, "dp_us": 52.93, "splitk_GBps": 313, "dp_GBps": 161},
}


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class Workload:
    """Device-resident inputs for one shape, with `sets` distinct weight sets to rotate through."""

    def __init__(self, m, n, k, g, sets, seed=0, bits=4):
        import torch

        from paper_2402_00025_amd.inputs import algorithmic_bytes, make_inputs, make_weight_sets

        self.m, self.n, self.k, self.g, self.bits = m, n, k, g, bits
        self.bytes = algorithmic_bytes(m, n, k, g, bits)
        x = make_inputs(m, n, k, g, seed=seed, bits=bits)
        self.host = x
        self.A = torch.from_numpy(x.A).cuda()
        self.C = torch.zeros((m, n), dtype=torch.float16, device="cuda")
        self.sets = [tuple(torch.from_numpy(t).cuda() for t in (x.qweight, x.scales, x.qzeros))]
        if sets > 1:
            for (qw, s, qz) in make_weight_sets(sets - 1, n, k, g, seed=seed, bits=bits):
                self.sets.append((torch.from_numpy(qw).cuda(), torch.from_numpy(s).cuda(), torch.from_numpy(qz).cuda()))
        torch.cuda.synchronize()

    def with_m(self, m):
        """A view of the same weights with the first m activation rows."""
        import copy

        from paper_2402_00025_amd.inputs import algorithmic_bytes

        w = copy.copy(self)
        w.m = m
        w.A = self.A[:m].contiguous()
        w.C = self.C[:m].contiguous()
        w.bytes = algorithmic_bytes(m, self.n, self.k, self.g, self.bits)
        return w


def make_call(w: Workload, kind: str, split_k=0, tile_cols=0, waves=0, reduce=0):
    """A closure launching call number i (weights rotate with i) through the C ABI on torch's
    current stream (looked up per call, so the same closure works under graph capture)."""
    import ctypes

    import torch

    from paper_2402_00025_amd import binding

    L = binding.lib()
    A, C = ctypes.c_void_p(w.A.data_ptr()), ctypes.c_void_p(w.C.data_ptr())
    ptrs = [tuple(ctypes.c_void_p(t.data_ptr()) for t in s) for s in w.sets]
    m, n, k, g = w.m, w.n, w.k, w.g
    nsets = len(ptrs)
    current_stream = torch.cuda.current_stream
    if kind == "splitk":
        def call(i):
            qw, s, qz = ptrs[i % nsets]
            rc = L.w4a16_gemm_ex(A, qw, s, qz, C, m, n, k, g, split_k, tile_cols, waves, reduce,
                                 ctypes.c_void_p(current_stream().cuda_stream))
            if rc:
                raise binding.W4A16Error(rc, "w4a16_gemm_ex")
    elif kind in ("splitk_bits", "dp_bits"):
        gemm = {2: L.w2a16_gemm, 3: L.w3a16_gemm, 8: L.w8a16_gemm}[w.bits]
        gemm_dp = {2: L.w2a16_gemm_dp, 3: L.w3a16_gemm_dp, 8: L.w8a16_gemm_dp}[w.bits]

        def call(i):
            qw, s, qz = ptrs[i % nsets]
            st = ctypes.c_void_p(current_stream().cuda_stream)
            rc = (gemm(A, qw, s, qz, C, m, n, k, g, split_k, st) if kind == "splitk_bits"
                  else gemm_dp(A, qw, s, qz, C, m, n, k, g, st))
            if rc:
                raise binding.W4A16Error(rc, f"w{w.bits}a16_gemm")
    elif kind == "read":
        nbytes = w.sets[0][0].numel() * 4
        read_shape = split_k   # the probe's launch shape rides in the split_k argument

        def call(i):
            qw, _s, _qz = ptrs[i % nsets]
            rc = L.w4a16_read_probe(qw, nbytes, read_shape, ctypes.c_void_p(current_stream().cuda_stream))
            if rc:
                raise binding.W4A16Error(rc, "w4a16_read_probe")
    elif kind == "streamk":
        def call(i):
            qw, s, qz = ptrs[i % nsets]
            rc = L.w4a16_gemm_streamk(A, qw, s, qz, C, m, n, k, g, 0, ctypes.c_void_p(current_stream().cuda_stream))
            if rc:
                raise binding.W4A16Error(rc, "w4a16_gemm_streamk")
    else:
        def call(i):
            qw, s, qz = ptrs[i % nsets]
            rc = L.w4a16_gemm_dp_ex(A, qw, s, qz, C, m, n, k, g, tile_cols, waves,
                                    ctypes.c_void_p(current_stream().cuda_stream))
            if rc:
                raise binding.W4A16Error(rc, "w4a16_gemm_dp_ex")
    call.nsets = nsets
    return call


def time_calls_eager(call, steps, warmup):
    """(wall seconds per call, HIP-event seconds per call) over exactly `steps` eager calls.
    With two launches per call from Python the host enqueues about one call per 7-8 us, so
    for small shapes this measures the host, not the GPU; see time_calls."""
    import torch

    for i in range(warmup):
        call(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record()
    for i in range(steps):
        call(warmup + i)
    e1.record()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    return (t1 - t0) / steps, e0.elapsed_time(e1) * 1e-3 / steps


_GRAPH_KEEP = []  # captured graphs must outlive their replays


def time_calls(call, steps, warmup, prewarm_s=0.03):
    """(wall seconds per call, HIP-event seconds per call) over exactly `steps` calls.

    The calls are captured once into HIP graphs (every kernel the library launches is
    captured; nothing is skipped or cached) and replayed, which takes the Python/ctypes
    enqueue cost out of the timed region: `chunk` consecutive calls (a whole rotation over the
    weight sets when possible) per graph, steps // chunk replays plus a second graph for the
    remainder.  Untimed before that: `warmup` eager calls, one replay of each graph, and
    `prewarm_s` seconds of replays so the GPU is at its running clocks."""
    import torch

    for i in range(max(warmup, 3)):
        call(i)
    torch.cuda.synchronize()
    chunk = min(steps, max(call.nsets, 64))
    reps, rem = divmod(steps, chunk)
    side = torch.cuda.Stream()
    graphs = []
    for count in ((chunk, rem) if rem else (chunk,)):
        g = torch.cuda.CUDAGraph()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.graph(g, stream=side):
            for i in range(count):
                call(i)
        graphs.append(g)
    _GRAPH_KEEP.append(graphs)
    for g in graphs:
        g.replay()
    torch.cuda.synchronize()
    t_end = time.perf_counter() + prewarm_s
    while time.perf_counter() < t_end:
        graphs[0].replay()
        torch.cuda.synchronize()
    # pass 1, wall clock: exactly `steps` calls between two synchronisations, nothing else enqueued
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        graphs[0].replay()
    if rem:
        graphs[1].replay()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # pass 2, HIP events on the launch stream around the same `steps` calls
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        graphs[0].replay()
    if rem:
        graphs[1].replay()
    e1.record()
    torch.cuda.synchronize()
    return (t1 - t0) / steps, e0.elapsed_time(e1) * 1e-3 / steps


def verify(w: Workload, call, oracle_ref):
    import torch

    w.C.fill_(float("nan"))
    call(0)
    torch.cuda.synchronize()
    got = w.C.cpu().numpy().astype(np.float64)
    rel = float(np.linalg.norm(got - oracle_ref) / np.linalg.norm(oracle_ref))
    emax = float(np.abs(got - oracle_ref).max())
    ok = bool(np.isfinite(got).all() and rel <= 2e-3 and emax <= 1e-2 * np.abs(oracle_ref).max())
    return ok, rel, emax


def cpu_baseline(w: Workload, budget_s=10.0):
    """The oracle as it stands (the definition, one output element at a time, OpenMP over the
    columns) on the host cores, on the whole timed workload; beside it the same function on one
    thread and the column-blocked arrangement kept for timing, each once."""
    from oracle import w4a16_oracle

    x = w.host
    times, threads = [], 0
    t_start = time.perf_counter()
    Cref = None
    while len(times) < 5 and (time.perf_counter() - t_start) < budget_s:
        t0 = time.perf_counter()
        Cref, _, threads = w4a16_oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, w.g, return_threads=True)
        times.append(time.perf_counter() - t0)
    med = float(np.median(times))
    t0 = time.perf_counter()
    w4a16_oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, w.g, threads=1)
    one = time.perf_counter() - t0
    w4a16_oracle.gemm(x.A, x.qweight, x.scales, x.qzeros, w.g, threads=int(threads))   # back to all threads
    t0 = time.perf_counter()
    w4a16_oracle.gemm_blocked(x.A, x.qweight, x.scales, x.qzeros, w.g)
    blocked = time.perf_counter() - t0
    return Cref, {
        "value": w.bytes / med / 1e9, "unit": "GB/s", "cores": int(threads), "kind": "oracle",
        "sample": f"full workload m={w.m} n={w.n} k={w.k}, {len(times)} calls, median {med * 1e3:.1f} ms/call, fp64 accumulation",
        "ms_per_call": med * 1e3,
        "single_thread": {"ms_per_call": one * 1e3, "GBps": w.bytes / one / 1e9, "cores": 1, "calls": 1},
        "blocked_arrangement": {"ms_per_call": blocked * 1e3, "GBps": w.bytes / blocked / 1e9, "cores": int(threads),
                                "calls": 1, "note": "same arithmetic in column blocks of 128 with a cached weight row"},
    }


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-sweep", action="store_true", help="headline workload only")
    ap.add_argument("--no-cpu", action="store_true", help="skip the oracle timing")
    ap.add_argument("--split-k", type=int, default=0, help="0 = library default")
    ap.add_argument("--tile-cols", type=int, default=0, help="launch knob of the timed workload (0 = library default)")
    ap.add_argument("--waves", type=int, default=0, help="launch knob of the timed workload (0 = library default)")
    ap.add_argument("--reduce", type=int, default=0,
                    help="reduction flavour of the timed workload, W4A16_REDUCE_* (0 = library default)")
    ap.add_argument("--dp", action="store_true", help="time the data-parallel kernel instead of the SplitK kernel")
    ap.add_argument("--table-steps", type=int, default=400, help="timed calls per entry of the tables")
    ap.add_argument("--shape", default="16,4096,4096",
                    help="m,n,k of the timed workload (default: the headline workload; another shape runs "
                         "without the tables, e.g. for a profile of the streaming kernel)")
    ap.add_argument("--bits", type=int, default=4, choices=(2, 3, 4, 8),
                    help="field width of the timed workload (default 4, the paper's; another width runs "
                         "without the tables and without the CPU leg, e.g. for a profile)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run plain 256 MiB device copies (reference traffic for rocprofv3 counter runs)")
    args = ap.parse_args()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        log("bench.py: this build runs on ONE GPU; the kernel has no multi-GPU path. Use --gpus 1.")
        sys.exit(2)

    import torch

    from paper_2402_00025_amd import binding

    assert torch.cuda.is_available(), "bench.py needs the MI355X"
    binding.lib()
    if args.calibrate_copy:
        calibrate_copy()
    dev_name = torch.cuda.get_device_name(0)
    g = 128
    m, n, k = (int(x) for x in args.shape.split(","))
    width = args.bits   # field width of the timed workload
    knobs = bool(args.tile_cols or args.waves or args.reduce or args.dp)
    if (m, n, k) != (16, 4096, 4096) or width != 4 or knobs:
        args.no_sweep = True   # the tables belong to the headline run
    if width != 4:
        args.no_cpu = True     # the CPU leg is the headline's

    def nsets(n_, k_):
        per = n_ * k_ * width // 8
        return max(2, -(-ROTATE_BYTES // per))

    log(f"[bench] device {dev_name}; building workload m={m} n={n} k={k} ({nsets(n, k)} weight sets)")
    w = Workload(m, n, k, g, nsets(n, k), seed=args.seed, bits=width)
    plan = (binding.w4a16_plan(m, n, k, g, dp=args.dp, split_k=args.split_k, tile_cols=args.tile_cols, waves=args.waves,
                               reduce=args.reduce) if width == 4
            else binding.w4a16_plan_bits(width, m, n, k, g, split_k=args.split_k))

    # oracle: reference for the correctness gate and the CPU baseline
    if args.no_cpu:
        from oracle import w4a16_oracle
        if width == 4:
            Cref, _ = w4a16_oracle.gemm(w.host.A, w.host.qweight, w.host.scales, w.host.qzeros, g)
        elif width == 3:
            Cref, _ = w4a16_oracle.gemm_3bit(w.host.A, w.host.qweight, w.host.scales, w.host.qzeros, g)
        else:
            Cref, _ = w4a16_oracle.gemm_bits(w.host.A, w.host.qweight, w.host.scales, w.host.qzeros, g, width)
        cpu = None
    else:
        Cref, cpu = cpu_baseline(w)
        log(f"[bench] oracle on {cpu['cores']} host threads: {cpu['ms_per_call']:.1f} ms/call = {cpu['value']:.2f} GB/s")

    if width == 4 and args.dp:
        head = make_call(w, "dp", tile_cols=plan["tile_cols"], waves=plan["waves"])
    elif width == 4:
        head = make_call(w, "splitk", split_k=plan["split_k"], tile_cols=plan["tile_cols"], waves=plan["waves"],
                         reduce=plan["reduce"])
    else:
        head = make_call(w, "splitk_bits", split_k=args.split_k)
    ok, rel, emax = verify(w, head, Cref)
    log(f"[bench] parity of the timed configuration: ok={ok} rel_fro={rel:.2e} max_err={emax:.2e}")
    if not ok:
        log("[bench] FAILED parity; refusing to report a number")
        sys.exit(1)

    wall, ev = time_calls(head, args.steps, args.warmup, prewarm_s=0.3)
    wall_eager, ev_eager = time_calls_eager(head, min(args.steps, 400), 50)
    value = w.bytes / wall / 1e9
    achieved = w.bytes / ev / 1e9
    log(f"[bench] splitk S={plan['split_k']}: {wall * 1e6:.2f} us/call wall, {ev * 1e6:.2f} us/launch by events, "
        f"{value:.0f} GB/s ({100 * achieved / HBM_PEAK_GBPS:.1f}% of 8 TB/s)")

    extra = {"device": dev_name, "plan": plan, "paper_context": PAPER_CONTEXT,
             "parity": {"rel_fro": rel, "max_abs_err": emax}, "weight_sets": len(w.sets),
             "us_per_call_wall": wall * 1e6, "us_per_launch_events": ev * 1e6,
             "timing": "calls captured in HIP graphs and replayed (all kernels of every call run)",
             "eager_us_per_call_400_steps": ev_eager * 1e6,
             "eager_note": "eager launches from Python cost the host ~7-8 us per call (two launches), so long eager "
                           "runs of the small shapes are host-bound"}

    # the achievable ceiling on this machine: a plain read of the packed weights alone, same protocol
    ev_read = min(time_calls(make_call(w, "read", split_k=shape), args.table_steps, 50)[1] for shape in range(10))
    packed_bytes = w.sets[0][0].numel() * 4
    extra["plain_read_of_packed_weights"] = {"bytes": packed_bytes, "us_per_launch": ev_read * 1e6,
                                             "note": "best of the probe's ten launch shapes (five, with and without the non-temporal hint)",
                                             "GBps": packed_bytes / ev_read / 1e9,
                                             "frac_of_peak": packed_bytes / ev_read / 1e9 / HBM_PEAK_GBPS,
                                             "gemm_over_read": ev / ev_read}
    log(f"[bench] plain read of the packed weights ({packed_bytes / 2**20:.0f} MiB): {ev_read * 1e6:.2f} us per launch, "
        f"{packed_bytes / ev_read / 1e9:.0f} GB/s; the GEMM takes {ev / ev_read:.2f}x that")

    if not args.no_sweep:
        sweep_steps, sweep_warm = args.table_steps, 50
        big_steps = max(20, args.table_steps // 2)
        # warm (single weight set: cache resident) figure for the headline shape
        w1 = Workload(m, n, k, g, 1, seed=args.seed)
        _, ev_warm = time_calls(make_call(w1, "splitk", split_k=plan["split_k"]), sweep_steps, sweep_warm)
        extra["warm_cache_resident"] = {"us_per_launch": ev_warm * 1e6, "GBps": w.bytes / ev_warm / 1e9,
                                        "note": "one weight set re-read every call: served by L2 / Infinity Cache, not HBM"}
        del w1
        # split_k sweep on the headline shape (configuration 2)
        sk = []
        for S in (1, 2, 4, 8, 16):
            _, e = time_calls(make_call(w, "splitk", split_k=S), sweep_steps, sweep_warm)
            sk.append({"split_k": S, "us": e * 1e6, "GBps": w.bytes / e / 1e9})
        extra["split_k_sweep_m16_nk4096"] = sk
        # configuration 1: m = 1, n = k = 1024, split_k = 4 as given, the library's own choice, and DP
        w1k = Workload(1, 1024, 1024, g, nsets(1024, 1024), seed=args.seed)
        _, e4 = time_calls(make_call(w1k, "splitk", split_k=4), sweep_steps, sweep_warm)
        _, e0 = time_calls(make_call(w1k, "splitk", split_k=0), sweep_steps, sweep_warm)
        _, edp = time_calls(make_call(w1k, "dp"), sweep_steps, sweep_warm)
        extra["cfg1_m1_nk1024"] = {"split_k_4_us": e4 * 1e6, "library_plan_us": e0 * 1e6, "dp_us": edp * 1e6,
                                   "plan_split_4": binding.w4a16_plan(1, 1024, 1024, g, split_k=4),
                                   "plan_library": binding.w4a16_plan(1, 1024, 1024, g),
                                   "GBps_split_k_4": w1k.bytes / e4 / 1e9, "speedup_over_dp": edp / e4,
                                   "note": "0.55 MB per call: a launch-latency measurement, not a bandwidth one"}
        log(f"[bench] m=1 n=k=1024: split_k=4 {e4 * 1e6:.2f} us, library plan {e0 * 1e6:.2f} us, dp {edp * 1e6:.2f} us")
        del w1k
        # The paper's own protocol for the split_k question (Section 3.3): tile, waves and everything
        # else held fixed, only split_k varies; split_k = 1 of that launch is the data-parallel kernel
        # of the comparison (one workgroup per 64-column tile over all of k, stored without atomics).
        fixed_rows = []
        for (mm, nk, splits) in ((16, 4096, (1, 2, 4, 8, 16)), (1, 4096, (1, 2, 4, 8, 16)), (16, 8192, (1, 2, 4, 8, 16, 32)),
                                 (8, 16384, (1, 4, 16, 32))):
            wb = w if (nk == n and mm == m) else Workload(mm, nk, nk, g, nsets(nk, nk), seed=args.seed)
            res = []
            for S in splits:
                _, e = time_calls(make_call(wb, "splitk", split_k=S, tile_cols=64, waves=2), big_steps, 30)
                res.append({"split_k": S, "us": e * 1e6, "GBps": wb.bytes / e / 1e9})
            best = min(res, key=lambda r: r["us"])
            fixed_rows.append({"m": mm, "n": nk, "k": nk, "tile_cols": 64, "waves": 2, "sweep": res,
                               "best_split_k": best["split_k"], "speedup_over_split_k_1": res[0]["us"] / best["us"]})
            log(f"[bench] fixed launch (64 columns, 2 waves) m={mm} n=k={nk}: " +
                ", ".join(f"S={r['split_k']}: {r['us']:.2f}" for r in res) +
                f" us; best S={best['split_k']}, x{res[0]['us'] / best['us']:.2f} over S=1")
            if wb is not w:
                del wb
        extra["split_k_sweep_fixed_launch"] = fixed_rows
        # SplitK vs DP, m in {1,2,4,8,16} x n=k in {4096, 8192} (configuration 3)
        rows = []
        for nk in (4096, 8192):
            wb = w if nk == n else Workload(16, nk, nk, g, nsets(nk, nk), seed=args.seed)
            for mm in (1, 2, 4, 8, 16):
                wm = wb.with_m(mm)
                best = None
                for S in (0, 2, 4, 8, 16):
                    _, e = time_calls(make_call(wm, "splitk", split_k=S), sweep_steps, sweep_warm)
                    if best is None or e < best[1]:
                        best = (S, e)
                _, e_def = time_calls(make_call(wm, "splitk", split_k=0), sweep_steps, sweep_warm)
                _, e_dp = time_calls(make_call(wm, "dp"), sweep_steps, sweep_warm)
                rows.append({"m": mm, "n": nk, "k": nk, "splitk_default_us": e_def * 1e6, "splitk_best_us": best[1] * 1e6,
                             "best_split_k": best[0], "dp_us": e_dp * 1e6, "speedup_over_dp": e_dp / best[1],
                             "splitk_GBps": wm.bytes / best[1] / 1e9, "frac_of_peak": wm.bytes / best[1] / 1e9 / HBM_PEAK_GBPS})
                log(f"[bench] m={mm:2d} n=k={nk}: splitk {best[1] * 1e6:7.2f} us (S={best[0]}), dp {e_dp * 1e6:7.2f} us, "
                    f"x{e_dp / best[1]:.2f}, {wm.bytes / best[1] / 1e9:.0f} GB/s")
            if wb is not w:
                del wb
        extra["splitk_vs_dp"] = rows
        # split_k sweeps of the two large configurations (m=16, 8192^2 and m=8, 16384^2)
        for (mm, nk, splits, key) in ((16, 8192, (1, 2, 4, 8, 16, 32), "split_k_sweep_m16_nk8192"),
                                      (8, 16384, (1, 4, 16, 32), "split_k_sweep_m8_nk16384")):
            wb = Workload(mm, nk, nk, g, nsets(nk, nk), seed=args.seed)
            res = []
            for S in splits:
                _, e = time_calls(make_call(wb, "splitk", split_k=S), big_steps, 30)
                res.append({"split_k": S, "us": e * 1e6, "GBps": wb.bytes / e / 1e9,
                            "frac_of_peak": wb.bytes / e / 1e9 / HBM_PEAK_GBPS})
            _, e_dp = time_calls(make_call(wb, "dp"), big_steps, 30)
            e_rd = min(time_calls(make_call(wb, "read", split_k=shape), big_steps, 30)[1] for shape in range(10))
            extra[key] = {"splitk": res, "dp_us": e_dp * 1e6, "plain_read_of_packed_weights_us": e_rd * 1e6}
            best = min(res, key=lambda r: r["us"])
            log(f"[bench] m={mm} n=k={nk}: best split_k={best['split_k']} {best['us']:.2f} us "
                f"({best['GBps']:.0f} GB/s, {100 * best['frac_of_peak']:.1f}% of peak), dp {e_dp * 1e6:.2f} us, "
                f"plain read of the packed weights {e_rd * 1e6:.2f} us")
            del wb

        # non-square shapes: the linear layers of llama-7B/13B/70B style decoders (fused qkv,
        # gate/up and down projections; k = 11008 and 13824 are 86 and 108 groups of 128)
        rows = []
        for (n_, k_) in ((12288, 4096), (11008, 4096), (4096, 11008), (13824, 5120), (5120, 13824),
                         (28672, 8192), (8192, 28672)):
            wb = Workload(16, n_, k_, g, nsets(n_, k_), seed=args.seed)
            for mm in (1, 16):
                wm = wb.with_m(mm)
                pl = binding.w4a16_plan(mm, n_, k_, g)
                _, e = time_calls(make_call(wm, "splitk", split_k=0), big_steps, 30)
                _, e_dp = time_calls(make_call(wm, "dp"), big_steps, 30)
                _, e_sk = time_calls(make_call(wm, "streamk"), big_steps, 30)
                rows.append({"m": mm, "n": n_, "k": k_, "plan": pl, "splitk_us": e * 1e6, "dp_us": e_dp * 1e6,
                             "streamk_us": e_sk * 1e6, "speedup_over_dp": e_dp / e, "splitk_GBps": wm.bytes / e / 1e9,
                             "frac_of_peak": wm.bytes / e / 1e9 / HBM_PEAK_GBPS})
                log(f"[bench] m={mm:2d} n={n_} k={k_}: splitk {e * 1e6:7.2f} us (S={pl['split_k']}, tile {pl['tile_cols']}), "
                    f"dp {e_dp * 1e6:7.2f} us, x{e_dp / e:.2f}, streamk {e_sk * 1e6:7.2f} us, {wm.bytes / e / 1e9:.0f} GB/s")
            del wb
        extra["decoder_projection_shapes"] = rows
        # more than 16 rows: row tiles of one launch (up to 64 rows share one pass over the weights)
        rows = []
        wb = Workload(64, 8192, 8192, g, nsets(8192, 8192), seed=args.seed)
        for mm in (16, 32, 48, 64):
            wm = wb.with_m(mm)
            _, e = time_calls(make_call(wm, "splitk", split_k=0), big_steps, 30)
            rows.append({"m": mm, "n": 8192, "k": 8192, "splitk_us": e * 1e6, "splitk_GBps": wm.bytes / e / 1e9,
                         "TFLOPs": 2.0 * mm * 8192 * 8192 / e / 1e12})
            log(f"[bench] m={mm:2d} n=k=8192: splitk {e * 1e6:7.2f} us, {wm.bytes / e / 1e9:.0f} GB/s, "
                f"{2.0 * mm * 8192 * 8192 / e / 1e12:.0f} TFLOP/s")
        del wb
        extra["row_tiles_nk8192"] = rows
        # 8-bit, 3-bit and 2-bit fields through the same kernels (2, 3/4 and 1/2 of the weight bytes per call)
        rows = []
        for bits in (8, 3, 2):
            # (8-bit fields also at 16384: 256 MiB of weights, the largest stream any of the kernels sees)
            for nk in (4096, 8192) + ((16384,) if bits == 8 else ()):
                wb = Workload(16, nk, nk, g, max(2, -(-ROTATE_BYTES // (nk * nk * bits // 8))), seed=args.seed, bits=bits)
                for mm in (1, 16):
                    wm = wb.with_m(mm)
                    _, e = time_calls(make_call(wm, "splitk_bits", split_k=0), big_steps, 30)
                    _, e_dp = time_calls(make_call(wm, "dp_bits"), big_steps, 30)
                    rows.append({"m": mm, "n": nk, "k": nk, "bits": bits, "splitk_us": e * 1e6, "dp_us": e_dp * 1e6,
                                 "splitk_GBps": wm.bytes / e / 1e9, "frac_of_peak": wm.bytes / e / 1e9 / HBM_PEAK_GBPS})
                    log(f"[bench] {bits}-bit m={mm:2d} n=k={nk}: splitk {e * 1e6:7.2f} us, dp {e_dp * 1e6:7.2f} us, "
                        f"{wm.bytes / e / 1e9:.0f} GB/s")
                del wb
        extra["other_field_widths"] = rows
        # activation ordering on the headline shape: rows sorted by group once, activations gathered per call
        kk = w.k
        rng = np.random.Generator(np.random.Philox(args.seed + 17))
        order = rng.permutation(kk).astype(np.int32)
        g_idx = np.empty(kk, np.int32)
        g_idx[order] = np.arange(kk, dtype=np.int32) // g
        d_gidx = torch.from_numpy(g_idx).cuda()
        perm = torch.empty(kk, dtype=torch.int32, device="cuda")
        status = torch.zeros(1, dtype=torch.int32, device="cuda")
        A_work = torch.empty_like(w.A)
        sorted_sets = []
        for (qw_t, s_t, qz_t) in w.sets:
            qs = torch.empty_like(qw_t)
            binding.w4a16_actorder_prepare(qw_t, d_gidx, qs, perm, status, w.n, kk, g)
            sorted_sets.append((qs, s_t, qz_t))
        torch.cuda.synchronize()
        assert int(status.item()) == 0
        L = binding.lib()
        import ctypes
        vp = ctypes.c_void_p
        ptrs = [tuple(vp(t.data_ptr()) for t in st) for st in sorted_sets]

        def call_actorder(i):
            qs, sc, qz = ptrs[i % len(ptrs)]
            rc = L.w4a16_gemm_actorder(vp(w.A.data_ptr()), qs, sc, qz, vp(perm.data_ptr()), vp(A_work.data_ptr()),
                                       vp(w.C.data_ptr()), w.m, w.n, kk, g, 0, vp(torch.cuda.current_stream().cuda_stream))
            if rc:
                raise binding.W4A16Error(rc, "w4a16_gemm_actorder")
        call_actorder.nsets = len(ptrs)
        _, e_ao = time_calls(call_actorder, sweep_steps, sweep_warm)
        extra["activation_ordering_m16_nk4096"] = {"us_per_call": e_ao * 1e6, "plain_us_per_call": ev * 1e6,
                                                   "note": "one more small launch per call (the gather of A[:, perm])"}
        log(f"[bench] activation ordering m={w.m} n=k={w.n}: {e_ao * 1e6:.2f} us per call against {ev * 1e6:.2f} plain")
        del sorted_sets

    out = {
        "metric": "effective HBM bandwidth of the fused W4A16 SplitK GEMM call (algorithmic bytes / time per call)",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": wall * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": f"f16 x int{width} -> f32 accumulate", "data": "synthetic",
        "config": {"workload": f"m={m}, n={n}, k={k}, group_size={g}, {width}-bit fields, split_k={plan['split_k']}, "
                               f"tile_cols={plan['tile_cols']}, weights rotated over {len(w.sets)} sets (cold HBM)", "seed": args.seed},
        "roofline": {"bound": "hbm", "achieved": achieved, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": achieved / HBM_PEAK_GBPS, "traffic": measured_traffic(m, n, k, width),
                     "kernel": "w4a16::gemm_stream_kernel (SplitK)" if plan["tile_cols"] == 256 else "w4a16::gemm_kernel (SplitK)", "algorithmic_bytes_per_launch": w.bytes},
        "cpu_baseline": cpu,
        "kernel_source_id": kernel_source_id(),
        "extra": extra,
    }
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
