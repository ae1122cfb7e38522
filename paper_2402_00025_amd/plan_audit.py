"""Audit of the library's launch plan on an MI355X: for a set of shapes, time every launch the
kernels offer (per-wave kernel with 16- to 64-column tiles, two strips per wave, streaming
kernel; every split_k that fits) and compare the best of them with the launch `split_k = 0`
chooses.  This is the measurement the plan's rules are fitted to and checked against.

    python -m paper_2402_00025_amd.plan_audit --random 40 --seed 1 --out profiles/plan_audit_seed1.txt
    python -m paper_2402_00025_amd.plan_audit --shapes 16,4096,4096 8,11008,4096
    python -m paper_2402_00025_amd.plan_audit --bits 8 --random 20 --seed 3

With --bits 8, 3 or 2 the candidates are the launches the entry points of that width expose: the
per-wave kernel with every split_k that divides k into whole groups (an explicit split_k never
selects the two-strip or the streaming kernel there), so the table bounds the plan from one side only.

Timing protocol: calls captured in a HIP graph over a rotation of weight sets (at least 512 MiB, so
the weights come from HBM), replayed 12 times, median of the HIP-event time per call.  The
output is a text table: one line per shape with the plan's launch, its time, the best candidate
and the ratio, then the candidates' times.
"""
from __future__ import annotations

import argparse
import ctypes
import statistics
import sys

import numpy as np

ROTATE_BYTES = 512 << 20


def candidates(binding, m, n, k, g=128):
    """Every (split_k, tile_cols, waves) the library accepts for this shape, as dicts."""
    groups = k // min(g, 128)
    out, seen = [], set()

    def add(split_k, tile_cols, waves):
        try:
            pl = binding.w4a16_plan(m, n, k, g, split_k=split_k, tile_cols=tile_cols, waves=waves)
        except binding.W4A16Error:
            return
        key = (pl["split_k"], pl["tile_cols"], pl["waves"], pl["reduce"])
        tiles = -(-n // pl["tile_cols"])
        if key in seen or not (96 <= tiles * pl["split_k"] <= 1100):
            return
        seen.add(key)
        out.append(pl)

    splits = [s for s in (1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16, 20, 24, 27, 32, 48, 64) if s <= groups]
    for s in splits:
        for w in (1, 2, 4) + ((8, 16) if g < 128 else ()):  # (short groups: larger workgroups as well)
            if s * w <= groups:
                add(s, 64, w)
        add(s, 256, 4)
        if groups % (2 * s) == 0:
            add(s, 256, 8)
    for w in (4, 2, 1):
        if groups % w == 0 and 2 <= groups // w <= 64:
            add(groups // w, 128, w)
    for tc in (16, 32):
        for w in (4, 8, 16):
            if w <= groups:
                add(1, tc, w)
    return out


def candidates_bits(binding, bits, m, n, k, g=128):
    """The other field widths: every explicit split_k their entry points accept, as dicts."""
    out = []
    for s in (1, 2, 3, 4, 5, 6, 7, 8, 10, 12, 14, 16, 20, 24, 27, 32, 48, 64):
        try:
            pl = binding.w4a16_plan_bits(bits, m, n, k, g, split_k=s)
        except binding.W4A16Error:
            continue
        if 96 <= -(-n // pl["tile_cols"]) * pl["split_k"] <= 1100:
            out.append(dict(pl, ask=s))
    return out


class Problem:
    def __init__(self, torch, m, n, k, g=128, seed=0, bits=4):
        per = n * k * bits // 8
        sets = max(2, -(-ROTATE_BYTES // per))
        gen = torch.Generator(device="cuda").manual_seed(seed)
        self.A = torch.randn((m, k), device="cuda", dtype=torch.float16, generator=gen)
        self.C = torch.empty((m, n), device="cuda", dtype=torch.float16)
        self.sets = []
        for _ in range(sets):
            # (every bit pattern is a valid word at every width)
            qw = torch.randint(-2 ** 31, 2 ** 31 - 1, (k * bits // 32, n), device="cuda", dtype=torch.int32, generator=gen)
            sc = (torch.rand((k // g, n), device="cuda", generator=gen) * 0.009 + 0.001).to(torch.float16)
            qz = torch.randint(-2 ** 31, 2 ** 31 - 1, (k // g, n * bits // 32), device="cuda", dtype=torch.int32, generator=gen)
            self.sets.append((qw, sc, qz))
        self.m, self.n, self.k, self.g, self.bits = m, n, k, g, bits


def time_launch(torch, binding, p: Problem, pl, replays=12):
    """Median HIP-event microseconds per call of one launch shape; None if the library refuses it."""
    L = binding.lib()
    vp = ctypes.c_void_p
    A, C = vp(p.A.data_ptr()), vp(p.C.data_ptr())
    ptrs = [tuple(vp(t.data_ptr()) for t in s) for s in p.sets]
    count = max(len(ptrs), 32)

    gemm_bits = {4: None, 8: L.w8a16_gemm, 3: L.w3a16_gemm, 2: L.w2a16_gemm}[p.bits]

    def call(i, stream):
        qw, sc, qz = ptrs[i % len(ptrs)]
        if gemm_bits is not None:  # `ask`: the split_k argument (0 = the library's plan)
            return gemm_bits(A, qw, sc, qz, C, p.m, p.n, p.k, p.g, pl["ask"], vp(stream.cuda_stream))
        return L.w4a16_gemm_ex(A, qw, sc, qz, C, p.m, p.n, p.k, p.g, pl["split_k"], pl["tile_cols"], pl["waves"],
                               pl["reduce"], vp(stream.cuda_stream))

    cur = torch.cuda.current_stream()
    for i in range(3):
        if call(i, cur) != 0:
            return None
    torch.cuda.synchronize()
    side = torch.cuda.Stream()
    side.wait_stream(cur)
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        for i in range(count):
            call(i, torch.cuda.current_stream())
    for _ in range(3):
        graph.replay()
    torch.cuda.synchronize()
    times = []
    for _ in range(replays):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        graph.replay()
        e1.record()
        torch.cuda.synchronize()
        times.append(e0.elapsed_time(e1) * 1e3 / count)
    del graph
    return statistics.median(times)


def random_shapes(count, seed):
    rng = np.random.Generator(np.random.Philox(seed))
    out = []
    for _ in range(count):
        n = int(rng.integers(128, 3600)) * 8
        k = int(rng.integers(8, 120)) * 128
        m = int(rng.choice([1, 2, 4, 6, 8, 12, 16]))
        if n * k // 2 > (160 << 20):
            k = max(1024, ((160 << 20) * 2 // n) // 128 * 128)
        out.append((m, n, k))
    return out


STRUCTURED = [(m, nk, nk) for nk in (4096, 8192) for m in (1, 4, 16)] + [(8, 16384, 16384)] + \
             [(m, n, k) for (n, k) in ((12288, 4096), (11008, 4096), (4096, 11008), (13824, 5120), (5120, 13824), (28672, 8192),
                                       (8192, 28672)) for m in (1, 16)]


def fmt(pl):
    return f"S{pl['split_k']}/t{pl['tile_cols']}/w{pl['waves']}/r{pl['reduce']}"


def main(argv=None):
    ap = argparse.ArgumentParser(description=__doc__, formatter_class=argparse.RawDescriptionHelpFormatter)
    ap.add_argument("--shapes", nargs="*", default=[], help="m,n,k triples")
    ap.add_argument("--structured", action="store_true", help="the square and decoder-projection shapes of the bench")
    ap.add_argument("--random", type=int, default=0, help="number of random shapes")
    ap.add_argument("--seed", type=int, default=1)
    ap.add_argument("--bits", type=int, default=4, choices=(2, 3, 4, 8), help="width of the packed fields")
    ap.add_argument("--group-size", type=int, default=128, choices=(32, 64, 128, 256), help="quantisation group size")
    ap.add_argument("--keep", type=int, default=8, help="candidates listed per shape, fastest first")
    ap.add_argument("--out", default=None, help="write the table here as well")
    args = ap.parse_args(argv)

    import torch

    from . import binding

    assert torch.cuda.is_available(), "plan_audit needs the GPU"
    shapes = [tuple(int(x) for x in s.split(",")) for s in args.shapes]
    if args.structured:
        shapes += STRUCTURED
    shapes += random_shapes(args.random, args.seed)
    bits = args.bits
    g = args.group_size
    lines = [f"# plan audit: {len(shapes)} shapes, group_size {g}, {bits}-bit fields; us per call (cold weights, median of 12 graph replays)",
             f"# command: python -m paper_2402_00025_amd.plan_audit {' '.join(sys.argv[1:] if argv is None else argv)}",
             "# shape m,n,k | plan launch, us | best launch, us | plan/best | the fastest candidates: launch=us",
             *(["# candidates: the per-wave kernel at every explicit split_k this width's entry point accepts"] if bits != 4 else []),
             "# launch = S<split_k>/t<tile_cols>/w<waves>/r<reduce>"]
    ratios = []
    for (m, n, k) in shapes:
        if bits != 4:
            n = -(-n // 32) * 32  # (3-bit fields need whole streams of 32 columns; kept for all three so that they share shapes)
        if m < 1 or n < 8 or n % 8 or k < 128 or k % 128:
            raise SystemExit(f"shape {m},{n},{k}: need m >= 1, n a multiple of 8, k a multiple of 128")
        p = Problem(torch, m, n, k, g=g, bits=bits)
        if bits == 4:
            plan = binding.w4a16_plan(m, n, k, g)
            cands = candidates(binding, m, n, k, g)
        else:
            plan = dict(binding.w4a16_plan_bits(bits, m, n, k, g), ask=0)
            cands = candidates_bits(binding, bits, m, n, k, g)
        if all(fmt(c) != fmt(plan) for c in cands):
            cands.append(plan)
        res = []
        for c in cands:
            t = time_launch(torch, binding, p, c)
            if t is not None:
                res.append((t, c))
        # the plan's own launch once more at the end: the two measurements bracket the drift over the sweep
        again = time_launch(torch, binding, p, plan)
        t_plan = min([t for (t, c) in res if fmt(c) == fmt(plan)] + ([again] if again is not None else []))
        res.sort(key=lambda r: r[0])
        best_t, best = res[0]
        ratios.append(t_plan / min(best_t, t_plan))
        line = (f"{m},{n},{k} | {fmt(plan)} {t_plan:.2f} | {fmt(best)} {best_t:.2f} | {t_plan / min(best_t, t_plan):.3f} | " +
                " ".join(f"{fmt(c)}={t:.2f}" for (t, c) in res[:args.keep]) +
                (f" (+{len(res) - args.keep} slower)" if len(res) > args.keep else ""))
        lines.append(line)
        print(line[:200], flush=True)
        del p
        torch.cuda.empty_cache()
    gm = float(np.exp(np.mean(np.log(ratios))))
    lines.append(f"# plan / best: geometric mean {gm:.4f}, worst {max(ratios):.3f}, within 3 % on {sum(r <= 1.03 for r in ratios)} of {len(ratios)} shapes")
    print(lines[-1], flush=True)
    if args.out:
        with open(args.out, "w") as f:
            f.write("\n".join(lines) + "\n")


if __name__ == "__main__":
    main()
