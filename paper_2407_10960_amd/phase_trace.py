#!/usr/bin/env python3
"""Where the time of one lutq_matmul launch goes (M = 1, 4-bit, the LLaMA-3 8B and 70B layer shapes).

Runs every shape through the measurement build of the fused kernel (lutq_calib_matmul_trace): every
wavefront reads the device's constant 100 MHz clock at eight points of the kernel.  32 launches on
distinct weight buffers (HBM-cold) are captured into one HIP graph, as bench.py replays its calls, so
that the idle time between two dependent launches is part of the record.  Prints one table per shape:
for every wave index of a workgroup the time, since the launch's first wave started, at which the wave
reached each point (median over the workgroups and launches of the last replay), in microseconds.

Usage: python -m paper_2407_10960_amd.phase_trace [--dtype f16|bf16] [--shapes 8b,70b]
"""
from __future__ import annotations

import argparse
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

SHAPES = {
    "8b": (128, {"qkv": (6144, 4096), "o": (4096, 4096), "gate_up": (28672, 4096), "down": (4096, 14336)}),
    "70b": (64, {"qkv": (10240, 8192), "o": (8192, 8192), "gate_up": (57344, 8192), "down": (8192, 28672)}),
}
LAUNCHES = 32
WAVE_SLOTS = 16
TICK_US = 0.01          # one tick of the 100 MHz clock


def q(v, f):
    v = np.sort(v)
    return float(v[min(len(v) - 1, int(f * len(v)))])


def trace_shape(lutq, torch, name, N, K, group, tdt, out):
    bits, M = 4, 1
    pb = lutq.lutq_packed_bytes(N, K, bits, group)
    ring = max(2, min(LAUNCHES, int(1.5e9 // pb) + 1))
    pk = [torch.randint(0, 256, (pb,), dtype=torch.uint8, device="cuda") for _ in range(ring)]
    S = (torch.rand((N, K // group), device="cuda") * 0.01 + 0.01).to(tdt)
    T = torch.linspace(-1, 1, 1 << bits, device="cuda").to(tdt)
    X = torch.randn((M, K), device="cuda").to(tdt)
    Y = torch.empty((M, N), dtype=tdt, device="cuda")
    ws = lutq.new_workspace(N, K, bits, group)
    plan = lutq.lutq_plan_default(bits, group, M, N, K, 0 if tdt == torch.float16 else 1)
    tr = torch.zeros((LAUNCHES, plan.grid, WAVE_SLOTS, 8), dtype=torch.int64, device="cuda")
    groups = [0]

    def traced():
        for i in range(LAUNCHES):
            groups[0] = lutq.calib_matmul_trace(X, pk[i % ring], S, T, bits, group, Y, ws, tr[i])

    def plain():
        for i in range(LAUNCHES):
            lutq.lutq_matmul(X, pk[i % ring], S, T, bits, group, Y, ws)

    def capture(fn):
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g

    gt, gp = capture(traced), capture(plain)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    times = {}
    for label, g in (("plain", gp), ("traced", gt)):
        for _ in range(100):                       # clocks up
            g.replay()
        torch.cuda.synchronize()
        e0.record()
        for _ in range(20):
            g.replay()
        e1.record()
        torch.cuda.synchronize()
        times[label] = e0.elapsed_time(e1) * 1e3 / (20 * LAUNCHES)
    G, NW = groups[0], plan.waves_per_workgroup
    assert G == plan.grid
    h = tr[:, :, :NW].cpu().numpy().astype(np.float64) * TICK_US          # [launch][workgroup][wave][stamp]
    names = lutq.TRACE_STAMPS
    out.append(f"## {name}: N={N} K={K} W4 g{group} {str(tdt).split('.')[-1]} M=1; plan R={plan.row_blocks_per_wave} "
               f"grid={plan.grid} waves={NW} teams={plan.row_groups_per_workgroup}; "
               f"{times['plain']:.2f} us per call in the replayed graph (measurement build: {times['traced']:.2f} us)")
    base = h[:, :, :, 0].min(axis=(1, 2))                                  # first wave start of each launch
    end = h[:, :, :, 7].max(axis=(1, 2))
    gaps = base[1:] - end[:-1]
    out.append(f"first wave start to last wave end: median {np.median(end - base):.2f} us; "
               f"previous launch's last end to this launch's first start: median {np.median(gaps):.2f} us")
    rel = h[1:] - base[1:, None, None, None]                               # launches 1..: us since the launch's first start
    rel[h[1:] == 0] = np.nan                                               # a point a wave never reached (a wave that got no work)

    def med(col):
        col = col[~np.isnan(col)]
        return f"{np.median(col):12.2f}" if col.size else f"{'-':>12s}"
    out.append("us since the launch's first wave started, median over workgroups (last column: 90 % quantile of the end)")
    out.append("wave   " + " ".join(f"{n[:12]:>12s}" for n in names) + "      end p90")
    for w in range(NW):
        v = rel[:, :, w, :].reshape(-1, 8)
        out.append(f"{w:4d}   " + " ".join(med(v[:, i]) for i in range(8)) + f" {q(v[:, 7], 0.9):12.2f}")
    v = rel.reshape(-1, 8)
    out.append(" all   " + " ".join(med(v[:, i]) for i in range(8)) + f" {q(v[:, 7], 0.9):12.2f}")
    out.append("")


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--dtype", default="f16", choices=("f16", "bf16"))
    ap.add_argument("--shapes", default="8b,70b")
    args = ap.parse_args()
    import torch
    import paper_2407_10960_amd as lutq
    torch.cuda.set_device(0)
    lutq.load_library()
    tdt = torch.float16 if args.dtype == "f16" else torch.bfloat16
    out = []
    for fam in args.shapes.split(","):
        group, shapes = SHAPES[fam]
        for name, (N, K) in shapes.items():
            trace_shape(lutq, torch, f"llama3-{fam} {name}", N, K, group, tdt, out)
            print("\n".join(out), flush=True)
            out.clear()


if __name__ == "__main__":
    main()
