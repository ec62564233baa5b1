#!/usr/bin/env python3
"""Runs one lutq_matmul configuration repeatedly on a ring of weight buffers larger than the caches and
prints its time per call -- the program to put after `rocprofv3 ... --` when one kernel instance is to
be profiled (kernel trace or counters) without the rest of bench.py around it.

  python -m paper_2407_10960_amd.run_case --shape 28672x4096 --bits 4 --group 128 --dtype f16 --m 32

Weights, scales and activations are random (the kernel's time does not depend on the values).
"""
from __future__ import annotations

import argparse
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--shape", required=True, help="NxK, e.g. 28672x4096")
    ap.add_argument("--bits", type=int, default=4)
    ap.add_argument("--group", type=int, default=128)
    ap.add_argument("--dtype", default="f16", choices=("f16", "bf16"))
    ap.add_argument("--m", type=int, default=1)
    ap.add_argument("--calls", type=int, default=200, help="timed calls (after as many untimed ones)")
    ap.add_argument("--plan", default="", help="R/grid/waves/tiles_in_flight/row_groups[/scheduling/tiles_per_item]; empty = default")
    ap.add_argument("--channel", action="store_true", help="lutq_matmul_channel (one table per output row)")
    args = ap.parse_args()
    import torch
    import paper_2407_10960_amd as lutq
    torch.cuda.set_device(0)
    lutq.load_library()
    N, K = (int(v) for v in args.shape.lower().split("x"))
    tdt = torch.float16 if args.dtype == "f16" else torch.bfloat16
    pb = lutq.lutq_packed_bytes(N, K, args.bits, args.group)
    ring = max(2, min(32, int(1.5e9 // pb) + 1))
    pk = [torch.randint(0, 256, (pb,), dtype=torch.uint8, device="cuda") for _ in range(ring)]
    S = (torch.rand((N, K // args.group), device="cuda") * 0.01 + 0.01).to(tdt)
    E = 1 << args.bits
    T = (torch.randn((N, E), device="cuda") * 0.5).to(tdt) if args.channel else torch.linspace(-1, 1, E, device="cuda").to(tdt)
    X = torch.randn((args.m, K), device="cuda").to(tdt)
    Y = torch.empty((args.m, N), dtype=tdt, device="cuda")
    ws = lutq.new_workspace(N, K, args.bits, args.group)
    plan = lutq.Plan(*[int(v) for v in args.plan.split("/")]) if args.plan else None

    def call(i):
        if args.channel:
            lutq.lutq_matmul_channel(X, pk[i % ring], S, T, args.bits, args.group, Y, ws)
        else:
            lutq.lutq_matmul(X, pk[i % ring], S, T, args.bits, args.group, Y, ws, plan=plan)

    for i in range(args.calls):
        call(i)
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for i in range(args.calls):
        call(i)
    e1.record()
    torch.cuda.synchronize()
    dp = lutq.lutq_plan_default(args.bits, args.group, args.m, N, K, 0 if args.dtype == "f16" else 1)
    print(f"N={N} K={K} bits={args.bits} group={args.group} {args.dtype} M={args.m} ring={ring} plan={plan or dp}: "
          f"{e0.elapsed_time(e1) * 1e3 / args.calls:.2f} us per call (launched from Python one by one: includes the host's launch time)")


if __name__ == "__main__":
    main()
