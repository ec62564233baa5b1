#!/usr/bin/env python3
"""Benchmark of the LUT-quantised matmul hot path on one MI355X.

A step is one decode token's pass through the quantised linear layers of a LLaMA-3-8B-shaped model:
32 layers x [fused QKV (6144x4096), O (4096x4096), fused gate+up (28672x4096), down (4096x14336)],
4-bit NormalFloat table, group 128, fp16, M = 1 -- 128 calls of lutq_matmul on 128 distinct weight
buffers (3.4 GB), so every call streams its weights from HBM.  Inputs are synthetic and seeded
(lutq_inputs.py); one layer is quantised on the host and its packed bytes are replicated on the
device for the other layers.

Prints ONE JSON line.  `value` is the whole step's algorithmic bytes (packed weights + scales + X + Y)
divided by the step time.  `roofline` prices the fused kernel against the 8 TB/s HBM peak with HIP
events over the same timed region; `cpu_baseline` times the CPU oracle on a bounded sample.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import lutq_inputs as gen  # noqa: E402

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of this workload (fetched + written), from the FETCH_SIZE / WRITE_SIZE counter runs
# summarised in profiles/matmul_kernel_llama3_8b_w4g128_m1_hbm_traffic.txt (counters scaled by a copy
# kernel of known size).  A counter run cannot be made from inside this script; the figure belongs to
# this exact workload and is reported as measured there.
MEASURED_TRAFFIC_BYTES_PER_LAUNCH = 28.35e6
LAYERS = 32
BITS, GROUP, DTYPE, M = 4, 128, "f16", 1


def _to_dev(bits_u16, torch):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16).copy()).view(torch.float16).cuda()


def build_layer(lutq, torch, seed):
    """One layer's four quantised matrices (host-quantised, seeded), uploaded once."""
    mats = {}
    for i, (name, (N, K)) in enumerate(gen.LLAMA3_8B_SHAPES.items()):
        c = gen.make_case(seed * 16 + i, M, N, K, BITS, GROUP, DTYPE, "nf")
        packed = torch.from_numpy(lutq.lutq_pack(c.Q, BITS, GROUP)).cuda()
        mats[name] = dict(N=N, K=K, case=c, packed=packed, S=_to_dev(c.S, torch), T=_to_dev(c.T, torch),
                          X=_to_dev(c.X, torch))
    return mats


def warm(torch, fn, seconds=0.1):
    """Runs fn (untimed) for a while: after any idle period the GPU needs some tens of milliseconds of
    load before its clocks are back up, and a single replay is far shorter than that."""
    torch.cuda.synchronize()
    t = time.perf_counter()
    while time.perf_counter() - t < seconds:
        fn()
        torch.cuda.synchronize()


def time_region(torch, fn, iters):
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    torch.cuda.synchronize()
    e0.record()
    for _ in range(iters):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / iters          # seconds per iteration


def cpu_baseline(case, budget_s=12.0):
    """The oracle as it stands, on the host cores, on the O-projection shape of the same workload."""
    from oracle import lutq_oracle as orc
    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
    except Exception:
        threads = os.cpu_count() or 1
    packed = orc.pack(case.Q, case.bits)
    t0 = time.perf_counter()
    n = 0
    while True:
        orc.lut_matmul(case.X, packed, case.S, case.T, case.bits, case.group_size, case.N, case.K, case.dtype)
        n += 1
        if time.perf_counter() - t0 > budget_s:
            break
    dt = (time.perf_counter() - t0) / n
    by = gen.algorithmic_bytes(case.M, case.N, case.K, case.bits, case.group_size)
    return {"value": by / dt * 1e-9, "unit": "GB/s", "cores": int(threads), "kind": "oracle",
            "sample": f"{n} calls of the numpy oracle (unpack + table lookup + scale + fp64 matmul) on the "
                      f"O-projection shape N={case.N} K={case.K} M={case.M} W4 g128; {dt * 1e3:.0f} ms per call; "
                      f"only the fp64 matmul step is multi-threaded"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the per-shape table and the dense fp16 comparison")
    ap.add_argument("--pmc-calib", action="store_true",
                    help="also launch the plain copy kernel on 256 MiB a few times, so that a counter run "
                         "(rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE) holds a dispatch of known traffic to scale by")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on exactly one GPU (the path has no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch
    import paper_2407_10960_amd as lutq
    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(2)
    torch.cuda.set_device(0)
    lutq.load_library()          # fails loudly if liblutq.so is missing: there is no fallback path

    layer0 = build_layer(lutq, torch, seed=0)
    names = list(layer0.keys())
    # 32 layers of distinct device buffers (replicas of layer 0's bytes: only the addresses matter for HBM)
    layers = []
    for li in range(LAYERS):
        L = {}
        for n in names:
            m = layer0[n]
            L[n] = dict(packed=m["packed"] if li == 0 else m["packed"].clone(),
                        S=m["S"] if li == 0 else m["S"].clone())
        layers.append(L)
    Y = {n: torch.empty((M, layer0[n]["N"]), dtype=torch.float16, device="cuda") for n in names}
    ws = lutq.new_workspace(28672, 4096, BITS, GROUP)

    def one_call(n, li):
        m = layer0[n]
        lutq.lutq_matmul(m["X"], layers[li][n]["packed"], layers[li][n]["S"], m["T"], BITS, GROUP, Y[n], ws)

    def step_direct():
        for li in range(LAYERS):
            for n in names:
                one_call(n, li)

    step_bytes = LAYERS * sum(gen.algorithmic_bytes(M, layer0[n]["N"], layer0[n]["K"], BITS, GROUP) for n in names)
    launches = LAYERS * len(names)

    step_direct()          # first launches: module load, device query
    torch.cuda.synchronize()
    if args.pmc_calib:
        src = torch.empty(256 << 20, dtype=torch.uint8, device="cuda").random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(4):
            lutq.calib_copy(src, dst, 2048)
        torch.cuda.synchronize()
        del src, dst

    use_graph = not args.no_graph

    def capture(fn):
        """A HIP graph of fn's launches (replayed as one unit: no per-call Python or launch-API time)."""
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

    step = capture(step_direct).replay if use_graph else step_direct

    for _ in range(args.warmup):
        step()
    # the GPU raises its clocks only after some tens of milliseconds of load: keep warming up (untimed)
    # until the step time has had that long to settle, whatever --warmup says
    warm(torch, step, 0.15)
    sec = time_region(torch, step, args.steps)
    value = step_bytes / sec * 1e-9
    per_launch_s = sec / launches
    roof_achieved = (step_bytes / launches) / per_launch_s * 1e-9

    out = {
        "metric": "effective HBM GB/s of LUT-GEMM (packed weights + scales + X + Y bytes per call / time), M=1",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "llama3-8b decode linears, W4 NormalFloat table g128 fp16 M=1: 32 layers x "
                               "[qkv 6144x4096, o 4096x4096, gate_up 28672x4096, down 4096x14336] = 128 lutq_matmul "
                               "calls per step on 128 distinct weight buffers (3.4 GB, HBM-cold)",
                   "bits": BITS, "group_size": GROUP, "M": M, "launch": "hipgraph replay" if use_graph else "python loop",
                   "calls_per_step": launches, "bytes_per_step": step_bytes,
                   "percent_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "achieved": roof_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": roof_achieved / HBM_PEAK_GBS, "traffic": MEASURED_TRAFFIC_BYTES_PER_LAUNCH,
                     "kernel": "lutq::matmul_kernel<4,128,1,1,F16,2,true,4,true,0,false> (all 128 launches of the step)",
                     "bytes_per_launch": step_bytes / launches, "us_per_launch": per_launch_s * 1e6},
    }

    if not args.no_extras:
        per_shape = {}
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        for n in names:
            m = layer0[n]
            N, K = m["N"], m["K"]
            by = gen.algorithmic_bytes(M, N, K, BITS, GROUP)

            def shape_pass(n=n):
                for li in range(LAYERS):
                    one_call(n, li)
            run = capture(shape_pass).replay if use_graph else shape_pass
            warm(torch, run)
            t = time_region(torch, run, 10) / LAYERS
            # a plain streaming read of the same packed bytes (no table, no arithmetic): what one launch
            # per call can reach on this shape at all
            def read_pass(n=n):
                for li in range(LAYERS):
                    lutq.calib_stream_read(layers[li][n]["packed"], 512, sink)
            rrun = capture(read_pass).replay if use_graph else read_pass
            warm(torch, rrun)
            tr = time_region(torch, rrun, 10) / LAYERS
            # dense fp16 GEMM on the same shape (torch.mm -> hipBLASLt/rocBLAS), ring of weights > 1 GB
            dense_bytes = N * K * 2
            ring = max(2, min(LAYERS, int(1.3e9 // dense_bytes) + 1))
            Wd = [torch.randn((N, K), dtype=torch.float16, device="cuda") * 0.02 for _ in range(ring)]
            Yd = torch.empty((M, N), dtype=torch.float16, device="cuda")

            def dense_pass(Wd=Wd, Yd=Yd, m=m):
                for w in Wd:
                    torch.mm(m["X"], w.t(), out=Yd)
            drun = capture(dense_pass).replay if use_graph else dense_pass
            warm(torch, drun)
            td = time_region(torch, drun, 10) / ring
            # hot regime: the same weight buffer on every call (what a repetition loop over one matrix
            # measures: the small shapes then come from the caches, not from HBM)
            def hot_pass(n=n):
                for _ in range(LAYERS):
                    one_call(n, 0)
            hrun = capture(hot_pass).replay if use_graph else hot_pass
            warm(torch, hrun)
            th = time_region(torch, hrun, 10) / LAYERS
            per_shape[n] = {"N": N, "K": K, "us": t * 1e6, "GBps": by / t * 1e-9, "frac_of_8TBps": by / t * 1e-9 / HBM_PEAK_GBS,
                            "TFLOPs": 2.0 * M * N * K / t * 1e-12, "dense_fp16_us": td * 1e6, "speedup_vs_dense_fp16": td / t,
                            "stream_read_us": tr * 1e6, "stream_read_GBps": m["packed"].numel() / tr * 1e-9,
                            "hot_us": th * 1e6, "hot_GBps": by / th * 1e-9}
            # the other batch sizes of the metric (M = 2..32) on the same cold rings, each beside the dense GEMM
            by_m = {}
            for m2 in (2, 4, 8, 16, 32):
                X2 = torch.randn((m2, K), device="cuda").to(torch.float16)
                Y2 = torch.empty((m2, N), dtype=torch.float16, device="cuda")
                Yd2 = torch.empty((m2, N), dtype=torch.float16, device="cuda")

                def m_pass(n=n, X2=X2, Y2=Y2):
                    for li in range(LAYERS):
                        lutq.lutq_matmul(X2, layers[li][n]["packed"], layers[li][n]["S"], m["T"], BITS, GROUP, Y2, ws)

                def dense_m_pass(Wd=Wd, X2=X2, Yd2=Yd2):
                    for w in Wd:
                        torch.mm(X2, w.t(), out=Yd2)
                mrun = capture(m_pass).replay if use_graph else m_pass
                warm(torch, mrun)
                tm = time_region(torch, mrun, 10) / LAYERS
                dmrun = capture(dense_m_pass).replay if use_graph else dense_m_pass
                warm(torch, dmrun)
                tdm = time_region(torch, dmrun, 10) / ring
                bm = gen.algorithmic_bytes(m2, N, K, BITS, GROUP)
                by_m[str(m2)] = {"us": tm * 1e6, "GBps": bm / tm * 1e-9, "frac_of_8TBps": bm / tm * 1e-9 / HBM_PEAK_GBS,
                                 "TFLOPs": 2.0 * m2 * N * K / tm * 1e-12, "dense_fp16_us": tdm * 1e6,
                                 "speedup_vs_dense_fp16": tdm / tm}
                del mrun, dmrun
            per_shape[n]["by_M"] = by_m
            del Wd, drun
        out["per_shape_cold"] = per_shape
        # a chain of dependent launches that do nothing (one workgroup reading 16 bytes): the cost of a
        # launch itself, part of every call above
        tiny = torch.zeros(16, dtype=torch.uint8, device="cuda")

        def empty_pass():
            for _ in range(LAYERS):
                lutq.calib_stream_read(tiny, 1, sink)
        erun = capture(empty_pass).replay if use_graph else empty_pass
        warm(torch, erun)
        out["empty_launch_us"] = time_region(torch, erun, 10) / LAYERS * 1e6
        # the LLaMA-3-70B layer shapes (4-bit, group 64, M = 1; bf16 as in the 70B configuration, fp16 next
        # to it), each on a ring of weight buffers larger than the caches.  The packed bytes and scales
        # are random (drawn on the GPU): the kernel's time does not depend on the values.  Parity at these
        # sizes and in these launch configurations is tests/test_gpu_parity.py::test_largest_shapes_sampled_rows
        # and ::test_full_size_sampled_rows.
        shapes70 = {"qkv": (10240, 8192), "o": (8192, 8192), "gate_up": (57344, 8192), "down": (8192, 28672)}
        g70 = 64
        per70 = {}
        for tname, tdt in (("bf16", torch.bfloat16), ("f16", torch.float16)):
            for n, (N, K) in shapes70.items():
                pb = lutq.lutq_packed_bytes(N, K, BITS, g70)
                ring = max(2, min(24, int(1.2e9 // pb) + 1))
                pk = [torch.randint(0, 256, (pb,), dtype=torch.uint8, device="cuda") for _ in range(ring)]
                S70 = (torch.rand((N, K // g70), device="cuda") * 0.01 + 0.01).to(tdt)
                T70 = torch.linspace(-1, 1, 1 << BITS, device="cuda").to(tdt)
                X70 = torch.randn((M, K), device="cuda").to(tdt)
                Y70 = torch.empty((M, N), dtype=tdt, device="cuda")
                ws70 = lutq.new_workspace(N, K, BITS, g70)

                def pass70(pk=pk, S70=S70, T70=T70, X70=X70, Y70=Y70, ws70=ws70):
                    for w in pk:
                        lutq.lutq_matmul(X70, w, S70, T70, BITS, g70, Y70, ws70)
                run = capture(pass70).replay if use_graph else pass70
                warm(torch, run)
                t = time_region(torch, run, 10) / ring
                by = gen.algorithmic_bytes(M, N, K, BITS, g70)
                per70[f"{n}_{tname}"] = {"N": N, "K": K, "us": t * 1e6, "GBps": by / t * 1e-9,
                                         "frac_of_8TBps": by / t * 1e-9 / HBM_PEAK_GBS}
                del pk, run
        out["per_shape_cold_llama3_70b_w4g64_m1"] = per70

    if not args.no_extras:
        # the entry points beyond the M <= 32 shared-table call, on the gate+up shape (cold rings as above)
        g = layer0["gate_up"]
        N, K = g["N"], g["K"]
        more = {}
        # one table per output row (Section 2.3: tables at the output-channel level), M = 1
        Tn = (torch.randn((N, 1 << BITS), device="cuda") * 0.5).to(torch.float16)

        def chan_pass():
            for li in range(LAYERS):
                lutq.lutq_matmul_channel(g["X"], layers[li]["gate_up"]["packed"], layers[li]["gate_up"]["S"], Tn,
                                         BITS, GROUP, Y["gate_up"], ws)
        run = capture(chan_pass).replay if use_graph else chan_pass
        warm(torch, run)
        t = time_region(torch, run, 10) / LAYERS
        by = gen.algorithmic_bytes(M, N, K, BITS, GROUP) + Tn.numel() * 2
        more["per_row_tables_m1"] = {"N": N, "K": K, "us": t * 1e6, "GBps": by / t * 1e-9, "frac_of_8TBps": by / t * 1e-9 / HBM_PEAK_GBS}
        # 33..128 activation rows (slices of 32 rows, one launch each)
        for m2 in (64, 128):
            X2 = torch.randn((m2, K), device="cuda").to(torch.float16)
            Y2 = torch.empty((m2, N), dtype=torch.float16, device="cuda")

            def big_pass(X2=X2, Y2=Y2):
                for li in range(LAYERS):
                    lutq.lutq_matmul(X2, layers[li]["gate_up"]["packed"], layers[li]["gate_up"]["S"], g["T"], BITS, GROUP, Y2, ws)
            run = capture(big_pass).replay if use_graph else big_pass
            warm(torch, run)
            t = time_region(torch, run, 5) / LAYERS
            by = gen.algorithmic_bytes(m2, N, K, BITS, GROUP)
            more[f"m{m2}"] = {"N": N, "K": K, "us": t * 1e6, "GBps": by / t * 1e-9, "TFLOPs": 2.0 * m2 * N * K / t * 1e-12}
            del run, X2, Y2
        # GPU quantiser: dense fp32 weights -> scales + packed indices (reads 4 B, writes b/8 + 2/group B per weight)
        Wq = torch.randn((N, K), device="cuda") * 0.02
        Sq = torch.empty((N, K // GROUP), dtype=torch.float16, device="cuda")
        Pq = torch.empty(lutq.lutq_packed_bytes(N, K, BITS, GROUP), dtype=torch.uint8, device="cuda")

        def quant_pass():
            lutq.lutq_quantize(Wq, g["T"], BITS, GROUP, Sq, Pq)
        warm(torch, quant_pass)
        t = time_region(torch, quant_pass, 10)
        by = Wq.numel() * 4 + Sq.numel() * 2 + Pq.numel()
        more["quantize_fp32"] = {"N": N, "K": K, "us": t * 1e6, "GBps": by / t * 1e-9, "Gweights_per_s": N * K / t * 1e-9}
        del Wq, Sq, Pq
        out["other_entry_points_llama3_8b_gate_up_w4g128"] = more

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layer0["o"]["case"])
    else:
        out["cpu_baseline"] = None

    print(json.dumps(out))


if __name__ == "__main__":
    main()
