#!/usr/bin/env python3
"""Benchmark of the LUT-quantised matmul hot path on one MI355X.

A step is one decode token's pass through the quantised linear layers of a LLaMA-3-8B-shaped model:
32 layers x [fused QKV (6144x4096), O (4096x4096), fused gate+up (28672x4096), down (4096x14336)],
4-bit NormalFloat table, group 128, fp16, M = 1 -- 128 calls of lutq_matmul on 128 distinct weight
buffers (3.4 GB), so every call streams its weights from HBM.  Inputs are synthetic and seeded
(lutq_inputs.py).  Three data sets (seeds 0, 1, 2; Section 4.1 of the paper times three random data
sets per shape) take turns step by step: seed 0 is NormalFloat-quantised Gaussian weights, seeds 1 and
2 are uniform random indices; each is replicated on the device for the 32 layers.

Prints ONE JSON line.  `value` is the whole step's algorithmic bytes (packed weights + scales + X + Y)
divided by the step time.  `roofline` prices the fused kernel against the 8 TB/s HBM peak with HIP
events over the same timed region; `cpu_baseline` times the CPU oracle on a bounded sample.  The
extras hold every other configuration of the metric (3-bit, the LLaMA-3-70B shapes in bf16, N = K =
8192 with group 32, M = 1..32), each beside a plain streaming read of the same packed bytes and, where
M varies, beside the dense 16-bit GEMM.
"""
from __future__ import annotations

import argparse
import json
import os
import re
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import lutq_inputs as gen  # noqa: E402

HBM_PEAK_GBS = 8000.0
# HBM bytes per launch of the headline workload (fetched + written) come from counter runs that cannot be
# made from inside this script (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a copy kernel of
# known size); their summary is this file, and the figure is read from its last "fetched + written" line.
TRAFFIC_SUMMARY = os.path.join(ROOT, "profiles", "matmul_and_decode_kernels_llama3_8b_w4g128_m1_hbm_traffic.txt")
LAYERS = 32
BITS, GROUP, DTYPE, M = 4, 128, "f16", 1
SEEDS = (0, 1, 2)


def measured_traffic_bytes():
    try:
        text = open(TRAFFIC_SUMMARY).read()
    except OSError:
        return None
    m = re.findall(r"fetched \+ written = ([0-9.]+) MB", text)
    return float(m[-1]) * 1e6 if m else None


def _to_dev(bits_u16, torch):
    return torch.from_numpy(np.ascontiguousarray(bits_u16).view(np.int16).copy()).view(torch.float16).cuda()


def build_layer(lutq, torch, seed):
    """One layer's four quantised matrices (host-quantised, seeded), uploaded once."""
    mats = {}
    for i, (name, (N, K)) in enumerate(gen.LLAMA3_8B_SHAPES.items()):
        c = gen.make_case(seed * 16 + i, M, N, K, BITS, GROUP, DTYPE, "nf" if seed == 0 else "random_index")
        packed = torch.from_numpy(lutq.lutq_pack(c.Q, BITS, GROUP)).cuda()
        mats[name] = dict(N=N, K=K, case=c, packed=packed, S=_to_dev(c.S, torch), T=_to_dev(c.T, torch),
                          X=_to_dev(c.X, torch))
    return mats


class Timer:
    def __init__(self, torch, use_graph):
        self.torch, self.use_graph = torch, use_graph

    def capture(self, fn):
        """A HIP graph of fn's launches (replayed as one unit: no per-call Python or launch-API time)."""
        torch = self.torch
        if not self.use_graph:
            return fn
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            fn()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            fn()
        return g.replay

    def warm(self, fn, seconds=0.1):
        """Runs fn (untimed) for a while: after any idle period the GPU needs some tens of milliseconds
        of load before its clocks are back up, and a single replay is far shorter than that."""
        torch = self.torch
        torch.cuda.synchronize()
        t = time.perf_counter()
        while time.perf_counter() - t < seconds:
            fn()
            torch.cuda.synchronize()

    def region(self, fns, iters):
        """Seconds per iteration; iteration i runs fns[i % len(fns)]."""
        torch = self.torch
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        torch.cuda.synchronize()
        e0.record()
        for i in range(iters):
            fns[i % len(fns)]()
        e1.record()
        torch.cuda.synchronize()
        return e0.elapsed_time(e1) * 1e-3 / iters

    def per_call(self, fn, calls, iters=10):
        run = self.capture(fn)
        self.warm(run)
        return self.region([run], iters) / calls


def cpu_baseline(case, budget_s=12.0):
    """The oracle as it stands, on the host cores, on the O-projection shape of the same workload."""
    from oracle import lutq_oracle as orc
    packed = orc.pack(case.Q, case.bits)
    t0, c0 = time.perf_counter(), time.process_time()
    n = 0
    while True:
        orc.lut_matmul(case.X, packed, case.S, case.T, case.bits, case.group_size, case.N, case.K, case.dtype)
        n += 1
        if time.perf_counter() - t0 > budget_s:
            break
    wall, cpu = time.perf_counter() - t0, time.process_time() - c0
    dt = wall / n
    by = gen.algorithmic_bytes(case.M, case.N, case.K, case.bits, case.group_size)
    return {"value": by / dt * 1e-9, "unit": "GB/s", "cores": max(1, int(round(cpu / wall))), "kind": "oracle",
            "sample": f"{n} calls of the numpy oracle (unpack + table lookup + scale + fp64 matmul) on the "
                      f"O-projection shape N={case.N} K={case.K} M={case.M} W4 g128; {dt * 1e3:.0f} ms per call; "
                      f"cores = process CPU time / wall time (only the fp64 matmul step is multi-threaded)"}


def r2(x):
    return round(float(x), 2)


class Weights:
    """A ring of random packed weight buffers of one shape, larger than the caches (the kernel's time does
    not depend on the values; parity at these sizes and in these launch configurations is
    tests/test_gpu_parity.py::test_largest_shapes_sampled_rows and ::test_full_size_sampled_rows)."""

    def __init__(self, lutq, torch, N, K, bits, group, tdt):
        self.N, self.K, self.bits, self.group, self.tdt = N, K, bits, group, tdt
        pb = lutq.lutq_packed_bytes(N, K, bits, group)
        ring = max(2, min(24, int(1.2e9 // pb) + 1))
        self.pk = [torch.randint(0, 256, (pb,), dtype=torch.uint8, device="cuda") for _ in range(ring)]
        self.S = (torch.rand((N, K // group), device="cuda") * 0.01 + 0.01).to(tdt)
        self.T = torch.linspace(-1, 1, 1 << bits, device="cuda").to(tdt)
        self.ws = lutq.new_workspace(N, K, bits, group)
        self.packed_bytes = pb


def time_lutq(lutq, torch, timer, w, m):
    X = torch.randn((m, w.K), device="cuda").to(w.tdt)
    Y = torch.empty((m, w.N), dtype=w.tdt, device="cuda")

    def run():
        for p in w.pk:
            lutq.lutq_matmul(X, p, w.S, w.T, w.bits, w.group, Y, w.ws)
    t = timer.per_call(run, len(w.pk))
    by = gen.algorithmic_bytes(m, w.N, w.K, w.bits, w.group)
    return t, {"us": r2(t * 1e6), "GBps": round(by / t * 1e-9), "frac_of_8TBps": round(by / t * 1e-9 / HBM_PEAK_GBS, 3)}


def time_stream_read(lutq, torch, timer, w, sink):
    def run():
        for p in w.pk:
            lutq.calib_stream_read(p, 512, sink)
    return timer.per_call(run, len(w.pk))


class Dense:
    """Dense 16-bit GEMM on the same shape (torch.mm -> hipBLASLt/rocBLAS) over a ring of weights > 1 GB."""

    def __init__(self, torch, N, K, tdt):
        ring = max(2, min(LAYERS, int(1.3e9 // (N * K * 2)) + 1))
        self.W = [(torch.randn((N, K), dtype=torch.float32, device="cuda") * 0.02).to(tdt) for _ in range(ring)]
        self.N, self.K, self.tdt = N, K, tdt

    def time(self, torch, timer, m):
        X = torch.randn((m, self.K), device="cuda").to(self.tdt)
        Y = torch.empty((m, self.N), dtype=self.tdt, device="cuda")

        def run():
            for w in self.W:
                torch.mm(X, w.t(), out=Y)
        return timer.per_call(run, len(self.W))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=60)
    ap.add_argument("--warmup", type=int, default=6)
    ap.add_argument("--no-graph", action="store_true", help="launch every call from Python instead of replaying a HIP graph")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="only the headline workload")
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
    use_graph = not args.no_graph
    timer = Timer(torch, use_graph)

    # ---------------------------------------------------------------- headline: the LLaMA-3-8B decode step
    names = list(gen.LLAMA3_8B_SHAPES.keys())
    ws = lutq.new_workspace(28672, 4096, BITS, GROUP)
    sets = []                                   # per seed: layer 0 on the host + 32 layers of device buffers
    for seed in SEEDS:
        layer0 = build_layer(lutq, torch, seed)
        layers = []
        for li in range(LAYERS):                # replicas of layer 0's bytes: only the addresses matter for HBM
            layers.append({n: dict(packed=layer0[n]["packed"] if li == 0 else layer0[n]["packed"].clone(),
                                   S=layer0[n]["S"] if li == 0 else layer0[n]["S"].clone()) for n in names})
        sets.append((layer0, layers))
    layer0, layers = sets[0]
    Y = {n: torch.empty((M, layer0[n]["N"]), dtype=torch.float16, device="cuda") for n in names}

    def one_call(n, li, data=0):
        l0, ls = sets[data]
        m = l0[n]
        lutq.lutq_matmul(m["X"], ls[li][n]["packed"], ls[li][n]["S"], m["T"], BITS, GROUP, Y[n], ws)

    def step_direct(data=0):
        for li in range(LAYERS):
            for n in names:
                one_call(n, li, data)

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

    steps = [timer.capture(lambda d=d: step_direct(d)) for d in range(len(SEEDS))]
    for i in range(args.warmup):
        steps[i % len(steps)]()
    # the GPU raises its clocks only after some tens of milliseconds of load: keep warming up (untimed)
    # until the step time has had that long to settle, whatever --warmup says
    for s in steps:
        timer.warm(s, 0.05)
    sec = timer.region(steps, args.steps)
    value = step_bytes / sec * 1e-9
    per_launch_s = sec / launches
    roof_achieved = (step_bytes / launches) / per_launch_s * 1e-9
    plan = {n: lutq.lutq_plan_default(BITS, GROUP, M, layer0[n]["N"], layer0[n]["K"]) for n in names}

    out = {
        "metric": "effective HBM GB/s of LUT-GEMM (packed weights + scales + X + Y bytes per call / time), M=1",
        "value": value, "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": sec * 1e3, "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f16", "data": "synthetic",
        "config": {"workload": "llama3-8b decode linears, W4 NormalFloat table g128 fp16 M=1: 32 layers x "
                               "[qkv 6144x4096, o 4096x4096, gate_up 28672x4096, down 4096x14336] = 128 lutq_matmul "
                               "calls per step on 128 distinct weight buffers (3.4 GB, HBM-cold); three seeded data "
                               "sets take turns step by step",
                   "bits": BITS, "group_size": GROUP, "M": M, "launch": "hipgraph replay" if use_graph else "python loop",
                   "calls_per_step": launches, "bytes_per_step": step_bytes,
                   "percent_of_hbm_peak": 100.0 * value / HBM_PEAK_GBS},
        "roofline": {"bound": "hbm", "achieved": roof_achieved, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                     "frac": roof_achieved / HBM_PEAK_GBS, "traffic": measured_traffic_bytes(),
                     "traffic_source": "profiles/" + os.path.basename(TRAFFIC_SUMMARY) + " (rocprofv3 --pmc FETCH_SIZE and WRITE_SIZE "
                                       "runs of this workload, scaled by a copy kernel of known size; not re-measured by this run)",
                     "kernel": "all 128 launches of the step: lutq::decode_kernel<4,128,1,F16,2,false,false> (o, qkv and gate_up: 96 launches, 74 % "
                               "of the time) and lutq::matmul_kernel<4,128,1,1,F16,2,true,4,true,0,false,false> (down: 32 launches)",
                     "bytes_per_launch": step_bytes / launches, "us_per_launch": per_launch_s * 1e6},
    }

    if not args.no_extras:
        sink = torch.zeros(4, dtype=torch.int32, device="cuda")
        # ---- configs 1-2: the headline's four shapes one by one (4-bit g128 fp16), M = 1..32, hot and cold
        per_shape = {}
        for n in names:
            m = layer0[n]
            N, K = m["N"], m["K"]
            by = gen.algorithmic_bytes(M, N, K, BITS, GROUP)
            t = timer.per_call(lambda n=n: [one_call(n, li) for li in range(LAYERS)], LAYERS)
            # a plain streaming read of the same packed bytes (no table, no arithmetic): what one launch
            # per call can reach on this shape at all
            tr = timer.per_call(lambda n=n: [lutq.calib_stream_read(layers[li][n]["packed"], 512, sink) for li in range(LAYERS)], LAYERS)
            # hot regime: the same weight buffer on every call (what a repetition loop over one matrix
            # measures: the small shapes then come from the caches, not from HBM)
            th = timer.per_call(lambda n=n: [one_call(n, 0) for _ in range(LAYERS)], LAYERS)
            dense = Dense(torch, N, K, torch.float16)
            td = dense.time(torch, timer, M)
            per_shape[n] = {"N": N, "K": K, "us": r2(t * 1e6), "GBps": round(by / t * 1e-9), "frac_of_8TBps": round(by / t * 1e-9 / HBM_PEAK_GBS, 3),
                            "TFLOPs": r2(2.0 * M * N * K / t * 1e-12), "dense_fp16_us": r2(td * 1e6), "speedup_vs_dense_fp16": r2(td / t),
                            "stream_read_us": r2(tr * 1e6), "lutq_over_stream_read": r2(t / tr), "hot_us": r2(th * 1e6),
                            "plan": repr(plan[n])}
            by_m = {}
            for m2 in (2, 4, 8, 16, 32):
                X2 = torch.randn((m2, K), device="cuda").to(torch.float16)
                Y2 = torch.empty((m2, N), dtype=torch.float16, device="cuda")

                def m_pass(n=n, X2=X2, Y2=Y2, m=m):
                    for li in range(LAYERS):
                        lutq.lutq_matmul(X2, layers[li][n]["packed"], layers[li][n]["S"], m["T"], BITS, GROUP, Y2, ws)
                tm = timer.per_call(m_pass, LAYERS)
                tdm = dense.time(torch, timer, m2)
                bm = gen.algorithmic_bytes(m2, N, K, BITS, GROUP)
                by_m[str(m2)] = {"us": r2(tm * 1e6), "frac_of_8TBps": round(bm / tm * 1e-9 / HBM_PEAK_GBS, 3),
                                 "TFLOPs": r2(2.0 * m2 * N * K / tm * 1e-12), "dense_fp16_us": r2(tdm * 1e6),
                                 "speedup_vs_dense_fp16": r2(tdm / tm)}
            per_shape[n]["by_M"] = by_m
            del dense
        out["per_shape_cold"] = per_shape
        # a chain of dependent launches that do nothing (one workgroup reading 16 bytes): the cost of a
        # launch itself, part of every call above
        tiny = torch.zeros(16, dtype=torch.uint8, device="cuda")
        out["empty_launch_us"] = r2(timer.per_call(lambda: [lutq.calib_stream_read(tiny, 1, sink) for _ in range(LAYERS)], LAYERS) * 1e6)
        del steps
        for s in sets[1:]:
            s[1].clear()
        del sets[1:]
        torch.cuda.empty_cache()

        def sweep(shapes, bits_list, group, tdt, Ms, dense_for=()):
            """{shape: {"w<bits>": {"stream_read_us", "M<m>": {us, GBps, frac_of_8TBps, lutq_over_stream_read[, dense_us, speedup_vs_dense]}}}}"""
            res = {}
            for n, (N, K) in shapes.items():
                res[n] = {"N": N, "K": K}
                dense = Dense(torch, N, K, tdt) if dense_for else None
                td = {m: dense.time(torch, timer, m) for m in dense_for} if dense else {}
                del dense
                for bits in bits_list:
                    w = Weights(lutq, torch, N, K, bits, group, tdt)
                    tr = time_stream_read(lutq, torch, timer, w, sink)
                    e = {"stream_read_us": r2(tr * 1e6)}
                    for m in Ms:
                        t, d = time_lutq(lutq, torch, timer, w, m)
                        d["lutq_over_stream_read"] = r2(t / tr)
                        if m in td:
                            d["dense_us"] = r2(td[m] * 1e6)
                            d["speedup_vs_dense"] = r2(td[m] / t)
                        e[f"M{m}"] = d
                    res[n][f"w{bits}"] = e
                    del w
                torch.cuda.empty_cache()
            return res

        # ---- config 3: 3-bit NormalFloat-sized table on the 8B shapes, groups 128 and 64, fp16
        out["config3_llama3_8b_w3_f16"] = {f"g{g}": sweep(gen.LLAMA3_8B_SHAPES, (3,), g, torch.float16, (1, 8, 32)) for g in (128, 64)}
        # ---- config 4: the LLaMA-3-70B shapes, 4- and 3-bit, group 64, bf16 (the 70B configuration's dtype),
        # beside the dense bf16 GEMM; fp16 at 4 bits and M = 1 next to it
        out["config4_llama3_70b_g64_bf16"] = sweep(gen.LLAMA3_70B_SHAPES, (4, 3), 64, torch.bfloat16, (1, 16, 32), dense_for=(1, 16, 32))
        out["config4_llama3_70b_w4g64_f16_m1"] = sweep(gen.LLAMA3_70B_SHAPES, (4,), 64, torch.float16, (1,))
        # ---- config 5: N = K = 8192, group 32, 2- and 4-bit, fp16, M = 1..32 beside the dense fp16 GEMM
        out["config5_8192sq_g32_f16"] = sweep({"sq": (8192, 8192)}, (2, 4), 32, torch.float16, (1, 2, 4, 8, 16, 32),
                                              dense_for=(1, 2, 4, 8, 16, 32))

        # ---- the entry points beyond the M <= 32 shared-table call, on the 8B gate+up shape (cold rings)
        g = layer0["gate_up"]
        N, K = g["N"], g["K"]
        more = {}
        # one table per output row (Section 2.3: tables at the output-channel level), M = 1
        Tn = (torch.randn((N, 1 << BITS), device="cuda") * 0.5).to(torch.float16)
        t = timer.per_call(lambda: [lutq.lutq_matmul_channel(g["X"], layers[li]["gate_up"]["packed"], layers[li]["gate_up"]["S"], Tn,
                                                             BITS, GROUP, Y["gate_up"], ws) for li in range(LAYERS)], LAYERS)
        by = gen.algorithmic_bytes(M, N, K, BITS, GROUP) + Tn.numel() * 2
        more["per_row_tables_m1"] = {"us": r2(t * 1e6), "frac_of_8TBps": round(by / t * 1e-9 / HBM_PEAK_GBS, 3),
                                     "over_shared_table": r2(t * 1e6 / per_shape["gate_up"]["us"])}
        # a codebook of 256 pairs of adjacent weights (Section 5: vector codebooks), M = 1: the same kernels, the same bytes + 1 KiB
        Cb = torch.randn((256, 2), device="cuda").to(torch.float16)
        t = timer.per_call(lambda: [lutq.lutq_matmul_pairs(g["X"], layers[li]["gate_up"]["packed"], layers[li]["gate_up"]["S"], Cb,
                                                           GROUP, Y["gate_up"], ws) for li in range(LAYERS)], LAYERS)
        more["pair_codebook_m1"] = {"us": r2(t * 1e6), "frac_of_8TBps": round((gen.algorithmic_bytes(M, N, K, BITS, GROUP) + 1024) / t * 1e-9 / HBM_PEAK_GBS, 3),
                                    "over_scalar_table": r2(t * 1e6 / per_shape["gate_up"]["us"])}
        # ... and at M = 16 (the row-streaming kernel with four row blocks' tables per pass)
        X16 = torch.randn((16, K), device="cuda").to(torch.float16)
        Y16 = torch.empty((16, N), dtype=torch.float16, device="cuda")
        t = timer.per_call(lambda: [lutq.lutq_matmul_channel(X16, layers[li]["gate_up"]["packed"], layers[li]["gate_up"]["S"], Tn,
                                                             BITS, GROUP, Y16, ws) for li in range(LAYERS)], LAYERS)
        t16 = per_shape["gate_up"]["by_M"].get("16", {}).get("us")
        more["per_row_tables_m16"] = {"us": r2(t * 1e6), "over_shared_table": r2(t * 1e6 / t16) if t16 else None}
        del X16, Y16
        # 33..128 activation rows
        dense = Dense(torch, N, K, torch.float16)
        for m2 in (48, 64, 96, 128):
            X2 = torch.randn((m2, K), device="cuda").to(torch.float16)
            Y2 = torch.empty((m2, N), dtype=torch.float16, device="cuda")
            t = timer.per_call(lambda X2=X2, Y2=Y2: [lutq.lutq_matmul(X2, layers[li]["gate_up"]["packed"], layers[li]["gate_up"]["S"], g["T"],
                                                                      BITS, GROUP, Y2, ws) for li in range(LAYERS)], LAYERS, iters=5)
            td = dense.time(torch, timer, m2)
            more[f"m{m2}"] = {"us": r2(t * 1e6), "TFLOPs": r2(2.0 * m2 * N * K / t * 1e-12), "dense_fp16_us": r2(td * 1e6)}
            del X2, Y2
        del dense
        # GPU quantiser: dense fp32 weights -> scales + packed indices (reads 4 B, writes b/8 + 2/group B per weight)
        Wq = torch.randn((N, K), device="cuda") * 0.02
        Sq = torch.empty((N, K // GROUP), dtype=torch.float16, device="cuda")
        Pq = torch.empty(lutq.lutq_packed_bytes(N, K, BITS, GROUP), dtype=torch.uint8, device="cuda")
        timer.warm(lambda: lutq.lutq_quantize(Wq, g["T"], BITS, GROUP, Sq, Pq))
        t = timer.region([lambda: lutq.lutq_quantize(Wq, g["T"], BITS, GROUP, Sq, Pq)], 10)
        by = Wq.numel() * 4 + Sq.numel() * 2 + Pq.numel()
        more["quantize_fp32"] = {"us": r2(t * 1e6), "GBps": round(by / t * 1e-9), "Gweights_per_s": round(N * K / t * 1e-9)}
        del Wq, Sq, Pq
        out["other_entry_points_llama3_8b_gate_up_w4g128"] = more

    if not args.no_cpu_baseline:
        out["cpu_baseline"] = cpu_baseline(layer0["o"]["case"])
    else:
        out["cpu_baseline"] = None

    print(json.dumps(out))


if __name__ == "__main__":
    main()
