#!/usr/bin/env python3
"""Benchmark of the ITQ3_S hot path on one MI355X.

A step is one decode pass (M = 1) over every weight tensor of a transformer-shaped stack, in the
order of the layer's data flow: q, k, v (same input) -> o -> gate, up (same input) -> down.  Tensors
that read the same activations go into one itq3s_matmul_grouped call (one launch: activation
rotation + streaming contraction + epilogue); `--ungrouped` issues one itq3s_matmul per tensor.
The default workload is the full 70B-shaped stream (80 layers, 560 tensors, 26.74 GB of packed
weights resident in HBM: no tensor is re-read from a cache); `--workload llama7b_decode` runs the
7B-shaped stack (32 layers, 2.5 GB), which the default run also times as an extra leg.  Weights are
synthetic (Student-t, see paper_2603_27914_amd/synth.py), generated on the device and packed by
itq3s_quantize, which is timed as well.

Prints ONE JSON line.  `value` = packed-weight bytes streamed per second over the whole step (wall
clock over the replayed graph, launch gaps included).  `roofline` prices the streaming contraction
kernel alone: algorithmic bytes of a call over the kernel's own duration, which
itq3s_matmul_grouped_timed reads from HIP events attached to the kernel's dispatch, averaged over
every call of the step (three more passes through the step, the middle reading of each call: the
same quantity rocprofv3 --kernel-trace --stats lists as the kernel's average duration).  The other
configurations of the metric (single 2048 x 2048 GEMV, 7B and 70B shapes one by one at several M, the
prefill GEMM at M = 512 and 2048 against the fp16 matrix-core peak) are extra legs of the same line.
"""
import argparse
import json
import os
import re
import sys
import time
from concurrent.futures import ThreadPoolExecutor

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

FP64_VECTOR_PEAK_TFLOPS = 78.6
HBM_PEAK_GBPS = 8000.0
MFMA_F16_PEAK_TFLOPS = 2516.6  # 256 CU x 4 SIMD x 1024 flop/clk x 2.4 GHz

WORKLOADS = {
    # name: (layers, stages of one layer in paper_2603_27914_amd.synth, M)
    "llama7b_decode": (32, "LLAMA7B_STAGES", 1),
    "llama70b_decode": (80, "LLAMA70B_STAGES", 1),
}


def student_t_weights(torch, gen, N, K):
    """0.02 * Student-t(nu=4) on the device, round(0.001 K) input channels times 20."""
    z = torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32)
    chi = torch.zeros((N, K), device="cuda", dtype=torch.float32)
    for _ in range(4):
        chi += torch.randn((N, K), generator=gen, device="cuda", dtype=torch.float32) ** 2
    W = z / torch.sqrt(chi / 4.0) * 0.02
    ncol = int(round(0.001 * K))
    cols = torch.randperm(K, generator=gen, device="cuda")[:ncol]
    W[:, cols] *= 20.0
    return W


def activations(torch, gen, M, K, outliers=True):
    X = torch.randn((M, K), generator=gen, device="cuda", dtype=torch.float32)
    if outliers:
        cols = torch.randperm(K, generator=gen, device="cuda")[: int(round(0.005 * K))]
        X[:, cols] *= 10.0
    return X.to(torch.float16)


def packed_bytes(N, K):
    return ((N + 15) // 16) * (K // 256) * 1600


def alg_bytes(N, K, M, y_bytes=4):
    return packed_bytes(N, K) + M * K * 2 + M * N * y_bytes


def measured_traffic(workload):
    """HBM bytes per launch of the streaming kernel from the committed rocprofv3 --pmc summary of
    this workload (FETCH_SIZE and WRITE_SIZE passes, scaled by the calibration copy), or None."""
    path = os.path.join(ROOT, "profiles", "gemv_%s.hbm_traffic.txt" % workload)
    if not os.path.exists(path):
        return None
    tot = {"FETCH_SIZE": [0.0, 0], "WRITE_SIZE": [0.0, 0]}
    for line in open(path):
        m = re.match(r"\s*gemv_kernel\S*.*?\s(\d+)\s+(FETCH_SIZE|WRITE_SIZE)\s+(\d+)\s+([\d.]+)\s+([\d.]+)\s*$", line)
        if m:
            calls, scaled = int(m.group(3)), float(m.group(5))
            tot[m.group(2)][0] += calls * scaled
            tot[m.group(2)][1] += calls
    if not tot["FETCH_SIZE"][1] or not tot["WRITE_SIZE"][1]:
        return None
    fetch = tot["FETCH_SIZE"][0] / tot["FETCH_SIZE"][1] * 1024.0
    write = tot["WRITE_SIZE"][0] / tot["WRITE_SIZE"][1] * 1024.0
    return {"bytes_per_launch": int(fetch + write), "fetch_bytes": int(fetch), "write_bytes": int(write), "source": os.path.relpath(path, ROOT)}


def build_stack(torch, binding, gen, stages, layers, flags=None):
    """Generate and pack every tensor of `layers` layers.  -> (tensors, quantize ms, quantize bytes);
    tensors = [(N, K, codes, scales, layer, stage, name)]."""
    tensors, q_ms, q_bytes = [], 0.0, 0
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    for li in range(layers):
        for si, stage in enumerate(stages):
            for name, N, K in stage:
                W = student_t_weights(torch, gen, N, K)
                codes, scales = binding.alloc_packed(N, K)
                ev0.record()
                binding.itq3s_quantize(W, codes, scales, status_flags=flags)
                ev1.record()
                ev1.synchronize()
                q_ms += ev0.elapsed_time(ev1)
                q_bytes += N * K * 4 + packed_bytes(N, K)
                tensors.append((N, K, codes, scales, li, si, name))
                del W
    return tensors, q_ms, q_bytes


def step_calls(tensors, stages, layers, ys, grouped=True):
    """The library calls of a step, in order: one per stage of every layer (the tensors of a stage read
    the same activations: one grouped call), or one per tensor."""
    calls = []  # (K, [(codes, scales, N)], [Y])
    for li in range(layers):
        for si in range(len(stages)):
            group = [t for t in tensors if t[4] == li and t[5] == si]
            if grouped:
                calls.append((group[0][1], [(c, s, N) for N, K, c, s, *_ in group], [ys[t[6]] for t in group]))
            else:
                calls.extend((K, [(c, s, N)], [ys[name]]) for N, K, c, s, _, _, name in group)
    return calls


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="llama70b_decode", choices=sorted(WORKLOADS))
    ap.add_argument("--layers", type=int, default=0, help="override the number of layers (0 = the workload's own)")
    ap.add_argument("--no-extras", action="store_true", help="only the timed step and the roofline pass")
    ap.add_argument("--ungrouped", action="store_true", help="one library call (one launch) per tensor instead of one per stage")
    ap.add_argument("--prefill-m", default="512,2048", help="activation row counts of the prefill leg")
    ap.add_argument("--legs", default="single,per_shape,stream7b,read_floor,prefill,dequantize,sub,ablation,copy,cpu", help="comma list of the extra legs to run")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (no sharding, no collectives); --gpus %d is not supported" % args.gpus, file=sys.stderr)
        sys.exit(2)

    import torch

    from paper_2603_27914_amd import binding, synth

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(2)
    binding.lib()
    torch.cuda.set_device(0)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(synth.MASTER_SEED)

    layers, stages_name, M = WORKLOADS[args.workload]
    if args.layers > 0:
        layers = args.layers
    stages = getattr(synth, stages_name)
    grouped = not args.ungrouped

    # ------------------------------------------------------------------ build the resident weights
    flags = torch.zeros(1, dtype=torch.int32, device="cuda")
    tensors, q_ms, q_bytes = build_stack(torch, binding, gen, stages, layers, flags)
    assert int(flags.item()) == 0, "quantizer raised data flags on synthetic weights"
    xs = {}
    for stage in stages:
        K = stage[0][2]
        if K not in xs:
            xs[K] = activations(torch, gen, M, K)
    ys = {name: torch.empty((M, N), dtype=torch.float32, device="cuda") for stage in stages for name, N, K in stage}
    ws = torch.empty(max(binding.itq3s_matmul_workspace_bytes(M, N, K) for stage in stages for _, N, K in stage), dtype=torch.uint8, device="cuda")
    calls = step_calls(tensors, stages, layers, ys, grouped)

    def step():
        for K, wts, outs in calls:
            binding.itq3s_matmul_grouped(wts, K, xs[K], outs=outs, workspace=ws, status_flags=flags)

    # ------------------------------------------------------------------ timed region
    # The step is captured once into a HIP graph and replayed, so that the timed region measures
    # the GPU and not the Python interpreter issuing the launches.
    step()
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for _ in range(args.warmup):
        graph.replay()
    torch.cuda.synchronize()
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(args.steps):
        graph.replay()
    ev1.record()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    ev_ms = ev0.elapsed_time(ev1)
    assert int(flags.item()) == 0, "a matmul raised data flags on synthetic inputs"
    ms_per_step = wall_ms / args.steps
    step_packed = sum(packed_bytes(N, K) for N, K, *_ in tensors)
    step_alg = sum(alg_bytes(N, K, M) for N, K, *_ in tensors)
    value = step_packed / (ms_per_step * 1e-3) / 1e9
    # dominant kernel = the streaming contraction (gemv_kernel), one launch per call: its duration by
    # the events attached to each dispatch, passes over the step's calls in step order (every
    # tensor comes from HBM: the whole stack lies between two uses of the same one)
    # (three passes, the middle value per call: the call waits for its kernel, so the GPU idles between
    # launches and single readings scatter upwards; the average below is over the step's calls)
    passes = []
    for _ in range(3):
        passes.append([binding.itq3s_matmul_grouped_timed(wts, K, xs[K], outs=outs, workspace=ws)[1] for K, wts, outs in calls])
    kern_ms = {}
    for i, (K, wts, outs) in enumerate(calls):
        kern_ms.setdefault((K, tuple(N for _, _, N in wts)), []).append(sorted(p[i] for p in passes)[1])
    all_ms = [m for v in kern_ms.values() for m in v]
    avg_launch_ms = sum(all_ms) / len(all_ms)
    achieved = (step_alg / len(calls)) / (avg_launch_ms * 1e-3) / 1e9
    per_kernel = []
    for (K, Ns), v in kern_ms.items():
        v = sorted(v)
        nbytes = sum(alg_bytes(N, K, M) for N in Ns)
        mean = sum(v) / len(v)
        per_kernel.append({"K": K, "N": list(Ns), "launches": len(v), "us_mean": round(1e3 * mean, 3), "us_median": round(1e3 * v[len(v) // 2], 3),
                           "us_min": round(1e3 * v[0], 3), "alg_bytes": nbytes, "GBps_mean": round(nbytes / (mean * 1e-3) / 1e9, 1),
                           "frac": round(nbytes / (mean * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)})
    measured = measured_traffic(args.workload) if layers == WORKLOADS[args.workload][0] and grouped else None

    out = {
        "metric": "ITQ3_S GEMV effective HBM GB/s on packed-weight bytes @M=1",
        "value": round(value, 1),
        "unit": "GB/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": "f16",
        "data": "synthetic",
        "config": {
            "workload": "%s: %d layers x [%s], M=%d, %d tensors in %d library calls (%s), %.2f GB packed resident in HBM"
            % (args.workload, layers, " -> ".join("+".join("%s %dx%d" % t for t in st) for st in stages), M, len(tensors), len(calls),
               "tensors that read the same activations share a launch" if grouped else "one call per tensor", step_packed / 1e9),
            "frac_of_hbm_peak": round(value / HBM_PEAK_GBPS, 4),
        },
        "roofline": {
            "bound": "hbm",
            "kernel": "gemv_kernel (itq3s_matmul / itq3s_matmul_grouped, M<=4 path)",
            "achieved": round(achieved, 1),
            "peak": HBM_PEAK_GBPS,
            "unit": "GB/s",
            "frac": round(achieved / HBM_PEAK_GBPS, 4),
            "traffic": measured["bytes_per_launch"] if measured else None,
            "traffic_detail": measured,
            "avg_launch_us": round(avg_launch_ms * 1e3, 3),
            "alg_bytes_per_launch": int(step_alg / len(calls)),
            "launches_timed": len(all_ms),
            "per_kernel": per_kernel,
            "step_wall_us_per_call": round(ev_ms / (args.steps * len(calls)) * 1e3, 3),
        },
        "quantize": {"GBps": round(q_bytes / (q_ms * 1e-3) / 1e9, 1), "bytes": q_bytes, "ms": round(q_ms, 2), "frac_of_hbm_peak": round(q_bytes / (q_ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4)},
    }

    legs = [] if args.no_extras else [x for x in args.legs.split(",") if x]
    if "single" in legs:
        out["single_gemv"] = single_leg(torch, binding, gen)
    if "per_shape" in legs:
        out["per_shape"] = per_shape_leg(torch, binding, tensors, gen, (1, 4, 16), torch.float16)
    if "read_floor" in legs:
        out["read_floor"] = read_floor_leg(torch, binding, tensors)
    if "dequantize" in legs:
        out["dequantize"] = dequantize_leg(torch, binding, tensors)
    if "cpu" in legs:
        out["cpu_baseline"] = cpu_baseline_leg(torch, binding, tensors, xs, M)
    if "stream7b" in legs and args.workload != "llama7b_decode":
        out["stream7b"] = stream7b_leg(torch, binding, synth, gen)
    if "prefill" in legs:
        out["prefill"] = prefill_leg(torch, binding, synth, gen, [int(m) for m in args.prefill_m.split(",")])
        best = max((r for r in out["prefill"] if r["M"] == max(x["M"] for x in out["prefill"])), key=lambda r: r["kernel_TFLOPs"])
        out["roofline_gemm"] = {"bound": "mfma", "kernel": "gemm_kernel (itq3s_matmul, M>16 path)", "achieved": best["kernel_TFLOPs"], "peak": MFMA_F16_PEAK_TFLOPS,
                                "unit": "TFLOP/s", "frac": round(best["kernel_TFLOPs"] / MFMA_F16_PEAK_TFLOPS, 4),
                                "workload": "X fp16 [%d, %d] x ITQ3_S W %dx%d, fp16 out" % (best["M"], best["K"], best["N"], best["K"]),
                                "whole_call_TFLOPs": best["TFLOPs"], "whole_call_frac": best["frac_of_mfma_peak"]}
    if "sub" in legs:
        out["sub_block_variant"] = sub_variant_leg(torch, binding, gen)
    if "ablation" in legs:
        out["block_size_ablation"] = ablation_leg(torch, binding, gen)
    if "copy" in legs:
        out["copy_ceiling"] = copy_leg(torch)
    print(json.dumps(out))


def time_calls(torch, fn, n_iter, warm=3):
    for _ in range(warm):
        fn()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(n_iter):
        fn()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / n_iter


def graph_time(torch, fn, n_calls, reps=10):
    """fn() enqueues n_calls library calls; capture once, replay, -> milliseconds per call."""
    fn()
    torch.cuda.synchronize()
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        fn()
    for _ in range(3):
        g.replay()
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record()
    for _ in range(reps):
        g.replay()
    e1.record()
    e1.synchronize()
    return e0.elapsed_time(e1) / (reps * n_calls)


def single_leg(torch, binding, gen, N=2048, K=2048, copies=256):
    """The single 2048 x 2048 GEMV (M = 1, fp32 out, no activation outliers): latency of one call, as a
    replayed graph cycling through `copies` packed copies (420 MB: weights come from HBM) and on one
    copy (weights stay in the last-level cache).  1.64 MB is 0.2 us of traffic at peak, far below
    the cost of any launch: this configuration shows latency, not bandwidth."""
    W = student_t_weights(torch, gen, N, K)
    first = binding.itq3s_quantize(W)
    packed = [first] + [(first[0].clone(), first[1].clone()) for _ in range(copies - 1)]
    del W
    X = activations(torch, gen, 1, K, outliers=False)
    Y = torch.empty((1, N), dtype=torch.float32, device="cuda")
    ws = torch.empty(binding.itq3s_matmul_workspace_bytes(1, N, K), dtype=torch.uint8, device="cuda")

    def run(which):
        for c, s in which:
            binding.itq3s_matmul(c, s, N, K, X, out=Y, workspace=ws)

    ms = graph_time(torch, lambda: run(packed), copies)
    ms_hot = graph_time(torch, lambda: run(packed[:1] * 32), 32)
    return {"N": N, "K": K, "M": 1, "us": round(ms * 1e3, 2), "GBps": round(packed_bytes(N, K) / (ms * 1e-3) / 1e9, 1),
            "frac_of_hbm_peak": round(packed_bytes(N, K) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4), "copies": copies, "us_cache_resident": round(ms_hot * 1e3, 2)}


def per_shape_leg(torch, binding, tensors, gen, Ms, out_dtype):
    """Each tensor shape of the stack on its own, one call per launch, for several M, as a replayed
    graph cycling through the resident copies of that shape (at most 24 of them, at least 0.5 GB:
    weights come from HBM)."""
    res = []
    shapes = []
    for t in tensors:
        if (t[0], t[1]) not in shapes:
            shapes.append((t[0], t[1]))
    for N, K in shapes:
        same = [t for t in tensors if (t[0], t[1]) == (N, K)]
        same = same[: max(2, min(len(same), 24, int(2e9 // packed_bytes(N, K)) + 1))]
        for M in Ms:
            X = activations(torch, gen, M, K)
            Y = torch.empty((M, N), dtype=out_dtype, device="cuda")
            ws = torch.empty(binding.itq3s_matmul_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")

            def run():
                for N_, K_, codes, scales, *_ in same:
                    binding.itq3s_matmul(codes, scales, N_, K_, X, out=Y, workspace=ws)

            ms = graph_time(torch, run, len(same))
            res.append({"N": N, "K": K, "M": M, "out": str(out_dtype).replace("torch.", ""), "us": round(ms * 1e3, 2),
                        "GBps": round(packed_bytes(N, K) / (ms * 1e-3) / 1e9, 1), "frac_of_hbm_peak": round(packed_bytes(N, K) / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                        "copies": len(same)})
    return res


def sub_variant_leg(torch, binding, gen, N=28672, K=8192, copies=8):
    """The 116-byte sub-block-scale variant of the format (Sec. 4.1) on the largest tensor shape:
    itq3s_quantize_sub (fp32 in), then itq3s_matmul_sub for M = 1, 4, 16 and 512 as a replayed graph
    cycling through `copies` packed copies (0.85 GB: weights come from HBM).  Bytes per block: 116."""
    nb = ((N + 15) // 16) * 16 * (K // 256)
    packed = nb * 116
    W = student_t_weights(torch, gen, N, K)
    first = binding.itq3s_quantize_sub(W)
    q_ms = time_calls(torch, lambda: binding.itq3s_quantize_sub(W, out=first), 5)
    sets = [first] + [tuple(t.clone() for t in first) for _ in range(copies - 1)]
    del W
    res = {"N": N, "K": K, "bytes_per_block": 116, "quantize_us": round(q_ms * 1e3, 1),
           "quantize_GBps": round((N * K * 4 + packed) / (q_ms * 1e-3) / 1e9, 1), "matmul": []}
    for M in (1, 4, 16, 512):
        X = activations(torch, gen, M, K)
        ws = torch.empty(max(256, binding.itq3s_matmul_workspace_bytes(min(M, 16), N, K)), dtype=torch.uint8, device="cuda")
        Y = torch.empty((M, N), dtype=torch.float16, device="cuda")

        def run():
            for c, sc, su in sets:
                binding.itq3s_matmul_sub(c, sc, su, N, K, X, out=Y, workspace=ws)

        ms = graph_time(torch, run, len(sets), reps=4 if M > 16 else 10)
        row = {"M": M, "us": round(ms * 1e3, 2)}
        if M <= 16:
            row.update(GBps=round(packed / (ms * 1e-3) / 1e9, 1), frac_of_hbm_peak=round(packed / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4))
        else:
            row.update(TFLOPs=round(2.0 * M * N * K / (ms * 1e-3) / 1e12, 1))
        res["matmul"].append(row)
    return res


def stream7b_leg(torch, binding, synth, gen):
    """The 7B-shaped decode stack (32 layers, 2.53 GB packed, fp32 out) as a replayed graph of grouped
    calls, and its shapes one by one at M = 1 and 8."""
    stages = synth.LLAMA7B_STAGES
    tensors, _, _ = build_stack(torch, binding, gen, stages, 32)
    xs = {K: activations(torch, gen, 1, K) for K in sorted({st[0][2] for st in stages})}
    ys = {name: torch.empty((1, N), dtype=torch.float32, device="cuda") for st in stages for name, N, K in st}
    ws = torch.empty(256, dtype=torch.uint8, device="cuda")
    calls = step_calls(tensors, stages, 32, ys)
    nbytes = sum(packed_bytes(t[0], t[1]) for t in tensors)

    def step():
        for K, wts, outs in calls:
            binding.itq3s_matmul_grouped(wts, K, xs[K], outs=outs, workspace=ws)

    ms = graph_time(torch, step, 1, reps=20)
    return {"workload": "llama7b_decode shapes, 32 layers, M=1, fp32 out, %d grouped calls, %.2f GB packed" % (len(calls), nbytes / 1e9),
            "ms_per_step": round(ms, 4), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "per_shape": per_shape_leg(torch, binding, tensors, gen, (1, 8), torch.float32)}


def prefill_leg(torch, binding, synth, gen, m_list=(512, 2048)):
    """The MFMA path: X fp16 [M, K] times the two FFN-shaped tensors, M = 512 and 2048.  `us` / `TFLOPs`
    are whole calls (rotation launch, contraction, and for shapes with few tiles the launch that adds
    the split-K shares); `kernel_us` / `kernel_TFLOPs` the contraction launch alone."""
    res = []
    for name, N, K in synth.SHAPES["prefill"]:
        W = student_t_weights(torch, gen, N, K)
        codes, scales = binding.itq3s_quantize(W)
        del W
        for M in m_list:
            X = activations(torch, gen, M, K)
            Y = torch.empty((M, N), dtype=torch.float16, device="cuda")
            ws = torch.empty(binding.itq3s_matmul_workspace_bytes(M, N, K), dtype=torch.uint8, device="cuda")
            ms = time_calls(torch, lambda: binding.itq3s_matmul(codes, scales, N, K, X, out=Y, workspace=ws), 20)
            tf = 2.0 * M * N * K / (ms * 1e-3) / 1e12
            kms = sorted(binding.itq3s_matmul_timed(codes, scales, N, K, X, out=Y, workspace=ws)[1] for _ in range(3))[1]
            # the paper's placement of the transform (inside the weight tile loader), for comparison
            binding.itq3s_matmul_weight_side(codes, scales, N, K, X, out=Y)
            wms = sorted(binding.itq3s_matmul_weight_side_timed(codes, scales, N, K, X, out=Y)[1] for _ in range(3))[1]
            res.append({"N": N, "K": K, "M": M, "us": round(ms * 1e3, 1), "TFLOPs": round(tf, 1), "frac_of_mfma_peak": round(tf / MFMA_F16_PEAK_TFLOPS, 4),
                        "kernel_us": round(kms * 1e3, 1), "kernel_TFLOPs": round(2.0 * M * N * K / (kms * 1e-3) / 1e12, 1),
                        "kernel_frac_of_mfma_peak": round(2.0 * M * N * K / (kms * 1e-3) / 1e12 / MFMA_F16_PEAK_TFLOPS, 4),
                        "weight_side_kernel_us": round(wms * 1e3, 1), "weight_side_TFLOPs": round(2.0 * M * N * K / (wms * 1e-3) / 1e12, 1),
                        "weight_side_overhead_pct": round(100.0 * (wms / kms - 1.0), 1),
                        # workgroups per launch: the weight-side kernel (512 x 128 tiles, no split of K) fills the chip only
                        # when it has at least one per compute unit -- compare the overhead where both kernels do
                        "weight_side_workgroups": ((M + 511) // 512) * ((N + 127) // 128)})
    return res


def dequantize_leg(torch, binding, tensors):
    """itq3s_dequantize (fp32 out) of the largest tensor shape, cycling over its resident copies and
    over enough output buffers (> 512 MB) that neither side is served from the last-level cache."""
    N, K = max(((t[0], t[1]) for t in tensors), key=lambda nk: nk[0] * nk[1])
    same = [t for t in tensors if (t[0], t[1]) == (N, K)][:8]
    nout = max(2, int(6e8 // (N * K * 4)) + 1)
    outs = [torch.empty((N, K), dtype=torch.float32, device="cuda") for _ in range(nout)]
    state = {"i": 0}

    def run():
        i = state["i"]
        state["i"] = i + 1
        t = same[i % len(same)]
        binding.itq3s_dequantize(t[2], t[3], N, K, out=outs[i % nout])

    ms = time_calls(torch, run, 4 * nout, warm=nout)
    nbytes = packed_bytes(N, K) + N * K * 4
    return {"N": N, "K": K, "us": round(ms * 1e3, 1), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
            "output_buffers": nout}


def ablation_leg(torch, binding, gen, N=8192, K=8192, copies=3):
    """Block-size ablation (Sec. 6): the rotate - quantize - reconstruct round trip with transform
    lengths 32 .. 512 over the same heavy-tailed fp32 weights; the error sums are reduced on the
    device (no output tensors), so a launch reads 4 bytes per weight.  The copies (768 MB together)
    are cycled so that the reads come from HBM."""
    Ws = [student_t_weights(torch, gen, N, K) for _ in range(copies)]
    res = []
    for n in (32, 64, 128, 256, 512):
        err2 = torch.zeros(2, dtype=torch.float64, device="cuda")
        binding.itq3s_roundtrip(Ws[0], n, codes=False, scales=False, w_hat=False, err2=err2)
        e = err2.cpu().numpy()
        state = {"i": 0}

        def run():
            state["i"] += 1
            binding.itq3s_roundtrip(Ws[state["i"] % copies], n, codes=False, scales=False, w_hat=False, err2=err2)

        ms = time_calls(torch, run, 4 * copies, warm=copies)
        nbytes = N * K * 4
        # fp64 operations per weight: two transforms of log2(n) additions each, about 20 more for the
        # scaling, statistics, thresholds, reconstruction and error sums; none of them fused, so the
        # ceiling is half the chip's fp64 vector rate (which counts a fused multiply-add as two)
        ops = (2 * (n.bit_length() - 1) + 20) * N * K
        res.append({"block_size": n, "bits_per_weight": round(3.0 + 32.0 / n, 4), "rel_rmse": round(float((e[0] / e[1]) ** 0.5), 5),
                    "us": round(ms * 1e3, 1), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1), "frac_of_hbm_peak": round(nbytes / (ms * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
                    "fp64_Tops": round(ops / (ms * 1e-3) / 1e12, 2), "frac_of_unfused_fp64_peak": round(ops / (ms * 1e-3) / 1e12 / (FP64_VECTOR_PEAK_TFLOPS / 2), 4)})
    return {"N": N, "K": K, "dtype": "f64", "bound": "alu", "sizes": res}


def read_floor_leg(torch, binding, tensors):
    """A plain read of the packed code arrays of every tensor shape of the step (the resident copies in
    turn, replayed graph): what a launch costs that only moves the bytes."""
    res = []
    sink = torch.zeros(1, dtype=torch.int32, device="cuda")
    shapes = []
    for t in tensors:
        if (t[0], t[1]) not in shapes:
            shapes.append((t[0], t[1]))
    for N, K in shapes:
        same = [t for t in tensors if (t[0], t[1]) == (N, K)]
        same = same[: max(2, min(len(same), 24))]

        def run():
            for t in same:
                binding.itq3s_read_probe(t[2], sink)

        ms = graph_time(torch, run, len(same))
        nbytes = same[0][2].numel() * 4
        res.append({"N": N, "K": K, "bytes": nbytes, "us": round(ms * 1e3, 2), "GBps": round(nbytes / (ms * 1e-3) / 1e9, 1)})
    return res


def copy_leg(torch):
    """A plain device-to-device copy of known size: the practical ceiling next to the 8 TB/s peak, and
    the kernel whose known traffic calibrates the FETCH_SIZE / WRITE_SIZE counters."""
    n = 1 << 28  # 1 GiB of fp32 read + 1 GiB written
    src = torch.empty(n, dtype=torch.float32, device="cuda").normal_()
    dst = torch.empty_like(src)
    ms = time_calls(torch, lambda: dst.copy_(src), 10)
    return {"bytes_read": 4 * n, "bytes_written": 4 * n, "us": round(ms * 1e3, 1), "GBps_read_plus_write": round(8 * n / (ms * 1e-3) / 1e9, 1)}


def cpu_baseline_leg(torch, binding, tensors, xs, M):
    """The CPU oracle, as it stands, on a bounded sample of the same workload: the M = 1 matmuls of the
    first layers' tensors -- once on one core, once with the output rows of every tensor dealt to all
    host cores this process may use (the oracle itself unchanged: each thread calls it for its own
    range of rows).  Also checks the GPU result of those calls against it."""
    from oracle import itq3s_ref as ref

    ref.build()
    ref.lib()
    ncores = len(os.sched_getaffinity(0)) if hasattr(os, "sched_getaffinity") else (os.cpu_count() or 1)
    omp = os.environ.get("OMP_NUM_THREADS")
    if omp and omp.isdigit():
        ncores = max(1, min(ncores, int(omp)))  # the machine's CPU share
    per_layer = sum(packed_bytes(t[0], t[1]) for t in tensors if t[4] == 0)
    n_layers = max(1, min(tensors[-1][4] + 1, int(1.1e9 // per_layer)))  # about 12 s of single-thread work
    sample = [t for t in tensors if t[4] < n_layers]
    host = [(N, K, codes.cpu().numpy().view(np.uint32), scales.cpu().numpy().view(np.uint32), xs[K].cpu().numpy()) for N, K, codes, scales, *_ in sample]
    nbytes = sum(packed_bytes(N, K) for N, K, *_ in host)

    t0 = time.perf_counter()
    one = [ref.matmul(hc, hs, N, K, X) for N, K, hc, hs, X in host]
    secs1 = time.perf_counter() - t0

    def rows_of(N, parts):
        edges = [N * i // parts for i in range(parts + 1)]
        return [(a, b) for a, b in zip(edges[:-1], edges[1:]) if b > a]

    t0 = time.perf_counter()
    with ThreadPoolExecutor(max_workers=ncores) as pool:
        futs = [[pool.submit(ref.matmul, hc, hs, N, K, X, r) for r in rows_of(N, ncores)] for N, K, hc, hs, X in host]
        many = [sum(f.result() for f in fs) for fs in futs]  # each part fills its own columns, zeros elsewhere
    secsn = time.perf_counter() - t0
    assert all(np.array_equal(a, b) for a, b in zip(one, many)), "row-partitioned oracle differs from the single-thread oracle"

    worst = 0.0
    for (N, K, codes, scales, *_), Yr in zip(sample, one):
        Y = binding.itq3s_matmul(codes, scales, N, K, xs[K]).cpu().numpy()
        worst = max(worst, float(np.max(np.linalg.norm(Y - Yr, axis=1) / np.linalg.norm(Yr, axis=1))))
    return {
        "value": round(nbytes / secsn / 1e9, 4),
        "unit": "GB/s",
        "cores": ncores,
        "kind": "oracle",
        "sample": "M=%d matmul of every tensor of the first %d layer(s) (%d tensors, %.1f MB packed): %.1f s on 1 core, %.1f s with the rows of each tensor dealt to %d threads"
        % (M, n_layers, len(sample), nbytes / 1e6, secs1, secsn, ncores),
        "single_core": {"value": round(nbytes / secs1 / 1e9, 4), "unit": "GB/s", "cores": 1, "seconds": round(secs1, 2)},
        "host_cpus_visible": os.cpu_count(),
        "gpu_vs_oracle_max_rel_l2": worst,
    }


if __name__ == "__main__":
    main()
