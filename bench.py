#!/usr/bin/env python3
"""Benchmark of the W4A16 GPTQ matrix multiply on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W]

Workload (the decode batch sweep configuration at M = 1, the case the HBM metric is quoted on):
one "step" is a decode pass over LAYERS distinct Llama-7B-shaped layers, four GEMVs each
(fused QKV 4096x12288, O 4096x4096, fused gate+up 4096x22016, down 11008x4096; group 128).
Every layer has its own weights, so the working set (LAYERS x 105 MB) is far larger than the
256 MB memory-side cache and every launch streams its weights from HBM.  All inputs are
resident in HBM before the timed region.  value = algorithmic bytes of a step / time of a step.

The same JSON line also carries the prefill half of the metric (fp16 MFMA TFLOP/s at M = 2048
on the three Llama-7B shapes), the roofline of the dominant kernel of each regime, and the CPU
oracle timed on this machine's host cores on a bounded sample of the same workload.
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

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E, published
MFMA_FP16_PEAK_TFLOPS = 2500.0  # MI355X dense fp16, published
GROUP = 128
QUICK = False


def algorithmic_bytes(M, K, N, group=GROUP, act_order=False):
    """Each operand once: packed weights, scales, packed zeros, activations, output (+ g_idx)."""
    groups = K // group
    b = K * N // 2 + groups * N * 2 + groups * (N // 8) * 4 + 2 * M * K + 2 * M * N
    return b + (4 * K if act_order else 0)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--layers", type=int, default=32, help="distinct layers per decode step")
    ap.add_argument("--no-cpu-baseline", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-prefill", action="store_true", help="skip the prefill (MFMA) leg")
    ap.add_argument("--no-graph", action="store_true", help="launch every kernel eagerly instead of replaying a HIP graph")
    ap.add_argument("--no-context", action="store_true", help="skip the device-copy / dense-matmul context lines")
    ap.add_argument("--no-sweep", action="store_true", help="skip the batch-size / act-order / 70B side tables")
    ap.add_argument("--ablation", action="store_true",
                    help="time the vector kernel with each of the paper's three techniques taken out (part of the "
                         "default run; this switch keeps it when --no-sweep drops the other side tables)")
    ap.add_argument("--quick", action="store_true",
                    help="few launches per leg and no clock settling: for runs under a profiler, where the launch "
                         "counts matter and the printed rates do not")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one 1 GiB device copy (reference kernel for the HBM traffic counters)")
    args = ap.parse_args()
    global QUICK
    QUICK = args.quick
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no sharding, no collectives); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        sys.exit(1)
    from paper_2511_19438_amd import binding as B
    from paper_2511_19438_amd import workloads

    B.load()
    torch.cuda.set_device(0)
    shapes = workloads.LLAMA_7B
    M = 1

    # ---- inputs: distinct seeded weights per layer, resident in HBM ----
    layers = []
    host_layer0 = None
    for layer in range(args.layers):
        mats = []
        for si, sh in enumerate(shapes):
            seed = workloads.case_seed(1, si) + 100 * layer
            w = workloads.make_weights(sh.K, sh.N, GROUP, seed=seed)
            x = workloads.make_activations(M, sh.K, seed=seed)
            if layer == 0:
                host_layer0 = host_layer0 or []
                host_layer0.append(dict(w, x=x))
            mats.append({
                "x": torch.from_numpy(x).cuda(),
                "qweight": torch.from_numpy(w["qweight"]).cuda(),
                "qzeros": torch.from_numpy(w["qzeros"]).cuda(),
                "scales": torch.from_numpy(w["scales"]).cuda(),
                "out": torch.empty((M, sh.N), dtype=torch.float16, device="cuda"),
            })
        layers.append(mats)
    launches_per_step = args.layers * len(shapes)
    bytes_per_step = args.layers * sum(algorithmic_bytes(M, sh.K, sh.N) for sh in shapes)

    def step():
        for mats in layers:
            for t in mats:
                B.gptq_w4a16_gemm(t["x"], t["qweight"], t["qzeros"], t["scales"], None, t["out"], GROUP)

    # One step = one HIP graph of all launches (captured once; replaying it removes the host's per-launch
    # cost, which at 1-10 us per kernel would otherwise be what is measured).  --no-graph launches eagerly.
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        step()  # first call sizes the library's split-K scratch (the only allocation it ever makes)
        torch.cuda.synchronize()
        run_step = step
        if not args.no_graph:
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=stream):
                step()
            run_step = graph.replay
        for _ in range(args.warmup):
            run_step()
        torch.cuda.synchronize()
        # events are recorded on the stream the kernels run on
        ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        ev0.record(stream)
        for _ in range(args.steps):
            run_step()
        ev1.record(stream)
        torch.cuda.synchronize()
        wall = time.perf_counter() - t0
    gpu_s = ev0.elapsed_time(ev1) * 1e-3
    ms_per_step = wall * 1e3 / args.steps
    value = bytes_per_step * args.steps / wall / 1e9

    # sanity: the timed path computed the right thing (layer 0, smallest shape, against the oracle)
    import oracle

    chk = host_layer0[1]
    ref = oracle.gemm_ref(chk["x"], chk["qweight"], chk["qzeros"], chk["scales"], None, GROUP)
    got = layers[0][1]["out"].cpu().numpy().astype(np.float64)
    max_ratio = float((np.abs(got - ref) / (2e-2 * np.maximum(1.0, np.abs(ref)))).max())
    if not max_ratio <= 1.0:
        print(f"bench.py: GPU result outside the tolerance band (err/tol = {max_ratio})", file=sys.stderr)
        sys.exit(1)

    # ---- roofline of the dominant kernel: the M=1 vector kernel, averaged over the launches of the timed region ----
    avg_launch_s = gpu_s / (args.steps * launches_per_step)
    bytes_per_launch = bytes_per_step / launches_per_step
    achieved = bytes_per_launch / avg_launch_s / 1e9
    roofline = {"bound": "hbm", "kernel": "decode_kernel<MB=1> (split-K vector kernel)",
                "achieved": round(achieved, 1), "peak": HBM_PEAK_GBS, "unit": "GB/s",
                "frac": round(achieved / HBM_PEAK_GBS, 4), "traffic": measured_traffic("decode_m1_llama7b"),
                "bytes_per_launch": int(bytes_per_launch), "avg_launch_us": round(avg_launch_s * 1e6, 3)}
    if args.calibrate_copy:
        # a plain copy of known size in the same process: the scale for the FETCH_SIZE / WRITE_SIZE counters
        src = torch.empty(256 * 1024 * 1024, dtype=torch.int32, device="cuda").random_()
        dst = torch.empty_like(src)
        dst.copy_(src)
        torch.cuda.synchronize()
        del src, dst

    # ---- prefill half of the metric: M = 2048 on the 7B shapes ----
    prefill = None
    if not args.no_prefill:
        prefill = prefill_leg(torch, B, workloads, layers)

    # ---- CPU oracle on this machine's host cores, bounded sample: layer 0 of the same workload ----
    cpu = None
    if not args.no_cpu_baseline:
        reps, spent = 0, 0.0
        while spent < 10.0 and reps < 50:
            t = time.perf_counter()
            for c in host_layer0:
                oracle.gemm_ref(c["x"], c["qweight"], c["qzeros"], c["scales"], None, GROUP)
            spent += time.perf_counter() - t
            reps += 1
        layer_bytes = sum(algorithmic_bytes(M, sh.K, sh.N) for sh in shapes)
        cpu = {"value": round(layer_bytes * reps / spent / 1e9, 3), "unit": "GB/s", "cores": oracle.num_threads(),
               "kind": "oracle",
               "sample": f"layer 0 of the step (4 GEMVs, {layer_bytes / 1e6:.1f} MB algorithmic), {reps} repetitions, "
                         f"{spent:.1f} s"}
        # the prefill half of the metric on the same cores: a row sample of the M = 2048 problem on the qkv shape
        rows = 16
        c = host_layer0[0]
        xs = workloads.make_activations(2048, shapes[0].K, seed=workloads.case_seed(3, 0))[:rows]
        t = time.perf_counter()
        oracle.gemm_ref(xs, c["qweight"], c["qzeros"], c["scales"], None, GROUP)
        dt = time.perf_counter() - t
        cpu["prefill"] = {"value": round(2.0 * rows * shapes[0].K * shapes[0].N / dt / 1e9, 2), "unit": "GFLOP/s",
                          "sample": f"{rows} of the 2048 rows of M=2048 K={shapes[0].K} N={shapes[0].N} "
                                    f"(all columns), {dt:.1f} s; the full problem would take {dt * 2048 / rows:.0f} s"}

    line = {
        "metric": "W4A16 GEMM: HBM GB/s at M=1 decode; TFLOP/s at M=2048 prefill",
        "value": round(value, 1), "unit": "GB/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "fp16 x int4 -> fp32 accumulate", "data": "synthetic",
        "config": {"workload": f"decode M=1, {args.layers} distinct Llama-7B-shaped layers x "
                               "{qkv 4096x12288, o 4096x4096, gate_up 4096x22016, down 11008x4096}, group 128",
                   "launches_per_step": launches_per_step, "algorithmic_bytes_per_step": int(bytes_per_step),
                   "launch": "eager" if args.no_graph else "hip_graph",
                   "check_err_over_tol": round(max_ratio, 4)},
        "roofline": roofline,
        "cpu_baseline": cpu,
    }
    if prefill:
        line["prefill"] = prefill["summary"]
        line["roofline_prefill"] = prefill["roofline"]
    if not args.no_sweep:
        line["sweep"] = sweep_tables(torch, B, workloads, layers)
    if args.ablation or not args.no_sweep:
        line["ablation"] = ablation_table(torch, B, workloads, layers)
    if not args.no_context:
        line["context"] = context_lines(torch, B)
    print(json.dumps(line))


def graph_us(torch, launches, reps=4, batches=3):
    """Microseconds per launch of a list of zero-argument launch functions, replayed as one HIP graph: the median
    of `batches` timed batches of `reps` replays each (a single batch now and then catches a hiccup of the box)."""
    stream = torch.cuda.Stream()
    with torch.cuda.stream(stream):
        for f in launches:
            f()
        torch.cuda.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=stream):
            for f in launches:
                f()
        graph.replay()
        torch.cuda.synchronize()
        times = []
        for _ in range(batches):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(reps):
                graph.replay()
            e1.record(stream)
            torch.cuda.synchronize()
            times.append(e0.elapsed_time(e1) * 1e3 / (reps * len(launches)))
    del graph
    return sorted(times)[len(times) // 2]


def sweep_tables(torch, B, workloads, layers):
    """Side tables (not the headline): the decode and mid batch sweep on the Llama-7B shapes, the act-order layer with
    its g_idx kernels and repacked, and the Llama-70B shapes at M = 1, 16 and 64.  Every launch streams its weights from
    HBM (the launches of a graph rotate over distinct weight copies larger than the caches).  Per shape also:
    `read_probe`, a plain read kernel over the same packed-weight buffers timed the same way (what any kernel of
    that footprint pays for launch, latency and ramp), and `vector_dot`, the single-row kernel with its inner loop
    on the vector ALU only (v_dot2_f32_f16) instead of 4x4x4 MFMAs."""
    shapes = workloads.LLAMA_7B
    out = {"unit": "us per launch (GB/s of algorithmic bytes[, fraction of the 8 TB/s peak])", "llama7b": [],
           "act_order": [], "llama70b": []}
    sink = torch.zeros(256, dtype=torch.int32, device="cuda")
    vdot = B.Plan(kernel=1, flags=8)
    for si, sh in enumerate(shapes):
        row = {"shape": f"{sh.name} K={sh.K} N={sh.N}"}
        for M in workloads.DECODE_BATCHES + workloads.MID_BATCHES:
            x = torch.randn((M, sh.K), device="cuda").half()
            o = torch.empty((M, sh.N), dtype=torch.float16, device="cuda")
            fns = [(lambda t=mats[si]: B.gptq_w4a16_gemm(x, t["qweight"], t["qzeros"], t["scales"], None, o, GROUP))
                   for mats in layers]
            us = graph_us(torch, fns)
            gbs = algorithmic_bytes(M, sh.K, sh.N) / us / 1e3
            row[f"M={M}"] = [round(us, 2), round(gbs), round(gbs / HBM_PEAK_GBS, 3)]
        x = torch.randn((1, sh.K), device="cuda").half()
        o = torch.empty((1, sh.N), dtype=torch.float16, device="cuda")
        us = graph_us(torch, [(lambda t=mats[si]: B.gptq_w4a16_gemm(x, t["qweight"], t["qzeros"], t["scales"], None, o,
                                                                    GROUP, vdot)) for mats in layers])
        row["vector_dot M=1"] = [round(us, 2), round(algorithmic_bytes(1, sh.K, sh.N) / us / 1e3)]
        us = graph_us(torch, [(lambda t=mats[si]: B.gptq_w4a16_stream_probe(t["qweight"], sink)) for mats in layers])
        row["read_probe"] = [round(us, 2), round(sh.K * sh.N // 2 / us / 1e3)]
        # the three MFMA kernels side by side at 64 rows (explicit plans; the automatic one is in "M=64")
        x = torch.randn((64, sh.K), device="cuda").half()
        o = torch.empty((64, sh.N), dtype=torch.float16, device="cuda")
        side = {}
        for name, kid in (("mid_batch", 4), ("big_tile", 2), ("small_batch", 3)):
            plan = B.Plan(kernel=kid)
            side[name] = round(graph_us(torch, [(lambda t=mats[si]: B.gptq_w4a16_gemm(
                x, t["qweight"], t["qzeros"], t["scales"], None, o, GROUP, plan)) for mats in layers], batches=1), 2)
        row["kernels at M=64"] = side
        out["llama7b"].append(row)
    gen = torch.Generator(device="cuda")
    gen.manual_seed(1234)

    # act-order layer (rows of a group scattered over K): the kernels that look g_idx up per row, and the same
    # layer after the one-time repack
    sh = workloads.ACT_ORDER_SHAPE
    copies = 24
    qws, qz, sc = device_weights(torch, sh.K, sh.N, copies, gen)
    g_idx = (torch.randperm(sh.K, device="cuda", generator=gen) // GROUP).int()
    sorted_qws = [torch.empty_like(q) for q in qws]
    perm = torch.empty(sh.K, dtype=torch.int32, device="cuda")
    for q, qs in zip(qws, sorted_qws):
        B.gptq_w4a16_act_order_prepare(q, g_idx, qs, perm, GROUP)
    for M in (1, 8):
        x = torch.randn((M, sh.K), device="cuda").half()
        o = torch.empty((M, sh.N), dtype=torch.float16, device="cuda")
        a = graph_us(torch, [(lambda q=q: B.gptq_w4a16_gemm(x, q, qz, sc, g_idx, o, GROUP)) for q in qws])
        b = graph_us(torch, [(lambda q=q: B.gptq_w4a16_gemm_prepared(x, q, qz, sc, perm, o, GROUP)) for q in sorted_qws])
        c = graph_us(torch, [(lambda q=q: B.gptq_w4a16_gemm(x, q, qz, sc, None, o, GROUP)) for q in qws])
        nbytes = algorithmic_bytes(M, sh.K, sh.N, act_order=True)
        out["act_order"].append({"shape": f"K={sh.K} N={sh.N} M={M}", "g_idx_kernel": [round(a, 2), round(nbytes / a / 1e3)],
                                 "repacked": [round(b, 2), round(nbytes / b / 1e3)],
                                 "plain_format_same_shape": [round(c, 2), round(nbytes / c / 1e3)]})
    del qws, sorted_qws
    torch.cuda.empty_cache()
    # format variants: smaller quantisation groups on the qkv shape (M = 1: vector kernel; M = 8: small-batch kernel
    # with two / four groups per 128-k unit; M = 2048: big-tile kernel, pipelined for multiples of 64)
    sh = shapes[0]
    out["group_sizes"] = []
    for group in (128, 64, 32):
        copies = 24
        qws = [torch.randint(-2**31, 2**31 - 1, (sh.K // 8, sh.N), dtype=torch.int32, device="cuda", generator=gen)
               for _ in range(copies)]
        qz = torch.randint(-2**31, 2**31 - 1, (sh.K // group, sh.N // 8), dtype=torch.int32, device="cuda", generator=gen)
        sc = (torch.rand((sh.K // group, sh.N), device="cuda", generator=gen) * 0.009 + 0.001).half()
        row = {"shape": f"{sh.name} K={sh.K} N={sh.N} group={group}"}
        for M in (1, 8):
            x = torch.randn((M, sh.K), device="cuda").half()
            o = torch.empty((M, sh.N), dtype=torch.float16, device="cuda")
            us = graph_us(torch, [(lambda q=q: B.gptq_w4a16_gemm(x, q, qz, sc, None, o, group)) for q in qws])
            row[f"M={M}"] = [round(us, 2), round(algorithmic_bytes(M, sh.K, sh.N, group) / us / 1e3)]
        x = torch.randn((2048, sh.K), device="cuda").half()
        o = torch.empty((2048, sh.N), dtype=torch.float16, device="cuda")
        sec = timed_launches(torch, lambda: B.gptq_w4a16_gemm(x, qws[0], qz, sc, None, o, group))
        row["M=2048"] = [round(sec * 1e6, 1), f"{2.0 * 2048 * sh.K * sh.N / sec / 1e12:.0f} TFLOP/s"]
        out["group_sizes"].append(row)
        del qws, qz, sc, x, o
        torch.cuda.empty_cache()
    for sh in workloads.LLAMA_70B:
        copies = max(2, int(1.3e9 // (sh.K * sh.N // 2)) + 1)
        qws, qz, sc = device_weights(torch, sh.K, sh.N, copies, gen)
        row = {"shape": f"{sh.name} K={sh.K} N={sh.N}"}
        for M in (1, 16, 64):
            x = torch.randn((M, sh.K), device="cuda").half()
            o = torch.empty((M, sh.N), dtype=torch.float16, device="cuda")
            us = graph_us(torch, [(lambda q=q: B.gptq_w4a16_gemm(x, q, qz, sc, None, o, GROUP)) for q in qws])
            gbs = algorithmic_bytes(M, sh.K, sh.N) / us / 1e3
            row[f"M={M}"] = [round(us, 2), round(gbs), round(gbs / HBM_PEAK_GBS, 3)]
        us = graph_us(torch, [(lambda q=q: B.gptq_w4a16_stream_probe(q, sink)) for q in qws])
        row["read_probe"] = [round(us, 2), round(sh.K * sh.N // 2 / us / 1e3)]
        out["llama70b"].append(row)
        del qws
        torch.cuda.empty_cache()
    return out


def ablation_table(torch, B, workloads, layers):
    """The vector kernel at M = 1 with each of the paper's three techniques taken out (and all of them): on-chip
    hierarchical reduction (SMB, Section 3.1), vectorised activation loads (VML, Section 3.2), packed half
    arithmetic (ILA, Section 3.3).  All variants on 64-column tiles with the same automatic K split."""
    names = {0: "all_on", 1: "no_smb", 2: "no_vml", 4: "no_ila", 7: "none_on"}
    out = {"unit": "us per launch", "M": 1, "rows": []}
    x_cache = {}
    for si, sh in enumerate(workloads.LLAMA_7B):
        row = {"shape": f"{sh.name} K={sh.K} N={sh.N}"}
        for flags, name in names.items():
            plan = B.Plan(kernel=1, tile=64, flags=flags)
            fns = [(lambda t=mats[si]: B.gptq_w4a16_gemm(t["x"], t["qweight"], t["qzeros"], t["scales"], None, t["out"],
                                                         GROUP, plan)) for mats in layers]
            row[name] = round(graph_us(torch, fns), 2)
        out["rows"].append(row)
    return out


def measured_traffic(key):
    """HBM bytes per launch measured with rocprofv3 counters (profiles/traffic.json), or None if not recorded."""
    path = os.path.join(ROOT, "profiles", "traffic.json")
    try:
        with open(path) as f:
            return json.load(f).get(key, {}).get("hbm_bytes_per_launch")
    except (OSError, ValueError):
        return None


def context_lines(torch, B):
    """What the box itself achieves, as context for the roofline fractions: a device copy, the dense fp16 matmul of
    the vendor library on the prefill shape, the matrix pipe alone (MFMA-only loop on random register operands,
    no memory traffic) under the same power budget, and the price of vector instructions beside an MFMA."""
    n = 256 * 1024 * 1024
    src = torch.empty(n, dtype=torch.int32, device="cuda").random_()
    dst = torch.empty_like(src)
    sec = timed_launches(torch, lambda: dst.copy_(src), min_warm_s=0.02, min_timed_s=0.02)
    copy_gbs = 2.0 * n * 4 / sec / 1e9
    del src, dst
    M, K, N = 2048, 4096, 22016
    x = torch.randn((M, K), device="cuda").half()
    w = torch.randn((K, N), device="cuda").half()
    sec = timed_launches(torch, lambda: torch.matmul(x, w))
    dense = 2.0 * M * K * N / sec / 1e12
    del x, w
    ops = (torch.rand(1 << 16, device="cuda") * 2.0 - 1.0).half()
    sink = torch.zeros(64, dtype=torch.float32, device="cuda")
    flops = [0.0]

    def probe():
        flops[0] = B.gptq_w4a16_mfma_probe(ops, sink, 4000)

    sec = timed_launches(torch, probe)
    mfma_only = flops[0] / sec / 1e12
    # what vector work beside an MFMA costs: ns per (one 32x32x16 MFMA + V packed-fp16 instructions) per SIMD,
    # with one and with two wavefronts per SIMD
    issue = {}
    for waves in (1, 2):
        row = {}
        for v in (0, 4, 8, 12, 16):
            count = [0.0]

            def group():
                count[0] = B.gptq_w4a16_issue_probe(ops, sink, 1000, v, waves)

            sec = timed_launches(torch, group, min_warm_s=0.03, min_timed_s=0.02)
            row[f"V={v}"] = round(sec * 1e9 / count[0], 2)
        issue[f"{waves} wavefront(s) per SIMD"] = row
    props = torch.cuda.get_device_properties(0)
    device = {"name": props.name, "arch": getattr(props, "gcnArchName", ""), "compute_units": props.multi_processor_count,
              "memory_GiB": round(props.total_memory / 2**30, 1)}
    clock_khz = getattr(props, "clock_rate", 0)
    if clock_khz:
        device["max_clock_MHz"] = round(clock_khz / 1e3)
    return {"device": device, "device_copy_GBps_read_plus_write": round(copy_gbs, 1),
            "torch_matmul_fp16_dense_TFLOPs_M2048_K4096_N22016": round(dense, 1),
            "mfma_only_loop_random_operands_TFLOPs": round(mfma_only, 1),
            "ns_per_mfma_with_V_vector_instructions": issue}


def timed_launches(torch, fn, min_warm_s=0.06, min_timed_s=0.03):
    """Mean seconds per call of fn (one kernel launch), after at least min_warm_s of the same launches: the chip's
    clock governor needs some tens of milliseconds of load before it settles (after an idle gap the first
    launches run 10-25 % slower), so short bursts measure the ramp, not the kernel."""
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    fn()
    torch.cuda.synchronize()
    e0.record()
    for _ in range(4):
        fn()
    e1.record()
    torch.cuda.synchronize()
    est = max(e0.elapsed_time(e1) * 1e-3 / 4, 1e-6)
    if QUICK:
        return est
    for _ in range(max(4, int(min_warm_s / est))):
        fn()
    reps = max(8, int(min_timed_s / est))
    torch.cuda.synchronize()
    e0.record()
    for _ in range(reps):
        fn()
    e1.record()
    torch.cuda.synchronize()
    return e0.elapsed_time(e1) * 1e-3 / reps


def device_weights(torch, K, N, copies, gen):
    """Random packed weights drawn on the device (uniform words: every nibble an independent uniform code)."""
    qws = [torch.randint(-2**31, 2**31 - 1, (K // 8, N), dtype=torch.int32, device="cuda", generator=gen)
           for _ in range(copies)]
    qz = torch.randint(-2**31, 2**31 - 1, (K // GROUP, N // 8), dtype=torch.int32, device="cuda", generator=gen)
    sc = (torch.rand((K // GROUP, N), device="cuda", generator=gen) * 0.009 + 0.001).half()
    return qws, qz, sc


def prefill_leg(torch, B, workloads, layers):
    """TFLOP/s of the big-tile MFMA kernel: the prefill configuration (M = 512 and 2048 on the three Llama-7B
    shapes) and the Llama-70B layer set at M = 2048."""
    gen = torch.Generator(device="cuda")
    gen.manual_seed(4321)

    def run(M, K, N, qw, qz, sc):
        x = (torch.randn((M, K), device="cuda", generator=gen)).half()
        out = torch.empty((M, N), dtype=torch.float16, device="cuda")
        sec = timed_launches(torch, lambda: B.gptq_w4a16_gemm(x, qw, qz, sc, None, out, GROUP))
        tf = 2.0 * M * K * N / sec / 1e12
        return {"shape": f"M={M} K={K} N={N}", "us": round(sec * 1e6, 1), "tflops": round(tf, 1),
                "frac_of_peak": round(tf / MFMA_FP16_PEAK_TFLOPS, 3)}

    shapes = workloads.LLAMA_7B
    rows7 = []
    for M in (2048, 512):
        for si in (0, 2, 3):  # qkv, gate_up, down
            sh, t = shapes[si], layers[0][si]
            rows7.append(run(M, sh.K, sh.N, t["qweight"], t["qzeros"], t["scales"]))
    rows70 = []
    for sh in workloads.LLAMA_70B:
        qws, qz, sc = device_weights(torch, sh.K, sh.N, 1, gen)
        rows70.append(run(2048, sh.K, sh.N, qws[0], qz, sc))
        del qws, qz, sc
        torch.cuda.empty_cache()
    head = rows7[:3]
    total_flops = sum(2.0 * 2048 * shapes[si].K * shapes[si].N for si in (0, 2, 3))
    agg = total_flops / (sum(r["us"] for r in head) * 1e-6) / 1e12
    dominant = max(head, key=lambda r: r["us"])
    return {
        "summary": {"value": round(agg, 1), "unit": "TFLOP/s", "M": 2048, "shapes": head,
                    "llama7b_M512": rows7[3:], "llama70b_M2048": rows70,
                    "timing": "per shape: >= 60 ms of untimed launches, then >= 30 ms timed (HIP events)"},
        "roofline": {"bound": "mfma", "kernel": f"prefill_pipelined_kernel (fp16 MFMA), {dominant['shape']}",
                     "achieved": dominant["tflops"], "peak": MFMA_FP16_PEAK_TFLOPS, "unit": "TFLOP/s",
                     "frac": round(dominant["tflops"] / MFMA_FP16_PEAK_TFLOPS, 4),
                     "traffic": measured_traffic("prefill_m2048_k4096_n22016")},
    }


if __name__ == "__main__":
    main()
