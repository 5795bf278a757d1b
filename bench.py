#!/usr/bin/env python3
"""Benchmark of the SRFT int4 KV-cache write + read path on one MI355X.

A step is one pass of the whole hot path over the workload's cache: every plan's fp16 K/V tensor is
quantized, then every plan's int4 record is dequantized.  By default (--batched auto) the read path goes through the
batched entry point, up to 64 plans per launch (measured faster than a launch per plan: fewer pipeline prologues),
and the write path does so only for plans with fewer than 65,536 vectors (for large plans a launch each is faster);
--batched on|off forces one way for both.
Inputs are synthetic, seeded, and resident in HBM before the timed region.  Prints ONE JSON line.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload NAME] [--no-cpu-baseline]

Beside the contract's keys the line carries per-path figures ("quantize", "dequantize"), for the default workload a
side measurement of the same launch shape at d = 256 ("d256_same_launch_shape", skip with --no-d256) and one timed
step of each of the other four configurations ("all_configs", skip with --no-all-configs: they are parity-test
cases, cache-resident or launch-bound except the d = 96 prefix read, and are flagged so), and on request the
streaming ceilings of the memory system (--ceiling), power and clock per path (--power), the decode-step append
(--decode-append) and scores against the stored keys (--scores).

Clocks: every duration in the line is HIP-event time on the stream the kernels are launched on (torch's current
stream, which is the stream handed to the library); "value" alone uses the host clock around the synchronised
timed region.  Back-to-back launches overlap their tails by a few per cent, so the per-launch average from events
is slightly below the kernel durations a profiler lists.
"""
from __future__ import annotations

import argparse
import json
import sys
import time

HBM_PEAK_GBPS = 8000.0          # MI355X published HBM3E peak

# HBM traffic measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE; profiles/hbm_traffic_d128_d256.txt), in bytes per
# vector, keyed by the kernel symbol and head dimension the measurement was taken on: a kernel without a recorded
# counter run reports null.  (FETCH_SIZE x its copy-kernel factor + WRITE_SIZE x its factor) KiB per dispatch x 1024 /
# vectors per dispatch.
MEASURED_TRAFFIC_PER_VECTOR = {
    ("srft_quantize_fold_batched_kernel", 128): 336.41,
    ("srft_dequantize_fold4_batched_kernel", 128): 336.23,
    ("srft_quantize_fold4_batched_kernel", 256): 672.66,
    ("srft_dequantize_fold4_batched_kernel", 256): 672.67,
}

# What a kernel that only streams the same bytes reaches on this machine (bench.py --ceiling, best over grid sizes and
# access kinds; profiles/stream_ceiling_d128_mixes.txt), GB/s: context beside the roofline, not the roofline.
MEASURED_STREAM_CEILING_GBPS = {
    "quantize": 5857.0,       # 8192 B read : 2560 B written per tile, non-temporal accesses, 512 workgroups (plain: 5439)
    "dequantize": 5475.0,     # 2560 : 8192, non-temporal, 768 workgroups (plain: 5403)
}

PAPER_CONTEXT = {   # Apple M1 GPU, Metal, fp32 input (paper Sec. 7.1): another machine, not a target
    "d128_ns_per_vec": 24.6, "d256_ns_per_vec": 50.0, "d128_gflops": 182.0,
}


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=3)
    ap.add_argument("--warmup", type=int, default=1)
    ap.add_argument("--workload", default="llama3-70b-128k")
    ap.add_argument("--plans", type=int, default=0, help="use only the first N plans (debugging; 0 = all)")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-all-configs", action="store_true",
                    help="skip the timed step of each of the other four configurations")
    ap.add_argument("--cpu-baseline-full", action="store_true",
                    help="time the oracle's two forms on 2^20 vectors per head dimension (minutes) instead of a "
                         "bounded sample each")
    ap.add_argument("--no-d256", action="store_true",
                    help="skip the d = 256 side measurement that rides along with the default workload")
    ap.add_argument("--max-workgroups", type=int, default=0)
    ap.add_argument("--batched", choices=["auto", "on", "off"], default="auto",
                    help="several plans per launch (auto: when a plan has fewer than 65,536 vectors)")
    ap.add_argument("--plans-per-launch", type=int, default=0,
                    help="plans per batched launch, both directions (at most 64); 0 = 64 for small plans, and for plans of "
                         "65536 vectors or more 16 on the write path and 4 on the read path")
    ap.add_argument("--plans-per-launch-write", type=int, default=0, help="the same for the write path only")
    ap.add_argument("--plans-per-launch-read", type=int, default=0, help="the same for the read path only")
    ap.add_argument("--ceiling", action="store_true",
                    help="also time the streaming kernel that has each path's read:write byte mix (HBM ceiling)")
    ap.add_argument("--decode-append", action="store_true",
                    help="also time the decode-step append of the decode-d96 workload: a launch per plan against "
                         "one batched launch")
    ap.add_argument("--scores", action="store_true",
                    help="also time srft_kv_scores (8 queries against plan 0's stored keys, read from the int4 record) "
                         "beside dequantizing those keys")
    ap.add_argument("--butterfly", action="store_true",
                    help="also time the write path in its butterfly form (fp32 FFT on the vector ALU, "
                         "srft_kv_quantize_butterfly) over the same plans, a launch per plan; also on the d = 256 side "
                         "measurement unless --no-d256")
    ap.add_argument("--power", action="store_true",
                    help="also run each path at d = 128 and d = 256 (8 x 1,048,576 vectors), on N(0,1) and on all-zero "
                         "data, and the streaming kernel with its byte mix, for about 3 s each while sampling socket "
                         "power and shader clock with amd-smi")
    ap.add_argument("--formats", action="store_true",
                    help="also time one 8,388,608-vector launch shape over every head dimension and record format "
                         "(group sizes, 8-bit codes, Walsh-Hadamard comparator), 30 launches each way")
    ap.add_argument("--copy-bytes", type=int, default=0,
                    help="also run the library's plain copy kernel over this many bytes (counter calibration)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU (vectors are independent; more GPUs would each take a share "
              "of the layers with no exchange); --gpus must be 1", file=sys.stderr)
        return 2

    import numpy as np
    import torch
    from paper_2605_05699_amd import binding as B
    from paper_2605_05699_amd import measure as M
    from paper_2605_05699_amd import workloads as W

    if not torch.cuda.is_available():
        print("bench.py: no GPU visible", file=sys.stderr)
        return 2
    B.lib()
    w = W.WORKLOADS[args.workload]
    dev = torch.device("cuda:0")
    n_plans = args.plans if args.plans > 0 else w.n_plans
    n = w.vectors_per_plan
    d, g, G = w.d, w.g, w.d // w.g
    bytes_per_vec = 2 * d + d // 2 + 4 * G

    # the whole cache, resident: fp16 in, int4 + scales record, fp16 out
    x = torch.empty(n_plans, n, d, dtype=torch.float16, device=dev)
    codes = torch.empty(n_plans, n, d // 2, dtype=torch.uint8, device=dev)
    scales = torch.empty(n_plans, n, G, dtype=torch.float32, device=dev)
    out = torch.empty(n_plans, n, d, dtype=torch.float16, device=dev)
    plans = []
    for p in range(n_plans):
        seed, lam, _ = W.plan_constants(w, p)
        plans.append(B.Plan(d, g, seed, lam))
        if args.max_workgroups:
            B.srft_plan_set_max_workgroups(plans[-1].handle, args.max_workgroups)
        W.fill_kv(x[p], w, p)
    torch.cuda.synchronize()

    stream = torch.cuda.current_stream()
    h = [pl.handle for pl in plans]
    # Plans per launch.  Small plans go 64 to a launch (a launch per plan would be launch-bound).  With plans of a
    # million vectors a few per launch are best, and the two directions differ: measured on this workload with 2 / 4 /
    # 8 / 16 plans per launch, write 5.36-5.56 / 5.43-5.60 / 5.56-5.61 / 5.61-5.70 TB/s (fewer launch tails), read
    # 5.29-5.32 / 5.40-5.55 / 5.33-5.44 / 5.18-5.21 TB/s (its workgroups spread over as many output buffers).
    batched_q = args.batched == "on" or (args.batched == "auto" and n_plans > 1)
    batched_d = args.batched == "on" or (args.batched == "auto" and n_plans > 1)
    small = n < 65536
    per_launch_q = args.plans_per_launch_write or args.plans_per_launch or (64 if small else 16)
    per_launch_d = args.plans_per_launch_read or args.plans_per_launch or (64 if small else 4)
    per_launch_q, per_launch_d = min(per_launch_q, 64), min(per_launch_d, 64)
    launches_q = -(-n_plans // per_launch_q) if batched_q else n_plans      # per step
    launches_d = -(-n_plans // per_launch_d) if batched_d else n_plans
    chunks_q = [slice(i, min(i + per_launch_q, n_plans)) for i in range(0, n_plans, per_launch_q)]
    chunks_d = [slice(i, min(i + per_launch_d, n_plans)) for i in range(0, n_plans, per_launch_d)]
    if batched_q:
        tables_q = [B.BatchTable(h[c], list(x[c]), list(codes[c]), list(scales[c])) for c in chunks_q]
    if batched_d:
        tables_d = [B.BatchTable(h[c], list(out[c]), list(codes[c]), list(scales[c])) for c in chunks_d]

    def step(ev=None):
        if ev:
            ev[0].record(stream)
        if batched_q:
            for t in tables_q:
                B.srft_kv_quantize_batched(t, stream)
        else:
            for p in range(n_plans):
                B.srft_kv_quantize(h[p], x[p], codes[p], scales[p], stream)
        if ev:
            ev[1].record(stream)
        if batched_d:
            for t in tables_d:
                B.srft_kv_dequantize_batched(t, stream)
        else:
            for p in range(n_plans):
                B.srft_kv_dequantize(h[p], codes[p], scales[p], out[p], stream)
        if ev:
            ev[2].record(stream)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    events = [[torch.cuda.Event(enable_timing=True) for _ in range(3)] for _ in range(args.steps)]
    t0 = time.perf_counter()
    for k in range(args.steps):
        step(events[k])
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    tq = sum(e[0].elapsed_time(e[1]) for e in events) / args.steps / 1e3     # seconds per step, write path
    td = sum(e[1].elapsed_time(e[2]) for e in events) / args.steps / 1e3     # read path
    total_vec = n_plans * n
    ms_per_step = wall / args.steps * 1e3

    def roof(t_phase, launches):
        per_launch_s = t_phase / launches
        achieved = total_vec * bytes_per_vec / t_phase / 1e9
        return per_launch_s, achieved

    ql, qa = roof(tq, launches_q)
    dl, da = roof(td, launches_d)
    launches = launches_q if tq >= td else launches_d
    dominant = "quantize" if tq >= td else "dequantize"
    # the symbol the profiler shows for it
    symbol = kernel_symbol(B, h[0], "quantize", batched_q) if tq >= td else kernel_symbol(B, h[0], "dequantize", batched_d)
    dom_l, dom_a = (ql, qa) if tq >= td else (dl, da)
    result = {
        "metric": "quantize+dequantize vectors/s (full write pass then full read pass over the cache)",
        "value": total_vec / (wall / args.steps),
        "unit": "vectors/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        # what the contraction runs in: exact fp16 inputs, matrices as fp16 hi + fp16 lo on f16 MFMA (about 22 bits),
        # fp32 accumulation and fp32 vector arithmetic for the quantizer
        "dtype": "f16 hi+lo MFMA, f32 accumulate",
        "data": "synthetic",
        "config": {"workload": w.name, "d": d, "group": g, "plans": n_plans, "vectors_per_plan": n,
                   "total_vectors": total_vec, "bytes_per_vector_each_direction": bytes_per_vec,
                   "launches_per_step": launches_q + launches_d,
                   "plans_per_launch": {"quantize": per_launch_q if batched_q else 1,
                                        "dequantize": per_launch_d if batched_d else 1},
                   "batched": {"quantize": batched_q, "dequantize": batched_d}},
        "quantize": {"vectors_per_s": total_vec / tq, "ns_per_vec": tq / total_vec * 1e9, "GBps": qa,
                     "hbm_frac": qa / HBM_PEAK_GBPS, "avg_launch_ms": ql * 1e3},
        "dequantize": {"vectors_per_s": total_vec / td, "ns_per_vec": td / total_vec * 1e9, "GBps": da,
                       "hbm_frac": da / HBM_PEAK_GBPS, "avg_launch_ms": dl * 1e3},
        "roofline": {"kernel": symbol, "bound": "hbm", "achieved": dom_a, "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                     "frac": dom_a / HBM_PEAK_GBPS,
                     "traffic": (MEASURED_TRAFFIC_PER_VECTOR[(symbol, d)] * total_vec / launches
                                 if (symbol, d) in MEASURED_TRAFFIC_PER_VECTOR else None),
                     "clock": "HIP events on the launch stream, average over the launches of the timed steps",
                     "algorithmic_bytes_per_launch": total_vec * bytes_per_vec // launches,
                     "avg_launch_ms": dom_l * 1e3,
                     # context, not the roofline: the rate of a pure stream with this kernel's byte mix
                     "stream_ceiling_GBps": MEASURED_STREAM_CEILING_GBPS.get(dominant) if d == 128 else None},
        "paper_context_apple_m1": PAPER_CONTEXT,
    }

    if w.name == "llama3-70b-128k" and not args.no_d256:
        # the metric names d = 256 beside d = 128: the same launch shape (1,048,576 vectors per plan) at d = 256
        result["d256_same_launch_shape"] = side_d256(B, W, torch, dev, stream, per_launch_q=per_launch_q, per_launch_d=per_launch_d,
                                                     butterfly=args.butterfly)
    if args.butterfly and d == 128 and g == 32:
        def b_pass():
            for p in range(n_plans):
                B.srft_kv_quantize_butterfly(h[p], x[p], codes[p], scales[p], stream)
        def m_pass():                            # the matrix-core form the same way: a launch per plan
            for p in range(n_plans):
                B.srft_kv_quantize(h[p], x[p], codes[p], scales[p], stream)
        tb, _ = timed_passes(torch, stream, b_pass, None, args.steps)
        tm, _ = timed_passes(torch, stream, m_pass, None, args.steps)      # (also restores the record)
        qm = total_vec * bytes_per_vec / tm / 1e9
        result["quantize_butterfly_form"] = {
            "what": "same plans, same record, the transform as fp32 FFT butterflies on the vector ALU (one vector per "
                    "lane) instead of the matrix-core contraction; a launch per plan",
            "GBps": total_vec * bytes_per_vec / tb / 1e9, "hbm_frac": total_vec * bytes_per_vec / tb / 1e9 / HBM_PEAK_GBPS,
            "vectors_per_s": total_vec / tb, "avg_launch_ms": tb / n_plans * 1e3,
            "matrix_core_form_GBps": qm, "ratio_matrix_core_over_butterfly": qm / (total_vec * bytes_per_vec / tb / 1e9)}
    if args.ceiling:
        result["hbm_ceiling"] = mix_ceiling(M, torch, x, out, n_plans * n, d, G, stream)
    if args.power:
        result["power"] = {"d128": power_phases(B, M, W, torch, dev, stream, 128),
                           "d256": power_phases(B, M, W, torch, dev, stream, 256)}
    if args.formats:
        result["formats"] = formats_sweep(B, W, torch, dev, stream)
    if args.scores:
        n_q = 8
        q = W.make_kv(w, 1, n_vec=n_q, device=dev)
        sc_out = torch.empty(n_q, n, dtype=torch.float32, device=dev)
        ws = torch.empty(B.lib().srft_scores_workspace_bytes(h[0]), dtype=torch.uint8, device=dev)
        B.srft_kv_quantize(h[0], x[0], codes[0], scales[0], stream)

        def timed(fn, iters=20):
            for _ in range(3):
                fn()
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(iters):
                fn()
            e1.record(stream)
            torch.cuda.synchronize()
            return e0.elapsed_time(e1) / iters * 1e-3
        ts = timed(lambda: B.srft_kv_scores(h[0], q, codes[0], scales[0], sc_out, ws, stream))
        tdq = timed(lambda: B.srft_kv_dequantize(h[0], codes[0], scales[0], out[0], stream))
        rec_bytes = d // 2 + 4 * G
        result["scores"] = {"queries": n_q, "keys": n, "us": ts * 1e6, "keys_per_s": n / ts,
                            "GBps_record_plus_scores": n * (rec_bytes + 4 * n_q) / ts / 1e9,
                            "dequantize_same_keys_us": tdq * 1e6}
        # the value side: weights (the softmax of those scores) times plan 1's stored values, and the whole decode step
        if n_plans > 1:
            B.srft_kv_quantize(h[1], x[1], codes[1], scales[1], stream)
            wts = torch.softmax(sc_out * d ** -0.5, dim=1)
            att = torch.empty(n_q, d, dtype=torch.float32, device=dev)
            wsa = torch.empty(B.lib().srft_attend_workspace_bytes(h[1]), dtype=torch.uint8, device=dev)
            ta = timed(lambda: B.srft_kv_attend(h[1], wts, codes[1], scales[1], att, wsa, stream))
            wsd = torch.empty(B.lib().srft_decode_attention_workspace_bytes(h[0], h[1], n_q, n), dtype=torch.uint8,
                              device=dev)
            tda = timed(lambda: B.srft_kv_decode_attention(h[0], h[1], q, codes[0], scales[0], codes[1], scales[1],
                                                           d ** -0.5, att, wsd, stream))
            # the same decode step recorded once into a HIP graph and replayed: the gaps between its launches close
            side = torch.cuda.Stream()
            side.wait_stream(stream)
            graph = torch.cuda.CUDAGraph()
            with torch.cuda.graph(graph, stream=side):
                B.srft_kv_decode_attention(h[0], h[1], q, codes[0], scales[0], codes[1], scales[1], d ** -0.5, att, wsd,
                                           torch.cuda.current_stream())
            torch.cuda.synchronize()
            tdg = timed(graph.replay)
            result["attend"] = {
                "queries": n_q, "values": n, "us": ta * 1e6, "values_per_s": n / ta,
                "bytes_read_per_value": {"record": rec_bytes, "weights": 4 * n_q, "dequantized_prefix_instead": 2 * d},
                "GBps_record_plus_weights": n * (rec_bytes + 4 * n_q) / ta / 1e9,
                "hbm_frac": n * (rec_bytes + 4 * n_q) / ta / 1e9 / HBM_PEAK_GBPS}
            result["decode_attention"] = {
                "queries": n_q, "keys": n, "us": tda * 1e6,
                "what": "scores over the K record (the scan keeps the row maxima), the V record weighted with "
                        "exp(scale * score - maximum) formed from the raw scores as they are loaded, divided by the sums "
                        "of those weights at the end: both records read once, the n_q x n_keys scores written once and "
                        "read once",
                "replayed_from_a_hip_graph_us": tdg * 1e6,
                "dequantize_K_and_V_instead_us": 2 * tdq * 1e6}
    if args.decode_append:
        result["decode_append"] = decode_append(B, W, torch, dev, stream)
    if args.copy_bytes:
        nb = args.copy_bytes // 16 * 16
        src = out.view(torch.uint8).reshape(-1)[:nb]
        dst = x.view(torch.uint8).reshape(-1)[:nb]
        for _ in range(2):
            M.srft_stream_copy(dst, src, stream)
        c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        c0.record(stream)
        for _ in range(5):
            M.srft_stream_copy(dst, src, stream)
        c1.record(stream)
        torch.cuda.synchronize()
        result["copy_kernel"] = {"bytes_each_way": nb, "GBps_read_plus_write": 2 * nb / (c0.elapsed_time(c1) / 5 * 1e-3) / 1e9}
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(w, x, plans, W, full=args.cpu_baseline_full)
    for pl in plans:
        pl.close()
    if w.name == "llama3-70b-128k" and not args.no_all_configs:
        del x, codes, scales, out
        torch.cuda.empty_cache()
        result["all_configs"] = all_configs(B, W, torch, dev, stream)
    print(json.dumps(result))
    return 0


def kernel_symbol(B, plan_handle, path, batched):
    """Name of the kernel the plan's launches of `path` ("quantize" / "dequantize") run: the form comes from the
    library (srft_plan_form), so the name cannot drift from what is launched."""
    form = B.lib().srft_plan_form(plan_handle, 0 if path == "quantize" else 1)
    if form < 0:
        raise RuntimeError(f"srft_plan_form: {form}")
    if path == "dequantize":
        stem = "srft_dequantize_fold4" if form == 2 else "srft_dequantize"
        return stem + ("_batched_kernel" if batched else "_kernel")
    stem = ("srft_quantize", "srft_quantize_fold", "srft_quantize_fold4")[form]
    return stem + ("_batched_kernel" if batched else "_kernel")


def timed_passes(torch, stream, q_pass, d_pass, reps, warm=1):
    """(seconds per write pass, seconds per read pass) from HIP events on `stream`; either pass may be None.
    `warm` untimed passes of each come first."""
    for fn in (q_pass, d_pass):
        for _ in range(warm if fn else 0):
            fn()
    torch.cuda.synchronize()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record(stream)
    for _ in range(reps if q_pass else 0):
        q_pass()
    ev[1].record(stream)
    for _ in range(reps if d_pass else 0):
        d_pass()
    ev[2].record(stream)
    torch.cuda.synchronize()
    return ev[0].elapsed_time(ev[1]) / reps / 1e3, ev[1].elapsed_time(ev[2]) / reps / 1e3


def all_configs(B, W, torch, dev, stream):
    """One timed step of each of the other four configurations, each with its full shape and its own buffers (freed
    before the next).  `regime` says what the figure is: "hbm" streams from HBM; "cache-resident" fits the 256 MB
    last-level cache, so its GB/s is not an HBM fraction; "launch-bound" is a few microseconds of work."""
    res = {}
    for name, regime, reps in (("tiny", "launch-bound", 200), ("qwen2.5-1.5b-4k", "cache-resident", 50),
                               ("gemma3-1b-4k", "cache-resident", 50)):
        w = W.WORKLOADS[name]
        n, d, G, k = w.vectors_per_plan, w.d, w.d // w.g, w.n_plans
        plans = [B.Plan(d, w.g, *W.plan_constants(w, p)[:2]) for p in range(k)]
        x = torch.empty(k, n, d, dtype=torch.float16, device=dev)
        for p in range(k):
            W.fill_kv(x[p], w, p)
        codes = torch.empty(k, n, d // 2, dtype=torch.uint8, device=dev)
        scales = torch.empty(k, n, G, dtype=torch.float32, device=dev)
        out = torch.empty(k, n, d, dtype=torch.float16, device=dev)
        h = [pl.handle for pl in plans]
        tq_tab = B.BatchTable(h, list(x), list(codes), list(scales))
        td_tab = B.BatchTable(h, list(out), list(codes), list(scales))
        tq, td = timed_passes(torch, stream, lambda: B.srft_kv_quantize_batched(tq_tab, stream),
                              lambda: B.srft_kv_dequantize_batched(td_tab, stream), reps, warm=reps)
        nbytes = k * n * (2 * d + d // 2 + 4 * G)
        res[name] = {"d": d, "plans": k, "vectors_per_plan": n, "regime": regime, "launches_per_step": 2,
                     "bytes_each_direction": nbytes, "us_per_step": (tq + td) * 1e6,
                     "quantize": {"us": tq * 1e6, "GBps": nbytes / tq / 1e9, "vectors_per_s": k * n / tq},
                     "dequantize": {"us": td * 1e6, "GBps": nbytes / td / 1e9, "vectors_per_s": k * n / td}}
        for pl in plans:
            pl.close()
        del x, codes, scales, out, tq_tab, td_tab
        torch.cuda.empty_cache()
    # configuration 4: the decode step appends 512 vectors to each of 64 plans (one batched launch), then every
    # plan's 4,194,304-vector int4 prefix is read (one batched launch over all 64 plans: 16 GB in, 51.5 GB out)
    w = W.WORKLOADS["decode-d96"]
    n, na, d, G, k = w.vectors_per_plan, w.append_vectors_per_plan, w.d, w.d // w.g, w.n_plans
    plans = [B.Plan(d, w.g, *W.plan_constants(w, p)[:2]) for p in range(k)]
    h = [pl.handle for pl in plans]
    xa = torch.empty(k, na, d, dtype=torch.float16, device=dev)
    for p in range(k):
        W.fill_kv(xa[p], w, p)
    ca = torch.empty(k, na, d // 2, dtype=torch.uint8, device=dev)
    sa = torch.empty(k, na, G, dtype=torch.float32, device=dev)
    ta = B.BatchTable(h, list(xa), list(ca), list(sa))
    t_app, _ = timed_passes(torch, stream, lambda: B.srft_kv_quantize_batched(ta, stream), None, 200)
    codes = torch.empty(k, n, d // 2, dtype=torch.uint8, device=dev)
    scales = torch.empty(k, n, G, dtype=torch.float32, device=dev)
    xbuf = torch.empty(n, d, dtype=torch.float16, device=dev)         # the prefix is produced plan after plan
    for p in range(k):
        W.fill_kv(xbuf, w, p)
        B.srft_kv_quantize(h[p], xbuf, codes[p], scales[p], stream)
    torch.cuda.synchronize()
    del xbuf
    out = torch.empty(k, n, d, dtype=torch.float16, device=dev)
    tp = B.BatchTable(h, list(out), list(codes), list(scales))
    _, t_pre = timed_passes(torch, stream, None, lambda: B.srft_kv_dequantize_batched(tp, stream), 2)
    ab, pb = k * na * (2 * d + d // 2 + 4 * G), k * n * (2 * d + d // 2 + 4 * G)
    res["decode-d96"] = {
        "d": d, "plans": k,
        "append": {"vectors_per_plan": na, "regime": "launch-bound", "launches_per_step": 1, "us": t_app * 1e6,
                   "bytes": ab, "GBps": ab / t_app / 1e9, "vectors_per_s": k * na / t_app},
        "prefix_read": {"vectors_per_plan": n, "regime": "hbm", "launches_per_step": 1, "ms": t_pre * 1e3,
                        "bytes": pb, "GBps": pb / t_pre / 1e9, "hbm_frac": pb / t_pre / 1e9 / HBM_PEAK_GBPS,
                        "vectors_per_s": k * n / t_pre}}
    for pl in plans:
        pl.close()
    return res


def side_d256(B, W, torch, dev, stream, n_plans=8, n=1 << 20, reps=10, warm=10, per_launch_q=16, per_launch_d=4,
              butterfly=False):
    """Write pass and read pass (plans per launch as in the main step, at most n_plans) over n_plans x n vectors of d = 256, g = 32:
    N(0,1) times a lognormal(0,1) channel scale and lognormal(0,0.5) lambda per plan, as in the d = 256 config.
    `warm` untimed passes of each path precede the `reps` timed ones (about 25 ms each way): after the idle gap in
    which the plans are built the first few milliseconds of work run 20-30 % slower than the steady state that the
    main step (160 launches, warmed up by a whole step) is timed in."""
    d, g = 256, 32
    G = d // g
    gen = torch.Generator(device=dev)
    x = torch.empty(n_plans, n, d, dtype=torch.float16, device=dev)
    plans = []
    for p in range(n_plans):
        gen.manual_seed(256_000 + p)
        gain = torch.exp(torch.randn(d, generator=gen, device=dev))
        x[p] = (torch.randn(n, d, generator=gen, device=dev) * gain).half()
        plans.append(B.Plan(d, g, 256_000 + p, W.lognormal_lambda(d, 256_000 + p)))
    codes = torch.empty(n_plans, n, d // 2, dtype=torch.uint8, device=dev)
    scales = torch.empty(n_plans, n, G, dtype=torch.float32, device=dev)
    out = torch.empty(n_plans, n, d, dtype=torch.float16, device=dev)
    h = [pl.handle for pl in plans]
    per_launch_q, per_launch_d = min(per_launch_q, n_plans), min(per_launch_d, n_plans)
    chunks_q = [slice(i, min(i + per_launch_q, n_plans)) for i in range(0, n_plans, per_launch_q)]
    chunks_d = [slice(i, min(i + per_launch_d, n_plans)) for i in range(0, n_plans, per_launch_d)]
    tables_q = [B.BatchTable(h[c], list(x[c]), list(codes[c]), list(scales[c])) for c in chunks_q]
    tables_d = [B.BatchTable(h[c], list(out[c]), list(codes[c]), list(scales[c])) for c in chunks_d]

    def pass_q():
        for t in tables_q:
            B.srft_kv_quantize_batched(t, stream)

    def pass_d():
        for t in tables_d:
            B.srft_kv_dequantize_batched(t, stream)

    for _ in range(warm):
        pass_q()
    for _ in range(warm):
        pass_d()
    for _ in range(2):
        pass_q()
    ev = [torch.cuda.Event(enable_timing=True) for _ in range(3)]
    ev[0].record(stream)
    for _ in range(reps):
        pass_q()
    ev[1].record(stream)
    for _ in range(reps):
        pass_d()
    ev[2].record(stream)
    torch.cuda.synchronize()
    nbytes = n_plans * n * (2 * d + d // 2 + 4 * G)
    tq, td = ev[0].elapsed_time(ev[1]) / reps / 1e3, ev[1].elapsed_time(ev[2]) / reps / 1e3
    bfly = None
    if butterfly:                                # the same record through the butterfly form, a launch per plan both ways
        def b_pass():
            for p in range(n_plans):
                B.srft_kv_quantize_butterfly(h[p], x[p], codes[p], scales[p], stream)
        def m_pass():
            for p in range(n_plans):
                B.srft_kv_quantize(h[p], x[p], codes[p], scales[p], stream)
        tb, _ = timed_passes(torch, stream, b_pass, None, reps, warm=2)
        tm, _ = timed_passes(torch, stream, m_pass, None, reps, warm=2)
        bfly = {"what": "the transform as fp32 FFT butterflies on the vector ALU, a vector on two lanes (length-64 FFTs in "
                        "registers, one decimation step and the Hermitian unpack across the lane pair); a launch per plan",
                "GBps": nbytes / tb / 1e9, "hbm_frac": nbytes / tb / 1e9 / HBM_PEAK_GBPS,
                "avg_launch_ms": tb / n_plans * 1e3, "matrix_core_form_GBps": nbytes / tm / 1e9,
                "ratio_matrix_core_over_butterfly": tb / tm}
    for pl in plans:
        pl.close()
    return {"d": d, "group": g, "plans": n_plans, "vectors_per_plan": n,
            "plans_per_launch": {"quantize": per_launch_q, "dequantize": per_launch_d},
            **({"quantize_butterfly_form": bfly} if bfly else {}),
            "quantize": {"GBps": nbytes / tq / 1e9, "hbm_frac": nbytes / tq / 1e9 / HBM_PEAK_GBPS,
                         "vectors_per_s": n_plans * n / tq},
            "dequantize": {"GBps": nbytes / td / 1e9, "hbm_frac": nbytes / td / 1e9 / HBM_PEAK_GBPS,
                           "vectors_per_s": n_plans * n / td}}


def mix_ceiling(M, torch, x, out, total_vec, d, G, stream):
    """Streaming kernel with the write path's and the read path's byte mix, no arithmetic: GB/s over a few grids."""
    big, small = 32 * 2 * d, 32 * (d // 2 + 4 * G)
    n_tiles = min(total_vec // 32, (2 << 30) // big)         # at most 2 GiB on the large side
    a, b = x.view(torch.uint8).reshape(-1), out.view(torch.uint8).reshape(-1)
    res = {"tiles": n_tiles, "read_write_bytes_per_tile": {"quantize_mix": [big, small], "dequantize_mix": [small, big]}}
    for name, (rb, wb), nt_acc in (("quantize_mix", (big, small), False), ("dequantize_mix", (small, big), False),
                                   ("quantize_mix_streaming_accesses", (big, small), 1),
                                   ("dequantize_mix_streaming_accesses", (small, big), 1),
                                   # every die walks a contiguous eighth of the tiles (plain / streaming accesses)
                                   ("quantize_mix_die_contiguous", (big, small), 4),
                                   ("dequantize_mix_die_contiguous", (small, big), 4),
                                   ("quantize_mix_die_contiguous_streaming_accesses", (big, small), 5),
                                   ("dequantize_mix_die_contiguous_streaming_accesses", (small, big), 5),
                                   # the write mix at d = 256 (16 KiB in : 5 KiB out per tile): 16 bytes per lane and
                                   # load, against every lane reading 64 contiguous bytes with four loads
                                   ("quantize_mix_d256", (16384, 5120), 0),
                                   ("quantize_mix_d256_streaming_accesses", (16384, 5120), 1),
                                   ("quantize_mix_d256_64B_per_lane", (16384, 5120), 2),
                                   ("quantize_mix_d256_64B_per_lane_streaming_accesses", (16384, 5120), 3)):
        n_tiles = min(total_vec // 32, (2 << 30) // max(rb, wb))
        best = {}
        for wgs in (512, 768, 1024, 2048, 4096, 8192):
            for _ in range(3):
                M.srft_stream_mix(a, b, n_tiles, rb, wb, wgs, nt_acc, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                M.srft_stream_mix(a, b, n_tiles, rb, wb, wgs, nt_acc, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            best[str(wgs)] = n_tiles * (rb + wb) / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9
        res[name + "_GBps_by_workgroups"] = best
        res[name + "_GBps"] = max(best.values())
    # what the machine gives plain streams (16 KiB per tile on the side that moves): read only, write only, copy
    plain = {}
    for name, (rb, wb) in (("read_only", (16384, 0)), ("write_only", (0, 16384)), ("copy", (16384, 16384)),
                           ("read4_write1", (16384, 4096)), ("read1_write4", (4096, 16384))):
        nt = min(2 << 30, a.numel(), b.numel()) // 16384       # up to 2 GiB per side, inside both buffers
        best = 0.0
        for wgs in (512, 1024, 4096, 16384):
            for _ in range(2):
                M.srft_stream_mix(a, b, nt, rb, wb, wgs, False, stream)
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record(stream)
            for _ in range(10):
                M.srft_stream_mix(a, b, nt, rb, wb, wgs, False, stream)
            e1.record(stream)
            torch.cuda.synchronize()
            best = max(best, nt * (rb + wb) / (e0.elapsed_time(e1) / 10 * 1e-3) / 1e9)
        plain[name] = best
    res["plain_streams_GBps"] = plain
    return res


def sampled_phase(torch, fn, bytes_per_call, seconds=3.0):
    """Run fn back to back for `seconds`; a thread samples `amd-smi metric --power --clock` meanwhile.
    Returns the sustained GB/s and the mean socket power / shader clock over the samples (the first is dropped)."""
    import subprocess
    import threading
    samples, stop = [], threading.Event()

    def sampler():
        while not stop.is_set():
            try:
                js = json.loads(subprocess.run(["amd-smi", "metric", "--power", "--clock", "--json"],
                                               capture_output=True, text=True, timeout=10).stdout)
                g = js["gpu_data"][0] if isinstance(js, dict) else js[0]
                clk = [v["clk"]["value"] for k, v in g["clock"].items() if k.startswith("gfx_") and
                       isinstance(v.get("clk"), dict)]
                samples.append((g["power"]["socket_power"]["value"], sum(clk) / max(1, len(clk))))
            except Exception:
                pass
            stop.wait(0.2)

    fn()
    torch.cuda.synchronize()
    th = threading.Thread(target=sampler, daemon=True)
    th.start()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0, calls = time.perf_counter(), 0
    e0.record()
    while time.perf_counter() - t0 < seconds:
        fn()
        calls += 1
        torch.cuda.synchronize()
    e1.record()
    torch.cuda.synchronize()
    stop.set()
    th.join()
    use = samples[1:] if len(samples) > 2 else samples
    return {"GBps": calls * bytes_per_call / (e0.elapsed_time(e1) * 1e-3) / 1e9, "samples": len(use),
            "socket_power_W": sum(a for a, _ in use) / max(1, len(use)),
            "shader_clock_MHz": sum(b for _, b in use) / max(1, len(use))}


def formats_sweep(B, W, torch, dev, stream, n=1 << 23, reps=30, warm=10):
    """Steady-state rate of both paths for every head dimension and record format: one plan, n vectors per launch,
    N(0,1) input, lognormal lambda; `warm` untimed launches, then `reps` timed ones, each way."""
    rows = []
    for d, g, bits, tr in [(32, 32, 4, "dft"), (64, 32, 4, "dft"), (96, 32, 4, "dft"), (128, 32, 4, "dft"),
                           (192, 32, 4, "dft"), (256, 32, 4, "dft"),
                           (128, 16, 4, "dft"), (128, 64, 4, "dft"), (128, 128, 4, "dft"), (128, 32, 8, "dft"),
                           (128, 128, 8, "dft"), (128, 32, 4, "hadamard"), (256, 32, 8, "dft"), (256, 256, 4, "dft"),
                           (96, 32, 8, "dft")]:
        plan = B.Plan(d, g, 3, W.lognormal_lambda(d, 1), bits=bits, transform=tr)
        x = torch.randn(n, d, device=dev, dtype=torch.float16)
        codes, scales = plan.quantize(x)
        out = plan.dequantize(codes, scales)
        tq, td = timed_passes(torch, stream, lambda: B.srft_kv_quantize(plan.handle, x, codes, scales, stream),
                              lambda: B.srft_kv_dequantize(plan.handle, codes, scales, out, stream), reps, warm=warm)
        nb = n * (2 * d + d * bits // 8 + 4 * d // g)
        rows.append({"d": d, "group": g, "bits": bits, "transform": tr, "bytes_per_vector": nb // n,
                     "quantize_GBps": nb / tq / 1e9, "dequantize_GBps": nb / td / 1e9,
                     "quantize_us": tq * 1e6, "dequantize_us": td * 1e6})
        plan.close()
        del x, codes, scales, out
        torch.cuda.empty_cache()
    # the lambda calibration statistic (per-channel abs-max of the transform's output): reads 2 d bytes per vector
    cal = []
    for d in (96, 128, 256):
        plan = B.Plan(d, 32, 3, None)
        x = torch.randn(n, d, device=dev, dtype=torch.float16)
        amax = torch.zeros(d, dtype=torch.float32, device=dev)
        tc, _ = timed_passes(torch, stream, lambda: B.srft_kv_channel_absmax(plan.handle, x, amax, stream), None, reps,
                             warm=warm)
        cal.append({"d": d, "us": tc * 1e6, "GBps_input_read": n * 2 * d / tc / 1e9})
        plan.close()
        del x
        torch.cuda.empty_cache()
    return {"vectors_per_launch": n, "launches_timed": reps, "rows": rows, "channel_absmax": cal}


def power_phases(B, M, W, torch, dev, stream, d, n_plans=8, n=1 << 20):
    """Sustained rate, socket power and shader clock of both paths over n_plans x n vectors of head dimension d
    (g = 32, 4 bits): on N(0,1) input, on all-zero input (the same instruction stream with nothing toggling in the
    data paths), and of a pure stream with each path's byte mix."""
    G = d // 32
    x = torch.randn(n_plans, n, d, device=dev).half()
    plans = [B.Plan(d, 32, 7_000 + p, W.lognormal_lambda(d, 7_000 + p)) for p in range(n_plans)]
    codes = torch.empty(n_plans, n, d // 2, dtype=torch.uint8, device=dev)
    scales = torch.empty(n_plans, n, G, dtype=torch.float32, device=dev)
    out = torch.empty_like(x)
    h = [pl.handle for pl in plans]
    table = B.BatchTable(h, list(out), list(codes), list(scales))

    def q_pass():
        for p in range(n_plans):
            B.srft_kv_quantize(h[p], x[p], codes[p], scales[p], stream)

    def d_pass():
        B.srft_kv_dequantize_batched(table, stream)
    nbytes = n_plans * n * (2 * d + d // 2 + 4 * G)
    big, small = 32 * 2 * d, 32 * (d // 2 + 4 * G)
    tiles = min(n_plans * n // 32, (2 << 30) // big)
    xa, xb = x.view(torch.uint8).reshape(-1), out.view(torch.uint8).reshape(-1)
    res = {"plans": n_plans, "vectors_per_plan": n}
    res["quantize"] = sampled_phase(torch, q_pass, nbytes)
    res["dequantize"] = sampled_phase(torch, d_pass, nbytes)
    res["stream_quantize_mix"] = sampled_phase(
        torch, lambda: M.srft_stream_mix(xa, xb, tiles, big, small, 768, False, stream), tiles * (big + small))
    res["stream_dequantize_mix"] = sampled_phase(
        torch, lambda: M.srft_stream_mix(xa, xb, tiles, small, big, 768, False, stream), tiles * (big + small))
    x.zero_()
    res["quantize_all_zero_input"] = sampled_phase(torch, q_pass, nbytes)       # leaves zero codes and scales
    res["dequantize_all_zero_record"] = sampled_phase(torch, d_pass, nbytes)
    for pl in plans:
        pl.close()
    return res


def decode_append(B, W, torch, dev, stream, iters=200):
    """One decode step of the decode-d96 workload: every plan appends batch x kv_heads new vectors (write path)
    and, for comparison, reads the same few back.  Microseconds per step, a launch per plan against one batched
    launch per direction."""
    w = W.WORKLOADS["decode-d96"]
    n, d, G, k = w.append_vectors_per_plan, w.d, w.d // w.g, w.n_plans
    plans = [B.Plan(d, w.g, *W.plan_constants(w, p)[:2]) for p in range(k)]
    x = torch.empty(k, n, d, dtype=torch.float16, device=dev)
    for p in range(k):
        W.fill_kv(x[p], w, p)
    codes = torch.empty(k, n, d // 2, dtype=torch.uint8, device=dev)
    scales = torch.empty(k, n, G, dtype=torch.float32, device=dev)
    out = torch.empty(k, n, d, dtype=torch.float16, device=dev)
    h = [pl.handle for pl in plans]
    tq = B.BatchTable(h, list(x), list(codes), list(scales))
    td = B.BatchTable(h, list(out), list(codes), list(scales))

    def timed(fn):
        for _ in range(10):
            fn()
        torch.cuda.synchronize()
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        t0 = time.perf_counter()
        e0.record(stream)
        for _ in range(iters):
            fn()
        e1.record(stream)
        torch.cuda.synchronize()
        return {"gpu_us": e0.elapsed_time(e1) / iters * 1e3, "wall_us": (time.perf_counter() - t0) / iters * 1e6}

    def per_plan_q():
        for p in range(k):
            B.srft_kv_quantize(h[p], x[p], codes[p], scales[p], stream)

    def per_plan_d():
        for p in range(k):
            B.srft_kv_dequantize(h[p], codes[p], scales[p], out[p], stream)

    res = {"workload": w.name, "plans": k, "vectors_per_plan": n, "d": d,
           "bytes_per_step_each_direction": k * n * (2 * d + d // 2 + 4 * G),
           "quantize_per_plan": timed(per_plan_q),
           "quantize_batched": timed(lambda: B.srft_kv_quantize_batched(tq, stream)),
           "dequantize_per_plan": timed(per_plan_d),
           "dequantize_batched": timed(lambda: B.srft_kv_dequantize_batched(td, stream))}
    # the same step through the cache manager: 15 steps of 16 only copy the token into the window, the 16th also
    # quantizes the full page of every plan and writes its reconstruction into the view (three launches)
    R, steps = 16, 320
    cache = B.Cache(plans, n, steps, R, device=dev)
    new = [x[p].view(n, 1, d) for p in range(k)]
    prepared = cache.prepare(new)                            # static buffers: the pointer table is built once
    cache.append_prepared(prepared, stream)                  # first call outside the timed region
    torch.cuda.synchronize()
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    e0.record(stream)
    for _ in range(steps - 1):
        cache.append_prepared(prepared, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    res["cache_manager_step"] = {"residual_tokens": R, "steps": steps - 1, "flushes": (steps // R),
                                 "gpu_us": e0.elapsed_time(e1) / (steps - 1) * 1e3,
                                 "wall_us": (time.perf_counter() - t0) / (steps - 1) * 1e6}
    cache.close()
    for pl in plans:
        pl.close()
    return res


def cpu_baseline(w, x, plans, W, budget_s=8.0, max_vectors=1 << 23, full=False):
    """The oracle as it stands, timed on this host's cores (rank 0, N = 1 only).

    `value`: write + read path over a bounded sample of the workload (chunks of 131,072 vectors, plan after plan, until
    about `budget_s` seconds are spent), in the oracle's dense form.  `forms`: the oracle's two forms of the transform
    (the dense d x d definition, and its mixed-radix FFT with the packing of Eq. 2) at d = 96, 128, 256, write and read
    path each, on a bounded sample per entry (about 1.5 s; 2^20 vectors each with --cpu-baseline-full).  The dense
    form is a BLAS product and uses every core numpy's BLAS is given; the FFT form is numpy element-wise code on one
    core.  A baseline, not a target."""
    import numpy as np
    from oracle import srft_oracle as O
    try:
        from threadpoolctl import threadpool_info
        cores = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        cores = 1
    tq = td = 0.0
    sample = 0
    used_plans = 0
    for p in range(len(plans)):
        _, lam, _ = W.plan_constants(w, p)
        s = plans[p].signs
        used_plans += 1
        for lo in range(0, x[p].shape[0], 1 << 17):
            xs = x[p][lo:lo + (1 << 17)].cpu().numpy()
            t0 = time.perf_counter()
            q = O.quantize(xs, s, lam, w.g)
            t1 = time.perf_counter()
            O.dequantize(q["codes"], q["scales"], s, lam, w.g)
            t2 = time.perf_counter()
            tq += t1 - t0
            td += t2 - t1
            sample += xs.shape[0]
            if tq + td > budget_s or sample >= max_vectors:
                break
        if tq + td > budget_s or sample >= max_vectors:
            break
    forms = []
    for d in (96, 128, 256):
        lam = W.lognormal_lambda(d, seed=d)
        s = O.signs_from_seed(d, d)
        for form in ("dense", "fft"):
            # sized from the rates of an 8-core host so that an entry takes about 1.5 s
            n = (1 << 20) if full else {"dense": 1 << 17, "fft": 1 << 14}[form] * (2 if d <= 128 else 1)
            xs = W.gaussian_with_outliers(n, d, seed=d, outliers=1, gain=20.0)
            t0 = time.perf_counter()
            q = O.quantize(xs, s, lam, 32, form=form)
            t1 = time.perf_counter()
            O.dequantize(q["codes"], q["scales"], s, lam, 32, form=form)
            t2 = time.perf_counter()
            used = cores if form == "dense" else 1
            forms.append({"d": d, "form": form, "vectors": n, "cores": used,
                          "quantize_vectors_per_s": n / (t1 - t0), "dequantize_vectors_per_s": n / (t2 - t1),
                          "quantize_ns_per_vec_per_core": (t1 - t0) / n * 1e9 * used,
                          "dequantize_ns_per_vec_per_core": (t2 - t1) / n * 1e9 * used})
    return {"value": sample / (tq + td), "unit": "vectors/s", "cores": cores, "kind": "oracle",
            "sample": f"the first {sample} vectors of {w.name} (plans 0..{used_plans - 1}): oracle quantize {tq:.2f} s + "
                      f"dequantize {td:.2f} s (numpy, float64, dense d x d form)",
            "quantize_vectors_per_s": sample / tq, "dequantize_vectors_per_s": sample / td,
            "forms": forms}


if __name__ == "__main__":
    sys.exit(main())
