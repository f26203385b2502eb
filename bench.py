#!/usr/bin/env python3
"""Benchmark of the trajectory-generation attention hot path on one MI355X.

A step is one pass of the whole decode hot path over one batch: host split-K plan, plan
upload, split-K decode kernel, log-sum-exp combine kernel (one heddle_attn_decode call),
on the Qwen3-8B-shaped long-tail workload (64 trajectories, 32 query / 8 kv heads,
head_dim 128, lognormal context lengths).  Inputs are synthetic and resident in HBM
before the timed region.  Prints one JSON line.

  python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload 2..9] [--op attention|pack|placement] [--seed S]
"""
from __future__ import annotations

import argparse
import gc
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

HBM_PEAK_GBPS = 8000.0        # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


FP32_VECTOR_PEAK_TFLOPS = 157.3   # published fp32 vector rate (packed); two-way bf16 dot instructions run at the same rate
FP32_FMA_PEAK_TFLOPS = 78.6       # 256 CUs x 4 SIMDs x 16 lanes x 2 flops x 2.4 GHz: plain (unpacked) fp32 FMA
PER_CONFIG = (3, 4, 5)            # the other named full-size workloads, reported after the headline


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--workload", type=int, default=None, choices=[2, 3, 4, 5, 6, 7, 8, 9],
                    help="one workload only; default: workload 2 as the headline plus per_config entries for "
                         "workloads 3, 4 and 5")
    ap.add_argument("--op", default="attention", choices=["attention", "pack", "placement"],
                    help="attention: the workload's decode or append pass (default); pack: gather of every "
                         "trajectory's blocks into one contiguous staging buffer (whole-block copy); placement: decode step time per batch size -> interference table -> "
                         "presorted dynamic programming for 6400 trajectories on 16 workers")
    ap.add_argument("--seed", type=int, default=0)
    ap.add_argument("--no-cpu-baseline", action="store_true")
    return ap.parse_args()


def main():
    args = parse()
    if args.gpus != 1 or int(os.environ.get("WORLD_SIZE", "1")) != 1:
        print("bench.py: this path runs on one GPU only (no sharding or collectives are built); "
              "run with --gpus 1", file=sys.stderr)
        sys.exit(2)

    import numpy as np
    import torch

    import heddle_workloads as hw
    import paper_2603_28101_amd as heddle

    torch.cuda.set_device(0)
    mods = (np, torch, hw, heddle)
    if args.op == "placement":
        print(json.dumps(run_placement(args, np, torch, hw, heddle)))
        return
    if args.workload is not None or args.op == "pack":
        print(json.dumps(measure(args, args.workload or 2, mods, cpu_budget_s=20.0)))
        return
    result = measure(args, 2, mods, cpu_budget_s=15.0)
    per_config = {}
    for cfg in PER_CONFIG:
        r = measure(args, cfg, mods, cpu_budget_s=8.0)
        per_config[r["config"]["workload"]] = {
            k: r[k] for k in ("metric", "value", "unit", "ms_per_step", "us_per_step", "step_us_p10_p50_p90",
                              "frac_of_hbm_peak_whole_step", "frac_of_mfma_peak_whole_step", "roofline",
                              "alu_ceiling", "cpu_baseline", "config") if k in r}
    result["per_config"] = per_config
    print(json.dumps(result))


def measure(args, workload, mods, cpu_budget_s):
    """Times one workload; returns the result record.  Three passes over the same resident inputs:
    (1) wall clock of `steps` whole steps with the library's timers off: `value`; (2) the same
    steps with one event per step boundary: spread of the whole step; (3) the same steps with an
    event pair around every kernel launch: the roofline of the dominant kernel."""
    np, torch, hw, heddle = mods
    w = hw.WORKLOADS[workload]
    case = hw.make_workload(workload, args.seed, threads=min(16, os.cpu_count() or 1))

    def dev_bf16(bits):
        return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)

    def dev_i32(a):
        return torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()

    pool = dev_bf16(case["pool"])
    row_off, block_ids, q = dev_i32(case["row_off"]), dev_i32(case["block_ids"]), dev_bf16(case["q"])
    out = torch.empty(case["q"].shape, dtype=torch.bfloat16, device="cuda")
    ctx = heddle.Context(w.n_q_heads, w.n_kv_heads, w.head_dim, case["n_blocks"], kv_pool=pool, device=0)
    # a stream of its own: work queued on the null stream pays for its implicit
    # synchronisation with every other stream of the process
    stream = torch.cuda.Stream()

    kind = "pack" if args.op == "pack" else w.kind
    shared = False
    if kind == "pack":
        used = np.concatenate([case["block_ids"][case["row_off"][b]:case["row_off"][b + 1]]
                               for b in range(w.B)]).astype(np.int32)
        block_elems = w.n_kv_heads * 2 * 16 * w.head_dim
        staging = torch.empty((len(used), block_elems), dtype=torch.bfloat16, device="cuda")
        unit_bytes = 2 * len(used) * block_elems * 2          # every byte is read once and written once

        def step():
            ctx.kv_pack(used, staging, stream=stream)

        dominant, bound = 4, "hbm"
    elif kind == "decode":
        lens = case["lens"]
        # a decode step stores the K/V row of its own position (len - 1) before it attends
        gen = torch.Generator(device="cuda").manual_seed(args.seed)
        k_row = torch.randn((w.B, w.n_kv_heads, w.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
        v_row = torch.randn((w.B, w.n_kv_heads, w.head_dim), generator=gen, device="cuda").to(torch.bfloat16)
        case["k_row"] = k_row.view(torch.int16).cpu().numpy().view(np.uint16)      # for the oracle's timed pass
        case["v_row"] = v_row.view(torch.int16).cpu().numpy().view(np.uint16)
        unit_bytes = hw.kv_bytes(lens, w.n_kv_heads, w.head_dim)   # algorithmic bytes of one step
        shared = "group_of" in case
        if shared:
            # blocks that several trajectories name are read once: bytes of the distinct tokens
            logical_bytes = unit_bytes
            unit_bytes = hw.kv_bytes([hw.unique_kv_tokens(case)], w.n_kv_heads, w.head_dim)
            plan = ctx.plan_decode_shared(lens, case["row_off"], case["block_ids"])
            private_tokens = int(lens.astype(np.int64).sum() - 16 * plan["traj_prefix"].astype(np.int64).sum())
            private_bytes = hw.kv_bytes([private_tokens], w.n_kv_heads, w.head_dim)

            def step():
                ctx.attn_decode_shared(lens, case["row_off"], case["block_ids"], row_off, block_ids, q, out, None,
                                       k_row, v_row, stream=stream)
        else:
            def step():
                ctx.attn_decode(lens, case["row_off"], row_off, block_ids, q, out, None, k_row, v_row, stream=stream)

        dominant, bound = 0, "hbm"
    else:
        k_new, v_new = dev_bf16(case["k_new"]), dev_bf16(case["v_new"])
        L, cu = case["lens"], case["cu_chunk"]
        C = case["chunk_lens"].astype(np.int64)
        # 4*d*Hq flops per (query row, visible key) pair; causal part counted once
        unit_flops = int(4 * w.head_dim * w.n_q_heads * (C * (L.astype(np.int64) + (C + 1) / 2)).sum())
        unit_bytes = hw.kv_bytes(L.astype(np.int64) + C, w.n_kv_heads, w.head_dim)

        def step():
            ctx.attn_append(L, cu, case["row_off"], row_off, block_ids, q, k_new, v_new, out, None, stream=stream)

        # below the machine balance (flops per byte of K/V) the pass is priced in bytes
        dominant = 2
        bound = "mfma" if unit_flops / unit_bytes > MFMA_BF16_PEAK_TFLOPS * 1e3 / HBM_PEAK_GBPS else "hbm"

    # a full Python garbage collection (tens of ms with torch loaded) must not land in the
    # timed region: collect now, keep the collector off while timing.  It comes before all GPU work
    # of the measurement: tens of ms of host work between warm-up and timed steps would let the GPU
    # fall back to its idle clocks, and the first timed steps would pay for the ramp.
    gc.collect()
    gc.disable()
    # measured streaming-read ceiling over the same pool (context for the roofline fraction); run
    # ahead of the timed passes, it also brings the GPU out of its idle clocks
    sink = torch.zeros(4096, dtype=torch.int32, device="cuda")
    nbytes = pool.numel() * 2
    for _ in range(3):
        heddle.stream_read(pool, nbytes, sink, stream)
    e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    e0.record(stream)
    for _ in range(10):
        heddle.stream_read(pool, nbytes, sink, stream)
    e1.record(stream)
    torch.cuda.synchronize()
    stream_gbps = nbytes * 10 / (e0.elapsed_time(e1) * 1e-3) / 1e9

    # plain device-to-device copy of known size: the reference the FETCH_SIZE / WRITE_SIZE
    # counters of a profiling run are scaled by
    cal_src = pool.view(torch.int16).reshape(-1)[: 64 * 1024 * 1024]
    cal_dst = torch.empty_like(cal_src)
    with torch.cuda.stream(stream):
        cal_dst.copy_(cal_src)
    torch.cuda.synchronize()
    del cal_dst

    torch.cuda.synchronize()
    for _ in range(args.warmup):
        step()
    # ---- pass 1: wall clock of the whole steps, nothing recorded on the stream but the work itself
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    # ---- pass 2: one event per step boundary (about 3 us of stream time each): spread of the whole step
    marks = [torch.cuda.Event(enable_timing=True) for _ in range(args.steps + 1)]
    marks[0].record(stream)
    for i in range(args.steps):
        step()
        marks[i + 1].record(stream)
    torch.cuda.synchronize()
    step_us = np.array([marks[i].elapsed_time(marks[i + 1]) * 1e3 for i in range(args.steps)])
    # ---- pass 3: HIP events around every launch of each kernel, on the launch stream
    ctx.timing_enable(1)
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    gc.enable()
    kernel_us, n_launch = ctx.timing_read(dominant)
    timer_of_kernel = dominant
    kernel_name = {0: "decode_splitk_kernel", 2: "append_dma_kernel", 4: "kv_move_kernel"}[dominant]
    if kind == "decode" and n_launch == 0:
        # with 8 query heads per kv head (or 3, 5, 6, 7 ...) the library runs decode in the matrix-core kernel
        # for short-row tiles
        (kernel_us, n_launch), kernel_name, timer_of_kernel = ctx.timing_read(7), "narrow_attn_kernel", 7
    if kind == "append":
        # tiles of at most 32 query rows per kv head run in the kernel that splits the keys over its waves
        narrow_us, narrow_n = ctx.timing_read(7)
        if narrow_n > 0 and (n_launch == 0 or narrow_us > kernel_us):
            other_us, kernel_us, n_launch, kernel_name = kernel_us, narrow_us, narrow_n, "narrow_attn_kernel"
            timer_of_kernel = 7
        else:
            other_us = narrow_us
    aux_us = ctx.timing_read({"decode": 1, "append": 3, "pack": 5}[kind])[0]
    group_us = ctx.timing_read(6)[0] if shared else 0.0
    ctx_combine_us = ctx.timing_read(1)[0]
    kernel_samples = ctx.timing_samples(timer_of_kernel)
    ctx.timing_enable(0)

    ms_per_step = (t1 - t0) * 1e3 / args.steps
    if kind == "pack":
        value = unit_bytes / (ms_per_step * 1e-3) / 1e9
        metric, unit = "kv-pack read+write GB/s", "GB/s"
        achieved = unit_bytes / (kernel_us * 1e-6) / 1e9
        roofline = {"bound": bound, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                    "kernel": "kv_move_kernel", "kernel_avg_us": round(kernel_us, 2), "launches_timed": n_launch}
    elif kind == "decode":
        value = unit_bytes / (ms_per_step * 1e-3) / 1e9
        metric, unit = "decode-attention KV GB/s", "GB/s"
        # the split-K kernel reads every block exactly one trajectory names (all blocks without sharing)
        achieved = (private_bytes if shared else unit_bytes) / (kernel_us * 1e-6) / 1e9
        roofline = {"bound": bound, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                    "kernel": kernel_name, "kernel_avg_us": round(kernel_us, 2),
                    "launches_timed": n_launch, "combine_avg_us": round(aux_us, 2)}
        if shared:
            roofline["kernel_bytes"] = private_bytes
            roofline["shared_prefix_kernel_avg_us"] = round(group_us, 2)
    elif bound == "hbm":
        value = unit_bytes / (ms_per_step * 1e-3) / 1e9
        metric, unit = "append-attention KV GB/s", "GB/s"
        achieved = unit_bytes / (kernel_us * 1e-6) / 1e9
        roofline = {"bound": bound, "achieved": round(achieved, 1), "peak": HBM_PEAK_GBPS, "unit": "GB/s",
                    "frac": round(achieved / HBM_PEAK_GBPS, 4), "traffic": None,
                    "kernel": kernel_name, "kernel_avg_us": round(kernel_us, 2),
                    "launches_timed": n_launch, "other_attn_kernel_avg_us": round(other_us, 2),
                    "kv_write_avg_us": round(aux_us, 2),
                    "combine_avg_us": round(ctx_combine_us, 2), "flops_per_step": unit_flops}
    else:
        value = unit_flops / (ms_per_step * 1e-3) / 1e12
        metric, unit = "append-attention TFLOP/s", "TFLOP/s"
        achieved = unit_flops / (kernel_us * 1e-6) / 1e12
        roofline = {"bound": bound, "achieved": round(achieved, 1), "peak": MFMA_BF16_PEAK_TFLOPS,
                    "unit": "TFLOP/s", "frac": round(achieved / MFMA_BF16_PEAK_TFLOPS, 4), "traffic": None,
                    "kernel": "append_dma_kernel", "kernel_avg_us": round(kernel_us, 2),
                    "launches_timed": n_launch, "kv_write_avg_us": round(aux_us, 2),
                    "flops_per_step": unit_flops}

    if bound == "mfma":
        # What the matrix cores sustain on this machine: the vendor library's bf16 GEMM (8192^3 through
        # torch.matmul, a measurement aid, not part of the path) on N(0,1) data and on constant data.
        # The part is power-limited under matrix-core load and draws more on data that toggles, so the
        # published peak (2.4 GHz) is out of reach of any kernel fed with real values.
        def gemm_tflops(make):
            n = 8192
            ga, gb = make(n), make(n)
            with torch.cuda.stream(stream):
                for _ in range(3):
                    gc_ = ga @ gb
                g0, g1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                g0.record(stream)
                for _ in range(20):
                    gc_ = ga @ gb
                g1.record(stream)
            torch.cuda.synchronize()
            del gc_
            return 2 * n ** 3 * 20 / (g0.elapsed_time(g1) * 1e-3) / 1e12
        rand = gemm_tflops(lambda n: torch.randn(n, n, device="cuda", dtype=torch.bfloat16))
        const = gemm_tflops(lambda n: torch.full((n, n), 0.001, device="cuda", dtype=torch.bfloat16))
        roofline["library_gemm_bf16_TFLOPs"] = {"normal_data": round(rand, 1), "constant_data": round(const, 1)}
        roofline["frac_of_library_gemm_normal_data"] = round(roofline["achieved"] / rand, 4)

    # HBM bytes per launch as rocprofv3's counters gave them when the profile summary was written
    # (not measured by this run); null once the kernel's source has changed since
    roofline["traffic"], roofline["traffic_source"] = recorded_traffic(w, roofline["kernel"])
    if kernel_samples.size:
        # spread of the timed launches of that kernel (the roofline uses their mean)
        p10, p50, p90 = np.percentile(kernel_samples.astype(np.float64), [10, 50, 90])
        roofline["kernel_us_p10_p50_p90"] = [round(float(p10), 2), round(float(p50), 2), round(float(p90), 2)]

    extra = {}
    if bound == "hbm":
        roofline["frac_of_stream_read_ceiling"] = round(roofline["achieved"] / stream_gbps, 4)
    if kind == "decode":
        # The arithmetic next to the bytes: per context token and kv head the step does 4*d*G flops
        # (logits and P.V for the G query heads of the group) on 4*d bytes of K and V, G flops per byte.
        # Time the plain vector ALUs would need at their published rate, next to the time HBM needs.
        G = w.n_q_heads // w.n_kv_heads
        flops = (private_bytes if shared else unit_bytes) * G
        extra["alu_ceiling"] = {
            "flops_per_step": flops, "flops_per_kv_byte": G,
            "us_at_hbm_peak": round(unit_bytes / HBM_PEAK_GBPS * 1e-3, 1),
            "us_at_fp32_vector_peak": round(flops / FP32_VECTOR_PEAK_TFLOPS * 1e-6, 1),
            "us_at_fp32_fma_unpacked_peak": round(flops / FP32_FMA_PEAK_TFLOPS * 1e-6, 1),
            "fp32_vector_peak_TFLOPs": FP32_VECTOR_PEAK_TFLOPS, "fp32_fma_unpacked_peak_TFLOPs": FP32_FMA_PEAK_TFLOPS,
            "achieved_TFLOPs": round(flops / (kernel_us * 1e-6) / 1e12, 1),
            "note": "logits and P.V use two-way bf16 dot instructions (vector-peak rate) or, for "
                    "narrow_attn_kernel, the matrix cores; packed fp32 instructions are compiled out"}
    if kind == "decode" and not shared:
        # bytes the step moves besides K/V, left out of the rate (listed so that the omission can be judged)
        plan = ctx.plan_decode(lens)
        n_parts = int(plan["nsplit"][plan["nsplit"] > 1].sum())
        n_blk = int(((np.asarray(lens, dtype=np.int64) + 15) // 16).sum())
        extra["bytes_not_counted"] = {
            "q_and_out": 2 * w.B * w.n_q_heads * w.head_dim * 2,
            "block_table": 4 * n_blk * w.n_kv_heads,
            "partials_written_and_read": 2 * n_parts * w.n_q_heads * (w.head_dim + 4) * 4}
    if kind == "decode" and shared:
        # the same batch through the plain decode entry point, which reads a shared block once per
        # trajectory that names it
        for _ in range(5):
            ctx.attn_decode(lens, case["row_off"], row_off, block_ids, q, out, None, k_row, v_row, stream=stream)
        torch.cuda.synchronize()
        t2 = time.perf_counter()
        for _ in range(20):
            ctx.attn_decode(lens, case["row_off"], row_off, block_ids, q, out, None, k_row, v_row, stream=stream)
        torch.cuda.synchronize()
        plain_us = (time.perf_counter() - t2) * 1e6 / 20
        extra.update({"kv_bytes_if_every_trajectory_read_its_own": logical_bytes,
                      "plain_decode_us_per_step": round(plain_us, 1),
                      "speedup_over_plain_decode": round(plain_us / (ms_per_step * 1e3), 3)})

    sp10, sp50, sp90 = np.percentile(step_us, [10, 50, 90])
    result = {
        "metric": metric, "value": round(value, 1), "unit": unit, "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": f"{w.name}{' / kv-pack' if kind == 'pack' else ''} (config {w.cfg_id}, seed {args.seed})",
                   "trajectories": w.B,
                   "n_q_heads": w.n_q_heads, "n_kv_heads": w.n_kv_heads, "head_dim": w.head_dim,
                   "kv_bytes_per_step": unit_bytes, "tokens": int(np.asarray(case["lens"], dtype=np.int64).sum())},
        "us_per_step": round(ms_per_step * 1e3, 1),
        # pass 2: one event per step boundary; these intervals include that event's stream time
        "step_us_p10_p50_p90": [round(float(sp10), 1), round(float(sp50), 1), round(float(sp90), 1)],
        "frac_of_hbm_peak_whole_step": round(unit_bytes / (ms_per_step * 1e-3) / 1e9 / HBM_PEAK_GBPS, 4),
        "stream_read_ceiling_GBps": round(stream_gbps, 1),
        "roofline": roofline,
        **extra,
    }
    if kind == "append":
        result["frac_of_mfma_peak_whole_step"] = round(unit_flops / (ms_per_step * 1e-3) / 1e12 / MFMA_BF16_PEAK_TFLOPS, 4)

    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(case, w, np, kind, unit, cpu_budget_s)
    # give the device memory back before the next workload is built
    ctx.close()
    del pool, q, out, row_off, block_ids, case
    gc.collect()
    torch.cuda.empty_cache()
    return result


def run_placement(args, np, torch, hw, heddle):
    """Sec. 5.2 end to end on this machine: (1) the profiler, decode step time of the Qwen3-8B
    shape at batch sizes 1..256 with every context at 4096 tokens; (2) the interference table
    F(s) = t(s)/t(1); (3) the presorted dynamic programming for n = 6400 trajectories with
    long-tailed lengths on m = 16 workers (the size the paper quotes a solve time for), in both
    modes; (4) the resulting makespan next to two placements that ignore lengths."""
    w = hw.WORKLOADS[2]
    sizes = [1, 2, 4, 8, 16, 32, 64, 128, 256]
    ctx_tokens = 4096
    Bmax = sizes[-1]
    lens = np.full(Bmax, ctx_tokens, dtype=np.int32)
    case = hw.build_case(entropy=[2, args.seed, 0x51], lens=lens, n_q_heads=w.n_q_heads, n_kv_heads=w.n_kv_heads,
                         head_dim=w.head_dim, threads=min(16, os.cpu_count() or 1), poison=False)
    bf = lambda bits: torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)
    i32 = lambda a: torch.from_numpy(np.ascontiguousarray(a, dtype=np.int32)).cuda()
    pool, q = bf(case["pool"]), bf(case["q"])
    row_off, block_ids = i32(case["row_off"]), i32(case["block_ids"])
    out = torch.empty_like(q)
    ctx = heddle.Context(w.n_q_heads, w.n_kv_heads, w.head_dim, case["n_blocks"], kv_pool=pool, device=0)
    stream = torch.cuda.Stream()
    step_us = []
    gc.collect()
    gc.disable()
    for s_ in sizes:
        f = lambda: ctx.attn_decode(lens[:s_], case["row_off"][: s_ + 1], row_off, block_ids, q, out, None,
                                    stream=stream)
        for _ in range(args.warmup):
            f()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            f()
        torch.cuda.synchronize()
        step_us.append((time.perf_counter() - t0) * 1e6 / args.steps)
    gc.enable()

    n, m = 6400, 16
    rng = np.random.default_rng([0x706C, args.seed])
    L = np.sort(np.clip(np.rint(np.exp(rng.normal(np.log(4096), 1.0, n))), 256, 40960))[::-1].astype(np.float64)
    F = heddle.interference_table(sizes, step_us, n)
    T = step_us[0]                                     # base time of one token at batch size 1, in us

    def timed(fn, reps):
        t0 = time.perf_counter()
        for _ in range(reps):
            r = fn()
        return r, (time.perf_counter() - t0) * 1e3 / reps

    (mk, sz), ms_fast = timed(lambda: heddle.placement_dp(L, m, F, T), 20)
    (mk2, sz2), ms_scan = timed(lambda: heddle.placement_dp(L, m, F, T, full_scan=True), 2)
    assert mk == mk2 and np.array_equal(sz, sz2)
    first, count = heddle.placement_aggregate(L, 2048.0, 8)
    (mk_a, sz_a), ms_agg = timed(lambda: heddle.placement_dp(L[first], m, F, T, counts=count, full_scan=True), 5)

    def objective(groups):            # Eq. 2 and the simulator, both in seconds
        eq2 = max((g.max() * T) * F[len(g)] for g in groups if len(g)) * 1e-6
        sim = max(heddle.simulate_group(g.astype(np.int32), sizes, step_us) for g in groups if len(g)) * 1e-6
        return round(eq2, 3), round(sim, 3)

    edges = np.concatenate([[0], np.cumsum(sz)])
    dp_groups = [L[edges[i]:edges[i + 1]] for i in range(m)]
    e_a = np.concatenate([[0], np.cumsum(sz_a)])
    starts = np.concatenate([first, [n]])
    agg_groups = [L[starts[e_a[i]]:starts[e_a[i + 1]]] for i in range(m)]
    shuffled = L[rng.permutation(n)]
    equal_groups = [shuffled[i::m] for i in range(m)]                  # length-oblivious: n/m each
    sorted_equal = [L[i * (n // m):(i + 1) * (n // m)] for i in range(m)]

    from oracle import placement as pl
    n_small = 400
    t0 = time.perf_counter()
    ref_mk, ref_sz = pl.placement_dp(L[:n_small].tolist(), m, F[: n_small + 1].tolist(), T)
    oracle_s = time.perf_counter() - t0
    lib_mk, lib_sz = heddle.placement_dp(L[:n_small], m, F[: n_small + 1], T)
    assert lib_mk == ref_mk and lib_sz.tolist() == ref_sz

    return {
        "metric": "presorted-DP placement solve time", "value": round(ms_fast, 3), "unit": "ms", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": round(ms_fast, 3), "higher_is_better": False,
        "scaling": "weak", "vs_baseline": None, "dtype": "f64", "data": "synthetic",
        "config": {"workload": f"placement of n={n} trajectories (lognormal(4096, 1.0) clip [256, 40960]) on m={m} "
                               f"workers; profile: qwen3-8b decode at {ctx_tokens} tokens per trajectory"},
        "profile": {"batch_sizes": sizes, "decode_step_us": [round(x, 1) for x in step_us],
                    "F_at_profile_points": [round(float(F[s_]), 3) for s_ in sizes]},
        "dp_ms": {"crossing_search": round(ms_fast, 3), "full_scan_eq3": round(ms_scan, 1),
                  "full_scan_after_bundling_short_tail": round(ms_agg, 2), "elements_after_bundling": int(len(first)),
                  "paper_reported_ms_n6400_m16": 42},
        "group_sizes": sz.tolist(),
        "makespan_s_eq2_and_simulated": {"dp": objective(dp_groups), "dp_after_bundling": objective(agg_groups),
                                         "equal_count_random": objective(equal_groups),
                                         "equal_count_sorted": objective(sorted_equal)},
        "cpu_baseline": {"value": round(oracle_s * 1e3, 1), "unit": "ms", "cores": 1, "kind": "oracle",
                         "sample": f"the oracle's Eq. 3 scan on the {n_small} longest trajectories, m={m} "
                                   f"(library result identical bit for bit)"},
    }


KERNEL_SOURCES = {"decode_splitk_kernel": "decode_kernels.hip", "append_dma_kernel": "append_kernels.hip",
                  "narrow_attn_kernel": "narrow_kernels.hip",
                  "kv_move_kernel": "misc_kernels.hip"}


def recorded_traffic(w, kernel):
    """HBM bytes per launch of the dominant kernel as measured with rocprofv3 counters and
    written into the kernel's summary under profiles/ (lines `traffic_bytes_per_launch = N` and
    `kernel_source_sha256 = H`); None if there is no record or the kernel source has changed
    since the counters were taken."""
    import hashlib
    import re
    path = os.path.join(ROOT, "profiles", f"{kernel}__{w.name}.md")
    src = os.path.join(ROOT, "paper_2603_28101_amd", "csrc", KERNEL_SOURCES[kernel])
    source = f"profiles/{os.path.basename(path)} (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE runs, recorded there)"
    try:
        text = open(path).read()
        digest = hashlib.sha256(open(src, "rb").read()).hexdigest()
    except OSError:
        return None, None
    m = re.search(r"traffic_bytes_per_launch\s*=\s*(\d+)", text)
    h = re.search(r"kernel_source_sha256\s*=\s*([0-9a-f]{64})", text)
    if not m or not h:
        return None, None
    if h.group(1) != digest:
        return None, source + "; the kernel source has changed since, so the record does not apply"
    return int(m.group(1)), source


def cpu_baseline(case, w, np, kind, unit, budget_s=20.0):
    """The oracle as it stands, timed on this host on a bounded sample."""
    from oracle import attention as oa
    try:
        from threadpoolctl import threadpool_info
        blas_threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        blas_threads = 1
    t0 = time.perf_counter()
    if kind == "pack":
        lens = (case["lens"].astype(np.int64) + (case["chunk_lens"] if "chunk_lens" in case else 0))
        moved = 0
        for b in range(len(lens)):
            moved += 2 * oa.pack(case["pool"], case["row_off"], case["block_ids"], b, int(lens[b])).nbytes
        dt = time.perf_counter() - t0
        return {"value": round(moved / dt / 1e9, 3), "unit": "GB/s", "cores": 1, "kind": "oracle",
                "sample": f"all {len(lens)} trajectories ({moved} bytes read+written in {dt:.2f} s)",
                "host_cpus": os.cpu_count(), "affinity": len(os.sched_getaffinity(0))}
    if kind == "decode":
        lens = case["lens"]
        done_bytes, n_done = 0, 0
        for b in range(len(lens)):
            pairs = [(b, j) for j in range(w.n_q_heads)]
            oa.write_kv(case["pool"], case["row_off"], case["block_ids"], [int(lens[b]) - 1], b,
                        case["k_row"][b:b + 1], case["v_row"][b:b + 1])
            oa.decode_rows(case["pool"], case["row_off"], case["block_ids"], lens, case["q"], w.n_kv_heads, pairs)
            done_bytes += int(lens[b]) * 2 * w.n_kv_heads * w.head_dim * 2
            n_done += 1
            if time.perf_counter() - t0 > budget_s:
                break
        dt = time.perf_counter() - t0
        return {"value": round(done_bytes / dt / 1e9, 4), "unit": "GB/s", "cores": blas_threads, "kind": "oracle",
                "sample": f"first {n_done} of {len(lens)} trajectories, all heads ({done_bytes} KV bytes in {dt:.1f} s)",
                "host_cpus": os.cpu_count(), "affinity": len(os.sched_getaffinity(0))}
    # append: the whole workload is minutes of float64 work; evaluate a fixed subset of chunk
    # rows (first, second, last two and every 97th of each trajectory), all heads, in one call
    pool = case["pool"].copy()
    L, cu = case["lens"], case["cu_chunk"]
    rows, flops, kv_bytes = [], 0, 0
    for b in range(len(L)):
        C = int(cu[b + 1] - cu[b])
        for r in sorted({0, 1, C - 2, C - 1} | set(range(0, C, 97))):
            if 0 <= r < C:
                rows.append(int(cu[b]) + r)
                flops += 4 * w.head_dim * w.n_q_heads * (int(L[b]) + r + 1)
                kv_bytes += (int(L[b]) + r + 1) * 2 * w.n_kv_heads * w.head_dim * 2
    oa.append(pool, case["row_off"], case["block_ids"], L, cu, case["q"], case["k_new"], case["v_new"],
              w.n_kv_heads, rows=rows)
    dt = time.perf_counter() - t0
    if unit == "GB/s":      # the pass is priced in K/V bytes: bytes of the keys the sampled rows visit
        value, what = round(kv_bytes / dt / 1e9, 4), f"{kv_bytes} bytes of visible K/V"
    else:
        value, what = round(flops / dt / 1e12, 6), f"{flops} flops"
    return {"value": value, "unit": unit, "cores": blas_threads, "kind": "oracle",
            "sample": f"{len(rows)} sampled chunk rows of all {len(L)} trajectories, all heads: {what} "
                      f"({dt:.1f} s, includes the oracle's KV write and gather)",
            "host_cpus": os.cpu_count(), "affinity": len(os.sched_getaffinity(0))}


if __name__ == "__main__":
    main()
