"""Benchmark of the HeatKV hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic activations:
calibration masses for every scale (Eq. 2) -> dataset average -> schedule
construction on the host (Eq. 3-5, Alg. 1) -> for every scale, attention over
the compressed cache followed by the cache append/compaction.  The default
workload is one Infinity-2B-like layer (16 heads, d=128, bf16, batch 2,
13 scales = 10521 tokens, 4x budget).

Prints ONE JSON line.  `value` is the headline metric on the default workload:
heatkv_attend_scale's algorithmic TFLOP/s (QK^T + PV over the *retained* keys)
over the 13 launches of a step, timed with HIP events on the launch stream
inside the timed region; `roofline` is the same kernel against the bf16 MFMA
peak; `whole_step_tflops` adds the calibration FLOPs and divides by the whole
step's wall time.  `roofline_hbm` is the metric's second leg, KV GB/s on the
launches bound by the K/V read (serving stack, batch 32, scales of 36-256
tokens), `stacks_20x` its third (per-image attention ms at the 20x budget, with
per-scale TFLOP/s, GB/s and the cache-update kernel's copy bandwidth);
`cpu_baseline` is the fp64 NumPy oracle on a bounded sample of the same work.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
if ROOT not in sys.path:
    sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0  # MI355X dense bf16 MFMA
PEAK_HBM_GBS = 8000.0      # MI355X HBM3E
METRIC = "attend_scale TFLOP/s + KV GB/s (% of MI355X peak); per-image attention ms at 20x"
TRAFFIC_PROFILE = os.path.join(ROOT, "profiles", "attend_hbm_traffic.txt")


def measured_traffic(key):
    """HBM bytes per launch of the attention kernel from the committed rocprofv3 counter summary (FETCH_SIZE and
    WRITE_SIZE, scaled by a plain copy of known size).  The summary carries one line `TRAFFIC <key> <bytes>` per
    workload it covers; anything else (file missing, workload not profiled) gives None: the figure is never typed
    into this file, so it cannot outlive the profile it came from."""
    try:
        for line in open(TRAFFIC_PROFILE):
            p = line.split()
            if len(p) == 3 and p[0] == "TRAFFIC" and p[1] == key:
                return float(p[2])
    except OSError:
        pass
    return None


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="layer2b",
                    choices=["layer2b", "serving_layer", "layer8b", "stack2b", "stack8b", "serving"],
                    help="layer2b (default): one 2B-like layer, the whole path.  *_layer / layer8b: one layer of the "
                         "named stack.  stack2b / stack8b / serving: every layer of the stack, attend + append only "
                         "(schedule from a fabricated beta table, no calibration pass), --steps passes")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--attend-only", action="store_true", help="profiling aid: skip calibrate/schedule in the step")
    ap.add_argument("--calibrate-per-scale", action="store_true",
                    help="calibrate with one call per scale instead of one launch for all scales")
    ap.add_argument("--separate-append", action="store_true",
                    help="call heatkv_attend_scale and heatkv_append_scale separately instead of the fused entry point")
    ap.add_argument("--stack-passes", default="both", choices=["both", "generation", "batched"],
                    help="stack workloads only: generation-order passes (attention + update fused, per-image time), "
                         "scale-batched passes (per-scale kernel durations of attention and update), or both")
    ap.add_argument("--fp8-cache", action="store_true",
                    help="stack workloads only: report the run with the cache rows stored as FP8 E4M3 codes "
                         "(same token budget, half the cache bytes); the native-format run is kept under native_cache")
    ap.add_argument("--no-stack-20x", action="store_true",
                    help="default workload only: skip the two 20x stacks that supply the per-image attention time")
    ap.add_argument("--no-mfma-probe", action="store_true",
                    help="skip the matrix-core probe (back-to-back bf16 MFMAs on zero and on random operands, "
                         "run after the timed region and reported next to the roofline)")
    ap.add_argument("--copy-probe-mb", type=int, default=0,
                    help="profiling aid: after the timed region run one plain device copy of this many MiB "
                         "(a kernel of known HBM traffic to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (no collectives, no sharding); use --gpus 1", file=sys.stderr)
        sys.exit(2)

    import torch

    import heatkv_inputs as hi
    import paper_2605_14877_amd as hk
    from paper_2605_14877_amd import probe as hp

    if not torch.cuda.is_available():
        print("bench.py needs a GPU", file=sys.stderr)
        sys.exit(1)
    torch.cuda.set_device(0)
    dev = torch.device("cuda:0")

    if args.workload in ("stack2b", "stack8b", "serving"):
        run_stack(args, dev)
        return
    base = {"layer2b": "layer2b", "serving_layer": "serving", "layer8b": "stack8b"}[args.workload]
    cfg = dict(hi.CONFIGS[base])
    cfg["L"] = 1  # one layer of the named stack: every attend/append/calibrate call is per layer
    t0 = hi.tokens_per_scale(cfg["sides"])
    c = hi.cumulative_tokens(t0)
    K, H, d, s, nb = len(t0), cfg["H"], cfg["d"], cfg["sinks"], cfg["batch"]
    esz = hi.elem_bytes(cfg["dtype"])
    sm = 1.0 / np.sqrt(d)
    B = hi.budget_tokens(cfg)
    budget_bytes = B * 2 * d * esz

    w = hi.head_weights(0, 1, H, K)
    gen_batch = min(nb, 2)
    q, k, v = hi.make_qkv(0, 0, cfg, w=w, batch=gen_batch)
    if nb > gen_batch:  # larger batches repeat the generated pair (same shapes and value distribution)
        rep = nb // gen_batch
        q, k, v = (x.repeat(rep, 1, 1, 1) for x in (q, k, v))
    dq, dk, dv = q.to(dev), k.to(dev), v.to(dev)
    sl = [slice(c[i] - t0[i], c[i]) for i in range(K)]
    q_s = [dq[:, :, sl[i]].contiguous() for i in range(K)]
    k_s = [dk[:, :, sl[i]].contiguous() for i in range(K)]
    v_s = [dv[:, :, sl[i]].contiguous() for i in range(K)]
    kall_s = [dk[:, :, :c[i]].contiguous() for i in range(K)]
    out_s = [torch.empty_like(x) for x in q_s]
    shape = hk.Shape(1, H, d, t0, nb, cfg["dtype"])

    beta = torch.zeros(1, H, K, K, device=dev)
    beta_pinned = torch.zeros(1, H, K, K, pin_memory=True)
    beta_host = beta_pinned.numpy()  # shares the pinned buffer
    mass = torch.empty(nb, H, K, device=dev)
    all_k1 = list(range(K))
    cal_ws = torch.empty(hk.binding.calibrate_scales_workspace_bytes(shape, all_k1), dtype=torch.uint8, device=dev)
    cal_ws_1 = [torch.empty(max(hk.binding.calibrate_workspace_bytes(shape, i), 4), dtype=torch.uint8, device=dev)
                for i in range(K)] if args.calibrate_per_scale else None

    def calibrate_and_plan():
        beta.zero_()
        # The scales of a calibration pass are independent (each fills its own row of beta) and the activations
        # of all of them are recorded before the pass starts: one launch for all scales, one for the reduction.
        if args.calibrate_per_scale:
            for k1 in reversed(range(K)):
                hk.heatkv_calibrate_accumulate(shape, 0, k1, q_s[k1], kall_s[k1], sm, 1.0 / nb, beta, mass,
                                               cal_ws_1[k1])
        else:
            hk.heatkv_calibrate_scales_accumulate(shape, 0, all_k1, q_s, kall_s, sm, 1.0 / nb, beta, None, cal_ws)
        beta_pinned.copy_(beta, non_blocking=True)  # 2.7 KB into pinned host memory, then one wait for the stream
        torch.cuda.current_stream().synchronize()
        plan = hk.heatkv_build_schedule(shape, beta_host, budget_bytes, s)
        plan.upload()
        return plan

    plan = calibrate_and_plan()
    arena_bytes = plan.arena_bytes
    ka = torch.zeros(max(arena_bytes, 16), dtype=torch.uint8, device=dev)
    va = torch.zeros(max(arena_bytes, 16), dtype=torch.uint8, device=dev)
    att_ws = [torch.empty(max(plan.attend_workspace_bytes(0, i), 4), dtype=torch.uint8, device=dev) for i in range(K)]

    run_len = [plan.runs(i, 0)[1].astype(np.int64) for i in range(K)]
    n_keys = [nb * int((run_len[i] + t0[i]).sum()) for i in range(K)]           # sum over (b,h) of n
    att_flops = [4.0 * t0[i] * d * n_keys[i] for i in range(K)]
    att_bytes = [2.0 * d * esz * (n_keys[i] + nb * H * t0[i]) for i in range(K)]
    cal_flops = [2.0 * d * t0[i] * c[i] * nb * H for i in range(K)]

    # Timed region: ONE event pair per step around the block of K attention launches (an event pair per launch
    # would put two event records and their host time between launches of 7 us).  The per-scale breakdown comes
    # from a second set of passes after the timed region, with a pair per launch.
    blk_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    cal_ev = [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(args.steps)]
    ev = [[(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
          for _ in range(args.steps)]

    def attend_block(pairs=None):
        for kk in range(K):
            if pairs is not None:
                pairs[kk][0].record()
            if args.separate_append:
                hk.heatkv_attend_scale(plan, 0, kk, q_s[kk], k_s[kk], v_s[kk], ka, va, sm, out_s[kk], att_ws[kk])
                if pairs is not None:
                    pairs[kk][1].record()
                hk.heatkv_append_scale(plan, 0, kk, k_s[kk], v_s[kk], ka, va)
            else:  # attention and cache update of the scale in one launch (an event pair then covers both)
                hk.heatkv_attend_append_scale(plan, 0, kk, q_s[kk], k_s[kk], v_s[kk], ka, va, sm, out_s[kk],
                                              att_ws[kk])
                if pairs is not None:
                    pairs[kk][1].record()

    def step(i_timed=None):
        nonlocal plan
        if not args.attend_only:
            if i_timed is not None:
                cal_ev[i_timed][0].record()
            plan = calibrate_and_plan()
            if i_timed is not None:
                cal_ev[i_timed][1].record()
            assert plan.arena_bytes <= arena_bytes
        if i_timed is not None:
            blk_ev[i_timed][0].record()
        attend_block()
        if i_timed is not None:
            blk_ev[i_timed][1].record()

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t_start = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    elapsed = time.perf_counter() - t_start
    ms_per_step = elapsed * 1e3 / args.steps
    total_att_ms = float(np.mean([a.elapsed_time(b) for a, b in blk_ev]))

    for i in range(args.steps):  # per-scale breakdown, outside the timed region
        attend_block(ev[i])
    torch.cuda.synchronize()
    att_ms = np.array([[ev[i][kk][0].elapsed_time(ev[i][kk][1]) for kk in range(K)] for i in range(args.steps)])
    att_ms_k = att_ms.mean(0)
    step_flops = sum(att_flops) + (0.0 if args.attend_only else sum(cal_flops))
    value = step_flops / (ms_per_step * 1e-3) / 1e12
    att_tflops = sum(att_flops) / (total_att_ms * 1e-3) / 1e12
    per_scale = []
    for kk in range(K):
        ai = att_flops[kk] / att_bytes[kk]
        per_scale.append({
            "k": kk, "t": t0[kk], "ms": round(float(att_ms_k[kk]), 4),
            "tflops": round(att_flops[kk] / (att_ms_k[kk] * 1e-3) / 1e12, 2),
            "gbs": round(att_bytes[kk] / (att_ms_k[kk] * 1e-3) / 1e9, 1),
            "flop_per_byte": round(ai, 1),
        })
    # KV-read-bound launches: arithmetic intensity below the chip's ridge (peak flops / peak bytes)
    ridge = PEAK_BF16_TFLOPS * 1e12 / (PEAK_HBM_GBS * 1e9)
    small = [kk for kk in range(K) if att_flops[kk] / att_bytes[kk] < ridge]
    small_gbs = (sum(att_bytes[kk] for kk in small) / (sum(att_ms_k[kk] for kk in small) * 1e-3) / 1e9) if small else None
    large = [kk for kk in range(K) if kk not in small]
    large_tflops = (sum(att_flops[kk] for kk in large) / (sum(att_ms_k[kk] for kk in large) * 1e-3) / 1e12) if large else None

    result = {
        "metric": METRIC,
        "value": round(att_tflops, 3),
        "unit": "TFLOP/s",
        "n_gpus": 1,
        "steps": args.steps,
        "warmup": args.warmup,
        "ms_per_step": round(ms_per_step, 4),
        "higher_is_better": True,
        "scaling": "weak",
        "vs_baseline": None,
        "dtype": cfg["dtype"],
        "data": "synthetic",
        "config": {"workload": f"{args.workload}: 1 layer x {H} heads x d{d} {cfg['dtype']}, batch {nb}, "
                               f"{K} scales ({c[-1]} tokens), {cfg['factor']}x budget, sinks {s}",
                   "attend_only": bool(args.attend_only), "fused_append": not args.separate_append,
                   "calibrate": "per scale" if args.calibrate_per_scale else "all scales in one launch"},
        "value_is": "heatkv_attend_scale algorithmic TFLOP/s over the 13 launches of a step (one HIP event pair "
                    "around the block of launches in every timed step; fused cache update included unless "
                    "--separate-append); per_scale: event pair per launch, passes after the timed region",
        "whole_step_tflops": round(value, 3),
        "attend_scale_tflops": round(att_tflops, 2),
        "attend_scale_ms_per_step": round(total_att_ms, 4),
        "attend_pct_of_bf16_peak": round(100 * att_tflops / PEAK_BF16_TFLOPS, 2),
        "attend_large_scales_tflops": None if large_tflops is None else round(large_tflops, 2),
        "attend_small_scales_kv_gbs": None if small_gbs is None else round(small_gbs, 1),
        "attend_small_scales_pct_of_hbm_peak": None if small_gbs is None else round(100 * small_gbs / PEAK_HBM_GBS, 2),
        "per_image_attention_ms": round(total_att_ms / max(nb // 2, 1), 4),
        "calibrate_ms_per_step": None if args.attend_only else round(
            float(np.mean([a.elapsed_time(b) for a, b in cal_ev])), 4),
        "arena_tokens_over_budget": round(plan.arena_tokens / max(B, 1), 4),
        "per_scale": per_scale,
        "roofline": {
            "kernel": "attend_bf16_kernel",
            "bound": "mfma",
            "achieved": round(att_tflops, 2),
            "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s",
            "frac": round(att_tflops / PEAK_BF16_TFLOPS, 4),
            "traffic": measured_traffic(args.workload),
            "algorithmic_bytes_per_launch": round(sum(att_bytes) / K),
            "flops_per_step": sum(att_flops),
            "launches_per_step": K,
            "avg_launch_ms": round(total_att_ms / K, 4),
        },
    }

    if not args.no_mfma_probe:
        probe = mfma_probe(dev)
        result["roofline"]["mfma_probe"] = probe
        # the same achieved figure against what the bare matrix pipes sustain on random operands on this GPU
        result["roofline"]["frac_of_probe_random"] = round(att_tflops / probe["random_operands"], 4)
        result["roofline"]["largest_scale_frac_of_probe_random"] = round(
            att_flops[K - 1] / (att_ms_k[K - 1] * 1e-3) / 1e12 / probe["random_operands"], 4)
        result["roofline"]["hbm_read_probe"] = hbm_read_probe(dev)
    if not args.no_stack_20x and not args.attend_only:
        del ka, va, q_s, k_s, v_s, kall_s, out_s, dq, dk, dv
        torch.cuda.empty_cache()
        stacks = {name: stack_measure(name, dev, passes=2, warmup=1, fp8_cache=(name == "serving"))
                  for name in ("stack8b", "serving")}
        result["per_image_attention_ms_at_20x"] = {name: r["ms_per_image"] for name, r in stacks.items()}
        result["stacks_20x"] = stacks
        result["roofline_hbm"] = hbm_leg(stacks["serving"])
        result["roofline_mfma_large_scales"] = mfma_leg(stacks["serving"])
        result["append_kernel"] = append_leg(stacks["serving"])
        # the same serving stack with the cache rows stored as FP8 E4M3 (same tokens kept, half the cache bytes)
        result["roofline_hbm_fp8_cache"] = hbm_leg(stacks["serving"]["fp8_cache"], "serving_small_scales_fp8_cache")
    if args.copy_probe_mb:
        src = torch.empty(args.copy_probe_mb << 20, dtype=torch.uint8, device=dev).fill_(1)
        dst = torch.empty_like(src)
        torch.cuda.synchronize()
        dst.copy_(src)
        torch.cuda.synchronize()
    if not args.no_cpu_baseline:
        result["cpu_baseline"] = cpu_baseline(q, k, v, t0, plan, sm, d)
    print(json.dumps(result))


def mfma_probe(dev):
    """What the matrix cores of this GPU sustain on back-to-back independent bf16 MFMAs (no memory traffic, no
    vector ALU work), for all-zero operands and for random operand bits.  The clock is power-limited, so the
    second figure, not the datasheet peak, is what a kernel working on real data can approach."""
    import torch

    import paper_2605_14877_amd as hk
    from paper_2605_14877_amd import probe as hp

    nbytes = hp.heatkv_probe_mfma_operand_bytes()
    workgroups, iters = 2048, 2000
    out = torch.empty(workgroups * 256, dtype=torch.float32, device=dev)
    flop = workgroups * 4 * iters * 32 * 32768.0
    res = {"unit": "TFLOP/s", "instruction": "v_mfma_f32_32x32x16_bf16", "workgroups": workgroups, "iters": iters}
    g = torch.Generator(device=dev)
    g.manual_seed(1234)
    for name in ("zero_operands", "random_operands"):
        if name == "zero_operands":
            ops = torch.zeros(nbytes // 2, dtype=torch.bfloat16, device=dev)
        else:
            ops = torch.randn(nbytes // 2, device=dev, generator=g).to(torch.bfloat16)
        best = None
        for _ in range(3):
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            hp.heatkv_probe_mfma(ops, out, workgroups, iters)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        res[name] = round(flop / best / 1e9, 1)
    # the attention kernel's tile step without its bookkeeping (same instruction mix, dependencies, LDS tiles,
    # barrier and tile copies, random bf16 tiles served from L2): what that mix sustains on this GPU
    tiles = torch.randn(hp.heatkv_probe_tile_step_bytes() // 2, device=dev, generator=g).to(torch.bfloat16)
    t_iters = 600
    out2 = torch.empty(workgroups * 256, dtype=torch.float32, device=dev)
    best = None
    for _ in range(3):
        e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
        e0.record()
        hp.heatkv_probe_tile_step(tiles, out2, workgroups, t_iters)
        e1.record()
        torch.cuda.synchronize()
        ms = e0.elapsed_time(e1)
        best = ms if best is None else min(best, ms)
    res["attention_tile_step_model"] = round(workgroups * 4 * t_iters * 32 * 32768.0 / best / 1e9, 1)
    return res


def hbm_read_probe(dev):
    """Read bandwidth of the attention kernel's own access pattern with the arithmetic taken out (tile copies
    HBM -> LDS, two stages, a barrier per step, two workgroups per compute unit): a long walk (1024 workgroups x
    64 steps = 2 GiB) and walks as short as those of the scales bound by the K/V read (1024 workgroups x 9 steps,
    each launch on memory it has not touched before)."""
    import torch

    import paper_2605_14877_amd as hk
    from paper_2605_14877_amd import probe as hp

    wgs = 1024
    src = torch.empty(hp.heatkv_probe_tile_stream_bytes(wgs, 64), dtype=torch.uint8, device=dev)
    src.random_(0, 256)
    out = torch.empty(wgs * 256, dtype=torch.int32, device=dev)
    res = {"unit": "GB/s", "workgroups": wgs}

    def best_of(n, steps, offset_steps):
        best = None
        for i in range(n):
            part = src[i * offset_steps * wgs * 32768:]
            e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
            e0.record()
            hp.heatkv_probe_tile_stream(part, out, wgs, steps)
            e1.record()
            torch.cuda.synchronize()
            ms = e0.elapsed_time(e1)
            best = ms if best is None else min(best, ms)
        return round(hp.heatkv_probe_tile_stream_bytes(wgs, steps) / best / 1e6, 1)

    res["walk_64_steps"] = best_of(4, 64, 0)
    res["walk_9_steps"] = best_of(6, 9, 9)  # six disjoint 288 MiB parts of the buffer, none read twice in a row
    return res


def run_stack(args, dev):
    """--workload stack2b / stack8b / serving: the stack measurement alone, as one JSON line (profiling aid)."""
    r = stack_measure(args.workload, dev, passes=args.steps, warmup=args.warmup,
                      generation=args.stack_passes in ("both", "generation"),
                      batched=args.stack_passes in ("both", "batched"), fp8_cache=args.fp8_cache)
    if args.fp8_cache:  # report the 8-bit cache run, keep the native one beside it
        native = {k: v for k, v in r.items() if k != "fp8_cache"}
        r = dict(r["fp8_cache"], native_cache=native)
    value = r.get("attend_tflops_generation_order")
    result = {
        "metric": METRIC, "value": value, "unit": "TFLOP/s", "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": r.get("ms_per_pass"), "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "bf16", "data": "synthetic",
        "config": {"workload": r["workload"] + "; schedule from a fabricated beta table; attend + append only",
                   "stack_passes": args.stack_passes},
        "value_is": "heatkv_attend_scale algorithmic TFLOP/s over a generation-order pass of the whole stack "
                    "(attention + cache update in one launch per layer and scale, host clock)",
        "stack": r,
    }
    if r.get("per_scale"):
        result["roofline"] = mfma_leg(r)
        result["roofline_hbm"] = hbm_leg(r, "serving_small_scales_fp8_cache" if args.fp8_cache else "serving_small_scales")
        result["append_kernel"] = append_leg(r)
    if not args.no_mfma_probe:
        result["mfma_probe"] = mfma_probe(dev)
        result["hbm_read_probe"] = hbm_read_probe(dev)
    print(json.dumps(result))


def stack_measure(name, dev, passes, warmup, generation=True, batched=True, fp8_cache=False):
    """One 20x stack (stack8b: one image with its CFG row; serving: 16 images), every layer with activations of
    its own (nothing a launch reads was touched by the launches just before it, so K/V, Q and the current scale
    come from HBM, not from L2 or the memory-side cache).  Two kinds of passes:
      * generation order (for every scale, for every layer: attention + cache update in one launch), timed as a
        whole on the host clock between device synchronisations: per-image attention time;
      * scale-batched (for every scale: the L attention launches back to back between one event pair, then the
        L cache-update launches between another): average duration per launch of either kernel at every scale,
        hence TFLOP/s, KV GB/s and the copy bandwidth of the update.  Legal because an update only retires its own
        layer's region of the scale, which only that layer's attention reads, and the updates keep their order.
    fp8_cache: the same passes once more over the same activations with the cache rows stored as FP8 E4M3 codes
    (same token budget, half the cache bytes), reported under "fp8_cache"."""
    import torch

    import heatkv_inputs as hi
    import paper_2605_14877_amd as hk

    cfg = hi.CONFIGS[name]
    t0 = hi.tokens_per_scale(cfg["sides"])
    c = hi.cumulative_tokens(t0)
    L, K, H, d, s, nb = cfg["L"], len(t0), cfg["H"], cfg["d"], cfg["sinks"], cfg["batch"]
    esz = hi.elem_bytes(cfg["dtype"])
    row = d * esz
    sm = 1.0 / np.sqrt(d)
    B = hi.budget_tokens(cfg)
    w = hi.head_weights(0, L, H, K)
    beta = hi.expected_beta_from_weights(w, t0).astype(np.float32)
    shape = hk.Shape(L, H, d, t0, nb, cfg["dtype"])
    sl = [slice(c[i] - t0[i], c[i]) for i in range(K)]
    acts = []  # acts[l][kk] = (q, k, v, out)
    for l in range(L):
        q, k, v = hi.make_qkv_device(l, l, cfg, w, dev)
        acts.append([(q[:, :, sl[i]].contiguous(), k[:, :, sl[i]].contiguous(), v[:, :, sl[i]].contiguous(),
                      torch.empty_like(q[:, :, sl[i]])) for i in range(K)])
        del q, k, v

    def measure(kv_format):
        kv_row = d * (1 if kv_format == hk.KV_FP8_E4M3 else esz)  # bytes of a cached K (or V) row
        plan = hk.heatkv_build_schedule(shape, beta, B * 2 * kv_row, s, kv_format=kv_format)
        plan.upload()
        assert plan.budget_tokens == B
        ka = torch.zeros(max(plan.arena_bytes, 16), dtype=torch.uint8, device=dev)
        va = torch.zeros_like(ka)
        flops, byts, app_bytes = np.zeros(K), np.zeros(K), np.zeros(K)
        for kk in range(K):
            for l in range(L):
                n_prior = nb * int(plan.runs(kk, l)[1].astype(np.int64).sum())
                n_cur = nb * H * t0[kk]
                flops[kk] += 4.0 * t0[kk] * d * (n_prior + n_cur)
                # K and V of the retained rows (cache format) and of the current scale, Q in, O out
                byts[kk] += 2.0 * kv_row * n_prior + 2.0 * row * n_cur + 2.0 * row * n_cur
                if kk + 1 < K:
                    # the update writes the whole region the next scale reads (K and V); it reads the rows kept from
                    # the old region in the cache format and the new scale's rows in the tensor dtype
                    nxt = nb * int(plan.runs(kk + 1, l)[1].astype(np.int64).sum())
                    ids = [plan.retained(kk + 1, l, h) for h in range(H)]
                    new_rows = nb * sum(t0[kk] for h in range(H) if len(ids[h]) and ids[h][-1] == c[kk] - 1)
                    app_bytes[kk] += 2.0 * (kv_row * nxt + kv_row * (nxt - new_rows) + row * new_rows)

        def generation_pass():
            for kk in range(K):
                for l in range(L):
                    q, k, v, o = acts[l][kk]
                    hk.heatkv_attend_append_scale(plan, l, kk, q, k, v, ka, va, sm, o)

        def batched_pass(ev_att, ev_app):
            for kk in range(K):
                ev_att[kk][0].record()
                for l in range(L):
                    q, k, v, o = acts[l][kk]
                    hk.heatkv_attend_scale(plan, l, kk, q, k, v, ka, va, sm, o)
                ev_att[kk][1].record()
                ev_app[kk][0].record()
                for l in range(L):
                    q, k, v, o = acts[l][kk]
                    hk.heatkv_append_scale(plan, l, kk, k, v, ka, va)
                ev_app[kk][1].record()

        out = {
            "workload": f"{name}: {L} layers x {H} heads x d{d} {cfg['dtype']}, batch {nb}, {K} scales, "
                        f"{cfg['factor']}x budget, sinks {s}; per-layer activations ({L} distinct sets)"
                        + ("; cache rows stored as FP8 E4M3" if kv_format == hk.KV_FP8_E4M3 else ""),
            "passes": passes, "images_per_pass": max(nb // 2, 1),
            "kv_cache_mb": round(2 * plan.arena_bytes / 1e6, 1),
            "arena_tokens_over_budget": round(plan.arena_tokens / B, 4), "launches_per_scale": L,
        }
        if generation:
            for _ in range(warmup):
                generation_pass()
            torch.cuda.synchronize()
            t_start = time.perf_counter()
            for _ in range(passes):
                generation_pass()
            torch.cuda.synchronize()
            ms_per_pass = (time.perf_counter() - t_start) * 1e3 / passes
            out.update({"ms_per_pass": round(ms_per_pass, 3), "ms_per_image": round(ms_per_pass / max(nb // 2, 1), 3),
                        "attend_tflops_generation_order": round(float(flops.sum()) / ms_per_pass / 1e9, 1)})
        if not batched:
            return out
        mk = lambda: [(torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)) for _ in range(K)]
        evs = [(mk(), mk()) for _ in range(passes)]
        if not generation:
            for _ in range(warmup):
                batched_pass(mk(), mk())
        for ea, ep in evs:
            batched_pass(ea, ep)
        torch.cuda.synchronize()
        att_us = np.array([[a.elapsed_time(b) for a, b in ea] for ea, _ in evs]).mean(0) * 1e3 / L
        app_us = np.array([[a.elapsed_time(b) for a, b in ep] for _, ep in evs]).mean(0) * 1e3 / L
        rows = []
        for kk in range(K):
            fl, by, ab = flops[kk] / L, byts[kk] / L, app_bytes[kk] / L  # per launch
            rows.append({
                "k": kk, "t": t0[kk], "attend_us": round(float(att_us[kk]), 2),
                "tflops": round(fl / att_us[kk] / 1e6, 1),
                "pct_mfma_peak": round(100 * fl / att_us[kk] / 1e6 / PEAK_BF16_TFLOPS, 2),
                "kv_mb": round(by / 1e6, 2), "kv_gbs": round(by / att_us[kk] / 1e3, 1),
                "pct_hbm_peak": round(100 * by / att_us[kk] / 1e3 / PEAK_HBM_GBS, 2),
                "flop_per_byte": round(fl / by, 1),
                "append_us": round(float(app_us[kk]), 2), "append_mb": round(ab / 1e6, 2),
                "append_gbs": round(ab / app_us[kk] / 1e3, 1) if kk + 1 < K else None,
            })
        out.update({"attend_ms_per_pass_kernel_only": round(float(att_us.sum()) * L / 1e3, 3),
                    "append_ms_per_pass_kernel_only": round(float(app_us.sum()) * L / 1e3, 3), "per_scale": rows})
        if kv_format == hk.KV_NATIVE:
            # The same launches of the largest scale on all-zero Q, K, V and cache rows: the same instructions, the
            # same memory traffic, but operand bits that do not make the chip lower its clock.  A diagnostic of
            # what the kernel's instruction stream sustains when power is not the limit; not a result.
            kk = K - 1
            zq, zk, zv = (torch.zeros_like(x) for x in acts[0][kk][:3])
            zo = torch.empty_like(zq)
            ka.zero_()
            va.zero_()
            n_l = min(L, 8)
            best = None
            for _ in range(3):
                e0, e1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
                e0.record()
                for l in range(n_l):
                    hk.heatkv_attend_scale(plan, l, kk, zq, zk, zv, ka, va, sm, zo)
                e1.record()
                torch.cuda.synchronize()
                us = e0.elapsed_time(e1) * 1e3 / n_l
                best = us if best is None else min(best, us)
            fl = sum(4.0 * t0[kk] * d * nb * (int(plan.runs(kk, l)[1].astype(np.int64).sum()) + H * t0[kk])
                     for l in range(n_l)) / n_l
            out["largest_scale_on_zero_inputs"] = {
                "t": t0[kk], "launches": n_l, "attend_us": round(best, 2), "tflops": round(fl / best / 1e6, 1),
                "pct_mfma_peak": round(100 * fl / best / 1e6 / PEAK_BF16_TFLOPS, 2)}
            del zq, zk, zv, zo
        return out

    result = measure(hk.KV_NATIVE)
    if fp8_cache:
        result["fp8_cache"] = measure(hk.KV_FP8_E4M3)
    return result


def hbm_leg(stack, traffic_key="serving_small_scales"):
    """Second leg of the headline metric: KV GB/s of the attention launches bound by the K/V read: scales of at
    most 256 tokens (arithmetic intensity 22-172 FLOP/B, under the chip's ridge of 312) whose launch moves at
    least 16 MB; on the serving stack those are the scales of 36, 64, 144 and 256 tokens."""
    rows = [r for r in stack["per_scale"] if r["kv_mb"] >= 16.0 and r["t"] <= 256]
    if not rows:
        return None
    by = sum(r["kv_mb"] for r in rows) * 1e6
    us = sum(r["attend_us"] for r in rows)
    gbs = by / us / 1e3
    return {"kernel": "attend_bf16_kernel", "workload": stack["workload"], "bound": "hbm",
            "launches": [r["t"] for r in rows], "achieved": round(gbs, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(gbs / PEAK_HBM_GBS, 4), "traffic": measured_traffic(traffic_key),
            "algorithmic_bytes_per_launch": round(by / max(len(rows), 1)),
            "avg_launch_us": round(us / max(len(rows), 1), 2),
            "per_scale": [{k: r[k] for k in ("t", "attend_us", "kv_mb", "kv_gbs", "pct_hbm_peak", "tflops",
                                             "flop_per_byte")} for r in rows]}


def mfma_leg(stack):
    """The matrix-core leg on a full chip: serving-stack launches of 1024 tokens and more."""
    rows = [r for r in stack["per_scale"] if r["t"] >= 1024]
    if not rows:
        return None
    fl = sum(r["tflops"] * r["attend_us"] for r in rows)
    us = sum(r["attend_us"] for r in rows)
    return {"kernel": "attend_bf16_kernel", "workload": stack["workload"], "bound": "mfma",
            "launches": [r["t"] for r in rows], "achieved": round(fl / us, 1), "peak": PEAK_BF16_TFLOPS,
            "unit": "TFLOP/s", "frac": round(fl / us / PEAK_BF16_TFLOPS, 4),
            "per_scale": [{k: r[k] for k in ("t", "attend_us", "tflops", "pct_mfma_peak")} for r in rows],
            # same kernel, same launches, all-zero operands (no clock throttling): diagnostic, see stack_measure
            "largest_scale_on_zero_inputs": stack.get("largest_scale_on_zero_inputs")}


def append_leg(stack):
    """The cache-update kernel as a copy: bytes read + written per launch over its duration, serving stack,
    launches that move at least 16 MB."""
    rows = [r for r in stack["per_scale"] if r["append_gbs"] is not None and r["append_mb"] >= 16.0]
    if not rows:
        return None
    by = sum(r["append_mb"] for r in rows) * 1e6
    us = sum(r["append_us"] for r in rows)
    return {"kernel": "append_kernel", "workload": stack["workload"], "bound": "hbm",
            "achieved": round(by / us / 1e3, 1), "peak": PEAK_HBM_GBS, "unit": "GB/s",
            "frac": round(by / us / 1e3 / PEAK_HBM_GBS, 4), "traffic": None,
            "bytes_per_launch": round(by / len(rows)), "avg_launch_us": round(us / len(rows), 2),
            "per_scale": [{k: r[k] for k in ("t", "append_us", "append_mb", "append_gbs")} for r in rows]}


def cpu_baseline(q, k, v, t0, plan, sm, d):
    """Times the fp64 oracle on the same step for a bounded sample of the workload: every scale, every head of
    the first two batch rows (the whole of the default workload); calibration masses (beta_row) and attention
    over the retained cache (attend_scale).  Reported in the metric's unit (algorithmic FLOPs of both legs
    over wall time)."""
    from oracle import heatkv_oracle as orc

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [1])
    except Exception:
        threads = len(os.sched_getaffinity(0))
    t1 = orc.one_based(t0)
    K = len(t0)
    H = q.shape[1]
    rows = list(range(min(q.shape[0], 2)))
    pairs = [(b, h) for b in rows for h in range(H)]
    c0 = np.cumsum([0] + list(t0))
    att_flops = cal_flops = 0.0
    kept = {}
    for kk in range(K):
        for h in range(H):
            idx = plan.retained(kk, 0, h)
            # which whole scales the retained positions cover (the plan only supplies the index list)
            kept[(kk, h)] = [i + 1 for i in range(kk) if idx.size and np.any(idx == c0[i])]
            att_flops += len(rows) * 4.0 * t0[kk] * d * (idx.size + t0[kk])
            cal_flops += len(rows) * 2.0 * d * t0[kk] * c0[kk + 1]
    t_cal = t_att = 0.0
    for (b, h) in pairs:
        qq, kk_, vv = (x[b, h].double().numpy() for x in (q, k, v))
        t_a = time.perf_counter()
        for kk in range(K):
            orc.beta_row(qq, kk_, t1, kk + 1, sm)
        t_b = time.perf_counter()
        for kk in range(K):
            orc.attend_scale(qq, kk_, vv, t1, kk + 1, kept[(kk, h)], sm)
        t_c = time.perf_counter()
        t_cal += t_b - t_a
        t_att += t_c - t_b
    dt = t_cal + t_att
    return {"value": round((att_flops + cal_flops) / dt / 1e12, 5), "unit": "TFLOP/s", "cores": int(threads),
            "kind": "oracle",
            "sample": f"oracle beta_row + attend_scale, batch rows 0-{rows[-1]}, all {H} heads, all {K} scales "
                      f"({cal_flops / 1e9:.0f} + {att_flops / 1e9:.0f} GFLOP algorithmic, "
                      f"{t_cal:.1f} + {t_att:.1f} s)"}


if __name__ == "__main__":
    main()
