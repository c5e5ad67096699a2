#!/usr/bin/env python3
"""Benchmark of the head-wise joint-attention layer on one MI355X.

A step is one difa_joint_attention call (the whole hot path: work-list lookup, cache copy for
cached heads, attention kernel for full/arrow heads) on synthetic FLUX-2K-shaped inputs that
are resident in HBM before the timed region starts.  Output and cache ping-pong between two
buffers, as a denoising loop would use them.  Prints ONE JSON line.
"""
import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA, published


def make_workload(name):
    from paper_2503_22796_amd import workloads as W
    if name in W.CONFIGS:
        return W.config(name)
    if name == "flux_2k_cache":
        return W.flux_2k_single_mode(W.CACHE)
    if name.startswith("flux_2k_arrow_w"):
        return W.flux_2k_single_mode(W.ARROW, int(name[len("flux_2k_arrow_w"):]))
    raise SystemExit(f"unknown workload {name}")


def cpu_baseline(wl, q, k, v, cache, every, block=None, image_first=False):
    """The oracle as it stands, timed on this host's cores, on every `every`-th query row."""
    from oracle import difa_oracle as O
    from paper_2503_22796_amd.accounting import allowed_pairs
    rows = list(range(0, wl.N, every))
    t0 = time.perf_counter()
    O.joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img, rows=rows, block=block,
                      image_first=image_first)
    dt = time.perf_counter() - t0
    # FLOPs of exactly the sampled rows (band length depends on the row)
    flops = 0
    for m, w in zip(wl.head_plan, wl.window):
        if m == 2:
            continue
        for i in rows:
            if m == 0 or i < wl.n_text or w >= wl.n_img - 1:
                n = wl.N
            else:
                ii = i - wl.n_text
                n = wl.n_text + min(ii + int(w), wl.n_img - 1) - max(ii - int(w), 0) + 1
            flops += 4 * wl.D * n
    flops *= wl.B
    return {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": O.threads(), "kind": "oracle",
            "sample": f"every {every}th query row of every head ({len(rows)} rows/head), {dt:.1f} s, "
                      f"extrapolated full layer {dt * every * 1e3:.0f} ms",
            "seconds": dt}


def run_schedule(args):
    """FLUX-like 2K full schedule: 57 joint-attention layers x 28 denoising steps, one plan object and
    two ping-pong output/cache buffers per layer, a seeded plan per (layer, step) with step 0 all full.
    A step of this workload is one layer call; --steps bounds the number of calls timed (0 = all 1596)."""
    import torch
    from paper_2503_22796_amd import binding as B
    from paper_2503_22796_amd import workloads as W
    from paper_2503_22796_amd.accounting import plan_flops

    L, T = 57, 28
    base = W.flux_2k_mixed()
    dev = torch.device("cuda:0")
    hp, win = W.schedule_plans(L, T, base.H, seed=5)
    gen = torch.Generator(device=dev)
    pos = torch.from_numpy(W.positional_term(base.n_img, base.D)).to(dev)
    qkv = []
    for t in range(T):                       # Q/K/V of a step, shared by its 57 layers, resident before timing
        gen.manual_seed(1000 + t)
        trio = []
        for _ in range(3):
            x = torch.randn((base.B, base.H, base.N, base.D), device=dev, dtype=torch.float32, generator=gen)
            x[:, :, base.n_text:, :] += pos
            trio.append(x.to(torch.bfloat16))
        qkv.append(trio)
    bufs = [[torch.zeros((base.B, base.H, base.N, base.D), device=dev, dtype=torch.bfloat16) for _ in range(2)]
            for _ in range(L)]
    plans = [B.difa_plan_create(base.B, base.H, base.D, max_tokens=base.N) for _ in range(L)]
    calls = [(t, l) for t in range(T) for l in range(L)]
    n_calls = len(calls) if args.steps <= 0 or args.steps > len(calls) else args.steps

    def run(n):
        for t, l in calls[:n]:
            q, k, v = qkv[t]
            B.difa_joint_attention(plans[l], q, k, v, bufs[l][(t + 1) % 2], bufs[l][t % 2], hp[l, t],
                                   base.n_text, base.n_img, win[l, t])

    run(min(args.warmup, n_calls))
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    run(n_calls)
    torch.cuda.synchronize()
    wall = time.perf_counter() - t0
    flops = sum(plan_flops(hp[l, t], win[l, t], base.n_text, base.n_img, base.D, base.B)["computed"]
                for t, l in calls[:n_calls])
    dense = 4 * base.D * base.N * base.N * base.H * base.B * n_calls
    for p in plans:
        B.difa_plan_destroy(p)
    out = {
        "metric": "ms per joint-attn layer + computed TFLOP/s (% bf16 MFMA peak), 2K MMDiT",
        "value": flops / wall * 1e-12, "unit": "TFLOP/s (computed, exact-mask FLOPs)",
        "n_gpus": 1, "steps": n_calls, "warmup": args.warmup, "ms_per_step": wall * 1e3 / n_calls,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "flux_2k_schedule", "layers": L, "denoising_steps": T, "calls_timed": n_calls,
                   "batch": base.B, "heads": base.H, "head_dim": base.D, "n_text": base.n_text,
                   "n_img": base.n_img, "flop_reduction": 1.0 - flops / dense,
                   "note": "every call carries a plan the library has not seen: work-list compilation is inside the timed region"},
        "ms_per_layer": wall * 1e3 / n_calls,
        "pct_of_bf16_peak": 100.0 * flops / wall * 1e-12 / PEAK_BF16_TFLOPS,
        "dense_equiv_tflops": dense / wall * 1e-12,
        "roofline": None, "cpu_baseline": None,
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="flux_2k_mixed")
    ap.add_argument("--cpu-every", type=int, default=1, help="oracle baseline on every n-th row; 0 = skip")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--block-band", action="store_true",
                    help="arrow heads use the block-granular band of the paper's kernel (Sec. 3.3) instead of the exact one")
    ap.add_argument("--image-first", action="store_true",
                    help="joint sequence [image, text] instead of [text, image] (same tokens, rotated)")
    args = ap.parse_args()
    if args.gpus != 1:
        raise SystemExit("bench.py: this build runs on one GPU only (heads would be sharded across GPUs, "
                         "see DESIGN.md); run with --gpus 1")

    import torch
    from paper_2503_22796_amd import binding as B
    from paper_2503_22796_amd import workloads as W
    from paper_2503_22796_amd.accounting import plan_bytes, plan_flops

    if not torch.cuda.is_available():
        raise SystemExit("bench.py needs a GPU (no CPU fallback exists)")
    if args.workload == "flux_2k_schedule":
        return run_schedule(args)
    dev = torch.device("cuda:0")
    wl = make_workload(args.workload)
    q, k, v = W.make_qkv(wl)
    cache0 = W.make_cache(wl)
    if args.image_first:
        rot = list(range(wl.n_text, wl.N)) + list(range(wl.n_text))
        q, k, v, cache0 = (t[:, :, rot].contiguous() for t in (q, k, v, cache0))
    qd, kd, vd = q.to(dev), k.to(dev), v.to(dev)
    bufs = [cache0.to(dev), torch.empty_like(qd)]
    plan = B.difa_plan_create(wl.B, wl.H, wl.D, max_tokens=wl.N,
                              flags=(B.DIFA_FLAG_BLOCK_BAND if args.block_band else 0) |
                                    (B.DIFA_FLAG_IMAGE_FIRST if args.image_first else 0))
    block = B.difa_tile_shape(wl.D) if args.block_band else None
    fl = plan_flops(wl.head_plan, wl.window, wl.n_text, wl.n_img, wl.D, wl.B, block=block)
    by = plan_bytes(wl.head_plan, wl.n_text, wl.n_img, wl.D, 2, wl.B)

    def step(i):
        # out of step i is the cache of step i+1
        B.difa_joint_attention(plan, qd, kd, vd, bufs[(i + 1) % 2], bufs[i % 2], wl.head_plan,
                               wl.n_text, wl.n_img, wl.window)

    for i in range(args.warmup):
        step(i)
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3 / args.steps

    # second pass with the library's HIP-event brackets around its kernels (same stream)
    B.difa_plan_timing_enable(plan, True)
    for i in range(args.steps):
        step(i)
    attn_ms, copy_ms, launches = B.difa_plan_timing_read(plan)
    B.difa_plan_timing_enable(plan, False)
    attn_avg = attn_ms / max(launches, 1)       # the one launch of a call: attention and the cached-head copy
    copy_avg = attn_avg if not fl["computed"] else 0.0   # a layer with every head cached is the copy alone

    # calibration helper (Sec. 3.4.1): the per-head influence metric of this layer's two output buffers,
    # an HBM-bound streaming pass over both
    rse_out = torch.empty(wl.H, dtype=torch.float32, device=dev)
    B.difa_head_rse(plan, bufs[0], bufs[1], wl.N, rse_out)
    B.difa_plan_timing_enable(plan, True)
    for _ in range(20):
        B.difa_head_rse(plan, bufs[0], bufs[1], wl.N, rse_out)
    rse_ms, rse_calls = B.difa_plan_timing_read_head_rse(plan)
    B.difa_plan_timing_enable(plan, False)
    rse_bytes = 2 * wl.B * wl.H * wl.N * wl.D * 2
    rse_avg = rse_ms / max(rse_calls, 1)
    head_rse = {"avg_kernel_ms": rse_avg, "bytes": rse_bytes, "GBps": rse_bytes / (rse_avg * 1e-3) * 1e-9 if rse_avg > 0 else None,
                "frac_of_hbm_peak": rse_bytes / (rse_avg * 1e-3) * 1e-9 / 8000.0 if rse_avg > 0 else None}

    bm, bn = B.difa_tile_shape(wl.D)
    _, items, _ = B.difa_worklist_build(wl.B, wl.H, wl.head_plan, wl.window, wl.n_text, wl.n_img, bm, bn,
                                        flags=B.DIFA_FLAG_IMAGE_FIRST if args.image_first else 0)
    items = items[items["q_tile"] >= 0] if items is not None else items
    executed = float(items["n_tiles"].sum()) * bm * bn * 4 * wl.D if items is not None and len(items) else 0.0

    computed_tflops = fl["computed"] / (wall_ms * 1e-3) * 1e-12 if fl["computed"] else 0.0
    achieved = fl["computed"] / (attn_avg * 1e-3) * 1e-12 if launches and fl["computed"] else 0.0
    traffic = None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")   # measured with rocprofv3 --pmc, see profiles/
    if os.path.exists(tpath):
        traffic = json.load(open(tpath)).get(wl.name, {}).get("traffic_bytes")
    if fl["computed"]:
        roofline = {"bound": "mfma", "kernel": f"attn_bf16_kernel<{wl.D}>", "achieved": achieved,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                    "traffic": traffic, "traffic_unit": "bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled on a known copy)",
                    "algorithmic_bytes": by["attention"], "avg_kernel_ms": attn_avg, "flop_per_launch": fl["computed"]}
        # what the matrix cores sustain on this workload's own operand bits with nothing else to do
        # (the published peak assumes the full clock; N(0,1) operands run into the power limit)
        sus, sus_ms = B.difa_probe_mfma_rate(kd, waves_per_simd=1, rounds=100000)
        roofline["sustained_mfma"] = {"value": sus, "unit": "TFLOP/s", "ms": sus_ms,
                                      "what": "independent v_mfma_f32_32x32x16_bf16 only, operands = this workload's K"}
        roofline["frac_of_sustained_mfma"] = achieved / sus if sus > 0 else None
    else:
        gbs = by["cache_copy"] / (copy_avg * 1e-3) * 1e-9 if copy_avg > 0 else 0.0
        roofline = {"bound": "hbm", "kernel": "cache_copy_kernel", "achieved": gbs, "peak": 8000.0,
                    "unit": "GB/s", "frac": gbs / 8000.0, "traffic": None, "avg_kernel_ms": copy_avg,
                    "bytes_per_launch": by["cache_copy"]}

    out = {
        "metric": "ms per joint-attn layer + computed TFLOP/s (% bf16 MFMA peak), 2K MMDiT",
        "value": computed_tflops, "unit": "TFLOP/s (computed, exact-mask FLOPs)",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "ms_per_step": wall_ms,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16",
        "data": "synthetic",
        "config": {"workload": wl.name + ("_block_band" if args.block_band else "") + ("_image_first" if args.image_first else ""), "batch": wl.B, "heads": wl.H, "head_dim": wl.D,
                   "n_text": wl.n_text, "n_img": wl.n_img,
                   "plan": {"full": int((wl.head_plan == 0).sum()),
                            "arrow": sorted(int(w) for w in wl.window[wl.head_plan == 1]),
                            "cache": int((wl.head_plan == 2).sum())},
                   "flop_reduction": fl["reduction"]},
        "ms_per_layer": wall_ms,
        "pct_of_bf16_peak": 100.0 * computed_tflops / PEAK_BF16_TFLOPS,
        "dense_equiv_tflops": fl["dense"] / (wall_ms * 1e-3) * 1e-12,
        "executed_tflops": executed / (wall_ms * 1e-3) * 1e-12,
        "cache_copy": {"avg_kernel_ms": copy_avg, "bytes": by["cache_copy"],
                       "GBps": (by["cache_copy"] / (copy_avg * 1e-3) * 1e-9) if copy_avg > 0 else None},
        "roofline": roofline,
        "head_rse": head_rse,
        "paper_context": "paper (one NVIDIA A100): ~68% fewer attention FLOPs and up to 1.5x end-to-end at "
                         "FLUX 2K; kernel speed-ups 1.44x/1.96x/3.55x at 25/50/75% sparsity (Table 3)",
    }
    B.difa_plan_destroy(plan)
    if not args.no_cpu and args.cpu_every > 0:
        has_cache = bool((wl.head_plan == 2).any())
        out["cpu_baseline"] = cpu_baseline(wl, q, k, v, cache0 if has_cache else None, args.cpu_every, block=block,
                                           image_first=args.image_first)
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
