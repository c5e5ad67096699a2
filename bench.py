#!/usr/bin/env python3
"""Benchmark of the head-wise joint-attention layer on one MI355X.

A step is one difa_joint_attention call, i.e. the whole hot path (work-list lookup, one kernel launch
that runs the full / arrow heads and copies the cached heads) on synthetic FLUX-2K-shaped inputs that
are resident in HBM before the timed region starts.  Output and cache ping-pong between two buffers,
as a denoising loop would use them.  Prints ONE JSON line.

Besides the headline workload (the mixed plan with about 68 % fewer attention FLOPs) the same run
measures, on the same inputs: the layer with every head full (how the time scales with the plan's
FLOP reduction), every head cached (HBM GB/s of the copy), every head an arrow head of half-width 128
(small-window heads: fraction of peak and GB/s), a long run of the headline workload (power-limited
steady state), the error of the timed configuration against the CPU oracle on every row, and the
oracle's own speed on the host cores.
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
PEAK_HBM_GBPS = 8000.0      # MI355X HBM3E, published
METRIC = "ms per joint-attn layer + computed TFLOP/s (% bf16 MFMA peak), 2K MMDiT"
PAPER_CONTEXT = ("paper (one NVIDIA A100): ~68% fewer attention FLOPs and up to 1.5x end-to-end at FLUX 2K; "
                 "kernel speed-ups 1.44x/1.96x/3.55x at 25/50/75% sparsity (Table 3)")


def make_workload(name):
    from paper_2503_22796_amd import workloads as W
    if name in W.CONFIGS:
        return W.config(name)
    if name == "flux_2k_cache":
        return W.flux_2k_single_mode(W.CACHE)
    if name.startswith("flux_2k_arrow_w"):
        return W.flux_2k_single_mode(W.ARROW, int(name[len("flux_2k_arrow_w"):]))
    raise SystemExit(f"unknown workload {name}")


def sampled_flops(wl, rows):
    """FLOPs of exactly the given rows of every computed head (the band length depends on the row)."""
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
    return flops * wl.B


def cpu_baseline(wl, q, k, v, cache, every, block=None, image_first=False):
    """The oracle as it stands, timed on this host's cores, on every `every`-th query row.
    Returns (report, fp64 reference [B, H, rows, D], raw cached rows, rows)."""
    from oracle import difa_oracle as O
    rows = list(range(0, wl.N, every))
    t0 = time.perf_counter()
    ref, ref_raw, _ = O.joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img, rows=rows,
                                        block=block, image_first=image_first)
    dt = time.perf_counter() - t0
    flops = sampled_flops(wl, rows)
    rep = {"value": flops / dt * 1e-12, "unit": "TFLOP/s", "cores": O.threads(), "kind": "oracle",
           "sample": f"every {every}th query row of every head ({len(rows)} rows/head), {dt:.1f} s, "
                     f"extrapolated full layer {dt * every * 1e3:.0f} ms",
           "seconds": dt}
    return rep, ref, ref_raw, rows


def error_against_oracle(got, ref, ref_raw, rows, head_plan):
    """Max abs error over the computed heads; cached heads must be bit-identical."""
    import torch
    g = got[:, :, rows]
    worst, cached_ok = 0.0, True
    for h, m in enumerate(head_plan):
        if m == 2:
            cached_ok &= bool(torch.equal(g[:, h].contiguous().view(torch.int16), ref_raw[:, h].contiguous().view(torch.int16)))
        else:
            worst = max(worst, float((g[:, h].double() - ref[:, h]).abs().max()))
    return worst, cached_ok


class Layer:
    """One plan object with resident inputs and two ping-pong output/cache buffers."""

    def __init__(self, wl, qd, kd, vd, cache_d, flags=0):
        import torch
        from paper_2503_22796_amd import binding as B
        self.B, self.wl, self.q, self.k, self.v = B, wl, qd, kd, vd
        self.bufs = [cache_d.clone(), torch.empty_like(qd)]
        self.plan = B.difa_plan_create(wl.B, wl.H, wl.D, max_tokens=wl.N, flags=flags)

    def step(self, i):
        wl = self.wl                      # the output of step i is the cache of step i + 1
        self.B.difa_joint_attention(self.plan, self.q, self.k, self.v, self.bufs[(i + 1) % 2], self.bufs[i % 2],
                                    wl.head_plan, wl.n_text, wl.n_img, wl.window)

    def wall_ms(self, steps, warmup):
        import torch
        # W untimed steps.  The library learns the dies' speeds from finished launches and may then make the
        # layer's schedule again (it tries two versions and keeps the faster); the pauses let that happen here,
        # in the warm-up, as it would have long before the steady state of a real run.
        for i in range(warmup):
            self.step(i)
            if i >= warmup - 9:
                torch.cuda.synchronize()
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for i in range(steps):
            self.step(i)
        torch.cuda.synchronize()
        return (time.perf_counter() - t0) * 1e3 / steps

    def kernel_ms(self, steps):
        """Mean duration of the call's kernel launch, from the library's HIP-event brackets on the call's stream."""
        B = self.B
        B.difa_plan_timing_enable(self.plan, True)
        for i in range(steps):
            self.step(i)
        attn_ms, _, launches = B.difa_plan_timing_read(self.plan)
        B.difa_plan_timing_enable(self.plan, False)
        return attn_ms / max(launches, 1)

    def close(self):
        self.B.difa_plan_destroy(self.plan)


def side_run(name, qd, kd, vd, cache_d, steps, warmup):
    """A second workload on the same resident inputs: wall and kernel time, rates."""
    from paper_2503_22796_amd.accounting import plan_bytes, plan_flops
    wl = make_workload(name)
    lay = Layer(wl, qd, kd, vd, cache_d)
    wall = lay.wall_ms(steps, warmup)
    kern = lay.kernel_ms(steps)
    lay.close()
    fl = plan_flops(wl.head_plan, wl.window, wl.n_text, wl.n_img, wl.D, wl.B)
    by = plan_bytes(wl.head_plan, wl.n_text, wl.n_img, wl.D, 2, wl.B)
    bytes_alg = by["attention"] + by["cache_copy"]
    rep = {"workload": name, "ms_per_step": wall, "avg_kernel_ms": kern, "steps": steps,
           "algorithmic_bytes": bytes_alg, "GBps": bytes_alg / (kern * 1e-3) * 1e-9}
    if fl["computed"]:
        rep.update({"computed_tflops": fl["computed"] / (wall * 1e-3) * 1e-12,
                    "frac_of_bf16_peak_kernel": fl["computed"] / (kern * 1e-3) * 1e-12 / PEAK_BF16_TFLOPS,
                    "flop_fraction_of_dense": fl["computed"] / fl["dense"]})
    else:
        rep["frac_of_hbm_peak"] = rep["GBps"] / PEAK_HBM_GBPS
    return rep, fl


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
    # the same calls again with the library's event brackets around its launches: summed kernel time
    for p in plans:
        B.difa_plan_timing_enable(p, True)
    run(n_calls)
    kern_ms, launches = 0.0, 0
    for p in plans:
        a_ms, _, n = B.difa_plan_timing_read(p)
        kern_ms += a_ms
        launches += n
        B.difa_plan_timing_enable(p, False)
    flops = sum(plan_flops(hp[l, t], win[l, t], base.n_text, base.n_img, base.D, base.B)["computed"]
                for t, l in calls[:n_calls])
    dense = 4 * base.D * base.N * base.N * base.H * base.B * n_calls
    achieved = flops / (kern_ms * 1e-3) * 1e-12
    roofline = {"bound": "mfma", "kernel": f"attn_bf16_kernel<{base.D}>", "achieved": achieved, "peak": PEAK_BF16_TFLOPS,
                "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS, "traffic": None,
                "avg_kernel_ms": kern_ms / max(launches, 1), "launches": launches,
                "flop_per_launch": flops / n_calls,
                "what": "computed FLOPs of all timed calls / summed kernel time of the same calls (HIP events)"}
    # the oracle on one call of the schedule (layer 0, step 1: the first step with a mixed plan), a sample of its rows
    cpu = None
    if not args.no_cpu:
        wl = W.flux_2k_mixed()
        wl.head_plan, wl.window = hp[0, 1].copy(), win[0, 1].copy()
        q, k, v = (x.cpu() for x in qkv[1])
        every = max(args.cpu_every, 4)
        cpu, _, _, _ = cpu_baseline(wl, q, k, v, torch.zeros_like(q), every)
        cpu["sample"] = "call (layer 0, step 1) of the schedule: " + cpu["sample"]
    for p in plans:
        B.difa_plan_destroy(p)
    out = {
        "metric": METRIC,
        "value": flops / wall * 1e-12, "unit": "TFLOP/s (computed, exact-mask FLOPs)",
        "n_gpus": 1, "steps": n_calls, "warmup": args.warmup, "ms_per_step": wall * 1e3 / n_calls,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "bf16", "data": "synthetic",
        "config": {"workload": "flux_2k_schedule", "layers": L, "denoising_steps": T, "calls_timed": n_calls,
                   "batch": base.B, "heads": base.H, "head_dim": base.D, "n_text": base.n_text,
                   "n_img": base.n_img, "flop_reduction": 1.0 - flops / dense,
                   "note": "every call carries a plan its plan object has not seen lately: work-list compilation "
                           "and upload are inside the timed region"},
        "ms_per_layer": wall * 1e3 / n_calls,
        "pct_of_bf16_peak": 100.0 * flops / wall * 1e-12 / PEAK_BF16_TFLOPS,
        "dense_equiv_tflops": dense / wall * 1e-12,
        "device": B.difa_device_info(0),
        "roofline": roofline, "cpu_baseline": cpu, "paper_context": PAPER_CONTEXT,
    }
    print(json.dumps(out))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="flux_2k_mixed")
    ap.add_argument("--cpu-every", type=int, default=1, help="oracle baseline on every n-th row; 0 = skip")
    ap.add_argument("--no-cpu", action="store_true")
    ap.add_argument("--no-extras", action="store_true", help="skip the side runs (all-full, all-cached, w=128, long run)")
    ap.add_argument("--long-steps", type=int, default=1000, help="steps of the steady-state run")
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
    qd, kd, vd, cd = q.to(dev), k.to(dev), v.to(dev), cache0.to(dev)
    flags = (B.DIFA_FLAG_BLOCK_BAND if args.block_band else 0) | (B.DIFA_FLAG_IMAGE_FIRST if args.image_first else 0)
    block = B.difa_tile_shape(wl.D) if args.block_band else None
    fl = plan_flops(wl.head_plan, wl.window, wl.n_text, wl.n_img, wl.D, wl.B, block=block)
    by = plan_bytes(wl.head_plan, wl.n_text, wl.n_img, wl.D, 2, wl.B)

    lay = Layer(wl, qd, kd, vd, cd, flags)
    wall_ms = lay.wall_ms(args.steps, args.warmup)
    attn_avg = lay.kernel_ms(args.steps)
    # the timed configuration once more from the initial cache, its output kept for the comparison with the oracle
    lay.bufs[0].copy_(cd)
    lay.bufs[1].fill_(float("nan"))
    lay.step(0)
    torch.cuda.synchronize()
    got = lay.bufs[1].cpu()
    steady = None
    if not args.no_extras and args.long_steps > 0:
        long_ms = lay.wall_ms(args.long_steps, 0)
        steady = {"steps": args.long_steps, "ms_per_step": long_ms,
                  "value": fl["computed"] / (long_ms * 1e-3) * 1e-12 if fl["computed"] else None}

    # calibration helper (Sec. 3.4.1): the per-head influence metric of this layer's two output buffers,
    # an HBM-bound streaming pass over both
    rse_out = torch.empty(wl.H, dtype=torch.float32, device=dev)
    B.difa_head_rse(lay.plan, lay.bufs[0], lay.bufs[1], wl.N, rse_out)
    B.difa_plan_timing_enable(lay.plan, True)
    for _ in range(20):
        B.difa_head_rse(lay.plan, lay.bufs[0], lay.bufs[1], wl.N, rse_out)
    rse_ms, rse_calls = B.difa_plan_timing_read_head_rse(lay.plan)
    B.difa_plan_timing_enable(lay.plan, False)
    rse_bytes = 2 * wl.B * wl.H * wl.N * wl.D * 2
    rse_avg = rse_ms / max(rse_calls, 1)
    head_rse = {"avg_kernel_ms": rse_avg, "bytes": rse_bytes, "GBps": rse_bytes / (rse_avg * 1e-3) * 1e-9 if rse_avg > 0 else None,
                "frac_of_hbm_peak": rse_bytes / (rse_avg * 1e-3) * 1e-9 / PEAK_HBM_GBPS if rse_avg > 0 else None}
    # what the plan object learnt about the dies' speeds from the workgroups' own run times, and how often
    # it made this layer's schedule again because of it
    speeds, speed_samples, retunes = B.difa_plan_die_speeds(lay.plan)
    die_info = {"relative_speed": [round(x, 4) for x in speeds], "launches_averaged": speed_samples,
                "schedules_made_again": retunes}
    lay.close()

    bm, bn = B.difa_tile_shape(wl.D)
    _, items, _ = B.difa_worklist_build(wl.B, wl.H, wl.head_plan, wl.window, wl.n_text, wl.n_img, bm, bn,
                                        flags=B.DIFA_FLAG_IMAGE_FIRST if args.image_first else 0)
    items = items[items["q_tile"] >= 0] if items is not None else items
    executed = float(items["n_tiles"].sum()) * bm * bn * 4 * wl.D if items is not None and len(items) else 0.0

    computed_tflops = fl["computed"] / (wall_ms * 1e-3) * 1e-12 if fl["computed"] else 0.0
    achieved = fl["computed"] / (attn_avg * 1e-3) * 1e-12 if fl["computed"] else 0.0
    traffic, traffic_src = None, None
    tpath = os.path.join(ROOT, "profiles", "hbm_traffic.json")   # measured with rocprofv3 --pmc, see profiles/
    if os.path.exists(tpath):
        entry = json.load(open(tpath)).get(wl.name, {})
        traffic, traffic_src = entry.get("traffic_bytes"), entry.get("source")
    if fl["computed"]:
        roofline = {"bound": "mfma", "kernel": f"attn_bf16_kernel<{wl.D}>", "achieved": achieved,
                    "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": achieved / PEAK_BF16_TFLOPS,
                    "traffic": traffic, "traffic_unit": "bytes per launch (FETCH_SIZE + WRITE_SIZE, scaled on a known copy)",
                    "traffic_source": traffic_src,
                    "algorithmic_bytes": by["attention"] + by["cache_copy"], "avg_kernel_ms": attn_avg,
                    "flop_per_launch": fl["computed"]}
        # what the matrix cores sustain on this workload's own operand bits with nothing else to do
        # (the published peak assumes the full clock; N(0,1) operands run into the power limit)
        sus, sus_ms = B.difa_probe_mfma_rate(kd, waves_per_simd=1, rounds=100000)
        roofline["sustained_mfma"] = {"value": sus, "unit": "TFLOP/s", "ms": sus_ms,
                                      "what": "independent v_mfma_f32_32x32x16_bf16 only, operands = this workload's K"}
        roofline["frac_of_sustained_mfma"] = achieved / sus if sus > 0 else None
    else:
        gbs = by["cache_copy"] / (attn_avg * 1e-3) * 1e-9 if attn_avg > 0 else 0.0
        roofline = {"bound": "hbm", "kernel": f"attn_bf16_kernel<{wl.D}> (cached-head copy only)", "achieved": gbs,
                    "peak": PEAK_HBM_GBPS, "unit": "GB/s", "frac": gbs / PEAK_HBM_GBPS, "traffic": traffic,
                    "avg_kernel_ms": attn_avg, "bytes_per_launch": by["cache_copy"]}

    out = {
        "metric": METRIC,
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
        "launches_per_step": 1,
        "steady_state": steady,
        "device": B.difa_device_info(0),
        "dies": die_info,
        "roofline": roofline,
        "head_rse": head_rse,
        "paper_context": PAPER_CONTEXT,
    }

    if not args.no_extras and wl.name == "flux_2k_mixed" and not (args.block_band or args.image_first):
        side_steps = max(20, args.steps)
        full, fl_full = side_run("flux_2k_full", qd, kd, vd, cd, side_steps, 5)
        out["all_full"] = full
        out["plan_scaling"] = {"t_mixed_over_t_full": wall_ms / full["ms_per_step"],
                               "kernel_t_mixed_over_t_full": attn_avg / full["avg_kernel_ms"],
                               "flop_mixed_over_flop_full": fl["computed"] / fl_full["computed"]}
        # The same all-full layer on all-zero operands: identical instruction stream, identical clock count,
        # but the matrix cores switch next to nothing, so the chip holds its clock.  The ratio of the two times
        # is what the power limit costs on realistic operand data.
        zq = torch.zeros_like(qd)
        zero, _ = side_run("flux_2k_full", zq, zq, zq, cd, side_steps, 5)
        out["power_limit_probe"] = {
            "workload": "flux_2k_full", "ms_per_step_workload_data": full["ms_per_step"],
            "ms_per_step_zero_operands": zero["ms_per_step"],
            "time_ratio_zero_over_data": zero["ms_per_step"] / full["ms_per_step"],
            "frac_of_bf16_peak_zero_operands": zero["frac_of_bf16_peak_kernel"],
            "what": "same kernel, same launch, Q = K = V = 0: the time the schedule takes when the clock is not lowered"}
        del zq
        out["all_cached"], _ = side_run("flux_2k_cache", qd, kd, vd, cd, side_steps, 5)
        out["arrow_w128"], _ = side_run("flux_2k_arrow_w128", qd, kd, vd, cd, side_steps, 5)

    if not args.no_cpu and args.cpu_every > 0:
        has_cache = bool((wl.head_plan == 2).any())
        rep, ref, ref_raw, rows = cpu_baseline(wl, q, k, v, cache0 if has_cache else None, args.cpu_every, block=block,
                                               image_first=args.image_first)
        out["cpu_baseline"] = rep
        err, cached_ok = error_against_oracle(got, ref, ref_raw, rows, wl.head_plan)
        out["max_abs_err"] = err
        out["cached_heads_bit_exact"] = cached_ok
        out["parity"] = {"against": "the CPU oracle (fp64) on the rows of cpu_baseline.sample", "max_abs_err": err,
                         "tolerance": 2e-2, "cached_heads_bit_exact": cached_ok}
    else:
        out["cpu_baseline"] = None
    print(json.dumps(out))


if __name__ == "__main__":
    main()
