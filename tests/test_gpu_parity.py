"""Parity of the HIP library (through the C ABI) against the CPU oracle, element by element.

Bars: max-abs 2e-2 for bf16 inputs (fp32 accumulation), 1e-5 for the fp32 debug path, cached
heads bit-exact."""
import numpy as np
import pytest
import torch

from paper_2503_22796_amd import workloads as W
from util import (ARROW, CACHE, FULL, TOL_BF16, TOL_F32, boundary_rows, check_against_oracle,
                  gpu_joint_attention, same_result_bf16)

pytestmark = pytest.mark.gpu


def small_workload(B, H, D, n_text, n_img, modes, wins, seed, positional=False):
    return W.Workload("case", B, H, D, n_text, n_img, np.asarray(modes, np.int32), np.asarray(wins, np.int32),
                      seed=seed, positional=positional)


def run_case(wl, dtype=torch.bfloat16, layout="bhnd", rows=None, scale=0.0, tol=None, flat_below=None):
    q, k, v = W.make_qkv(wl, dtype=dtype)
    cache = W.make_cache(wl, dtype=dtype) if (wl.head_plan == CACHE).any() else None
    out = gpu_joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img, scale=scale,
                              layout=layout)
    tol = tol if tol is not None else (TOL_BF16 if dtype == torch.bfloat16 else TOL_F32)
    err = check_against_oracle(out, q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img,
                               scale=(scale if scale > 0 else None), rows=rows, tol=tol, flat_below=flat_below)
    print(f"{wl.name}: dtype={dtype} layout={layout} max_abs_err={err:.3e} max|out|={float(out.float().abs().max()):.2f} "
          f"so far: worst excess over 2^-7|ref| {getattr(check_against_oracle, 'worst_excess', float('nan')):.3e}, "
          f"worst rms error / rms bar {getattr(check_against_oracle, 'worst_rms', float('nan')):.3f}", flush=True)
    return out


# ----------------------------------------------------------------------------- the named configs
def test_tiny_bf16():
    run_case(W.tiny())


def test_tiny_fp32_debug_path():
    run_case(W.tiny(), dtype=torch.float32)


def test_sd3_1k_all_rows():
    run_case(W.sd3_1k())


def test_flux_1k_all_rows():
    run_case(W.flux_1k())


def test_flux_2k_mixed_all_rows():
    run_case(W.flux_2k_mixed())


def test_flux_2k_full_all_rows():
    run_case(W.flux_2k_full())


def test_flux_2k_arrow_w128_all_rows():
    run_case(W.flux_2k_single_mode(ARROW, 128))


# ----------------------------------------------------------------------------- further layer shapes
@pytest.mark.parametrize("n_text", [77, 154, 256])
def test_flux_1k_other_prompt_lengths_all_rows(n_text):
    run_case(W.flux_1k_text(n_text), flat_below=4.0)


def test_sd3_2k_sampled_rows():
    wl = W.sd3_2k()
    rows = boundary_rows(wl.n_text, wl.n_img, wl.window[wl.head_plan == ARROW], extra=96, seed=6)
    run_case(wl, rows=rows, flat_below=4.0)


def test_video_like_layer_sampled_rows():
    wl = W.video_like()       # 13 x 30 x 52 latent: not a square grid, N = 20 536 is not a multiple of the tile sizes
    rows = boundary_rows(wl.n_text, wl.n_img, wl.window[wl.head_plan == ARROW], extra=96, seed=7)
    run_case(wl, rows=rows, flat_below=4.0)


# ----------------------------------------------------------------------------- shapes and edges
@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("n_text,n_img,wins", [
    (0, 300, [0, 1, 70]),          # no text: pure band, first band tile has fully masked rows
    (77, 0, [0, 5, 9]),            # no image tokens: every head is full attention
    (1, 1, [0, 0, 0]),             # two tokens
    (64, 256, [63, 64, 65]),       # band edges on tile edges
    (333, 1000, [7, 130, 998]),    # text edge mid-tile, ragged tail, window ~ n_img
    (130, 515, [200, 514, 9999]),  # w >= n_img - 1 is full attention
])
def test_edge_shapes_bf16(D, n_text, n_img, wins):
    wl = small_workload(2, 4, D, n_text, n_img, [FULL, ARROW, ARROW, ARROW], [0] + wins, seed=100 + n_img)
    run_case(wl)


def test_single_token():
    wl = small_workload(1, 2, 64, 1, 0, [FULL, ARROW], [0, 3], seed=7)
    run_case(wl)
    wl = small_workload(1, 2, 64, 0, 1, [FULL, ARROW], [0, 0], seed=8)
    run_case(wl)


@pytest.mark.parametrize("D", [64, 128])
def test_fp32_debug_path_mid_size(D):
    wl = small_workload(2, 5, D, 45, 400, [FULL, ARROW, ARROW, CACHE, ARROW], [0, 0, 33, 0, 399], seed=21,
                        positional=True)
    run_case(wl, dtype=torch.float32)


@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_bnhd_layout(dtype):
    wl = small_workload(2, 6, 64, 50, 256, [FULL, ARROW, CACHE, ARROW, CACHE, FULL], [0, 17, 0, 100, 0, 0],
                        seed=31, positional=True)
    run_case(wl, dtype=dtype, layout="bnhd")


def test_softmax_scale_override():
    wl = small_workload(1, 2, 64, 20, 144, [FULL, ARROW], [0, 12], seed=41)
    run_case(wl, scale=0.05)


def test_peaked_rows_with_large_values():
    # positional term makes rows sharply peaked; large values stress the P rounding and rescale
    wl = small_workload(1, 3, 128, 64, 1024, [FULL, ARROW, ARROW], [0, 64, 300], seed=51, positional=True)
    run_case(wl)


# ----------------------------------------------------------------------------- invariants on the GPU
def test_arrow_covering_window_equals_full_on_gpu():
    wl = small_workload(1, 3, 128, 70, 400, [FULL, ARROW, ARROW], [0, 399, 5000], seed=61)
    q, k, v = W.make_qkv(wl)
    q[:, 1:] = q[:, :1]; k[:, 1:] = k[:, :1]; v[:, 1:] = v[:, :1]
    out = gpu_joint_attention(q, k, v, None, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    assert torch.equal(out[:, 0], out[:, 1]) and torch.equal(out[:, 0], out[:, 2])


def test_keys_outside_band_do_not_matter_on_gpu():
    n_text, n_img, w = 100, 900, 150
    wl = small_workload(1, 1, 128, n_text, n_img, [ARROW], [w], seed=71)
    q, k, v = W.make_qkv(wl)
    base = gpu_joint_attention(q, k, v, None, wl.head_plan, wl.window, n_text, n_img)
    i = n_text + 500
    k2, v2 = k.clone(), v.clone()
    for j in (i + w + 1, i - w - 1):
        k2[0, 0, j] = 40.0
        v2[0, 0, j] = -30.0
    got = gpu_joint_attention(q, k2, v2, None, wl.head_plan, wl.window, n_text, n_img)
    assert torch.equal(got[0, 0, i], base[0, 0, i])
    k3 = k.clone()
    k3[0, 0, i + w] = 40.0
    got3 = gpu_joint_attention(q, k3, v, None, wl.head_plan, wl.window, n_text, n_img)
    assert not torch.equal(got3[0, 0, i], base[0, 0, i])


def test_cache_heads_bit_exact_and_cache_contents_never_leak():
    wl = small_workload(2, 4, 64, 33, 300, [CACHE, FULL, CACHE, ARROW], [0, 0, 0, 40], seed=81)
    q, k, v = W.make_qkv(wl)
    cache = W.make_cache(wl)
    cache[:, 1] = float("nan")
    cache[:, 3] = float("inf")
    cache.view(torch.int16)[0, 0, 0, 0] = 0x7FC1     # NaN payload must survive
    out = gpu_joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    for h in (0, 2):
        assert torch.equal(out[:, h].view(torch.int16), cache[:, h].view(torch.int16))
    check_against_oracle(out, q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img)


def test_all_heads_cached_launches_only_the_copy():
    wl = small_workload(1, 3, 128, 10, 200, [CACHE, CACHE, CACHE], [0, 0, 0], seed=91)
    q, k, v = W.make_qkv(wl)
    cache = W.make_cache(wl)
    out = gpu_joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    assert torch.equal(out.view(torch.int16), cache.view(torch.int16))


def test_out_may_alias_cache():
    wl = small_workload(1, 3, 64, 20, 300, [CACHE, ARROW, FULL], [0, 25, 0], seed=101)
    q, k, v = W.make_qkv(wl)
    cache = W.make_cache(wl)
    out = gpu_joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img,
                              alias_out_to_cache=True)
    check_against_oracle(out, q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img)


# ----------------------------------------------------------------------------- the plan object
def test_plan_reuse_many_plans_and_a_side_stream():
    from paper_2503_22796_amd import binding as B
    n_text, n_img, H, D = 40, 529, 4, 128
    N = n_text + n_img
    base = small_workload(1, H, D, n_text, n_img, [FULL] * H, [0] * H, seed=111, positional=True)
    q, k, v = W.make_qkv(base)
    cache = W.make_cache(base)
    plan = B.difa_plan_create(1, H, D, max_tokens=N)
    side = torch.cuda.Stream()
    try:
        rng = np.random.Generator(np.random.PCG64(5))
        cases = []
        for it in range(12):                      # more distinct plans than the memo keeps
            hp = rng.integers(0, 3, size=H).astype(np.int32)
            win = rng.integers(0, 300, size=H).astype(np.int32)
            cases.append((hp, win))
        for rep in range(2):                      # second pass: evicted plans are rebuilt
            for n, (hp, win) in enumerate(cases):
                stream = side if n % 2 else None
                out = gpu_joint_attention(q, k, v, cache, hp, win, n_text, n_img, plan=plan, stream=stream)
                check_against_oracle(out, q, k, v, cache, hp, win, n_text, n_img)
        # a shorter sequence on the same plan object
        wl2 = small_workload(1, H, D, 8, 100, [ARROW, FULL, CACHE, ARROW], [3, 0, 0, 50], seed=112)
        q2, k2, v2 = W.make_qkv(wl2)
        c2 = W.make_cache(wl2)
        out = gpu_joint_attention(q2, k2, v2, c2, wl2.head_plan, wl2.window, 8, 100, plan=plan)
        check_against_oracle(out, q2, k2, v2, c2, wl2.head_plan, wl2.window, 8, 100)
    finally:
        B.difa_plan_destroy(plan)


def test_argument_errors_launch_nothing():
    from paper_2503_22796_amd import binding as B
    H, D, N = 2, 64, 32
    plan = B.difa_plan_create(1, H, D, max_tokens=N)
    dev = torch.device("cuda:0")
    q = torch.zeros(1, H, N, D, dtype=torch.bfloat16, device=dev)
    out = torch.full_like(q, 7.0)
    try:
        bad = [
            dict(head_plan=[0, 3], window=[0, 0]),                 # unknown mode
            dict(head_plan=[1, 0], window=[-2, 0]),                # negative window
            dict(head_plan=[1, 0], window=None),                   # arrow without windows
            dict(head_plan=[2, 0], window=[0, 0]),                 # cache head, no cache tensor
            dict(head_plan=[0, 0], window=[0, 0], n_text=30, n_img=30),   # beyond max_tokens
            dict(head_plan=[0, 0], window=[0, 0], n_text=0, n_img=0),
            dict(head_plan=[0, 0], window=[0, 0], n_text=-1, n_img=5),
        ]
        for kw in bad:
            args = dict(n_text=16, n_img=16)
            args.update(kw)
            with pytest.raises(B.DifaError) as ei:
                B.difa_joint_attention(plan, q, q, q, out, None, args["head_plan"], args["n_text"],
                                       args["n_img"], args["window"])
            assert ei.value.status == B.DIFA_ERR_INVALID_ARG
            assert B.difa_last_error(plan) != ""
        with pytest.raises(B.DifaError):
            B.difa_joint_attention(plan, q, q, q, q, None, [0, 0], 16, 16, [0, 0])   # out aliases q
        torch.cuda.synchronize()
        assert bool((out == 7.0).all())
    finally:
        B.difa_plan_destroy(plan)


def test_too_many_tokens_for_32_bit_offsets_inside_a_head_are_refused():
    from paper_2503_22796_amd import binding as B
    # [B, N, H, D] with 24 heads of 128: a token row is 6 KiB, so 2 GiB of one head is 349 527 tokens
    plan = B.difa_plan_create(1, 24, 128, layout=B.DIFA_LAYOUT_BNHD, max_tokens=400000)
    try:
        t = torch.zeros(1, 64, 24, 128, dtype=torch.bfloat16, device="cuda:0")     # never read: the call is refused
        with pytest.raises(B.DifaError) as ei:
            B.difa_joint_attention(plan, t, t, t, torch.empty_like(t), None, [0] * 24, 0, 349600, [0] * 24)
        assert ei.value.status == B.DIFA_ERR_UNSUPPORTED
    finally:
        B.difa_plan_destroy(plan)


def test_kernel_timing_hook():
    from paper_2503_22796_amd import binding as B
    wl = small_workload(1, 4, 128, 64, 1024, [FULL, ARROW, CACHE, FULL], [0, 100, 0, 0], seed=121)
    q, k, v = (t.cuda() for t in W.make_qkv(wl))
    cache = W.make_cache(wl).cuda()
    out = torch.empty_like(q)
    plan = B.difa_plan_create(1, 4, 128, max_tokens=wl.N)
    try:
        B.difa_plan_timing_enable(plan, True)
        for _ in range(3):
            B.difa_joint_attention(plan, q, k, v, out, cache, wl.head_plan, wl.n_text, wl.n_img, wl.window)
        attn_ms, copy_ms, launches = B.difa_plan_timing_read(plan)
        assert launches == 3 and attn_ms > 0
        assert copy_ms == 0        # the cached head is copied inside the one launch
        assert B.difa_plan_timing_read(plan)[2] == 0
    finally:
        B.difa_plan_destroy(plan)


# ----------------------------------------------------------------------------- block-granular band
def run_block_case(wl, dtype=torch.bfloat16, rows=None):
    from paper_2503_22796_amd import binding as B
    bm, bn = B.difa_tile_shape(wl.D, B.DIFA_DTYPE_BF16 if dtype == torch.bfloat16 else B.DIFA_DTYPE_F32)
    q, k, v = W.make_qkv(wl, dtype=dtype)
    cache = W.make_cache(wl, dtype=dtype) if (wl.head_plan == CACHE).any() else None
    out = gpu_joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img,
                              flags=B.DIFA_FLAG_BLOCK_BAND)
    tol = TOL_BF16 if dtype == torch.bfloat16 else TOL_F32
    err = check_against_oracle(out, q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img, rows=rows,
                               tol=tol, block=(bm, bn))
    print(f"{wl.name} (block band {bm}x{bn}): dtype={dtype} max_abs_err={err:.3e}", flush=True)
    return out, q, k, v


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("n_text,n_img,wins", [
    (0, 700, [0, 1, 70]),
    (64, 1024, [63, 64, 300]),
    (333, 1000, [7, 130, 998]),
])
def test_block_band_edge_shapes(D, n_text, n_img, wins):
    wl = small_workload(2, 4, D, n_text, n_img, [FULL, ARROW, ARROW, ARROW], [0] + wins, seed=200 + n_img)
    run_block_case(wl)


def test_block_band_flux_1k_all_rows_and_it_differs_from_the_exact_band():
    wl = W.flux_1k()
    out, q, k, v = run_block_case(wl)
    exact = gpu_joint_attention(q, k, v, W.make_cache(wl), wl.head_plan, wl.window, wl.n_text, wl.n_img)
    arrow = [h for h in range(wl.H) if wl.head_plan[h] == ARROW and wl.window[h] < wl.n_img - 1]
    assert any(not torch.equal(out[:, h], exact[:, h]) for h in arrow)      # the flag is not a no-op
    others = [h for h in range(wl.H) if wl.head_plan[h] == FULL]
    # full heads compute the same thing in both runs (their records may be cut at other places)
    assert all(same_result_bf16(out[:, h], exact[:, h]) for h in others)


def test_block_band_flux_2k_mixed_sampled_rows():
    wl = W.flux_2k_mixed()
    rows = boundary_rows(wl.n_text, wl.n_img, wl.window[wl.head_plan == ARROW], extra=64, seed=14)
    run_block_case(wl, rows=rows)


# ----------------------------------------------------------------------------- image tokens first
def run_image_first_case(wl, dtype=torch.bfloat16, layout="bhnd", rows=None, block=False):
    """The workload's tensors with the text block moved behind the image block, DIFA_FLAG_IMAGE_FIRST."""
    from paper_2503_22796_amd import binding as B
    rot = list(range(wl.n_text, wl.N)) + list(range(wl.n_text))
    q, k, v = (t[:, :, rot].contiguous() for t in W.make_qkv(wl, dtype=dtype))
    cache = W.make_cache(wl, dtype=dtype) if (wl.head_plan == CACHE).any() else None
    flags = B.DIFA_FLAG_IMAGE_FIRST | (B.DIFA_FLAG_BLOCK_BAND if block else 0)
    out = gpu_joint_attention(q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img, layout=layout, flags=flags)
    tol = TOL_BF16 if dtype == torch.bfloat16 else TOL_F32
    blk = B.difa_tile_shape(wl.D) if block else None
    err = check_against_oracle(out, q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img, rows=rows,
                               tol=tol, block=blk, image_first=True)
    print(f"{wl.name} (image first{', block band' if block else ''}): dtype={dtype} layout={layout} "
          f"max_abs_err={err:.3e}", flush=True)
    return out


@pytest.mark.parametrize("D", [64, 128])
@pytest.mark.parametrize("n_text,n_img,wins", [
    (16, 64, [8, 16, 70]),         # the tiny shape
    (0, 700, [0, 1, 70]),          # no text at all
    (64, 1024, [63, 64, 300]),     # image length a multiple of the key tile
    (333, 1000, [7, 130, 998]),    # a key tile that holds image and text keys; ragged tail
    (700, 50, [3, 20, 49]),        # fewer image tokens than one key tile, long text
    (1, 4099, [0, 255, 2048]),
])
def test_image_first_edge_shapes(D, n_text, n_img, wins):
    wl = small_workload(2, 5, D, n_text, n_img, [FULL, ARROW, ARROW, ARROW, CACHE], [0] + wins + [0], seed=300 + n_img)
    run_image_first_case(wl)


def test_image_first_sd3_1k_all_rows():
    run_image_first_case(W.sd3_1k())


def test_image_first_flux_1k_bnhd_layout():
    run_image_first_case(W.flux_1k(), layout="bnhd")


def test_image_first_flux_2k_mixed_sampled_rows():
    wl = W.flux_2k_mixed()
    # edges of the rotated sequence: image rows are 0 .. n_img-1 now, text rows the last n_text
    rows = sorted({(r - wl.n_text) % wl.N for r in
                   boundary_rows(wl.n_text, wl.n_img, wl.window[wl.head_plan == ARROW], extra=64, seed=15)})
    run_image_first_case(wl, rows=rows)


def test_image_first_fp32_debug_path():
    wl = small_workload(1, 4, 64, 40, 300, [FULL, ARROW, ARROW, CACHE], [0, 5, 120, 0], seed=311)
    run_image_first_case(wl, dtype=torch.float32)


def test_image_first_with_block_band():
    wl = small_workload(2, 4, 128, 100, 1500, [FULL, ARROW, ARROW, ARROW], [0, 7, 130, 700], seed=312)
    run_image_first_case(wl, block=True)


def test_image_first_equals_text_first_on_rotated_inputs():
    from paper_2503_22796_amd import binding as B
    wl = small_workload(1, 3, 128, 128, 2048, [FULL, ARROW, ARROW], [0, 100, 600], seed=313)
    q, k, v = W.make_qkv(wl)
    ref = gpu_joint_attention(q, k, v, None, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    rot = list(range(wl.n_text, wl.N)) + list(range(wl.n_text))
    got = gpu_joint_attention(q[:, :, rot].contiguous(), k[:, :, rot].contiguous(), v[:, :, rot].contiguous(), None,
                              wl.head_plan, wl.window, wl.n_text, wl.n_img, flags=B.DIFA_FLAG_IMAGE_FIRST)
    # same pairs, visited in another order
    assert same_result_bf16(got, ref[:, :, rot])
