"""Pins for the CPU oracle: checks against things other than itself.

Each test names what a plausible mistake it would catch.  None of them needs a GPU
and none of them touches the HIP library.
"""
import math
import os

import numpy as np
import pytest
import torch

from oracle import difa_oracle as O
from paper_2503_22796_amd import workloads as W

FULL, ARROW, CACHE = 0, 1, 2
GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def rand(shape, seed, dtype=torch.float32):
    g = torch.Generator().manual_seed(seed)
    return torch.randn(shape, generator=g, dtype=torch.float32).to(dtype)


def brute_force(q, k, v, mode, w, n_text, scale):
    """Independent statement of Sec. 3.1 with explicit Python loops (one head)."""
    N, D = len(q), len(q[0])
    out = [[0.0] * D for _ in range(N)]
    for i in range(N):
        keys = []
        for j in range(N):
            if mode == FULL:
                ok = True
            else:
                text_involved = (i < n_text) or (j < n_text)
                ok = text_involved or (-w <= i - j <= w)
            if ok:
                keys.append(j)
        scores = [scale * sum(q[i][d] * k[j][d] for d in range(D)) for j in keys]
        top = max(scores)
        e = [math.exp(s - top) for s in scores]
        z = sum(e)
        for jj, j in enumerate(keys):
            wgt = e[jj] / z
            for d in range(D):
                out[i][d] += wgt * v[j][d]
    return torch.tensor(out, dtype=torch.float64)


def separately_built_mask(N, n_text, w):
    """Boolean [N,N] arrow mask built quadrant by quadrant (not via the oracle's predicate)."""
    m = torch.zeros(N, N, dtype=torch.bool)
    m[:n_text, :] = True          # language -> everything
    m[:, :n_text] = True          # everything -> language
    n_img = N - n_text
    idx = torch.arange(n_img)
    band = (idx[:, None] - idx[None, :]).abs() <= w
    m[n_text:, n_text:] = band
    return m


# --------------------------------------------------------------------------- brute force
def test_tiny_config_matches_brute_force():
    wl = W.tiny()
    q, k, v = W.make_qkv(wl)
    c = W.make_cache(wl)
    out, raw, _ = O.joint_attention(q, k, v, c, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    for h in range(3):
        ref = brute_force(q[0, h].double().tolist(), k[0, h].double().tolist(),
                          v[0, h].double().tolist(), int(wl.head_plan[h]), int(wl.window[h]),
                          wl.n_text, wl.scale)
        assert (out[0, h] - ref).abs().max() < 1e-12
    assert torch.equal(raw[0, 3].view(torch.int16), c[0, 3].view(torch.int16))


@pytest.mark.parametrize("n_text,n_img,w,D", [(0, 9, 0, 4), (0, 12, 3, 8), (1, 16, 1, 8),
                                               (5, 25, 3, 4), (5, 16, 16, 8), (5, 16, 40, 8),
                                               (7, 1, 0, 4), (3, 0, 2, 4)])
def test_random_tiny_shapes_match_brute_force(n_text, n_img, w, D):
    N = n_text + n_img
    q, k, v = (rand((1, 2, N, D), s) for s in (11, 12, 13))
    scale = 0.37
    out, _, _ = O.joint_attention(q, k, v, None, [FULL, ARROW], [0, w], n_text, n_img, scale=scale)
    for h, mode in enumerate([FULL, ARROW]):
        ref = brute_force(q[0, h].double().tolist(), k[0, h].double().tolist(),
                          v[0, h].double().tolist(), mode, w, n_text, scale)
        assert (out[0, h] - ref).abs().max() < 1e-12


# ------------------------------------------------------------------- library routine (SDPA)
def test_full_and_arrow_match_torch_sdpa_fp64():
    n_text, n_img, D, w = 13, 100, 16, 7
    N = n_text + n_img
    q, k, v = (rand((2, 3, N, D), s, torch.bfloat16) for s in (1, 2, 3))
    out, _, _ = O.joint_attention(q, k, v, None, [FULL, ARROW, ARROW], [0, w, 3 * w], n_text, n_img)
    qd, kd, vd = q.double(), k.double(), v.double()
    ref_full = torch.nn.functional.scaled_dot_product_attention(qd, kd, vd)
    assert (out[:, 0] - ref_full[:, 0]).abs().max() < 1e-12
    for h, ww in ((1, w), (2, 3 * w)):
        mask = separately_built_mask(N, n_text, ww)
        ref = torch.nn.functional.scaled_dot_product_attention(qd[:, h], kd[:, h], vd[:, h],
                                                               attn_mask=mask)
        assert (out[:, h] - ref).abs().max() < 1e-12


def test_scale_argument_is_used():
    q, k, v = (rand((1, 1, 20, 8), s) for s in (4, 5, 6))
    out, _, _ = O.joint_attention(q, k, v, None, [FULL], [0], 4, 16, scale=0.9)
    ref = torch.nn.functional.scaled_dot_product_attention(q.double(), k.double(), v.double(), scale=0.9)
    assert (out - ref).abs().max() < 1e-12


# ------------------------------------------------------------------- mask cardinality
def golden_pairs():
    rows = []
    with open(os.path.join(GOLDEN, "arrow_pair_counts.txt")) as f:
        for line in f:
            if line.strip() and not line.startswith("#"):
                rows.append(tuple(int(t) for t in line.split()))
    return rows


@pytest.mark.parametrize("n_text,n_img,w,pairs", golden_pairs())
def test_allowed_pair_count_matches_hand_counts(n_text, n_img, w, pairs):
    N = n_text + n_img
    got = sum(O.allowed(ARROW, i, j, n_text, w) for i in range(N) for j in range(N))
    assert got == pairs
    # and through the values: probabilities are non-zero exactly on allowed pairs
    q, k, v = (rand((1, 1, N, 4), s) for s in (7, 8, 9))
    _, _, P = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img, want_probs=True)
    assert int((P[0, 0] > 0).sum()) == pairs


def test_per_row_count_closed_form():
    n_text, n_img, w = 6, 30, 4
    N = n_text + n_img
    q, k, v = (rand((1, 1, N, 4), s) for s in (7, 8, 9))
    _, _, P = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img, want_probs=True)
    for i in range(N):
        if i < n_text:
            expect = N
        else:
            ii = i - n_text
            expect = n_text + min(ii + w, n_img - 1) - max(ii - w, 0) + 1
        assert int((P[0, 0, i] > 0).sum()) == expect


# ------------------------------------------------------------------- invariants
def test_arrow_with_window_covering_image_equals_full_exactly():
    n_text, n_img, D = 5, 40, 8
    N = n_text + n_img
    q, k, v = (rand((1, 3, N, D), s, torch.bfloat16) for s in (21, 22, 23))
    qq = q[:, :1].expand(1, 3, N, D).contiguous()
    kk = k[:, :1].expand(1, 3, N, D).contiguous()
    vv = v[:, :1].expand(1, 3, N, D).contiguous()
    out, _, _ = O.joint_attention(qq, kk, vv, None, [FULL, ARROW, ARROW], [0, n_img - 1, 10 * n_img],
                                  n_text, n_img)
    assert torch.equal(out[0, 0], out[0, 1]) and torch.equal(out[0, 0], out[0, 2])
    # one less than covering is NOT full (rows 0 and n_img-1 of the image lose one key)
    out2, _, _ = O.joint_attention(qq, kk, vv, None, [FULL, ARROW, ARROW], [0, n_img - 2, 0],
                                   n_text, n_img)
    assert not torch.equal(out2[0, 0], out2[0, 1])
    assert torch.equal(out2[0, 0, n_text + 1:N - 1], out2[0, 1, n_text + 1:N - 1])


def test_text_rows_of_arrow_head_equal_full():
    n_text, n_img, D = 9, 36, 8
    N = n_text + n_img
    q, k, v = (rand((1, 1, N, D), s).expand(1, 2, N, D).contiguous() for s in (31, 32, 33))
    out, _, _ = O.joint_attention(q, k, v, None, [FULL, ARROW], [0, 2], n_text, n_img)
    assert torch.equal(out[0, 0, :n_text], out[0, 1, :n_text])
    assert not torch.equal(out[0, 0, n_text:], out[0, 1, n_text:])


def test_rows_sum_to_one_and_zero_outside_mask():
    n_text, n_img, w = 4, 49, 5
    N = n_text + n_img
    q, k, v = (rand((2, 2, N, 8), s) for s in (41, 42, 43))
    _, _, P = O.joint_attention(q, k, v, None, [FULL, ARROW], [0, w], n_text, n_img, want_probs=True)
    assert (P.sum(-1) - 1).abs().max() < 1e-12
    mask = separately_built_mask(N, n_text, w)
    assert (P[:, 1][:, ~mask] == 0).all()
    assert (P[:, 1][:, mask] > 0).all()
    assert (P[:, 0] > 0).all()


# ------------------------------------------------------------------- closed forms
def test_zero_queries_give_mean_of_allowed_values():
    n_text, n_img, w, D = 3, 25, 4, 6
    N = n_text + n_img
    k, v = rand((1, 1, N, D), 51), rand((1, 1, N, D), 52)
    q = torch.zeros(1, 1, N, D)
    out, _, _ = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img)
    mask = separately_built_mask(N, n_text, w).double()
    expect = (mask @ v[0, 0].double()) / mask.sum(-1, keepdim=True)
    assert (out[0, 0] - expect).abs().max() < 1e-13


def test_constant_values_pass_through():
    N, D = 30, 8
    q, k = rand((1, 2, N, D), 61), rand((1, 2, N, D), 62)
    v = torch.full((1, 2, N, D), 0.75)
    out, _, _ = O.joint_attention(q, k, v, None, [FULL, ARROW], [0, 3], 5, 25)
    assert (out - 0.75).abs().max() < 1e-14


def test_zero_window_without_text_returns_values():
    N, D = 17, 8
    q, k, v = (rand((1, 1, N, D), s) for s in (71, 72, 73))
    out, _, _ = O.joint_attention(q, k, v, None, [ARROW], [0], 0, N)
    assert torch.equal(out[0, 0], v[0, 0].double())


def test_softmax_shift_invariance_under_common_key_offset():
    n_text, n_img, D = 4, 36, 8
    N = n_text + n_img
    q, k, v = (rand((1, 2, N, D), s).double() for s in (81, 82, 83))
    u = 3.0 * rand((D,), 84).double()
    a, _, _ = O.joint_attention(q.float(), k.float(), v.float(), None, [FULL, ARROW], [0, 5], n_text, n_img)
    k2 = (k + u).float()
    b, _, _ = O.joint_attention(q.float(), k2, v.float(), None, [FULL, ARROW], [0, 5], n_text, n_img)
    # k2 is rounded to fp32, so agreement is to fp32 rounding of the shift, not exact
    assert (a - b).abs().max() < 1e-5


def test_single_huge_logit_selects_that_value_row():
    N, D = 24, 8
    q, k, v = (rand((1, 1, N, D), s) for s in (91, 92, 93))
    j_star = 17
    k[0, 0, j_star] = 0
    k[0, 0, j_star, 0] = 1000.0
    q[0, 0, :, 0] = 1.0          # every query scores ~ +1000*scale on key j_star
    out, _, _ = O.joint_attention(q, k, v, None, [FULL], [0], 4, 20, scale=1.0)
    assert (out[0, 0] - v[0, 0, j_star].double()).abs().max() < 1e-12


# ------------------------------------------------------------------- structure
def test_head_permutation_commutes():
    wl = W.tiny()
    q, k, v = W.make_qkv(wl)
    c = W.make_cache(wl)
    out, raw, _ = O.joint_attention(q, k, v, c, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    perm = [2, 3, 0, 1]
    out_p, raw_p, _ = O.joint_attention(q[:, perm], k[:, perm], v[:, perm], c[:, perm],
                                        wl.head_plan[perm], wl.window[perm], wl.n_text, wl.n_img)
    assert torch.equal(out[:, perm], out_p)
    assert torch.equal(raw[:, perm].view(torch.int16), raw_p.view(torch.int16))


def test_text_key_permutation_leaves_output_unchanged():
    n_text, n_img, D = 6, 25, 8
    N = n_text + n_img
    q, k, v = (rand((1, 1, N, D), s) for s in (101, 102, 103))
    a, _, _ = O.joint_attention(q, k, v, None, [ARROW], [3], n_text, n_img)
    perm = torch.cat([torch.tensor([4, 2, 0, 5, 1, 3]), torch.arange(n_text, N)])
    b, _, _ = O.joint_attention(q, k[:, :, perm], v[:, :, perm], None, [ARROW], [3], n_text, n_img)
    assert (a - b).abs().max() < 1e-13   # summation order differs


def test_keys_just_outside_band_are_irrelevant_and_band_edge_is_not():
    n_text, n_img, D, w = 5, 40, 8, 6
    N = n_text + n_img
    q, k, v = (rand((1, 1, N, D), s) for s in (111, 112, 113))
    base, _, _ = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img)
    i = n_text + 20
    for delta, changes in ((w + 1, False), (-(w + 1), False), (w, True), (-w, True)):
        k2, v2 = k.clone(), v.clone()
        k2[0, 0, i + delta] += 5.0
        v2[0, 0, i + delta] -= 7.0
        got, _, _ = O.joint_attention(q, k2, v2, None, [ARROW], [w], n_text, n_img)
        same = torch.equal(got[0, 0, i], base[0, 0, i])
        assert same != changes


def test_band_is_on_flattened_image_index_not_joint_index():
    # image row 0 (joint index n_text) must see image keys 0..w of the image, and text
    # keys count as text, not as "within w of the diagonal"
    n_text, n_img, w = 10, 20, 2
    N = n_text + n_img
    q, k, v = (rand((1, 1, N, 4), s) for s in (121, 122, 123))
    _, _, P = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img, want_probs=True)
    row = P[0, 0, n_text]
    assert (row[:n_text] > 0).all() and (row[n_text:n_text + w + 1] > 0).all()
    assert (row[n_text + w + 1:] == 0).all()


# ------------------------------------------------------------------- cache heads
def test_cache_heads_are_bit_exact_and_cache_never_leaks_into_computed_heads():
    wl = W.tiny()
    q, k, v = W.make_qkv(wl)
    c = W.make_cache(wl)
    out, raw, _ = O.joint_attention(q, k, v, c, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    poisoned = c.clone()
    poisoned[:, :3] = float("nan")
    out2, raw2, _ = O.joint_attention(q, k, v, poisoned, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    assert torch.equal(out[:, :3], out2[:, :3])
    assert torch.equal(raw2[0, 3].view(torch.int16), c[0, 3].view(torch.int16))
    assert torch.equal(out[0, 3], c[0, 3].double())
    # a NaN payload survives a raw copy
    weird = c.clone()
    weird.view(torch.int16)[0, 3, 0, 0] = 0x7FC1
    _, raw3, _ = O.joint_attention(q, k, v, weird, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    assert int(raw3.view(torch.int16)[0, 3, 0, 0]) == 0x7FC1


# ------------------------------------------------------------------- interface
def test_row_subset_equals_rows_of_full_evaluation():
    wl = W.tiny()
    q, k, v = W.make_qkv(wl)
    c = W.make_cache(wl)
    full, raw, _ = O.joint_attention(q, k, v, c, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    rows = [79, 0, 15, 16, 17, 40]
    sub, raw_s, _ = O.joint_attention(q, k, v, c, wl.head_plan, wl.window, wl.n_text, wl.n_img, rows=rows)
    assert torch.equal(sub, full[:, :, rows])
    assert torch.equal(raw_s[:, 3].view(torch.int16), raw[:, 3][:, rows].view(torch.int16))


def test_fp32_inputs_and_bf16_inputs_agree_when_values_are_bf16_representable():
    wl = W.tiny()
    q, k, v = W.make_qkv(wl)
    c = W.make_cache(wl)
    a, _, _ = O.joint_attention(q, k, v, c, wl.head_plan, wl.window, wl.n_text, wl.n_img)
    b, rawf, _ = O.joint_attention(q.float(), k.float(), v.float(), c.float(), wl.head_plan,
                                   wl.window, wl.n_text, wl.n_img)
    assert torch.equal(a, b)
    assert torch.equal(rawf[0, 3], c[0, 3].float())


def test_invalid_arguments_are_rejected():
    q, k, v = (rand((1, 1, 8, 4), s) for s in (1, 2, 3))
    with pytest.raises(ValueError):
        O.joint_attention(q, k, v, None, [CACHE], [0], 4, 4)       # cache head without cache
    with pytest.raises(ValueError):
        O.joint_attention(q, k, v, None, [ARROW], [-1], 4, 4)      # negative window
    with pytest.raises(ValueError):
        O.joint_attention(q, k, v, None, [3], [0], 4, 4)           # unknown mode
    with pytest.raises(ValueError):
        O.joint_attention(q, k, v, None, [FULL], [0], 4, 4, rows=[8])


# ------------------------------------------------------------------- the input recipe
def test_generator_is_seeded_and_diagonal_local():
    wl = W.config("flux_1k")
    pos = W.positional_term(wl.n_img, wl.D)
    assert pos.shape == (4096, 128) and abs(float(np.abs(pos).max()) - 1.5) < 1e-3
    # the positional inner product peaks at distance 0 on the grid
    g = pos @ pos[64 * 30 + 30]
    assert int(g.argmax()) == 64 * 30 + 30
    small = W.Workload("s", 1, 2, 8, 3, 16, np.zeros(2, np.int32), np.zeros(2, np.int32), seed=9)
    a = W.make_qkv(small)
    b = W.make_qkv(small)
    assert all(torch.equal(x, y) for x, y in zip(a, b))
    assert not torch.equal(a[0], W.make_qkv(small, step=1)[0])


# --------------------------------------------------------------------------- block-granular band
def block_rule(n_text, N, w, bm, bn):
    """Sec. 3.3 / Fig. 4 restated with explicit loops: a block is kept whole iff it holds a kept pair."""
    kept = [[False] * N for _ in range(N)]
    for a in range(0, N, bm):
        for b in range(0, N, bn):
            hit = any((i < n_text) or (j < n_text) or abs(i - j) <= w
                      for i in range(a, min(a + bm, N)) for j in range(b, min(b + bn, N)))
            if hit:
                for i in range(a, min(a + bm, N)):
                    for j in range(b, min(b + bn, N)):
                        kept[i][j] = True
    return kept


def brute_force_masked(q, k, v, kept, scale):
    N, D = len(q), len(q[0])
    out = [[0.0] * D for _ in range(N)]
    for i in range(N):
        keys = [j for j in range(N) if kept[i][j]]
        scores = [scale * sum(q[i][d] * k[j][d] for d in range(D)) for j in keys]
        top = max(scores)
        e = [math.exp(s - top) for s in scores]
        z = sum(e)
        for jj, j in enumerate(keys):
            for d in range(D):
                out[i][d] += e[jj] / z * v[j][d]
    return torch.tensor(out, dtype=torch.float64)


@pytest.mark.parametrize("n_text,n_img,w,bm,bn", [(0, 16, 1, 4, 4), (3, 21, 2, 8, 4), (5, 14, 0, 4, 8),
                                                   (1, 30, 6, 16, 4), (7, 9, 3, 5, 3)])
def test_block_band_matches_brute_force(n_text, n_img, w, bm, bn):
    # catches: block index from the wrong axis, blocks anchored at n_text instead of 0, a dropped ragged block
    N, D = n_text + n_img, 4
    q, k, v = (rand((1, 1, N, D), 300 + s + N) for s in range(3))
    got, _, probs = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img, scale=0.7, block=(bm, bn),
                                      want_probs=True)
    kept = block_rule(n_text, N, w, bm, bn)
    ref = brute_force_masked(q[0, 0].tolist(), k[0, 0].tolist(), v[0, 0].tolist(), kept, 0.7)
    assert (got[0, 0] - ref).abs().max() < 1e-12
    assert torch.equal(probs[0, 0] > 0, torch.tensor(kept))


def test_block_band_pair_counts_match_hand_counts():
    for line in open(os.path.join(GOLDEN, "block_band_pair_counts.txt")):
        if line.startswith("#") or not line.strip():
            continue
        n_text, n_img, w, bm, bn, pairs = (int(x) for x in line.split())
        N = n_text + n_img
        q, k, v = (rand((1, 1, N, 2), 400 + s) for s in range(3))
        _, _, probs = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img, block=(bm, bn), want_probs=True)
        assert int((probs[0, 0] > 0).sum()) == pairs, line


def test_block_band_with_unit_blocks_is_the_exact_band_and_is_a_superset_otherwise():
    n_text, n_img, w = 6, 40, 5
    N = n_text + n_img
    q, k, v = (rand((1, 2, N, 8), 500 + s) for s in range(3))
    exact, _, p_exact = O.joint_attention(q, k, v, None, [ARROW, FULL], [w, 0], n_text, n_img, want_probs=True)
    unit, _, _ = O.joint_attention(q, k, v, None, [ARROW, FULL], [w, 0], n_text, n_img, block=(1, 1))
    assert torch.equal(exact, unit)
    blk, _, p_blk = O.joint_attention(q, k, v, None, [ARROW, FULL], [w, 0], n_text, n_img, block=(8, 4),
                                      want_probs=True)
    assert bool(((p_exact[0, 0] > 0) <= (p_blk[0, 0] > 0)).all())       # every exact pair is still kept
    assert int((p_blk[0, 0] > 0).sum()) > int((p_exact[0, 0] > 0).sum())
    assert torch.equal(blk[:, 1], exact[:, 1])                           # FULL heads are untouched
    assert (p_blk.sum(-1) - 1).abs().max() < 1e-12


def test_block_band_covering_window_equals_full():
    n_text, n_img = 4, 28
    q, k, v = (rand((1, 2, n_text + n_img, 8), 600 + s) for s in range(3))
    out, _, _ = O.joint_attention(q, k, v, None, [ARROW, FULL], [n_img - 1, 0], n_text, n_img, block=(8, 8))
    q2, k2, v2 = q.clone(), k.clone(), v.clone()
    q2[:, 1], k2[:, 1], v2[:, 1] = q[:, 0], k[:, 0], v[:, 0]
    full, _, _ = O.joint_attention(q2, k2, v2, None, [ARROW, FULL], [n_img - 1, 0], n_text, n_img, block=(8, 8))
    assert torch.equal(full[:, 0], full[:, 1])


# --------------------------------------------------------------------------- image tokens first
def image_first_rule(n_text, n_img, w):
    """Sec. 3.1 restated for the order [image, text] with explicit loops."""
    N = n_text + n_img
    kept = [[False] * N for _ in range(N)]
    for i in range(N):
        for j in range(N):
            i_text, j_text = i >= n_img, j >= n_img
            kept[i][j] = i_text or j_text or (-w <= i - j <= w)
    return kept


@pytest.mark.parametrize("n_text,n_img,w", [(0, 12, 2), (4, 16, 1), (7, 9, 3), (3, 20, 0), (16, 8, 5)])
def test_image_first_matches_brute_force(n_text, n_img, w):
    # catches: text interval taken at the front, band measured from the wrong origin, text rows not full
    N, D = n_text + n_img, 4
    q, k, v = (rand((1, 1, N, D), 500 + s + N) for s in range(3))
    got, _, probs = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img, scale=0.6, want_probs=True,
                                      image_first=True)
    kept = image_first_rule(n_text, n_img, w)
    ref = brute_force_masked(q[0, 0].tolist(), k[0, 0].tolist(), v[0, 0].tolist(), kept, 0.6)
    assert (got[0, 0] - ref).abs().max() < 1e-12
    assert torch.equal(probs[0, 0] > 0, torch.tensor(kept))


def test_image_first_is_text_first_with_the_tokens_rotated():
    # the operator does not care where a token sits, only what kind it is: moving the text block
    # behind the image block moves the output rows and nothing else
    n_text, n_img, H, D = 6, 25, 3, 8
    N = n_text + n_img
    q, k, v = (rand((2, H, N, D), 600 + s, torch.bfloat16) for s in range(3))
    hp, win = [ARROW, FULL, ARROW], [3, 0, 9]
    ref, _, _ = O.joint_attention(q, k, v, None, hp, win, n_text, n_img)
    rot = list(range(n_text, N)) + list(range(n_text))          # image tokens first, then the text tokens
    got, _, _ = O.joint_attention(q[:, :, rot], k[:, :, rot], v[:, :, rot], None, hp, win, n_text, n_img,
                                  image_first=True)
    assert (got - ref[:, :, rot]).abs().max() < 1e-13


def test_image_first_pair_counts_and_predicate():
    # same number of allowed pairs as with the text in front (hand counts of the golden file)
    for n_text, n_img, w, pairs in golden_pairs():
        N = n_text + n_img
        cnt = sum(O.allowed(ARROW, i, j, n_text, w, n_img=n_img, image_first=True) for i in range(N) for j in range(N))
        assert cnt == pairs
    # a few pairs by hand: n_img = 10, n_text = 3, w = 2 -> text tokens are 10, 11, 12
    a = lambda i, j: O.allowed(ARROW, i, j, 3, 2, n_img=10, image_first=True)
    assert a(0, 2) and not a(0, 3) and a(0, 10) and a(0, 12)      # band edge; text keys always
    assert a(9, 7) and not a(9, 6) and a(12, 0) and a(10, 5)      # text queries see everything
    assert not a(5, 8) and a(5, 7)


def test_image_first_text_rows_equal_full_and_covering_window_equals_full():
    n_text, n_img, D = 5, 18, 8
    N = n_text + n_img
    q, k, v = (rand((1, 2, N, D), 700 + s) for s in range(3))
    full, _, _ = O.joint_attention(q, k, v, None, [FULL, FULL], [0, 0], n_text, n_img, image_first=True)
    arrow, _, _ = O.joint_attention(q, k, v, None, [ARROW, ARROW], [2, n_img - 1], n_text, n_img, image_first=True)
    assert torch.equal(arrow[:, 0, n_img:], full[:, 0, n_img:])          # the text rows are the last ones now
    assert not torch.equal(arrow[:, 0, :n_img], full[:, 0, :n_img])
    assert torch.equal(arrow[:, 1], full[:, 1])


def test_image_first_block_band_matches_brute_force():
    n_text, n_img, w, bm, bn = 5, 19, 2, 8, 4
    N, D = n_text + n_img, 4
    q, k, v = (rand((1, 1, N, D), 800 + s) for s in range(3))
    got, _, probs = O.joint_attention(q, k, v, None, [ARROW], [w], n_text, n_img, scale=0.7, block=(bm, bn),
                                      want_probs=True, image_first=True)
    exact = image_first_rule(n_text, n_img, w)
    kept = [[False] * N for _ in range(N)]
    for a in range(0, N, bm):
        for b in range(0, N, bn):
            if any(exact[i][j] for i in range(a, min(a + bm, N)) for j in range(b, min(b + bn, N))):
                for i in range(a, min(a + bm, N)):
                    for j in range(b, min(b + bn, N)):
                        kept[i][j] = True
    ref = brute_force_masked(q[0, 0].tolist(), k[0, 0].tolist(), v[0, 0].tolist(), kept, 0.7)
    assert (got[0, 0] - ref).abs().max() < 1e-12
    assert torch.equal(probs[0, 0] > 0, torch.tensor(kept))
