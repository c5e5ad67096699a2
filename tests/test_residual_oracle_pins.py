"""Pins of oracle/residual_oracle.py (arrow attention with residual sharing; Sec. 2.4, Sec. 4.6.1, Table 4 name
the technique): brute force, algebraic identities and hand-rounded values, none of which calls the code under test
to produce its expectation."""
import math
import os

import numpy as np
import torch

from oracle import difa_oracle as O
from oracle import residual_oracle as R

FULL, ARROW, CACHE, RES = 0, 1, 2, 3
GOLDEN = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "residual_hand_values.txt")


def rand(shape, seed, dtype=torch.float32):
    g = np.random.Generator(np.random.PCG64(seed))
    return torch.from_numpy(g.standard_normal(size=shape).astype(np.float32)).to(dtype)


def brute(q, k, v, r, n_text, w, scale):
    """One head, explicit loops: arrow attention of Sec. 3.1 and the kept difference added to every output element."""
    N, D = q.shape
    out = [[0.0] * D for _ in range(N)]
    for i in range(N):
        js = [j for j in range(N) if i < n_text or j < n_text or abs(i - j) <= w]
        s = [scale * sum(float(q[i, d]) * float(k[j, d]) for d in range(D)) for j in js]
        m = max(s)
        p = [math.exp(x - m) for x in s]
        l = sum(p)
        for d in range(D):
            out[i][d] = sum(pj * float(v[j, d]) for pj, j in zip(p, js)) / l + float(r[i, d])
    return torch.tensor(out, dtype=torch.float64)


def test_brute_force_on_tiny_shapes():
    for seed, (n_text, n_img, D, w) in enumerate([(3, 9, 4, 2), (0, 11, 3, 1), (5, 6, 2, 0), (2, 7, 5, 9)]):
        N = n_text + n_img
        q, k, v, r = (rand((1, 1, N, D), 10 * seed + t) for t in range(4))
        out, _ = R.joint_attention(q, k, v, None, r, [RES], [w], n_text, n_img, scale=0.7)
        want = brute(q[0, 0], k[0, 0], v[0, 0], r[0, 0], n_text, w, 0.7)
        assert float((out[0, 0] - want).abs().max()) <= 1e-12


def test_zero_residual_is_arrow_attention():
    q, k, v = (rand((2, 3, 20, 8), 50 + t) for t in range(3))
    hp, win = [RES, RES, FULL], [3, 0, 0]
    out, _ = R.joint_attention(q, k, v, None, torch.zeros_like(q), hp, win, 4, 16)
    ref, _, _ = O.joint_attention(q, k, v, None, [ARROW, ARROW, FULL], win, 4, 16)
    assert torch.equal(out, ref)


def test_refresh_step_reproduces_full_attention():
    """With the difference of the two exact outputs kept unrounded, arrow + r is full attention again."""
    q, k, v = (rand((1, 2, 24, 8), 60 + t) for t in range(3))
    full, _, _ = O.joint_attention(q, k, v, None, [FULL, FULL], [0, 0], 5, 19)
    arrow, _, _ = O.joint_attention(q, k, v, None, [ARROW, ARROW], [2, 6], 5, 19)
    assert float((full - arrow).abs().max()) > 1e-3          # the two really differ
    out, _ = R.joint_attention(q, k, v, None, full - arrow, [RES, RES], [2, 6], 5, 19)
    assert float((out - full).abs().max()) <= 1e-14


def test_linear_in_the_residual_and_confined_to_its_head_row_and_feature():
    q, k, v, r1, r2 = (rand((2, 3, 18, 4), 70 + t) for t in range(5))
    hp, win = [RES, ARROW, RES], [2, 2, 5]
    a, _ = R.joint_attention(q, k, v, None, r1, hp, win, 3, 15)
    b, _ = R.joint_attention(q, k, v, None, r1 + r2, hp, win, 3, 15)
    d = b - a
    assert float((d[:, 0] - r2[:, 0].double()).abs().max()) <= 1e-6      # (r1 + r2 is formed in fp32)
    assert float((d[:, 2] - r2[:, 2].double()).abs().max()) <= 1e-6
    assert torch.equal(a[:, 1], b[:, 1])                                   # an ARROW head never reads it
    # one element of the residual moves exactly that element of the output
    r3 = r1.clone()
    r3[1, 2, 7, 3] += 1.0
    c, _ = R.joint_attention(q, k, v, None, r3, hp, win, 3, 15)
    diff = (c - a).abs()
    assert abs(float(diff[1, 2, 7, 3]) - 1.0) <= 1e-6
    diff[1, 2, 7, 3] = 0
    assert float(diff.max()) == 0.0


def test_window_covering_the_image_is_full_attention_plus_residual():
    q, k, v, r = (rand((1, 1, 15, 4), 80 + t) for t in range(4))
    out, _ = R.joint_attention(q, k, v, None, r, [RES], [11], 3, 12)
    full, _, _ = O.joint_attention(q, k, v, None, [FULL], [0], 3, 12)
    assert float((out - (full + r.double())).abs().max()) <= 1e-15


def test_row_subset_and_cached_heads_pass_through():
    q, k, v, r, cache = (rand((1, 3, 16, 4), 90 + t, torch.bfloat16) for t in range(5))
    hp, win = [RES, CACHE, FULL], [3, 0, 0]
    rows = [0, 5, 15]
    sub, raw = R.joint_attention(q, k, v, cache, r, hp, win, 4, 12, rows=rows)
    allr, _ = R.joint_attention(q, k, v, cache, r, hp, win, 4, 12)
    assert torch.equal(sub, allr[:, :, rows])
    assert torch.equal(raw[:, 1].view(torch.int16), cache[:, 1][:, rows].contiguous().view(torch.int16))


def test_residual_store_hand_rounded_values():
    rows = [tuple(float(x) for x in line.split()) for line in open(GOLDEN) if line.strip() and not line.startswith("#")]
    assert len(rows) >= 6
    full = torch.tensor([r[0] for r in rows], dtype=torch.bfloat16)
    arrow = torch.tensor([r[1] for r in rows], dtype=torch.bfloat16)
    want = torch.tensor([r[2] for r in rows], dtype=torch.float32)
    assert torch.equal(full.float(), torch.tensor([r[0] for r in rows])), "fixture values must be exact in bfloat16"
    assert torch.equal(arrow.float(), torch.tensor([r[1] for r in rows]))
    got = R.residual_store(full, arrow)
    assert got.dtype == torch.bfloat16 and torch.equal(got.float(), want)


def test_residual_store_then_add_returns_the_full_output_to_within_one_rounding():
    full, arrow = rand((1, 2, 9, 8), 101, torch.bfloat16), rand((1, 2, 9, 8), 102, torch.bfloat16)
    r = R.residual_store(full, arrow)
    back = arrow.double() + r.double()
    # r was rounded to 8 significant bits: the sum misses `full` by at most half a step of r (2^-8 |r| at most)
    assert bool(((back - full.double()).abs() <= 2.0 ** -8 * (full.double() - arrow.double()).abs() + 1e-30).all())
    assert R.residual_store(full.float(), arrow.float()).dtype == torch.float32
