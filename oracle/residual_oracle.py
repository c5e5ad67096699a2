"""Arrow attention with residual sharing -- TEST INFRASTRUCTURE, not the product.

DiTFastAttnV2 keeps "arrow attention with residual sharing" as an optional member of its method set
(Sec. 2.4 names the technique of its predecessor, Sec. 4.6.1 and Table 4 evaluate it); the technique
itself is defined in the predecessor's paper, not in this one.  The reading implemented here:

  * At a refresh step a head runs both full attention and arrow attention with its window, and the
    difference of the two outputs, as they were emitted, is kept:
        r = O_full - O_arrow                         (rounded once, to the tensors' element type).
  * At the following steps the head runs arrow attention only and adds the kept difference:
        O = ArrowAttention(Q, K, V; w) + r           (the sum taken before the result is rounded).
    The difference stands in for what the discarded image-image pairs would have contributed, which
    changes slowly from one denoising step to the next.

The arrow attention inside is the dense fp64 oracle of the operator (difa_oracle.joint_attention, pinned
on its own); this module adds exactly the two statements above.  Pinned by algebra and brute force
(tests/test_residual_oracle_pins.py); the paper prints no value of it.  Nothing in the product path may
import this module.
"""
import numpy as np
import torch

from . import difa_oracle as O

FULL, ARROW, CACHE, ARROW_RESIDUAL = 0, 1, 2, 3


def residual_store(o_full, o_arrow):
    """r = O_full - O_arrow, exact in fp64, rounded once (to nearest, ties to even) to the inputs' element type."""
    assert o_full.shape == o_arrow.shape and o_full.dtype == o_arrow.dtype
    return (o_full.double() - o_arrow.double()).to(o_full.dtype)


def joint_attention(q, k, v, cache, residual, head_plan, window, n_text, n_img, scale=None, rows=None,
                    block=None, image_first=False):
    """The head-wise operator with a fourth head mode, ARROW_RESIDUAL: arrow attention plus the head's kept
    difference.  `residual`: [B, H, N, D], any floating type (widened exactly to fp64), read only for
    ARROW_RESIDUAL heads.  Returns (out fp64 [B, H, R, D], raw cached rows) like the operator's oracle."""
    hp = np.asarray(head_plan, dtype=np.int32)
    as_arrow = np.where(hp == ARROW_RESIDUAL, ARROW, hp).astype(np.int32)
    out, raw, _ = O.joint_attention(q, k, v, cache, as_arrow, window, n_text, n_img, scale=scale, rows=rows,
                                    block=block, image_first=image_first)
    idx = list(range(q.shape[2])) if rows is None else [int(r) for r in rows]
    for h in np.nonzero(hp == ARROW_RESIDUAL)[0]:
        assert residual is not None and residual.shape == q.shape
        out[:, h] = out[:, h] + residual[:, h][:, idx].double()
    return out, raw
