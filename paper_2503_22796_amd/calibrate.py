"""Calibration pass of the plan search for one layer (Alg. 1, the part before the solver; Sec. 3.4.1).

One reference call with every head on full attention, then, per candidate method, one call with
every head on that method and one influence measurement (Eq. 1) of its output against the reference.
Only a loop over C-ABI calls: every attention and every measurement runs in the library's kernels
(difa_joint_attention, difa_head_rse); torch is used for the two output buffers and the result.
"""
import numpy as np
import torch

from . import binding as B

FULL, ARROW, CACHE = B.DIFA_HEAD_FULL, B.DIFA_HEAD_ARROW, B.DIFA_HEAD_CACHE


def influence_matrix(plan, heads, q, k, v, n_text, n_img, methods, prev_out=None, stream=None):
    """Influence[h, m] for one layer.  `plan` was created for q's batch, `heads`, head_dim, dtype and layout.

    methods: sequence of ("arrow", w) and/or ("cache",); the cached method compares the layer's
    previous-step output `prev_out` (same shape as q) with this step's full-attention output.
    Returns (influence [H, M] fp32 device tensor, full-attention output O).  Asynchronous on `stream`
    (default: torch's current stream); the caller synchronises before reading.
    """
    heads = int(heads)
    n_tokens = n_text + n_img
    full = np.full(heads, FULL, dtype=np.int32)
    zero_w = np.zeros(heads, dtype=np.int32)
    o_ref = torch.empty_like(q)
    o_m = torch.empty_like(q)
    infl = torch.empty((len(methods), heads), dtype=torch.float32, device=q.device)
    B.difa_joint_attention(plan, q, k, v, o_ref, None, full, n_text, n_img, zero_w, stream=stream)
    for j, m in enumerate(methods):
        if m[0] == "arrow":
            hp = np.full(heads, ARROW, dtype=np.int32)
            win = np.full(heads, int(m[1]), dtype=np.int32)
            B.difa_joint_attention(plan, q, k, v, o_m, None, hp, n_text, n_img, win, stream=stream)
            B.difa_head_rse(plan, o_m, o_ref, n_tokens, infl[j], stream=stream)
        elif m[0] == "cache":
            if prev_out is None:
                raise ValueError("the cached method needs the layer's previous-step output")
            B.difa_head_rse(plan, prev_out, o_ref, n_tokens, infl[j], stream=stream)
        else:
            raise ValueError(f"unknown method {m!r}")
    return infl.t(), o_ref

