"""FLOP and byte accounting for a head-wise plan (used by the benchmark's report only).

"Computed" work is what the method itself has to do: 4*D FLOPs (two contractions, multiply and
add) per allowed (query, key) pair of a full or arrow head, nothing for a cached head.
"Dense-equivalent" is the work of running every head as full attention.
"""
import numpy as np

FULL, ARROW, CACHE = 0, 1, 2


def allowed_pairs(mode: int, w: int, n_text: int, n_img: int) -> int:
    """Allowed (query, key) pairs of one head (Sec. 3.1: text quadrants whole, image band |i-j|<=w)."""
    N = n_text + n_img
    if mode == CACHE:
        return 0
    if mode == FULL or w >= n_img - 1:
        return N * N
    band = n_img * (2 * w + 1) - w * (w + 1)          # band rows clipped at both ends of the image
    return n_text * N + n_img * n_text + band


def plan_flops(head_plan, window, n_text, n_img, D, batch=1):
    N = n_text + n_img
    computed = sum(4 * D * allowed_pairs(int(m), int(w), n_text, n_img) for m, w in zip(head_plan, window))
    dense = 4 * D * N * N * len(head_plan)
    return {"computed": batch * computed, "dense": batch * dense,
            "reduction": 1.0 - computed / dense}


def plan_bytes(head_plan, n_text, n_img, D, elem=2, batch=1):
    """Compulsory HBM bytes: Q,K,V read + O written per computed head; read + write per cached head."""
    N = n_text + n_img
    hp = np.asarray(head_plan)
    n_cache = int((hp == CACHE).sum())
    n_comp = len(hp) - n_cache
    return {"attention": batch * n_comp * 4 * N * D * elem, "cache_copy": batch * n_cache * 2 * N * D * elem}
