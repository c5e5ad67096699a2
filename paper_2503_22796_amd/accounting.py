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


def block_band_pairs(w: int, n_text: int, n_img: int, bm: int, bn: int) -> int:
    """Pairs an arrow head keeps under the block-granular band (Sec. 3.3 / Fig. 4): every pair of a
    bm x bn block that holds at least one pair of the exact pattern, keys past the sequence end excluded."""
    N = n_text + n_img
    if w >= n_img - 1:
        return N * N
    total = 0
    for i0 in range(0, N, bm):
        i1 = min(i0 + bm, N)
        if i0 < n_text:                       # the block holds text rows: they keep every key
            total += (i1 - i0) * N
            continue
        kept = 0
        for j0 in range(0, N, bn):
            j1 = min(j0 + bn, N)
            if j0 < n_text or (max(j0, n_text) <= (i1 - 1) + w and (j1 - 1) >= i0 - w):
                kept += j1 - j0
        total += (i1 - i0) * kept
    return total


def plan_flops(head_plan, window, n_text, n_img, D, batch=1, block=None):
    """block: None for the exact band, (bm, bn) for the block-granular band."""
    N = n_text + n_img
    if block is None:
        computed = sum(4 * D * allowed_pairs(int(m), int(w), n_text, n_img) for m, w in zip(head_plan, window))
    else:
        computed = sum(4 * D * (block_band_pairs(int(w), n_text, n_img, *block) if m == ARROW
                                else allowed_pairs(int(m), int(w), n_text, n_img))
                       for m, w in zip(head_plan, window))
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
