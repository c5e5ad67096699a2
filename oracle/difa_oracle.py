"""ctypes wrapper over oracle/difa_oracle.c -- TEST INFRASTRUCTURE, not the product.

The oracle is the plain dense fp64 statement of the head-wise joint-attention
operator (Sec. 3.1-3.3 and the tail of Alg. 1 of DiTFastAttnV2): per head either
full softmax attention, arrow attention (text quadrants whole, image-image band
|i-j| <= w) or a bit-exact copy of the cached previous-step output.  Nothing in
the product path may import this module.
"""
import ctypes
import os

import numpy as np
import torch

from . import build as _build

FULL, ARROW, CACHE = 0, 1, 2
_DT = {torch.bfloat16: 0, torch.float32: 1}
_lib = None


def lib():
    global _lib
    if _lib is None:
        path = _build.build(force=False)
        L = ctypes.CDLL(path)
        L.difa_oracle_joint_attention.restype = ctypes.c_int
        L.difa_oracle_joint_attention.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.difa_oracle_joint_attention_blocks.restype = ctypes.c_int
        L.difa_oracle_joint_attention_blocks.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.difa_oracle_joint_attention_order.restype = ctypes.c_int
        L.difa_oracle_joint_attention_order.argtypes = [
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p,
            ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int, ctypes.c_double,
            ctypes.c_void_p, ctypes.c_int, ctypes.c_int, ctypes.c_int,
            ctypes.c_void_p, ctypes.c_void_p, ctypes.c_void_p]
        L.difa_oracle_allowed_order.restype = ctypes.c_int
        L.difa_oracle_allowed_order.argtypes = [ctypes.c_int] * 7
        L.difa_oracle_allowed.restype = ctypes.c_int
        L.difa_oracle_allowed.argtypes = [ctypes.c_int] * 5
        L.difa_oracle_threads.restype = ctypes.c_int
        _lib = L
    return _lib


def threads() -> int:
    return int(lib().difa_oracle_threads())


def allowed(mode: int, i: int, j: int, n_text: int, w: int, n_img: int = 0, image_first: bool = False) -> bool:
    """Sec. 3.1: does query i attend to key j for a head in `mode` with half-width w.
    image_first: the text tokens follow the n_img image tokens instead of preceding them."""
    if image_first:
        return bool(lib().difa_oracle_allowed_order(int(mode), int(i), int(j), int(n_text), int(n_img), int(w), 1))
    return bool(lib().difa_oracle_allowed(int(mode), int(i), int(j), int(n_text), int(w)))


def joint_attention(q, k, v, cache, head_plan, window, n_text, n_img, scale=None,
                    rows=None, want_probs=False, block=None, image_first=False):
    """Evaluate the operator on CPU tensors q, k, v (and cache) of shape [B,H,N,D].

    dtype bf16 or fp32; the values are widened exactly to fp64.
    rows: optional 1-D integer sequence of query rows (default: all).
    block: None for the exact band, or (bm, bn) for the block-granular band of Sec. 3.3 / Fig. 4
    (an ARROW head keeps every pair of a bm x bn block that holds a pair of the exact pattern).
    image_first: the joint sequence is [image tokens, text tokens] instead of [text, image].
    Returns (out_f64 [B,H,R,D], out_raw [B,H,R,D] of the input dtype -- meaningful
    on CACHE heads only, elsewhere zero --, probs [B,H,R,N] or None).
    """
    assert q.device.type == "cpu" and q.dtype in _DT
    B, H, N, D = q.shape
    assert N == n_text + n_img
    q, k, v = q.contiguous(), k.contiguous(), v.contiguous()
    assert k.shape == q.shape and v.shape == q.shape and k.dtype == q.dtype and v.dtype == q.dtype
    if cache is not None:
        cache = cache.contiguous()
        assert cache.shape == q.shape and cache.dtype == q.dtype
    hp = np.ascontiguousarray(np.asarray(head_plan, dtype=np.int32))
    win = np.ascontiguousarray(np.asarray(window, dtype=np.int32))
    assert hp.shape == (H,) and win.shape == (H,)
    if scale is None:
        scale = 1.0 / float(D) ** 0.5
    if rows is None:
        rows_arr, R, rows_ptr = None, N, None
    else:
        rows_arr = np.ascontiguousarray(np.asarray(rows, dtype=np.int32))
        R, rows_ptr = int(rows_arr.shape[0]), rows_arr.ctypes.data
    out = np.zeros((B, H, R, D), dtype=np.float64)
    out_raw = torch.zeros((B, H, R, D), dtype=q.dtype)
    probs = np.zeros((B, H, R, N), dtype=np.float64) if want_probs else None
    bm, bn = (0, 0) if block is None else (int(block[0]), int(block[1]))
    rc = lib().difa_oracle_joint_attention_order(
        q.data_ptr(), k.data_ptr(), v.data_ptr(), cache.data_ptr() if cache is not None else None,
        _DT[q.dtype], B, H, D, hp.ctypes.data, win.ctypes.data, int(n_text), int(n_img), 1 if image_first else 0,
        float(scale), rows_ptr, R, bm, bn, out.ctypes.data, out_raw.data_ptr(),
        probs.ctypes.data if probs is not None else None)
    if rc != 0:
        raise ValueError(f"difa_oracle_joint_attention: invalid argument (rc={rc})")
    return torch.from_numpy(out), out_raw, (torch.from_numpy(probs) if probs is not None else None)
