"""ctypes binding of libdifa.so: argument marshalling only, same names as include/difa.h.

PyTorch is used for device memory and streams; every step of the operator runs in the HIP
library.  There is no fallback: if the library is missing, importing this module fails.
"""
import ctypes
import os

import numpy as np

HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DIFA_LIBRARY", os.path.join(HERE, "libdifa.so"))   # override: another build of the same ABI

DIFA_OK, DIFA_ERR_INVALID_ARG, DIFA_ERR_UNSUPPORTED, DIFA_ERR_ALLOC, DIFA_ERR_HIP = range(5)
DIFA_HEAD_FULL, DIFA_HEAD_ARROW, DIFA_HEAD_CACHE, DIFA_HEAD_ARROW_RESIDUAL = 0, 1, 2, 3
DIFA_ITEM_ADD_RESIDUAL = 1
DIFA_DTYPE_BF16, DIFA_DTYPE_F32 = 0, 1
DIFA_LAYOUT_BHND, DIFA_LAYOUT_BNHD = 0, 1
DIFA_FLAG_BLOCK_BAND = 1
DIFA_FLAG_IMAGE_FIRST = 2


class difa_plan_desc_t(ctypes.Structure):
    _fields_ = [("batch", ctypes.c_int32), ("heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
                ("dtype", ctypes.c_int32), ("layout", ctypes.c_int32), ("max_tokens", ctypes.c_int32),
                ("softmax_scale", ctypes.c_float), ("device", ctypes.c_int32), ("flags", ctypes.c_uint32)]


class difa_work_item_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("bh", "q_tile", "kv0_end", "nm0_end", "kv1_begin", "kv1_end", "nm1_begin", "nm1_end",
                 "window", "n_tiles", "flags")]


class difa_segment_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in
                ("bh", "q_tile", "kv0_end", "nm0_end", "kv1_begin", "kv1_end", "nm1_begin", "nm1_end",
                 "window", "pos_begin", "pos_end", "part_slot", "merge_idx", "n_parts", "first_slot", "flags")]


class difa_merge_item_t(ctypes.Structure):
    _fields_ = [(n, ctypes.c_int32) for n in ("bh", "q_tile", "first_slot", "n_parts")]


def _load():
    if not os.path.exists(LIB_PATH):
        raise ImportError(f"{LIB_PATH} is missing: build it with `python -m paper_2503_22796_amd.build` "
                          "(there is no fallback path)")
    L = ctypes.CDLL(LIB_PATH)
    vp, i32, i32p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int32)
    L.difa_plan_create.restype = ctypes.c_int
    L.difa_plan_create.argtypes = [ctypes.POINTER(difa_plan_desc_t), ctypes.POINTER(vp)]
    L.difa_joint_attention.restype = ctypes.c_int
    L.difa_joint_attention.argtypes = [vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
    L.difa_joint_attention_static.restype = ctypes.c_int
    L.difa_joint_attention_static.argtypes = L.difa_joint_attention.argtypes
    L.difa_joint_attention_residual.restype = ctypes.c_int
    L.difa_joint_attention_residual.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i32, i32, vp, vp]
    L.difa_residual_store.restype = ctypes.c_int
    L.difa_residual_store.argtypes = [vp, vp, vp, vp, i32, vp]
    L.difa_plan_destroy.restype = ctypes.c_int
    L.difa_plan_destroy.argtypes = [vp]
    L.difa_status_string.restype = ctypes.c_char_p
    L.difa_status_string.argtypes = [ctypes.c_int]
    L.difa_last_error.restype = ctypes.c_char_p
    L.difa_last_error.argtypes = [vp]
    L.difa_tile_shape.restype = i32
    L.difa_tile_shape.argtypes = [i32, i32, i32p, i32p]
    L.difa_worklist_build.restype = ctypes.c_int
    L.difa_worklist_build.argtypes = [i32, i32, vp, vp, i32, i32, i32, i32, i32, ctypes.c_uint32, vp, i32, i32p, vp, i32p]
    L.difa_schedule_build.restype = ctypes.c_int
    L.difa_schedule_build.argtypes = [vp, i32, i32, i32, vp, i32, vp, i32p, vp, i32, i32p, i32p]
    L.difa_plan_timing_enable.restype = ctypes.c_int
    L.difa_plan_timing_enable.argtypes = [vp, i32]
    L.difa_plan_timing_read.restype = ctypes.c_int
    L.difa_plan_timing_read.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double),
                                        ctypes.POINTER(ctypes.c_int64), i32]
    L.difa_plan_solve.restype = ctypes.c_int
    L.difa_plan_solve.argtypes = [vp, vp, ctypes.c_double, i32, i32, ctypes.c_double, ctypes.c_double, vp,
                                  ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_double)]
    L.difa_head_rse.restype = ctypes.c_int
    L.difa_head_rse.argtypes = [vp, vp, vp, i32, vp, vp]
    L.difa_plan_die_speeds.restype = ctypes.c_int
    L.difa_plan_die_speeds.argtypes = [vp, ctypes.POINTER(ctypes.c_double), i32, i32p, i32p, i32p]
    L.difa_plan_timing_read_head_rse.restype = ctypes.c_int
    L.difa_plan_timing_read_head_rse.argtypes = [vp, ctypes.POINTER(ctypes.c_double), ctypes.POINTER(ctypes.c_int64), i32]
    L.difa_device_info.restype = ctypes.c_int
    L.difa_device_info.argtypes = [i32, i32p, i32p, i32p, i32p, ctypes.c_char_p, i32]
    L.difa_probe_mfma_rate.restype = ctypes.c_int
    L.difa_probe_mfma_rate.argtypes = [vp, ctypes.c_int64, i32, i32, vp, vp, ctypes.POINTER(ctypes.c_double),
                                       ctypes.POINTER(ctypes.c_double)]
    return L


lib = _load()


class DifaError(RuntimeError):
    def __init__(self, status, text):
        super().__init__(f"difa status {status} ({lib.difa_status_string(status).decode()}): {text}")
        self.status = status


def difa_status_string(status: int) -> str:
    return lib.difa_status_string(int(status)).decode()


def difa_last_error(plan=None) -> str:
    return lib.difa_last_error(plan).decode()


def difa_tile_shape(head_dim: int, dtype: int = DIFA_DTYPE_BF16):
    bm, bn = ctypes.c_int32(0), ctypes.c_int32(0)
    if lib.difa_tile_shape(head_dim, dtype, ctypes.byref(bm), ctypes.byref(bn)) != 0:
        raise DifaError(DIFA_ERR_UNSUPPORTED, "difa_tile_shape: unsupported head_dim/dtype")
    return bm.value, bn.value


def _i32(a):
    return None if a is None else np.ascontiguousarray(np.asarray(a, dtype=np.int32))


def difa_worklist_build(batch, heads, head_plan, window, n_text, n_img, bm, bn, n_xcd=1, flags=0):
    """Returns (status, items as a numpy structured array, CACHE-head indices)."""
    hp, win = _i32(head_plan), _i32(window)
    n_items, n_copy = ctypes.c_int32(0), ctypes.c_int32(0)
    copy_heads = np.zeros(max(int(heads), 1), dtype=np.int32)
    st = lib.difa_worklist_build(batch, heads, hp.ctypes.data if hp is not None else None,
                                 win.ctypes.data if win is not None else None, n_text, n_img, bm, bn, n_xcd,
                                 flags, None, 0, ctypes.byref(n_items), None, ctypes.byref(n_copy))
    if st != DIFA_OK:
        return st, None, None
    items = (difa_work_item_t * max(n_items.value, 1))()
    st = lib.difa_worklist_build(batch, heads, hp.ctypes.data, win.ctypes.data if win is not None else None,
                                 n_text, n_img, bm, bn, n_xcd, flags, ctypes.cast(items, ctypes.c_void_p), n_items.value,
                                 ctypes.byref(n_items), copy_heads.ctypes.data, ctypes.byref(n_copy))
    arr = np.frombuffer(items, dtype=np.dtype([(n, np.int32) for n, _ in difa_work_item_t._fields_]),
                        count=n_items.value).copy()
    return st, arr, copy_heads[:n_copy.value].copy()


def difa_schedule_build(items, n_wg, n_xcd):
    """items: structured array as difa_worklist_build returns.  Returns (status, segments, wg_begin,
    merge items, number of scratch slots); the arrays are numpy structured / int32 arrays."""
    items = np.ascontiguousarray(items)
    n = len(items)
    seg_cap, merge_cap = n + 2 * n_wg, 2 * n_wg
    segs = (difa_segment_t * max(seg_cap, 1))()
    merges = (difa_merge_item_t * max(merge_cap, 1))()
    wg_begin = np.zeros(n_wg + 1, dtype=np.int32)
    n_segs, n_merges, n_slots = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib.difa_schedule_build(items.ctypes.data if n else None, n, n_wg, n_xcd, ctypes.cast(segs, ctypes.c_void_p),
                                 seg_cap, wg_begin.ctypes.data, ctypes.byref(n_segs),
                                 ctypes.cast(merges, ctypes.c_void_p), merge_cap, ctypes.byref(n_merges),
                                 ctypes.byref(n_slots))
    if st != DIFA_OK:
        return st, None, None, None, 0
    sa = np.frombuffer(segs, dtype=np.dtype([(n_, np.int32) for n_, _ in difa_segment_t._fields_]),
                       count=n_segs.value).copy()
    ma = np.frombuffer(merges, dtype=np.dtype([(n_, np.int32) for n_, _ in difa_merge_item_t._fields_]),
                       count=n_merges.value).copy()
    return st, sa, wg_begin, ma, n_slots.value


def difa_plan_create(batch, heads, head_dim, dtype=DIFA_DTYPE_BF16, layout=DIFA_LAYOUT_BHND,
                     max_tokens=1, softmax_scale=0.0, device=0, flags=0):
    desc = difa_plan_desc_t(batch, heads, head_dim, dtype, layout, max_tokens, softmax_scale, device, flags)
    plan = ctypes.c_void_p()
    st = lib.difa_plan_create(ctypes.byref(desc), ctypes.byref(plan))
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(None))
    return plan


def difa_plan_destroy(plan):
    st = lib.difa_plan_destroy(plan)
    if st != DIFA_OK:
        raise DifaError(st, "difa_plan_destroy")


def _ptr(t):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def difa_joint_attention_static(plan, q, k, v, out, cache, head_plan, n_text, n_img, window, stream=None):
    """difa_joint_attention with the library's file-scope device array as scratch (no allocation anywhere)."""
    return difa_joint_attention(plan, q, k, v, out, cache, head_plan, n_text, n_img, window, stream=stream,
                                _entry=lib.difa_joint_attention_static)


def difa_joint_attention(plan, q, k, v, out, cache, head_plan, n_text, n_img, window, stream=None, _entry=None):
    """q, k, v, out, cache: torch tensors on the plan's device (cache may be None).

    `stream`: a torch.cuda.Stream, a raw hipStream_t integer, or None for torch's current stream.
    """
    import torch
    hp, win = _i32(head_plan), _i32(window)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    st = (_entry or lib.difa_joint_attention)(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(cache),
                                  hp.ctypes.data if hp is not None else None, int(n_text), int(n_img),
                                  win.ctypes.data if win is not None else None, ctypes.c_void_p(stream))
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(plan))


def difa_joint_attention_residual(plan, q, k, v, out, cache, residual, head_plan, n_text, n_img, window, stream=None):
    """difa_joint_attention with the kept differences of the DIFA_HEAD_ARROW_RESIDUAL heads (`residual`, may be None)."""
    import torch
    hp, win = _i32(head_plan), _i32(window)
    if stream is None:
        stream = torch.cuda.current_stream(q.device).cuda_stream
    elif hasattr(stream, "cuda_stream"):
        stream = stream.cuda_stream
    st = lib.difa_joint_attention_residual(plan, _ptr(q), _ptr(k), _ptr(v), _ptr(out), _ptr(cache), _ptr(residual),
                                           hp.ctypes.data if hp is not None else None, int(n_text), int(n_img),
                                           win.ctypes.data if win is not None else None, ctypes.c_void_p(stream))
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(plan))


def difa_residual_store(plan, o_full, o_arrow, residual, n_tokens, stream=None):
    """residual = o_full - o_arrow, element by element (device tensors of the plan's shape and dtype), asynchronous."""
    import torch
    s = stream if stream is not None else torch.cuda.current_stream(o_full.device).cuda_stream
    st = lib.difa_residual_store(plan, _ptr(o_full), _ptr(o_arrow), _ptr(residual), int(n_tokens), ctypes.c_void_p(s))
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(plan))


def difa_plan_timing_enable(plan, enable=True):
    st = lib.difa_plan_timing_enable(plan, 1 if enable else 0)
    if st != DIFA_OK:
        raise DifaError(st, "difa_plan_timing_enable")


def difa_plan_timing_read(plan, reset=True):
    """Returns (attention kernel ms, copy kernel ms, attention launches) accumulated so far."""
    a, c, n = ctypes.c_double(0), ctypes.c_double(0), ctypes.c_int64(0)
    st = lib.difa_plan_timing_read(plan, ctypes.byref(a), ctypes.byref(c), ctypes.byref(n), 1 if reset else 0)
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(plan))
    return a.value, c.value, n.value


def difa_device_info(device=0):
    """What the runtime reports for the device: a dict with compute_units, clock_khz, memory_clock_khz, l2_bytes, arch."""
    cu, clk, mclk, l2 = (ctypes.c_int32(0) for _ in range(4))
    arch = ctypes.create_string_buffer(64)
    st = lib.difa_device_info(int(device), ctypes.byref(cu), ctypes.byref(clk), ctypes.byref(mclk), ctypes.byref(l2),
                              arch, 64)
    if st != DIFA_OK:
        raise DifaError(st, "difa_device_info")
    return {"compute_units": cu.value, "clock_khz": clk.value, "memory_clock_khz": mclk.value, "l2_bytes": l2.value,
            "arch": arch.value.decode()}


def difa_probe_mfma_rate(data, waves_per_simd=1, rounds=50000, stream=None):
    """Sustained dense bf16 MFMA rate on the operand bits of `data` (a bf16 device tensor).
    Returns (TFLOP/s, milliseconds)."""
    import torch
    assert data.is_cuda and data.dtype == torch.bfloat16 and data.is_contiguous()
    scratch = torch.zeros(1, dtype=torch.float32, device=data.device)
    t, ms = ctypes.c_double(0), ctypes.c_double(0)
    s = stream if stream is not None else torch.cuda.current_stream(data.device).cuda_stream
    with torch.cuda.device(data.device):
        st = lib.difa_probe_mfma_rate(ctypes.c_void_p(data.data_ptr()), int(data.numel()), int(waves_per_simd),
                                      int(rounds), ctypes.c_void_p(scratch.data_ptr()), ctypes.c_void_p(s),
                                      ctypes.byref(t), ctypes.byref(ms))
    if st != DIFA_OK:
        raise DifaError(st, "difa_probe_mfma_rate")
    return t.value, ms.value


def difa_head_rse(plan, y_m, y_o, n_tokens, rse_out, stream=None):
    """rse_out[h] = sum (y_m - y_o)^2 / sum (y_o - mean y_o)^2 per head; device tensors, asynchronous."""
    import torch
    s = stream if stream is not None else torch.cuda.current_stream(y_m.device).cuda_stream
    st = lib.difa_head_rse(plan, ctypes.c_void_p(y_m.data_ptr()), ctypes.c_void_p(y_o.data_ptr()), int(n_tokens),
                           ctypes.c_void_p(rse_out.data_ptr()), ctypes.c_void_p(s))
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(plan))


def difa_plan_die_speeds(plan):
    """(relative die speeds, launches averaged, schedules made again)"""
    sp = (ctypes.c_double * 16)()
    n, samples, retunes = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    st = lib.difa_plan_die_speeds(plan, sp, 16, ctypes.byref(n), ctypes.byref(samples), ctypes.byref(retunes))
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(plan))
    return [float(sp[i]) for i in range(n.value)], samples.value, retunes.value


def difa_plan_timing_read_head_rse(plan, reset=True):
    """Returns (milliseconds, calls) of difa_head_rse accumulated while timing was enabled."""
    a, n = ctypes.c_double(0), ctypes.c_int64(0)
    st = lib.difa_plan_timing_read_head_rse(plan, ctypes.byref(a), ctypes.byref(n), 1 if reset else 0)
    if st != DIFA_OK:
        raise DifaError(st, difa_last_error(plan))
    return a.value, n.value


def difa_plan_solve(influence, latency, latency_full, delta, c):
    """Eq. 2 for one layer.  influence [H, M], latency [M] (host).  Returns (status, choice [H] with -1 = full
    attention, total latency, total influence)."""
    infl = np.ascontiguousarray(influence, dtype=np.float64)
    lat = np.ascontiguousarray(latency, dtype=np.float64)
    H, M = infl.shape
    assert lat.shape == (M,)
    choice = np.full(H, -2, dtype=np.int32)
    tl, ti = ctypes.c_double(0), ctypes.c_double(0)
    st = lib.difa_plan_solve(infl.ctypes.data, lat.ctypes.data, float(latency_full), H, M, float(delta), float(c),
                             choice.ctypes.data, ctypes.byref(tl), ctypes.byref(ti))
    return st, choice, tl.value, ti.value
