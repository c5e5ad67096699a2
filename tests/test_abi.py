"""The C-ABI library: it loads, exports every declared symbol, and rejects bad arguments.

No compute call is made here (no GPU in this tier)."""
import ctypes
import os
import re

import numpy as np
import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_symbols():
    text = open(os.path.join(ROOT, "include", "difa.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(difa_[a-z_]+)\s*\(", text)))


def test_header_declares_the_three_calls():
    syms = declared_symbols()
    for name in ("difa_plan_create", "difa_joint_attention", "difa_plan_destroy"):
        assert name in syms


def test_library_exports_every_declared_symbol():
    from paper_2503_22796_amd import binding as B
    for name in declared_symbols():
        assert hasattr(B.lib, name), f"{name} is declared in include/difa.h but not exported"


def test_binding_has_the_same_names():
    from paper_2503_22796_amd import binding as B
    for name in declared_symbols():
        assert hasattr(B, name), f"binding lacks {name}"


def test_status_strings():
    from paper_2503_22796_amd import binding as B
    assert B.difa_status_string(B.DIFA_OK) == "ok"
    assert "invalid" in B.difa_status_string(B.DIFA_ERR_INVALID_ARG)
    assert B.difa_status_string(99) == "unknown status"


def test_destroy_null_is_ok_and_create_rejects_bad_descriptors():
    from paper_2503_22796_amd import binding as B
    assert B.lib.difa_plan_destroy(None) == B.DIFA_OK
    plan = ctypes.c_void_p(123)
    assert B.lib.difa_plan_create(None, ctypes.byref(plan)) == B.DIFA_ERR_INVALID_ARG
    assert plan.value is None
    for kw, status in ((dict(batch=0), B.DIFA_ERR_INVALID_ARG), (dict(heads=0), B.DIFA_ERR_INVALID_ARG),
                       (dict(max_tokens=0), B.DIFA_ERR_INVALID_ARG), (dict(flags=4), B.DIFA_ERR_INVALID_ARG),
                       (dict(flags=1, dtype=1), B.DIFA_ERR_UNSUPPORTED),
                       (dict(softmax_scale=-1.0), B.DIFA_ERR_INVALID_ARG),
                       (dict(head_dim=96), B.DIFA_ERR_UNSUPPORTED), (dict(dtype=7), B.DIFA_ERR_UNSUPPORTED),
                       (dict(layout=5), B.DIFA_ERR_UNSUPPORTED)):
        args = dict(batch=1, heads=2, head_dim=64, max_tokens=16)
        args.update(kw)
        with pytest.raises(B.DifaError) as ei:
            B.difa_plan_create(**args)
        assert ei.value.status == status
        assert B.difa_last_error(None) != ""


def test_joint_attention_with_null_plan_is_an_error_not_a_crash():
    from paper_2503_22796_amd import binding as B
    hp = np.zeros(2, dtype=np.int32)
    st = B.lib.difa_joint_attention(None, None, None, None, None, None, hp.ctypes.data, 1, 1, None, None)
    assert st == B.DIFA_ERR_INVALID_ARG


def test_mfma_rate_probe_rejects_bad_arguments_before_touching_the_gpu():
    from paper_2503_22796_amd import binding as B
    t = ctypes.c_double(0)
    fake = ctypes.c_void_p(4096)
    call = B.lib.difa_probe_mfma_rate
    assert call(None, 1024, 1, 10, fake, None, ctypes.byref(t), None) == B.DIFA_ERR_INVALID_ARG      # no data
    assert call(fake, 1024, 3, 10, fake, None, ctypes.byref(t), None) == B.DIFA_ERR_INVALID_ARG      # 3 wavefronts per SIMD
    assert call(fake, 1024, 1, 0, fake, None, ctypes.byref(t), None) == B.DIFA_ERR_INVALID_ARG       # no rounds
    assert call(fake, 4, 1, 10, fake, None, ctypes.byref(t), None) == B.DIFA_ERR_INVALID_ARG         # fewer than 8 values
    assert call(ctypes.c_void_p(4100), 1024, 1, 10, fake, None, ctypes.byref(t), None) == B.DIFA_ERR_INVALID_ARG   # unaligned
    assert call(fake, 1024, 1, 10, fake, None, None, None) == B.DIFA_ERR_INVALID_ARG                 # nowhere to put the result


def test_head_rse_with_null_plan_is_an_error_not_a_crash():
    from paper_2503_22796_amd import binding as B
    assert B.lib.difa_head_rse(None, None, None, 1, None, None) == B.DIFA_ERR_INVALID_ARG
    assert B.lib.difa_plan_timing_read_head_rse(None, None, None, 0) == B.DIFA_ERR_INVALID_ARG
    assert B.lib.difa_plan_die_speeds(None, None, 0, None, None, None) == B.DIFA_ERR_INVALID_ARG


def test_product_package_does_not_import_the_oracle():
    pkg = os.path.join(ROOT, "paper_2503_22796_amd")
    for dirpath, _, files in os.walk(pkg):
        for f in files:
            if f.endswith((".py", ".cpp", ".hip", ".h")):
                text = open(os.path.join(dirpath, f)).read()
                assert "oracle" not in text.replace("oracle's callers", ""), f"{f} mentions the oracle"
