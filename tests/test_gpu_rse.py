"""difa_head_rse (influence metric, Sec. 3.4.1) through the C ABI against oracle/rse_oracle.py."""
import numpy as np
import pytest
import torch

pytestmark = pytest.mark.gpu

REL_TOL = 1e-5   # fp32 inside one 16-byte vector, fp64 across vectors (include/difa.h)


def make(B, H, N, D, dtype, seed, err=0.3, offset=0.0):
    g = torch.Generator().manual_seed(seed)
    yo = (torch.randn(B, H, N, D, generator=g) * (1.0 + 0.5 * torch.arange(H).view(1, H, 1, 1)) + offset).to(dtype)
    ym = (yo.float() + err * torch.randn(B, H, N, D, generator=g) * (torch.arange(H).view(1, H, 1, 1) % 3)).to(dtype)
    return ym, yo


def run_gpu(ym, yo, layout="bhnd", max_tokens=None, stream=None, plan=None):
    from paper_2503_22796_amd import binding as B
    dev = torch.device("cuda:0")
    Bn, H, N, D = yo.shape
    dt = B.DIFA_DTYPE_BF16 if yo.dtype == torch.bfloat16 else B.DIFA_DTYPE_F32
    lay = B.DIFA_LAYOUT_BHND if layout == "bhnd" else B.DIFA_LAYOUT_BNHD
    put = (lambda t: t.to(dev).transpose(1, 2).contiguous()) if layout == "bnhd" else (lambda t: t.to(dev).contiguous())
    ymd, yod = put(ym), put(yo)
    out = torch.full((H,), float("nan"), dtype=torch.float32, device=dev)
    own = plan is None
    if own:
        plan = B.difa_plan_create(Bn, H, D, dtype=dt, layout=lay, max_tokens=max_tokens or N)
    try:
        B.difa_head_rse(plan, ymd, yod, N, out, stream=stream)
        torch.cuda.synchronize()
    finally:
        if own:
            B.difa_plan_destroy(plan)
    return out.cpu().double().numpy()


def check(ym, yo, **kw):
    from oracle import rse_oracle as R
    got = run_gpu(ym, yo, **kw)
    want = R.head_rse(ym, yo)
    for h in range(len(want)):
        if want[h] == 0.0:
            assert got[h] == 0.0, (h, got[h])
        else:
            # the result is stored as fp32: half an ulp on top of the arithmetic's bound
            assert abs(got[h] - want[h]) <= (REL_TOL + 6e-8) * want[h], (h, got[h], want[h])
    return got, want


@pytest.mark.parametrize("layout", ["bhnd", "bnhd"])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
@pytest.mark.parametrize("shape", [(1, 4, 80, 64), (2, 3, 1000, 64), (1, 5, 2500, 128), (2, 2, 1, 128), (1, 1, 63, 64)])
def test_matches_the_oracle(shape, dtype, layout):
    ym, yo = make(*shape, dtype, seed=sum(shape))
    if shape[2] == 1 and dtype == torch.bfloat16:
        yo[..., 0] += 1.0          # one token: make sure the head is not constant
    check(ym, yo, layout=layout)


def test_perfect_method_is_exactly_zero_and_heads_do_not_mix():
    ym, yo = make(1, 6, 700, 128, torch.bfloat16, seed=5)
    ym[:, 0] = yo[:, 0]
    ym[:, 3] = yo[:, 3]
    got, want = check(ym, yo)
    assert got[0] == 0.0 and got[3] == 0.0 and got[1] > 0.0


def test_common_offset_costs_no_digits():
    ym, yo = make(2, 3, 900, 64, torch.float32, seed=6, offset=1000.0)
    check(ym, yo)


def test_fewer_tokens_than_the_plan_allows_and_two_calls_on_two_streams():
    from paper_2503_22796_amd import binding as B
    from oracle import rse_oracle as R
    dev = torch.device("cuda:0")
    plan = B.difa_plan_create(1, 4, 128, max_tokens=4096)
    try:
        s1, s2 = torch.cuda.Stream(dev), torch.cuda.Stream(dev)
        a_m, a_o = make(1, 4, 4096, 128, torch.bfloat16, seed=7)
        b_m, b_o = make(1, 4, 333, 128, torch.bfloat16, seed=8)
        amd, aod, bmd, bod = (t.to(dev) for t in (a_m, a_o, b_m, b_o))
        out_a = torch.empty(4, dtype=torch.float32, device=dev)
        out_b = torch.empty(4, dtype=torch.float32, device=dev)
        torch.cuda.synchronize()
        B.difa_head_rse(plan, amd, aod, 4096, out_a, stream=s1.cuda_stream)
        B.difa_head_rse(plan, bmd, bod, 333, out_b, stream=s2.cuda_stream)
        torch.cuda.synchronize()
        for got, (m, o) in ((out_a, (a_m, a_o)), (out_b, (b_m, b_o))):
            want = R.head_rse(m, o)
            np.testing.assert_allclose(got.cpu().double().numpy()[1:], want[1:], rtol=REL_TOL + 6e-8)
    finally:
        B.difa_plan_destroy(plan)


def test_full_size_flux_2k_layer():
    ym, yo = make(1, 24, 16896, 128, torch.bfloat16, seed=9)
    check(ym, yo)


def test_rejects_bad_arguments():
    from paper_2503_22796_amd import binding as B
    dev = torch.device("cuda:0")
    plan = B.difa_plan_create(1, 2, 64, max_tokens=64)
    try:
        y = torch.zeros(1, 2, 64, 64, dtype=torch.bfloat16, device=dev)
        out = torch.zeros(2, dtype=torch.float32, device=dev)
        with pytest.raises(B.DifaError):
            B.difa_head_rse(plan, y, y, 65, out)
        with pytest.raises(B.DifaError):
            B.difa_head_rse(plan, y, y, 0, out)
        assert B.lib.difa_head_rse(plan, None, None, 8, None, None) == B.DIFA_ERR_INVALID_ARG
    finally:
        B.difa_plan_destroy(plan)


def test_influence_matrix_of_one_layer_follows_the_oracle_pipeline():
    """Alg. 1 up to the solver: every method applied to every head, RSE against full attention."""
    from paper_2503_22796_amd import binding as B
    from paper_2503_22796_amd import calibrate as C
    from paper_2503_22796_amd import workloads as W
    from oracle import difa_oracle as O
    from oracle import rse_oracle as R
    wl = W.Workload("calib", 1, 4, 64, 48, 1024, np.zeros(4, np.int32), np.zeros(4, np.int32), seed=21)
    q, k, v = W.make_qkv(wl)
    prev = W.make_cache(wl)
    methods = [("arrow", 32), ("arrow", 128), ("arrow", 512), ("cache",)]
    dev = torch.device("cuda:0")
    plan = B.difa_plan_create(wl.B, wl.H, wl.D, max_tokens=wl.N)
    try:
        infl, o_ref = C.influence_matrix(plan, wl.H, q.to(dev), k.to(dev), v.to(dev), wl.n_text, wl.n_img,
                                         methods, prev_out=prev.to(dev))
        torch.cuda.synchronize()
    finally:
        B.difa_plan_destroy(plan)
    infl = infl.cpu().double().numpy()
    assert infl.shape == (wl.H, len(methods))
    full = np.zeros(wl.H, np.int32)
    ref_full, _, _ = O.joint_attention(q, k, v, None, full, np.zeros(wl.H, np.int32), wl.n_text, wl.n_img)
    for j, m in enumerate(methods):
        if m[0] == "arrow":
            ref_m, _, _ = O.joint_attention(q, k, v, None, np.full(wl.H, 1, np.int32), np.full(wl.H, m[1], np.int32),
                                            wl.n_text, wl.n_img)
        else:
            ref_m = prev.double()
        want = R.head_rse(ref_m, ref_full)
        # the GPU's outputs are rounded to bf16 (2^-9 relative) before the metric sees them: that adds a
        # noise floor of about 1e-5 to every entry and moves large entries by well under a percent
        assert np.all(np.abs(infl[:, j] - want) <= 1e-4 + 0.02 * want), (m, infl[:, j], want)
    # wider windows lose less
    assert np.all(infl[:, 0] >= infl[:, 1]) and np.all(infl[:, 1] >= infl[:, 2])
