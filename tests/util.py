"""Helpers shared by the GPU parity tests: run the C-ABI library, run the oracle, compare."""
import numpy as np
import torch

FULL, ARROW, CACHE = 0, 1, 2
TOL_BF16 = 2e-2   # max-abs bar for bf16 inputs, fp32 accumulation
TOL_F32 = 1e-5    # max-abs bar for the fp32 debug path


def gpu_joint_attention(q, k, v, cache, head_plan, window, n_text, n_img, scale=0.0, layout="bhnd",
                        poison=True, stream=None, plan=None, alias_out_to_cache=False, flags=0):
    """Run difa_joint_attention on cuda:0.  CPU tensors [B,H,N,D] in, CPU tensor [B,H,N,D] out."""
    from paper_2503_22796_amd import binding as B
    dev = torch.device("cuda:0")
    Bn, H, N, D = q.shape
    dt = B.DIFA_DTYPE_BF16 if q.dtype == torch.bfloat16 else B.DIFA_DTYPE_F32
    lay = B.DIFA_LAYOUT_BHND if layout == "bhnd" else B.DIFA_LAYOUT_BNHD

    def put(t):
        if t is None:
            return None
        t = t.to(dev)
        return t.transpose(1, 2).contiguous() if layout == "bnhd" else t.contiguous()

    qd, kd, vd, cd = put(q), put(k), put(v), put(cache)
    if alias_out_to_cache:
        od = cd
    else:
        od = torch.empty_like(qd)
        if poison:
            od.fill_(float("nan"))
    own = plan is None
    if own:
        plan = B.difa_plan_create(Bn, H, D, dtype=dt, layout=lay, max_tokens=N, softmax_scale=scale, flags=flags)
    try:
        B.difa_joint_attention(plan, qd, kd, vd, od, cd, head_plan, n_text, n_img, window, stream=stream)
        torch.cuda.synchronize()
    finally:
        if own:
            B.difa_plan_destroy(plan)
    o = od.transpose(1, 2) if layout == "bnhd" else od
    return o.contiguous().cpu()


def check_against_oracle(out, q, k, v, cache, head_plan, window, n_text, n_img, scale=None, rows=None,
                         tol=TOL_BF16, block=None, image_first=False):
    """Element-by-element comparison; returns the max abs error over computed heads."""
    from oracle import difa_oracle as O
    ref, ref_raw, _ = O.joint_attention(q, k, v, cache, head_plan, window, n_text, n_img,
                                        scale=scale, rows=rows, block=block, image_first=image_first)
    got = out if rows is None else out[:, :, list(rows)]
    hp = np.asarray(head_plan)
    worst = 0.0
    for h in range(q.shape[1]):
        if hp[h] == CACHE:
            a = got[:, h].contiguous().view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32)
            b = ref_raw[:, h].contiguous().view(torch.int16 if got.dtype == torch.bfloat16 else torch.int32)
            assert torch.equal(a, b), f"cached head {h} is not bit-exact"
        else:
            g = got[:, h].double()
            assert torch.isfinite(g).all(), f"head {h}: non-finite output (unwritten or NaN rows)"
            err = float((g - ref[:, h]).abs().max())
            assert err <= tol, f"head {h} (mode {hp[h]}, w {window[h]}): max abs err {err:.3e} > {tol}"
            worst = max(worst, err)
    return worst


def boundary_rows(n_text, n_img, windows, bm=128, extra=64, seed=0):
    """Rows that sit on every edge the kernel treats specially, plus seeded random rows."""
    N = n_text + n_img
    rows = {0, N - 1, max(n_text - 1, 0), min(n_text, N - 1), min(n_text + 1, N - 1)}
    for w in set(int(x) for x in windows):
        for r in (n_text + w - 1, n_text + w, n_text + w + 1, N - w - 2, N - w - 1, N - w):
            if 0 <= r < N:
                rows.add(r)
    for t in (0, 1, 2, (N // bm) // 2, N // bm - 1, N // bm):
        for r in (t * bm, t * bm + 31, t * bm + 32, t * bm + bm - 1):
            if 0 <= r < N:
                rows.add(r)
    g = np.random.Generator(np.random.PCG64(seed))
    rows.update(int(x) for x in g.integers(0, N, size=extra))
    return sorted(rows)
