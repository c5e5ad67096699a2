"""The plan object learns the relative speeds of the accelerator dies from the run times its workgroups
report, and makes a layer's schedule again when they have moved.  Checked here: the report arrives without
any call waiting for it, the speeds are sane, and a schedule made for other speeds computes the same layer
(against the oracle, and against the output of the first schedule)."""
import pytest
import torch

from paper_2503_22796_amd import workloads as W
from util import boundary_rows, check_against_oracle, same_result_bf16, ARROW

pytestmark = pytest.mark.gpu


def test_die_speeds_are_learnt_and_the_retuned_schedule_computes_the_same_layer():
    from paper_2503_22796_amd import binding as B
    wl = W.flux_2k_mixed()
    dev = torch.device("cuda:0")
    q, k, v = W.make_qkv(wl)
    cache = W.make_cache(wl)
    qd, kd, vd, cd = q.to(dev), k.to(dev), v.to(dev), cache.to(dev)
    plan = B.difa_plan_create(wl.B, wl.H, wl.D, max_tokens=wl.N)
    try:
        speeds, samples, retunes = B.difa_plan_die_speeds(plan)
        n_dies = len(speeds)
        first = torch.empty_like(qd)
        B.difa_joint_attention(plan, qd, kd, vd, first, cd, wl.head_plan, wl.n_text, wl.n_img, wl.window)
        torch.cuda.synchronize()
        out = torch.empty_like(qd)
        seen_retune = retunes
        for _ in range(14):                       # a report is picked up by the call after the launch has ended
            out.fill_(float("nan"))
            B.difa_joint_attention(plan, qd, kd, vd, out, cd, wl.head_plan, wl.n_text, wl.n_img, wl.window)
            torch.cuda.synchronize()
            speeds, samples, retunes = B.difa_plan_die_speeds(plan)
            seen_retune = max(seen_retune, retunes)
        if n_dies > 1:
            assert samples >= 6, "no run-time reports were picked up"
            assert all(0.85 <= s <= 1.15 for s in speeds), speeds
            assert abs(sum(speeds) / n_dies - 1.0) < 0.02, speeds
            assert retunes <= 2
        print(f"dies {n_dies} speeds {[round(s, 3) for s in speeds]} samples {samples} schedules made again {seen_retune}", flush=True)
        # whatever schedule the last call ran on: the same layer
        assert same_result_bf16(out.cpu(), first.cpu())
        rows = boundary_rows(wl.n_text, wl.n_img, wl.window[wl.head_plan == ARROW], extra=48, seed=3)
        check_against_oracle(out.cpu(), q, k, v, cache, wl.head_plan, wl.window, wl.n_text, wl.n_img, rows=rows)
    finally:
        B.difa_plan_destroy(plan)
