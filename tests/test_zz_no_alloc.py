"""difa_joint_attention_static (the entry point for callers that cannot allocate) against
difa_joint_attention: same inputs, same plan object, two calls in a row, the second on a smaller input.

Both go through the C ABI.  The layers are sized so that the schedule cuts records into pieces (that is
what the scratch is for); the second call leaves most of the array holding the first call's contents."""
import numpy as np
import pytest
import torch

from paper_2503_22796_amd import workloads as W
from util import ARROW, CACHE, FULL, TOL_BF16

pytestmark = pytest.mark.gpu


def _layer(n_text, n_img, seed):
    H = 12
    modes = np.asarray([FULL, ARROW, ARROW, CACHE, FULL, ARROW, ARROW, FULL, CACHE, ARROW, FULL, ARROW], np.int32)
    wins = np.asarray([0, 64, 300, 0, 0, 128, 1000, 0, 0, 17, 0, 512], np.int32)
    return W.Workload("static", 1, H, 128, n_text, n_img, modes, wins, seed=seed, positional=True)


def test_static_scratch_entry_matches_the_allocating_one_on_two_calls_in_a_row():
    from paper_2503_22796_amd import binding as B
    dev = torch.device("cuda:0")
    big, small = _layer(512, 4096, seed=31), _layer(77, 2048, seed=32)
    plan = B.difa_plan_create(1, 12, 128, max_tokens=big.N)
    try:
        for wl in (big, small):
            # the schedule of this layer does cut records: otherwise the scratch would not be exercised
            bm, bn = B.difa_tile_shape(wl.D)
            _, items, _ = B.difa_worklist_build(wl.B, wl.H, wl.head_plan, wl.window, wl.n_text, wl.n_img, bm, bn)
            _, _, _, merges, n_slots = B.difa_schedule_build(items[items["q_tile"] >= 0], 256, 8)
            assert n_slots > 0 and len(merges) > 0
            q, k, v = (t.to(dev) for t in W.make_qkv(wl))
            cache = W.make_cache(wl).to(dev)
            ref = torch.full_like(q, float("nan"))
            got = torch.full_like(q, float("nan"))
            print(f"static entry: N={wl.N} pieces={n_slots}", flush=True)
            B.difa_joint_attention(plan, q, k, v, ref, cache, wl.head_plan, wl.n_text, wl.n_img, wl.window)
            B.difa_joint_attention_static(plan, q, k, v, got, cache, wl.head_plan, wl.n_text, wl.n_img, wl.window)
            torch.cuda.synchronize()
            ref, got = ref.cpu(), got.cpu()
            for h in range(wl.H):
                if wl.head_plan[h] == CACHE:
                    assert torch.equal(got[:, h].view(torch.int16), ref[:, h].view(torch.int16)), f"cached head {h}"
                else:
                    assert torch.isfinite(got[:, h].float()).all(), f"head {h}: unwritten rows"
                    err = float((got[:, h].double() - ref[:, h].double()).abs().max())
                    assert err <= TOL_BF16, f"head {h}: {err}"
            print(f"static entry: N={wl.N} bit-identical={torch.equal(got.view(torch.int16), ref.view(torch.int16))}",
                  flush=True)
    finally:
        B.difa_plan_destroy(plan)
