"""hm_plan_static (the entry point that allocates nothing: its scratch is a static device array)
against hm_plan, through the C ABI, bit for bit, on two calls in a row, the second smaller."""
import numpy as np
import pytest
import torch

from paper_2508_09591_amd import binding as B
from paper_2508_09591_amd import workloads as W

pytestmark = pytest.mark.gpu

FIELDS = ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "row_weight", "rank_mask", "node_mask",
          "load_expert", "load_rank", "load_node")


def _run(fn, ids_d, w_d, e2r_d, wl, level, poison):
    T, K = ids_d.shape
    plan = B.alloc_plan(T, K, wl.E, wl.nodes, wl.ranks_per_node, level, loads=True)
    for f in FIELDS:
        getattr(plan, f).fill_(poison)
    plan.status.fill_(55)
    fn(ids_d, w_d, e2r_d, wl.nodes, wl.ranks_per_node, level, plan=plan)
    st, total = B.hm_plan_status(plan)
    return plan, st, total


def _same(a, b, total, T, K):
    n = {"dest_count": a.num_dest, "dest_offset": a.num_dest + 1, "row_token": total, "row_weight": total,
         "slot_row": T * K, "slot_keep": T * K, "rank_mask": T, "node_mask": T}
    for f in FIELDS:
        x, y = getattr(a, f), getattr(b, f)
        m = n.get(f, x.numel())
        xa, ya = x[:m].cpu().numpy(), y[:m].cpu().numpy()
        if xa.dtype == np.float32:                     # compare encodings, not values
            xa, ya = xa.view(np.uint32), ya.view(np.uint32)
        assert np.array_equal(xa, ya), f


def test_static_scratch_plan_equals_hm_plan():
    assert B.lib().hm_plan_static_max_bytes() == 1 << 20
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    # first call: the 64 Ki-token layer at rank level (512 workgroups x 64 destinations: the count
    # matrix takes the scan launch); second call: a smaller, ragged table at another level, whose
    # matrix covers only a corner of what the first call left in the scratch
    calls = [("stress", None, B.HM_DEDUP_GPU), ("qwen3", 1237, B.HM_DEDUP_NODE), ("tiny", 333, B.HM_DEDUP_NONE)]
    for name, rows, level in calls:
        wl = W.WORKLOADS[name]
        r = W.make_routing(wl)
        ids, w = (r.topk_ids, r.topk_weights) if rows is None else (r.topk_ids[:rows], r.topk_weights[:rows])
        ids_d, w_d, e2r_d = dev(ids), dev(w), dev(r.expert_to_rank)
        T, K = ids.shape
        got, st_g, tot_g = _run(B.hm_plan_static, ids_d, w_d, e2r_d, wl, level, -7)
        want, st_w, tot_w = _run(B.hm_plan, ids_d, w_d, e2r_d, wl, level, -9)
        assert (st_g, tot_g) == (st_w, tot_w) and st_g == 0 and tot_g > 0, (name, st_g, tot_g, st_w, tot_w)
        _same(got, want, tot_g, T, K)


def test_static_scratch_rejects_sizes_beyond_its_maximum():
    # 64 destinations, 8 slots per token: (workgroups + 1) * 64 * 4 bytes must fit 1 MiB
    T, K, E = 600_000, 8, 256
    assert B.hm_plan_workspace_bytes(T, K, E, 8, 8, B.HM_DEDUP_GPU) > B.lib().hm_plan_static_max_bytes()
    plan = B.alloc_plan(16, K, E, 8, 8, B.HM_DEDUP_GPU)       # never written: the call must refuse first
    fake = torch.zeros(16, dtype=torch.int32, device="cuda")
    rc = B.lib().hm_plan_static(fake.data_ptr(), fake.data_ptr(), fake.data_ptr(), T, K, E, B.hm_topology(8, 8),
                                B.HM_DEDUP_GPU, plan.ref(), None)
    assert rc == B.HM_ERR_WORKSPACE
