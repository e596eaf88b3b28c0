"""Shared plumbing of the GPU parity tests: upload inputs, run the HIP path through the C ABI,
download results.  No arithmetic of the method lives here."""
from __future__ import annotations

import numpy as np
import torch

from paper_2508_09591_amd import binding as B


def to_dev_bf16(bits: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(bits).view(np.int16)).cuda().view(torch.bfloat16)


def bf16_to_host(t: torch.Tensor) -> np.ndarray:
    return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)


def dev(a: np.ndarray) -> torch.Tensor:
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


class GpuPlan:
    """hm_plan on the GPU plus host copies of everything it produced."""

    def __init__(self, ids, w, e2r, nodes, rpn, level, row_capacity=None, loads=False):
        self.ids_d, self.w_d, self.e2r_d = dev(ids), dev(w), dev(e2r)
        T, K = ids.shape
        self.T, self.K = T, K
        self.loads = loads
        self.plan = B.alloc_plan(T, K, e2r.shape[0], nodes, rpn, level, row_capacity=row_capacity, loads=loads)
        # poison the outputs so that unwritten entries are noticed
        for name in ("dest_count", "dest_offset", "row_token", "slot_row"):
            getattr(self.plan, name).fill_(-12345)
        self.plan.slot_keep.fill_(77)
        self.plan.row_weight.fill_(float("nan"))
        self.plan.status.fill_(55)
        B.hm_plan(self.ids_d, self.w_d, self.e2r_d, nodes, rpn, level, plan=self.plan)
        self.status, self.total_rows = B.hm_plan_status(self.plan)

    def host(self):
        p = self.plan
        n = self.total_rows
        extra = {}
        if self.loads:   # the load counts hm_plan fills on request
            extra = dict(load_expert=p.load_expert.cpu().numpy(), load_rank=p.load_rank.cpu().numpy(),
                         load_node=p.load_node.cpu().numpy())
        return dict(
            **extra,
            dest_count=p.dest_count[:p.num_dest].cpu().numpy(),
            dest_offset=p.dest_offset[:p.num_dest + 1].cpu().numpy(),
            row_token=p.row_token[:min(n, p.row_capacity)].cpu().numpy(),
            row_weight=p.row_weight[:min(n, p.row_capacity)].cpu().numpy(),
            slot_row=p.slot_row[:self.T * self.K].cpu().numpy().reshape(self.T, self.K),
            slot_keep=p.slot_keep[:self.T * self.K].cpu().numpy().reshape(self.T, self.K),
            rank_mask=p.rank_mask[:self.T].cpu().numpy().view(np.uint64),
            node_mask=p.node_mask[:self.T].cpu().numpy().view(np.uint32),
        )


def assert_plan_equal(gpu: GpuPlan, ora, ctx=""):
    h = gpu.host()
    assert gpu.status == ora.status, ctx
    assert gpu.total_rows == ora.total_rows, ctx
    assert gpu.plan.num_dest == ora.num_dest, ctx
    for f in ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "rank_mask", "node_mask"):
        assert np.array_equal(h[f], getattr(ora, f)), (ctx, f)
    # weights: compare encodings, not values
    assert np.array_equal(h["row_weight"].view(np.uint32), ora.row_weight.view(np.uint32)), (ctx, "row_weight")


def combine_forms(fn, y, weights, plan, out, stream=None):
    """Run a combine entry point (hm_combine, hm_combine_f32, hm_combine_mix) in both of its
    forms -- with the caller's weights, and with the weights the plan merged (weights = NULL) --
    and require the same bits from both; `out` holds the result."""
    fn(y, weights, plan, out)
    other = torch.full_like(out, float("nan"))
    fn(y, None, plan, other)
    if plan.row_capacity >= y.shape[0]:      # rows past the plan's weight array count as outside y
        a, b = out.contiguous().view(torch.uint8).cpu().numpy(), other.contiguous().view(torch.uint8).cpu().numpy()
        assert np.array_equal(a, b), "the two forms of %s disagree" % fn.__name__
    return out
