"""GPU parity: the HIP path, called through the C ABI, against the CPU oracle on the same seeded
inputs.  Plans, maps and packed buffers must match bit for bit; combine must be within 1 bf16
ulp of the oracle's binary64 result rounded to bf16; the transpose is one fp32 multiply and
must match bit for bit."""
import numpy as np
import pytest

from helpers import GPU, NODE, NONE, bf16_ulp_distance
from paper_2508_09591_amd import workloads as W

pytestmark = pytest.mark.gpu

LEVEL = {NONE: "none", GPU: "gpu", NODE: "node"}


@pytest.fixture(scope="module")
def hw():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_harness
    from paper_2508_09591_amd import binding
    binding.lib()
    return gpu_harness


def _scaled_y(oracle, wl, r, p, packed_bits):
    """Test-harness expert model 'output = c[e] * input' in the packed layout: a row that serves
    several experts of one destination carries their weight-normalised mixture."""
    c = W.make_expert_scales(wl)
    num = np.zeros(p.total_rows)
    np.add.at(num, p.slot_row.reshape(-1), (r.topk_weights * c[r.topk_ids]).astype(np.float64).reshape(-1))
    s = (num / p.row_weight.astype(np.float64)).astype(np.float32)
    return W.f32_to_bf16_bits(s[:, None] * W.bf16_bits_to_f32(packed_bits))


def _run_layer(hw, oracle, wl, T, H, level, e2r=None, check_transpose=False, expert_model=None):
    import torch
    from paper_2508_09591_amd import binding as B
    r = W.make_routing(wl, T=T)
    e2r = r.expert_to_rank if e2r is None else e2r
    ctx = "%s T=%d H=%d level=%s" % (wl.name, T, H, LEVEL[level])
    print("case:", ctx, flush=True)
    ora = oracle.plan(r.topk_ids, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, level)
    g = hw.GpuPlan(r.topk_ids, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, level)
    hw.assert_plan_equal(g, ora, ctx)

    x = W.make_activations(wl, T=T, H=H)
    x_d = hw.to_dev_bf16(x)
    packed_d = torch.full((max(ora.total_rows, 1), H), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.hm_dispatch_pack(x_d, g.plan, packed_d[:ora.total_rows])
    packed = hw.bf16_to_host(packed_d[:ora.total_rows])
    packed_ref = oracle.dispatch_pack(x, ora.row_token)
    assert np.array_equal(packed, packed_ref), ctx

    model = expert_model or wl.expert_model
    y = packed_ref if model == "identity" else _scaled_y(oracle, wl, r, ora, packed_ref)
    y_d = hw.to_dev_bf16(y) if model != "identity" else packed_d[:ora.total_rows]
    out_d = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    hw.combine_forms(B.hm_combine, y_d, g.w_d, g.plan, out_d)
    out = hw.bf16_to_host(out_d)
    out_ref = oracle.combine(y, r.topk_weights, ora.slot_row)
    dist = bf16_ulp_distance(out, out_ref)
    assert dist.max() <= 1, (ctx, int(dist.max()))
    exact = float((dist == 0).mean())
    print("  combine: %.4f%% of elements bit-equal, rest 1 ulp" % (100 * exact), flush=True)
    assert exact > 0.98, ctx
    if model == "identity":
        # round trip: weights sum to 1, so the layer is the identity (a -0.0 input comes back as +0.0)
        assert bf16_ulp_distance(out, x).max() == 0, ctx

    if check_transpose:
        gout = W.make_output_grads(wl, T=T, H=H)
        gy_d = torch.full((max(ora.total_rows, 1), H), float("nan"), dtype=torch.float32, device="cuda")
        B.hm_combine_transpose(hw.dev(gout), g.plan, gy_d[:ora.total_rows])
        gy_ref = oracle.combine_transpose(gout, ora.row_token, ora.row_weight)
        assert np.array_equal(gy_d[:ora.total_rows].cpu().numpy().view(np.uint32), gy_ref.view(np.uint32)), ctx

    st, total = B.hm_plan_status(g.plan)
    assert st == 0 and total == ora.total_rows, ctx
    return r, ora, g


# ---- the five workloads, reduced so the oracle takes seconds: several tiles and a ragged tail ----
@pytest.mark.parametrize("name,T,H", [
    ("tiny", 1024, 256),          # configs[0] at full size
    ("qwen3", 1500, 2048),
    ("dsv3", 1111, 7168),
    ("skew", 2049, 2048),
    ("stress", 777, 7168),
])
def test_reduced_workloads_all_levels(hw, oracle, name, T, H):
    wl = W.WORKLOADS[name]
    for level in (NONE, GPU, NODE):
        _run_layer(hw, oracle, wl, T, H, level, check_transpose=True)


# ---- full sizes ----------------------------------------------------------------------------------
@pytest.mark.parametrize("name", ["qwen3", "dsv3"])
def test_full_size_layers(hw, oracle, name):
    wl = W.WORKLOADS[name]
    for level in wl.levels:
        _run_layer(hw, oracle, wl, wl.T, wl.H, level, check_transpose=(name == "dsv3"))


def test_combine_on_a_ragged_row_length(hw, oracle):
    """33001 tokens of 517 vectors per row (nine 1 KiB segments, the last one almost empty; two 4 KiB
    segments for the kernel that merges the caller's weights) with scaled experts, element by element."""
    import dataclasses
    wl = dataclasses.replace(W.WORKLOADS["skew"], name="wide", K=4, E=32, nodes=2, ranks_per_node=4, seed=77)
    for level in (GPU, NODE):
        _run_layer(hw, oracle, wl, 33001, 8 * 517, level)


def test_full_size_skew_both_placements(hw, oracle):
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["skew"]
    r = W.make_routing(wl)
    for e2r in (r.expert_to_rank, r.extras["expert_to_rank_swapped"]):
        le, lr, ln, st = oracle.expert_load(r.topk_ids, e2r, wl.nodes, wl.ranks_per_node)
        le_d = torch.full((wl.E,), -1, dtype=torch.int32, device="cuda")
        lr_d = torch.full((wl.G,), -1, dtype=torch.int32, device="cuda")
        ln_d = torch.full((wl.nodes,), -1, dtype=torch.int32, device="cuda")
        st_d = torch.full((1,), 9, dtype=torch.int32, device="cuda")
        B.hm_expert_load(hw.dev(r.topk_ids), hw.dev(e2r), wl.nodes, wl.ranks_per_node, le_d, lr_d, ln_d, st_d)
        assert np.array_equal(le_d.cpu().numpy(), le) and np.array_equal(lr_d.cpu().numpy(), lr)
        assert np.array_equal(ln_d.cpu().numpy(), ln) and int(st_d.item()) == st == 0
        for level in wl.levels:
            _, ora, g = _run_layer(hw, oracle, wl, wl.T, wl.H, level, e2r=e2r)
            # the dedup-aware loads are the plan's destination counts (Eq.(7))
            assert np.array_equal(ora.dest_count, lr if level == GPU else ln)


def test_full_size_stress_sampled(hw, oracle):
    """T=65536, H=7168: the plan is compared in full, the row buffers on sampled ranges."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["stress"]
    r = W.make_routing(wl)
    x = W.make_activations(wl)
    x_d = hw.to_dev_bf16(x)
    gout = W.make_output_grads(wl)
    gout_d = hw.dev(gout)
    rng = np.random.default_rng(1234)
    # T above the single-launch limit: the split (clear + atomics) path of hm_expert_load
    le, lr, ln, st = oracle.expert_load(r.topk_ids, r.expert_to_rank, wl.nodes, wl.ranks_per_node)
    le_d, lr_d, ln_d = (torch.full((m,), -1, dtype=torch.int32, device="cuda") for m in (wl.E, wl.G, wl.nodes))
    st_d = torch.full((1,), 9, dtype=torch.int32, device="cuda")
    B.hm_expert_load(hw.dev(r.topk_ids), hw.dev(r.expert_to_rank), wl.nodes, wl.ranks_per_node, le_d, lr_d, ln_d, st_d)
    assert np.array_equal(le_d.cpu().numpy(), le) and np.array_equal(lr_d.cpu().numpy(), lr)
    assert np.array_equal(ln_d.cpu().numpy(), ln) and int(st_d.item()) == 0
    bad = r.topk_ids.copy()
    bad[40000, 3] = wl.E + 5
    le, lr, ln, st = oracle.expert_load(bad, r.expert_to_rank, wl.nodes, wl.ranks_per_node)
    B.hm_expert_load(hw.dev(bad), hw.dev(r.expert_to_rank), wl.nodes, wl.ranks_per_node, le_d, lr_d, ln_d, st_d)
    assert np.array_equal(le_d.cpu().numpy(), le) and np.array_equal(lr_d.cpu().numpy(), lr)
    assert np.array_equal(ln_d.cpu().numpy(), ln) and int(st_d.item()) == st == B.HM_ERR_BAD_ID
    for level in wl.levels:
        ctx = "stress full level=%s" % LEVEL[level]
        print("case:", ctx, flush=True)
        ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        hw.assert_plan_equal(g, ora, ctx)
        n = ora.total_rows
        packed_d = torch.empty((n, wl.H), dtype=torch.bfloat16, device="cuda")
        packed_d.view(torch.int16).fill_(0x7FC1)
        B.hm_dispatch_pack(x_d, g.plan, packed_d)
        out_d = torch.empty((wl.T, wl.H), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine, packed_d, g.w_d, g.plan, out_d)
        gy_d = torch.empty((n, wl.H), dtype=torch.float32, device="cuda")
        B.hm_combine_transpose(gout_d, g.plan, gy_d)
        # whole-buffer property: identity experts and weights summing to 1 -> the layer is the identity
        assert torch.equal(out_d, x_d), ctx                     # compares values: -0.0 == +0.0
        # row ranges: first, last and random windows of 1500 rows, each row checked against the oracle
        starts = [0, n - 1500] + [int(v) for v in rng.integers(0, n - 1500, 4)]
        for a in starts:
            rows = slice(a, a + 1500)
            ref = oracle.dispatch_pack(x, ora.row_token[rows])
            assert np.array_equal(hw.bf16_to_host(packed_d[rows]), ref), (ctx, a)
            gref = oracle.combine_transpose(gout, ora.row_token[rows], ora.row_weight[rows])
            assert np.array_equal(gy_d[rows].cpu().numpy().view(np.uint32), gref.view(np.uint32)), (ctx, a)
        # token ranges for combine: the oracle gathers from the (already verified) packed rows it needs
        for t0 in [0, wl.T - 300] + [int(v) for v in rng.integers(0, wl.T - 300, 2)]:
            sr = ora.slot_row[t0:t0 + 300]
            uniq, inv = np.unique(sr, return_inverse=True)
            y_sub = oracle.dispatch_pack(x, ora.row_token[uniq])
            ref = oracle.combine(y_sub, r.topk_weights[t0:t0 + 300], inv.reshape(sr.shape).astype(np.int32))
            got = hw.bf16_to_host(out_d[t0:t0 + 300])
            assert bf16_ulp_distance(got, ref).max() <= 1, (ctx, t0)
        # scaled experts ("output = c[e] * input", a shared row carrying the weight-normalised mixture):
        # Y is built on the device from the verified packed rows by the harness (one fp32 multiply,
        # rounded to bf16 -- the numpy form below gives the same bits), combine is checked on token windows
        cexp = W.make_expert_scales(wl)
        num = np.zeros(n)
        np.add.at(num, ora.slot_row.reshape(-1), (r.topk_weights * cexp[r.topk_ids]).astype(np.float64).reshape(-1))
        scale = (num / ora.row_weight.astype(np.float64)).astype(np.float32)
        y_d = (packed_d.float() * hw.dev(scale)[:, None]).to(torch.bfloat16)
        hw.combine_forms(B.hm_combine, y_d, g.w_d, g.plan, out_d)
        for t0 in [0, wl.T - 300] + [int(v) for v in rng.integers(0, wl.T - 300, 2)]:
            sr = ora.slot_row[t0:t0 + 300]
            uniq, inv = np.unique(sr, return_inverse=True)
            y_sub = W.f32_to_bf16_bits(scale[uniq][:, None] * W.bf16_bits_to_f32(oracle.dispatch_pack(x, ora.row_token[uniq])))
            assert np.array_equal(hw.bf16_to_host(y_d[torch.from_numpy(uniq).cuda()]), y_sub), (ctx, t0)
            ref = oracle.combine(y_sub, r.topk_weights[t0:t0 + 300], inv.reshape(sr.shape).astype(np.int32))
            got = hw.bf16_to_host(out_d[t0:t0 + 300])
            assert bf16_ulp_distance(got, ref).max() <= 1, (ctx, "scaled", t0)
        del packed_d, out_d, gy_d, y_d
        torch.cuda.empty_cache()


def test_full_size_dsv3_at_the_other_levels(hw, oracle):
    """The DeepSeek-V3-shaped layer at full size at rank level and without dedup (about seven and
    exactly eight rows per token: combine runs with the cap on resident waves), scaled experts,
    element by element."""
    wl = W.WORKLOADS["dsv3"]
    for level in (GPU, NONE):
        _run_layer(hw, oracle, wl, wl.T, wl.H, level, expert_model="scaled")


def test_full_size_dsv3_scaled_experts_at_node_level(hw, oracle):
    wl = W.WORKLOADS["dsv3"]
    _run_layer(hw, oracle, wl, wl.T, wl.H, NODE, expert_model="scaled")


def test_worst_case_buffers_without_a_sync(hw, oracle):
    """The mode the header recommends to callers that do not want to synchronise: row buffers
    allocated for the worst case (row_capacity rows) and no hm_plan_status before the row calls.
    The launch shape then comes from the bound hm_plan left in the struct -- never from the buffer
    sizes -- and the results are the oracle's whatever shape a hint selects."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["dsv3"]
    T, H = 1500, 7168
    r = W.make_routing(wl, T=T)
    x = W.make_activations(wl, T=T, H=H)
    x_d = hw.to_dev_bf16(x)
    ids_d, w_d, e2r_d = hw.dev(r.topk_ids), hw.dev(r.topk_weights), hw.dev(r.expert_to_rank)
    for level, bound, shape in ((GPU, 8, (1, 8, 16)), (NODE, 4, (1, 8, 32)), (NONE, 8, (1, 8, 16))):
        ctx = "no-sync level=%s" % LEVEL[level]
        print("case:", ctx, flush=True)
        ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        plan = B.hm_plan(ids_d, w_d, e2r_d, wl.nodes, wl.ranks_per_node, level)       # no hm_plan_status
        assert plan.c.expected_rows == 0 and plan.c.max_rows_per_token == bound
        assert B.hm_combine_launch_shape(plan, H) == shape, ctx
        assert B.hm_combine_launch_shape(plan, H, weights_from_plan=False) == (4, 4, 32)
        cap = plan.row_capacity                                                       # T * min(K, destinations)
        packed_d = torch.full((cap, H), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.hm_dispatch_pack(x_d, plan, packed_d)
        n = ora.total_rows
        assert cap > n or level == NONE
        assert np.array_equal(hw.bf16_to_host(packed_d[:n]), oracle.dispatch_pack(x, ora.row_token)), ctx
        assert bool(torch.isnan(packed_d[n:]).all())                                  # nothing beyond total_rows
        ref = oracle.combine(hw.bf16_to_host(packed_d[:n]), r.topk_weights, ora.slot_row)
        outs = []
        for hint in (0, n, T, 64 * T):           # unknown, the true count, "one row per token", "very many"
            plan.c.expected_rows = hint
            out_d = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
            hw.combine_forms(B.hm_combine, packed_d, w_d, plan, out_d)
            outs.append(hw.bf16_to_host(out_d))
            assert bf16_ulp_distance(outs[-1], ref).max() <= 1, (ctx, hint)
            assert np.array_equal(outs[-1], outs[0]), (ctx, hint)                     # the shape never changes the bits
        plan.c.expected_rows = T
        assert B.hm_combine_launch_shape(plan, H) == (4, 2, 32)
        plan.c.expected_rows = 64 * T
        assert B.hm_combine_launch_shape(plan, H) == (1, 8, 16)
        st, total = B.hm_plan_status(plan)
        assert st == 0 and total == n and plan.c.expected_rows == n                   # the status call leaves the count as the hint
    # a hop-table plan (about one row per token, no useful bound): unknown means "few", whatever the buffer
    on3 = r.expert_to_rank == 3
    dm = hw.dev(np.where(on3, np.cumsum(on3) - 1, -1).astype(np.int32))      # experts of rank 3 -> 0, 1, 2, ...; others: no copy
    nd = int(on3.sum())
    mp = B.hm_plan_mapped(ids_d, w_d, dm, nd, False)
    assert mp.c.max_rows_per_token == 0 and mp.c.expected_rows == 0
    assert B.hm_combine_launch_shape(mp, H) == (4, 4, 32)
    o = oracle.plan_mapped(r.topk_ids, r.topk_weights, dm.cpu().numpy(), nd, False)
    big_d = torch.full((mp.row_capacity, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    B.hm_dispatch_pack(x_d, mp, big_d)
    assert np.array_equal(hw.bf16_to_host(big_d[:o.total_rows]), oracle.dispatch_pack(x, o.row_token))
    out_d = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    hw.combine_forms(B.hm_combine_mix, big_d, w_d, mp, out_d)
    refm = oracle.combine_mix(hw.bf16_to_host(big_d[:o.total_rows]), r.topk_weights, o.slot_row)
    assert bf16_ulp_distance(hw.bf16_to_host(out_d), refm).max() <= 1


def test_table4_grid(hw, oracle):
    """K in {6,8,10}, E in {64,128,256}, G in {8,16,32} (the grid of the paper's Table IV), all
    three levels, reduced T."""
    for wl in W.table4_variants():
        for level in (NONE, GPU, NODE):
            _run_layer(hw, oracle, wl, 1200, 512, level, expert_model="scaled")


# ---- edge cases ------------------------------------------------------------------------------------
@pytest.mark.parametrize("T,K,E,nodes,rpn,H", [
    (0, 2, 8, 2, 2, 64),        # empty
    (1, 1, 4, 1, 1, 8),         # one token, one destination
    (3, 64, 64, 8, 8, 72),      # K at its limit, 64 ranks, 9 vectors per row
    (130, 5, 30, 3, 5, 1000),   # K and G not powers of two, 125 vectors per row (ragged segment)
    (257, 6, 48, 2, 3, 100),    # H not a multiple of 8 -> element-wise kernels
    (64, 8, 256, 32, 2, 520),   # 32 nodes
    (1025, 3, 12, 1, 4, 264),   # slots straddle workgroup boundaries with K=3
])
def test_edge_shapes(hw, oracle, T, K, E, nodes, rpn, H):
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(T * 7 + K)
    G = nodes * rpn
    ids = rng.integers(0, E, (T, K), dtype=np.int32)           # repeated experts inside a token allowed
    w = rng.random((T, K), dtype=np.float32) + np.float32(0.05)
    e2r = rng.integers(0, G, E, dtype=np.int32)
    x = W.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    gout = rng.standard_normal((T, H)).astype(np.float32)
    for level in (NONE, GPU, NODE):
        ctx = "edge T=%d K=%d E=%d %dx%d H=%d level=%s" % (T, K, E, nodes, rpn, H, LEVEL[level])
        print("case:", ctx, flush=True)
        ora = oracle.plan(ids, w, e2r, nodes, rpn, level)
        g = hw.GpuPlan(ids, w, e2r, nodes, rpn, level)
        hw.assert_plan_equal(g, ora, ctx)
        n = ora.total_rows
        packed_d = torch.zeros((max(n, 1), H), dtype=torch.bfloat16, device="cuda")
        B.hm_dispatch_pack(hw.to_dev_bf16(x), g.plan, packed_d[:n])
        assert np.array_equal(hw.bf16_to_host(packed_d[:n]), oracle.dispatch_pack(x, ora.row_token)), ctx
        y = W.f32_to_bf16_bits(rng.random((max(n, 1), H)).astype(np.float32) + np.float32(0.5))[:n]  # same-sign terms
        out_d = torch.zeros((max(T, 1), H), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine, hw.to_dev_bf16(y) if n else packed_d[:0], g.w_d, g.plan, out_d[:T])
        ref = oracle.combine(y, w, ora.slot_row) if T else np.zeros((0, H), np.uint16)
        assert T == 0 or bf16_ulp_distance(hw.bf16_to_host(out_d[:T]), ref).max() <= 1, ctx
        gy_d = torch.zeros((max(n, 1), H), dtype=torch.float32, device="cuda")
        B.hm_combine_transpose(hw.dev(gout) if T else gy_d[:0], g.plan, gy_d[:n])
        gref = oracle.combine_transpose(gout, ora.row_token, ora.row_weight)
        assert np.array_equal(gy_d[:n].cpu().numpy().view(np.uint32), gref.view(np.uint32)), ctx
        le, lr, ln, st = oracle.expert_load(ids, e2r, nodes, rpn)
        le_d, lr_d, ln_d = (torch.full((m,), -1, dtype=torch.int32, device="cuda") for m in (E, G, nodes))
        B.hm_expert_load(g.ids_d, g.e2r_d, nodes, rpn, le_d, lr_d, ln_d)
        assert np.array_equal(le_d.cpu().numpy(), le) and np.array_equal(lr_d.cpu().numpy(), lr), ctx
        assert np.array_equal(ln_d.cpu().numpy(), ln), ctx


def test_vector_and_elementwise_kernels_agree_on_misaligned_views(hw, oracle):
    """The same problem through the 16-byte path and, via views offset by one element, through
    the element-wise path: identical bits."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["qwen3"]
    T, H = 300, 512
    r = W.make_routing(wl, T=T)
    x = W.make_activations(wl, T=T, H=H)
    ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, GPU)
    g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, GPU)
    n = ora.total_rows
    x_d = hw.to_dev_bf16(x)
    pad = torch.zeros(T * H + 1, dtype=torch.bfloat16, device="cuda")
    x_mis = pad[1:].view(T, H)
    x_mis.copy_(x_d)
    assert x_mis.data_ptr() % 16 != 0
    a = torch.zeros((n, H), dtype=torch.bfloat16, device="cuda")
    b_store = torch.zeros(n * H + 1, dtype=torch.bfloat16, device="cuda")
    b = b_store[1:].view(n, H)
    B.hm_dispatch_pack(x_d, g.plan, a)
    B.hm_dispatch_pack(x_mis, g.plan, b)
    assert torch.equal(a.view(torch.int16), b.contiguous().view(torch.int16))
    oa = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    ob_store = torch.zeros(T * H + 1, dtype=torch.bfloat16, device="cuda")
    ob = ob_store[1:].view(T, H)
    hw.combine_forms(B.hm_combine, a, g.w_d, g.plan, oa)
    hw.combine_forms(B.hm_combine, b, g.w_d, g.plan, ob)
    assert torch.equal(oa.view(torch.int16), ob.contiguous().view(torch.int16))
    assert bf16_ulp_distance(hw.bf16_to_host(oa), x).max() == 0


def test_bad_ids_and_small_buffers_are_flagged_not_faulted(hw, oracle):
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(2)
    T, K, E, nodes, rpn, H = 200, 4, 16, 2, 2, 128
    ids = rng.integers(0, E, (T, K), dtype=np.int32)
    ids[5, 1] = -3
    ids[17, 0] = E
    ids[199, 3] = 1 << 30
    w = rng.random((T, K), dtype=np.float32)
    e2r = W.contiguous_placement(E, nodes * rpn)
    e2r[9] = 4                                                   # rank that does not exist
    x = W.f32_to_bf16_bits(rng.standard_normal((T, H)).astype(np.float32))
    for level in (NONE, GPU, NODE):
        ora = oracle.plan(ids, w, e2r, nodes, rpn, level)
        g = hw.GpuPlan(ids, w, e2r, nodes, rpn, level)
        assert g.status == B.HM_ERR_BAD_ID == ora.status
        hw.assert_plan_equal(g, ora)
        n = ora.total_rows
        packed_d = torch.zeros((n, H), dtype=torch.bfloat16, device="cuda")
        B.hm_dispatch_pack(hw.to_dev_bf16(x), g.plan, packed_d)
        assert np.array_equal(hw.bf16_to_host(packed_d), oracle.dispatch_pack(x, ora.row_token))
        out_d = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine, packed_d, g.w_d, g.plan, out_d)
        ref = oracle.combine(hw.bf16_to_host(packed_d), w, ora.slot_row)
        assert bf16_ulp_distance(hw.bf16_to_host(out_d), ref).max() <= 1
        le, lr, ln, st = oracle.expert_load(ids, e2r, nodes, rpn)
        le_d, lr_d, ln_d = (torch.full((m,), -1, dtype=torch.int32, device="cuda") for m in (E, nodes * rpn, nodes))
        st_d = torch.zeros(1, dtype=torch.int32, device="cuda")
        B.hm_expert_load(g.ids_d, g.e2r_d, nodes, rpn, le_d, lr_d, ln_d, st_d)
        assert int(st_d.item()) == B.HM_ERR_BAD_ID == st
        assert np.array_equal(le_d.cpu().numpy(), le) and np.array_equal(lr_d.cpu().numpy(), lr)

    # a packed buffer that is too short: rows beyond it are skipped, the rest is correct
    good = rng.integers(0, E, (T, K), dtype=np.int32)
    e2r_ok = W.contiguous_placement(E, nodes * rpn)
    ora = oracle.plan(good, w, e2r_ok, nodes, rpn, GPU)
    g = hw.GpuPlan(good, w, e2r_ok, nodes, rpn, GPU)
    short = ora.total_rows - 37
    store = torch.full((ora.total_rows, H), 7.0, dtype=torch.bfloat16, device="cuda")
    B.hm_dispatch_pack(hw.to_dev_bf16(x), g.plan, store[:short])
    st, _ = B.hm_plan_status(g.plan)
    assert st == B.HM_ERR_CAPACITY
    ref = oracle.dispatch_pack(x, ora.row_token)
    assert np.array_equal(hw.bf16_to_host(store[:short]), ref[:short])
    assert bool((store[short:] == 7.0).all())                  # nothing written past the end
    # a plan whose row buffers are too small: counts stay exact, status says so
    g2 = hw.GpuPlan(good, w, e2r_ok, nodes, rpn, GPU, row_capacity=ora.total_rows - 5)
    assert g2.status == B.HM_ERR_CAPACITY and g2.total_rows == ora.total_rows
    assert np.array_equal(g2.host()["dest_count"], ora.dest_count)
    assert np.array_equal(g2.host()["row_token"], ora.row_token[:ora.total_rows - 5])


def test_dropped_slots_on_the_gpu(hw, oracle):
    """Capacity-limited routing: slots marked -1 are skipped by every entry point, without error."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["qwen3"]
    T, H = 1500, 256
    r = W.make_routing(wl, T=T)
    rng = np.random.default_rng(77)
    ids = r.topk_ids.copy()
    ids[rng.random(ids.shape) < 0.2] = -1
    ids[11, :] = -1                                              # a token with nothing left
    w, e2r = r.topk_weights, r.expert_to_rank
    x = W.make_activations(wl, T=T, H=H)
    for level in (NONE, GPU, NODE):
        ora = oracle.plan(ids, w, e2r, wl.nodes, wl.ranks_per_node, level)
        g = hw.GpuPlan(ids, w, e2r, wl.nodes, wl.ranks_per_node, level)
        assert g.status == 0 == ora.status
        hw.assert_plan_equal(g, ora, "dropped level %d" % level)
        n = ora.total_rows
        packed_d = torch.zeros((n, H), dtype=torch.bfloat16, device="cuda")
        B.hm_dispatch_pack(hw.to_dev_bf16(x), g.plan, packed_d)
        packed = hw.bf16_to_host(packed_d)
        assert np.array_equal(packed, oracle.dispatch_pack(x, ora.row_token))
        out_d = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine, packed_d, g.w_d, g.plan, out_d)
        out = hw.bf16_to_host(out_d)
        assert bf16_ulp_distance(out, oracle.combine(packed, w, ora.slot_row)).max() <= 1
        assert not out[11].any()
    le, lr, ln, st = oracle.expert_load(ids, e2r, wl.nodes, wl.ranks_per_node)
    le_d, lr_d, ln_d = (torch.full((m,), -1, dtype=torch.int32, device="cuda") for m in (wl.E, wl.G, wl.nodes))
    st_d = torch.full((1,), 3, dtype=torch.int32, device="cuda")
    B.hm_expert_load(hw.dev(ids), hw.dev(e2r), wl.nodes, wl.ranks_per_node, le_d, lr_d, ln_d, st_d)
    assert np.array_equal(le_d.cpu().numpy(), le) and np.array_equal(lr_d.cpu().numpy(), lr)
    assert np.array_equal(ln_d.cpu().numpy(), ln) and int(st_d.item()) == st == 0
    counts_d = torch.zeros((2, 64), dtype=torch.int32, device="cuda")
    B.hm_group_counts(hw.dev(ids), hw.dev(e2r), wl.G, [wl.G, wl.nodes], counts_d, st_d)
    ref, st = oracle.group_counts(ids, e2r, wl.G, [wl.G, wl.nodes])
    assert np.array_equal(counts_d.cpu().numpy(), ref) and int(st_d.item()) == st == 0
    Z = torch.zeros((wl.E, wl.E, wl.nodes), dtype=torch.int32, device="cuda")
    B.hm_swap_counts(hw.dev(ids), hw.dev(e2r), wl.G, wl.nodes, Z, st_d)
    zr, st = oracle.swap_counts(ids, e2r, wl.G, wl.nodes)
    assert np.array_equal(Z.cpu().numpy(), zr) and int(st_d.item()) == st == 0
    dm = (e2r // wl.ranks_per_node).astype(np.int32)
    ora = oracle.plan_mapped(ids, w, dm, wl.nodes, True)
    plan = B.hm_plan_mapped(hw.dev(ids), hw.dev(w), hw.dev(dm), wl.nodes, True)
    st, total = B.hm_plan_status(plan)
    assert st == 0 == ora.status and total == ora.total_rows
    assert np.array_equal(plan.slot_row.cpu().numpy().reshape(T, wl.K), ora.slot_row)


@pytest.mark.parametrize("name,T", [("tiny", 1024), ("qwen3", 3000), ("dsv3", 8192), ("skew", 16384), ("stress", 65536)])
def test_plan_with_fused_loads(hw, oracle, name, T):
    """hm_plan with the optional load arrays: same plan, plus the counts of hm_expert_load."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=T)
    ids = r.topk_ids.copy()
    e2r = r.extras.get("expert_to_rank_swapped", r.expert_to_rank)
    if name == "qwen3":
        ids[7, 2] = -1                                         # a dropped slot
        ids[100, 0] = wl.E + 1                                 # an invalid one
    le, lr, ln, st = oracle.expert_load(ids, e2r, wl.nodes, wl.ranks_per_node)
    ids_d, w_d, e2r_d = hw.dev(ids), hw.dev(r.topk_weights), hw.dev(e2r)
    for level in (NONE, GPU, NODE):
        ora = oracle.plan(ids, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, level)
        plan = B.alloc_plan(T, wl.K, wl.E, wl.nodes, wl.ranks_per_node, level, loads=True)
        for t in (plan.load_expert, plan.load_rank, plan.load_node):
            t.fill_(-99)
        B.hm_plan(ids_d, w_d, e2r_d, wl.nodes, wl.ranks_per_node, level, plan=plan)
        stg, total = B.hm_plan_status(plan)
        assert stg == ora.status == st and total == ora.total_rows
        assert np.array_equal(plan.slot_row.cpu().numpy().reshape(T, wl.K), ora.slot_row)
        assert np.array_equal(plan.row_token[:total].cpu().numpy(), ora.row_token)
        assert np.array_equal(plan.load_expert.cpu().numpy(), le), (name, level)
        assert np.array_equal(plan.load_rank.cpu().numpy(), lr), (name, level)
        assert np.array_equal(plan.load_node.cpu().numpy(), ln), (name, level)


def test_fused_loads_with_many_experts(hw, oracle):
    """More experts than the LDS histogram holds: the global-atomics path."""
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(404)
    T, K, E, nodes, rpn = 3000, 4, 9000, 4, 8
    ids = rng.integers(0, E, (T, K), dtype=np.int32)
    w = rng.random((T, K), dtype=np.float32)
    e2r = rng.integers(0, nodes * rpn, E).astype(np.int32)
    le, lr, ln, st = oracle.expert_load(ids, e2r, nodes, rpn)
    plan = B.alloc_plan(T, K, E, nodes, rpn, GPU, loads=True)
    B.hm_plan(hw.dev(ids), hw.dev(w), hw.dev(e2r), nodes, rpn, GPU, plan=plan)
    stg, total = B.hm_plan_status(plan)
    ora = oracle.plan(ids, w, e2r, nodes, rpn, GPU)
    assert stg == 0 and total == ora.total_rows
    assert np.array_equal(plan.load_expert.cpu().numpy(), le) and np.array_equal(plan.load_rank.cpu().numpy(), lr)
    assert np.array_equal(plan.load_node.cpu().numpy(), ln)


@pytest.mark.parametrize("T,K,nodes,rpn", [(400000, 8, 8, 8), (70000, 3, 2, 4), (32768, 8, 8, 8), (32640, 8, 8, 8)])
def test_plan_at_large_token_counts(hw, oracle, T, K, nodes, rpn):
    """Sizes on both sides of the point where hm_plan inserts its scan launch (count-matrix
    entries = ceil(T*K/1024) * destinations >= 16384), the whole plan compared with the oracle."""
    E = 256
    rng = np.random.default_rng(T % 97)
    ids = rng.integers(0, E, (T, K), dtype=np.int32)         # repeated ids inside a token are legal
    w = rng.random((T, K), dtype=np.float32)
    e2r = W.contiguous_placement(E, nodes * rpn)
    for level in (NONE, GPU, NODE):
        ctx = "large plan T=%d K=%d %dx%d level=%s" % (T, K, nodes, rpn, LEVEL[level])
        print("case:", ctx, flush=True)
        ora = oracle.plan(ids, w, e2r, nodes, rpn, level)
        g = hw.GpuPlan(ids, w, e2r, nodes, rpn, level)
        hw.assert_plan_equal(g, ora, ctx)


def test_plan_is_deterministic(hw, oracle):
    import torch
    wl = W.WORKLOADS["dsv3"]
    r = W.make_routing(wl, T=4096)
    first = None
    for _ in range(5):
        g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, NODE)
        h = g.host()
        blob = b"".join(np.ascontiguousarray(h[k]).tobytes() for k in sorted(h))
        first = first or blob
        assert blob == first


def test_plan_does_not_depend_on_the_launch_path(hw, oracle):
    """Small plans run as one launch by default; with the limit at 0 the same plans take the
    separate count / write launches (which otherwise only plans above 262,144 slots use), and a
    limit of 2 workgroups splits the cases between the two.  Every field must come out the same,
    fused load counts included, and equal to the oracle."""
    from paper_2508_09591_amd import binding as B
    cases = [("qwen3", 1500, GPU), ("dsv3", 4096, NODE), ("tiny", 1024, NONE), ("skew", 200, GPU)]
    blobs = {}
    try:
        for limit in (256, 0, 2):
            assert B.hm_plan_one_launch_limit(limit) in (256, 0, 2)
            for name, T, level in cases:
                wl = W.WORKLOADS[name]
                r = W.make_routing(wl, T=T)
                g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level, loads=True)
                h = g.host()
                blob = b"".join(np.ascontiguousarray(h[k]).tobytes() for k in sorted(h))
                assert blobs.setdefault((name, T, level), blob) == blob, (limit, name)
                if limit == 0:
                    hw.assert_plan_equal(g, oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node,
                                                        level), "separate launches: " + name)
    finally:
        assert B.hm_plan_one_launch_limit(256) in (256, 0, 2)
    assert B.hm_plan_one_launch_limit(10 ** 6) == 256 and B.hm_plan_one_launch_limit(-5) == 256      # clamped to [0, 256]
    assert B.hm_plan_one_launch_limit(256) == 0


def test_random_shapes_against_the_oracle(hw, oracle):
    """Seeded sweep over shapes nobody picked by hand: topology, K, E, H (vector and element-wise
    paths), uneven placements, repeated experts, dropped and invalid slots, all three levels."""
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(20260)
    for case in range(40):
        nodes = int(rng.choice([1, 2, 3, 4, 8]))
        rpn = int(rng.choice([1, 2, 4, 8]))
        G = nodes * rpn
        E = G * int(rng.integers(1, 9)) + int(rng.integers(0, 3))
        K = int(rng.integers(1, 13))
        T = int(rng.integers(1, 2600))
        H = int(rng.choice([8, 24, 64, 100, 520, 1024, 2048, 2056]))
        ids = rng.integers(0, E, (T, K), dtype=np.int32)
        if case % 3 == 0:
            ids[rng.random((T, K)) < 0.1] = -1
        if case % 4 == 0:
            ids[rng.integers(0, T), rng.integers(0, K)] = E + 7
        w = rng.random((T, K), dtype=np.float32) + np.float32(0.02)
        e2r = rng.integers(0, G, E).astype(np.int32)
        x = W.f32_to_bf16_bits((rng.random((T, H)) + 0.25).astype(np.float32))
        level = int(rng.integers(0, 3))
        ctx = "case %d: %dx%d E=%d K=%d T=%d H=%d level=%d" % (case, nodes, rpn, E, K, T, H, level)
        print(ctx, flush=True)
        ora = oracle.plan(ids, w, e2r, nodes, rpn, level)
        g = hw.GpuPlan(ids, w, e2r, nodes, rpn, level)
        hw.assert_plan_equal(g, ora, ctx)
        n = ora.total_rows
        packed_d = torch.zeros((max(n, 1), H), dtype=torch.bfloat16, device="cuda")
        B.hm_dispatch_pack(hw.to_dev_bf16(x), g.plan, packed_d[:n])
        packed = hw.bf16_to_host(packed_d[:n])
        assert np.array_equal(packed, oracle.dispatch_pack(x, ora.row_token)), ctx
        out_d = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine, packed_d[:n], g.w_d, g.plan, out_d)
        assert bf16_ulp_distance(hw.bf16_to_host(out_d), oracle.combine(packed, w, ora.slot_row)).max() <= 1, ctx
        gout = rng.standard_normal((T, H)).astype(np.float32)
        gy_d = torch.zeros((max(n, 1), H), dtype=torch.float32, device="cuda")
        B.hm_combine_transpose(hw.dev(gout), g.plan, gy_d[:n])
        gref = oracle.combine_transpose(gout, ora.row_token, ora.row_weight)
        assert np.array_equal(gy_d[:n].cpu().numpy().view(np.uint32), gref.view(np.uint32)), ctx


def test_dispatch_packs_rows_of_any_element_type(hw, oracle):
    """hm_dispatch_pack copies bytes: fp32 rows, fp8 / uint8 rows (with their fp32 scale rows) and
    int32 metadata rows pack through the same call when H is given in 2-byte units."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["dsv3"]
    T, H = 900, 7168
    r = W.make_routing(wl, T=T)
    rng = np.random.default_rng(8)
    ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, NODE)
    g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, NODE)
    n = ora.total_rows
    x32 = rng.standard_normal((T, H)).astype(np.float32)                 # fp32 rows: 2H units
    x8 = rng.integers(0, 256, (T, H), dtype=np.uint8)                    # one byte per element: H/2 units
    scales = rng.random((T, H // 128)).astype(np.float32)               # per-128 block scales: 2*(H/128) units
    for host, units in ((x32, 2 * H), (x8, H // 2), (scales, 2 * (H // 128))):
        src_d = hw.dev(host).view(torch.bfloat16).view(T, units)
        out_d = torch.zeros((n, units), dtype=torch.bfloat16, device="cuda")
        B.hm_dispatch_pack(src_d, g.plan, out_d)
        got = out_d.view(torch.uint8).cpu().numpy().reshape(n, -1)
        want = oracle.dispatch_pack(host, ora.row_token).view(np.uint8).reshape(n, -1)
        assert np.array_equal(got, want), host.dtype


@pytest.mark.parametrize("name,T,H", [("tiny", 1024, 256), ("qwen3", 1500, 2048), ("dsv3", 700, 7168),
                                      ("skew", 2049, 1030), ("skew", 300, 77)])
def test_combine_on_binary32_rows(hw, oracle, name, T, H):
    """hm_combine_f32 against the oracle's binary64 sum: within the bound of a K-term fp32 fma
    chain with merged weights, 2K * 2^-24 * sum_k |w y| (vector kernel, the ragged-H vector case
    and the element-wise kernel for H % 4 != 0)."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=T)
    rng = np.random.default_rng(T + H)
    for level in (NONE, GPU, NODE):
        ctx = "f32 %s T=%d H=%d level=%s" % (name, T, H, LEVEL[level])
        print("case:", ctx, flush=True)
        ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        y = rng.standard_normal((ora.total_rows, H)).astype(np.float32)
        out_d = torch.full((T, H), float("nan"), dtype=torch.float32, device="cuda")
        hw.combine_forms(B.hm_combine_f32, hw.dev(y), g.w_d, g.plan, out_d)
        got = out_d.cpu().numpy()
        ref = oracle.combine_f32(y, r.topk_weights, ora.slot_row)
        mag = np.einsum("tk,tkh->th", np.abs(r.topk_weights).astype(np.float64), np.abs(y).astype(np.float64)[ora.slot_row])
        err = np.abs(got.astype(np.float64) - ref.astype(np.float64))
        assert (err <= 2 * wl.K * 2.0 ** -24 * mag + 1e-45).all(), (ctx, float((err / np.maximum(mag, 1e-30)).max()))
        assert float((got == ref).mean()) > 0.25, ctx         # a good share of the elements round identically
        st, _ = B.hm_plan_status(g.plan)
        assert st == 0
    # a row index beyond the caller's buffer is skipped and flagged, as in hm_combine
    out_d.fill_(float("nan"))
    hw.combine_forms(B.hm_combine_f32, hw.dev(y)[:ora.total_rows - 3], g.w_d, g.plan, out_d)
    st, _ = B.hm_plan_status(g.plan)
    assert st == B.HM_ERR_CAPACITY and not torch.isnan(out_d).any()


@pytest.mark.parametrize("name,T,H", [("tiny", 1024, 256), ("qwen3", 1500, 2048), ("stress", 600, 7168), ("skew", 777, 90),
                                      ("skew", 300, 77)])
def test_transpose_on_bf16_gradients(hw, oracle, name, T, H):
    """hm_combine_transpose_bf16: the exact product rounded once, so bit for bit against the oracle
    (vector kernel, ragged H, and the element-wise kernel), including products that land on bf16
    ties after the binary32 rounding."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=T)
    gout = W.f32_to_bf16_bits(W.make_output_grads(wl, T=T, H=H))
    for level in (NONE, GPU, NODE):
        ctx = "transpose bf16 %s T=%d H=%d level=%s" % (name, T, H, LEVEL[level])
        print("case:", ctx, flush=True)
        ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        gy_d = torch.full((max(ora.total_rows, 1), H), float("nan"), dtype=torch.bfloat16, device="cuda")
        B.hm_combine_transpose_bf16(hw.to_dev_bf16(gout), g.plan, gy_d[:ora.total_rows])
        ref = oracle.combine_transpose_bf16(gout, ora.row_token, ora.row_weight)
        assert np.array_equal(hw.bf16_to_host(gy_d[:ora.total_rows]), ref), ctx
        st, _ = B.hm_plan_status(g.plan)
        assert st == 0
    # weights chosen so that the fp32 product sits exactly on a bf16 tie while the true product does not
    n_w = 1100
    w = (1.0 + np.arange(97000, 97000 + n_w) * 2.0 ** -23).astype(np.float32).reshape(n_w, 1)
    ids = np.zeros((n_w, 1), np.int32)
    e2r = np.zeros(1, np.int32)
    ora = oracle.plan(ids, w, e2r, 1, 1, GPU)
    g = hw.GpuPlan(ids, w, e2r, 1, 1, GPU)
    gg = W.f32_to_bf16_bits(np.full((n_w, 8), 1.0 + 2.0 ** -7, np.float32))
    gy_d = torch.zeros((n_w, 8), dtype=torch.bfloat16, device="cuda")
    B.hm_combine_transpose_bf16(hw.to_dev_bf16(gg), g.plan, gy_d)
    ref = oracle.combine_transpose_bf16(gg, ora.row_token, ora.row_weight)
    twice = W.f32_to_bf16_bits((w * np.float32(1.0 + 2.0 ** -7)).astype(np.float32))      # rounded twice
    assert (ref[:, :1] != twice).any()                     # the family does contain such traps
    assert np.array_equal(hw.bf16_to_host(gy_d), ref)
    # the same family with negative gradients, with several gradient values per row (products just
    # below, on and above a tie), and scaled down to where the fp32 product is still normal but
    # small (2^-100): the sign of the rounding error decides every one of them
    vals = np.array([1.0 + 2.0 ** -7, -(1.0 + 2.0 ** -7), 1.0 + 3 * 2.0 ** -7, -(1.0 + 5 * 2.0 ** -7),
                     (1.0 + 2.0 ** -7) * 2.0 ** -100, -(1.0 + 3 * 2.0 ** -7) * 2.0 ** -100, 1.5, -1.75], np.float32)
    gg = W.f32_to_bf16_bits(np.tile(vals, (n_w, 1)))
    assert np.array_equal(W.bf16_bits_to_f32(gg[0]), vals)                                # all exact in bf16
    B.hm_combine_transpose_bf16(hw.to_dev_bf16(gg), g.plan, gy_d)
    ref = oracle.combine_transpose_bf16(gg, ora.row_token, ora.row_weight)
    twice = W.f32_to_bf16_bits((w * vals[None, :]).astype(np.float32))
    assert (ref != twice)[:, [0, 1, 4]].any(axis=0).all()      # a trap in the negative and in the small column as well
    assert np.array_equal(hw.bf16_to_host(gy_d), ref)


def test_combine_with_cancelling_terms(hw, oracle):
    """Independent random-sign Y rows: the K terms of an output element can cancel, and an fp32
    accumulator is then only accurate relative to sum_k |w y|, not to the (tiny) result.  Bar: within
    1 bf16 ulp of the oracle, or within the fp32 chain's bound 2K * 2^-24 * sum_k |w y| plus half a
    bf16 ulp of the value returned; the share that needs the second clause is printed."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["qwen3"]
    T, H = 1200, 1024
    r = W.make_routing(wl, T=T)
    rng = np.random.default_rng(4242)
    for level in (NONE, GPU, NODE):
        ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        g = hw.GpuPlan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        y = W.f32_to_bf16_bits(rng.standard_normal((ora.total_rows, H)).astype(np.float32))
        out_d = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine, hw.to_dev_bf16(y), g.w_d, g.plan, out_d)
        got = hw.bf16_to_host(out_d)
        ref = oracle.combine(y, r.topk_weights, ora.slot_row)
        dist = bf16_ulp_distance(got, ref)
        yf = W.bf16_bits_to_f32(y)
        exact = oracle.combine_f32(yf, r.topk_weights, ora.slot_row).astype(np.float64)      # exact sum to 2^-24
        mag = oracle.combine_f32(np.abs(yf), np.abs(r.topk_weights), ora.slot_row).astype(np.float64)
        gotf = W.bf16_bits_to_f64(got)
        half_ulp = np.maximum(np.abs(gotf), 2.0 ** -126) * 2.0 ** -8
        second = np.abs(gotf - exact) <= (2 * wl.K + 1) * 2.0 ** -24 * mag + half_ulp
        ok = (dist <= 1) | second
        print("  level %s: %.4f%% bit-equal, %.4f%% within 1 ulp, %d of %d needed the magnitude clause"
              % (LEVEL[level], 100 * (dist == 0).mean(), 100 * (dist <= 1).mean(), int((dist > 1).sum()), dist.size), flush=True)
        assert ok.all(), (LEVEL[level], int((~ok).sum()))
        assert (dist <= 1).mean() > 0.999


def test_stream_probe_moves_what_it_says(hw):
    """The benchmark's measurement aid (a library of its own, not part of the product): every
    output stream is the XOR of the input streams, ragged tail included, for every launch shape."""
    import torch
    import bench
    rng = np.random.default_rng(3)
    shapes = [(64, 32), (128, 20), (256, 8), (64, 5), (256, 32)]
    for i, (nr, nw, n) in enumerate(((1, 1, 64), (1, 3, 1000), (3, 1, 4097), (7, 2, 130), (16, 16, 65))):
        src = rng.integers(-2 ** 31, 2 ** 31 - 1, (nr, n, 4), dtype=np.int64).astype(np.int32)
        dst_d = torch.full((nw, n, 4), 77, dtype=torch.int32, device="cuda")
        block, waves = shapes[i]
        bench.stream_probe(hw.dev(src), nr, dst_d, nw, block, waves)
        want = np.bitwise_xor.reduce(src, axis=0)
        got = dst_d.cpu().numpy()
        for j in range(nw):
            assert np.array_equal(got[j], want), (nr, nw, n, j)


def test_step_under_hip_graph_capture(hw, oracle):
    """The entry points only enqueue kernels (no allocation, no memset, no synchronisation), so a
    whole step can be captured in a HIP graph and replayed: every replay, with fresh routing and
    activations copied into the captured buffers, must match the oracle."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["dsv3"]
    T, H, level = 2048, 1024, NODE
    cases = []
    for seed_shift in range(4):
        import dataclasses
        r = W.make_routing(dataclasses.replace(wl, seed=500 + seed_shift), T=T)
        x = W.make_activations(dataclasses.replace(wl, seed=600 + seed_shift), T=T, H=H)
        cases.append((r, x))
    r0, x0 = cases[0]
    ids_d, w_d, e2r_d = hw.dev(r0.topk_ids), hw.dev(r0.topk_weights), hw.dev(r0.expert_to_rank)
    x_d = hw.to_dev_bf16(x0)
    plan = B.alloc_plan(T, wl.K, wl.E, wl.nodes, wl.ranks_per_node, level, loads=True)
    packed_d = torch.zeros((plan.row_capacity, H), dtype=torch.bfloat16, device="cuda")
    out_d = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    gy_d = torch.zeros((plan.row_capacity, H), dtype=torch.float32, device="cuda")
    gout_d = hw.dev(W.make_output_grads(wl, T=T, H=H))
    gout = gout_d.cpu().numpy()

    def step():
        B.hm_plan(ids_d, w_d, e2r_d, wl.nodes, wl.ranks_per_node, level, plan=plan)
        B.hm_dispatch_pack(x_d, plan, packed_d)
        B.hm_combine(packed_d, None, plan, out_d)           # the plan's merged weights: the form a step uses
        B.hm_combine_transpose(gout_d, plan, gy_d)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        step()                                              # warm-up outside capture
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for r, x in cases[1:] + cases[:1]:
        ids_d.copy_(hw.dev(r.topk_ids))
        w_d.copy_(hw.dev(r.topk_weights))
        x_d.copy_(hw.to_dev_bf16(x))
        packed_d.zero_()
        out_d.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        ora = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        st, total = B.hm_plan_status(plan)
        assert st == 0 and total == ora.total_rows
        assert np.array_equal(plan.slot_row.cpu().numpy().reshape(T, wl.K), ora.slot_row)
        assert np.array_equal(plan.row_token[:total].cpu().numpy(), ora.row_token)
        packed = hw.bf16_to_host(packed_d[:total])
        assert np.array_equal(packed, oracle.dispatch_pack(x, ora.row_token))
        assert bf16_ulp_distance(hw.bf16_to_host(out_d), oracle.combine(packed, r.topk_weights, ora.slot_row)).max() <= 1
        gref = oracle.combine_transpose(gout, ora.row_token, ora.row_weight)
        assert np.array_equal(gy_d[:total].cpu().numpy().view(np.uint32), gref.view(np.uint32))
        le, lr, ln, _ = oracle.expert_load(r.topk_ids, r.expert_to_rank, wl.nodes, wl.ranks_per_node)
        assert np.array_equal(plan.load_expert.cpu().numpy(), le) and np.array_equal(plan.load_node.cpu().numpy(), ln)


def test_table2_duplication_rates_on_the_gpu(hw):
    """The duplication rates printed in the paper's Table II, from hm_plan's own counts (uniform
    K-subsets of 256 experts, R groups): within 1.5 points of every printed entry."""
    import os
    from paper_2508_09591_amd import binding as B
    golden = os.path.join(os.path.dirname(__file__), "golden", "table2_duplication.txt")
    rows = [tuple(int(v) for v in ln.split()) for ln in open(golden) if ln.strip() and not ln.startswith("#")]
    E, T = 256, 20000
    topo = {32: (4, 8), 16: (2, 8), 8: (1, 8), 4: (1, 4)}
    for R, K, pct in rows:
        ids, w = W.uniform_subset_routing(T, E, K, seed=100 + K)
        nodes, rpn = topo[R]
        g = hw.GpuPlan(ids, w, W.contiguous_placement(E, R), nodes, rpn, GPU)
        assert g.status == 0
        dup = 100.0 * (1.0 - g.total_rows / (T * K))
        assert abs(dup - pct) <= 1.5, (R, K, dup, pct)
