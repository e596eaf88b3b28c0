"""GPU parity for the receiver side of the two-hop exchange: destination tables, the mapped plan,
the normalised merge, and the whole hierarchical layer run stage by stage through the C ABI
with every stage checked against the oracle on the same stage inputs."""
import numpy as np
import pytest

from helpers import GPU, NODE, NONE, bf16_ulp_distance
from paper_2508_09591_amd import workloads as W

pytestmark = pytest.mark.gpu
INTRA, LOCAL = 0, 1


@pytest.fixture(scope="module")
def hw():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_harness
    from paper_2508_09591_amd import binding
    binding.lib()
    return gpu_harness


def _gpu_dest_map(hw, e2r, nodes, rpn, me, stage):
    import torch
    from paper_2508_09591_amd import binding as B
    dm_d = torch.full((e2r.shape[0],), -77, dtype=torch.int32, device="cuda")
    nd_d = torch.full((1,), -77, dtype=torch.int32, device="cuda")
    B.hm_recv_dest_map(hw.dev(e2r), nodes, rpn, me, stage, dm_d, nd_d)
    return dm_d, int(nd_d.item())


def _gpu_plan_mapped(hw, ids, w, dm_d, nd, dedup):
    """hm_plan_mapped with poisoned outputs; returns (plan, status, total_rows, host copies)."""
    import torch
    from paper_2508_09591_amd import binding as B
    rows, K = ids.shape
    plan = B.alloc_plan(rows, K, dm_d.shape[0], 1, 1, B.HM_DEDUP_GPU if dedup else B.HM_DEDUP_NONE, num_dest=nd)
    for name in ("dest_count", "dest_offset", "row_token", "slot_row"):
        getattr(plan, name).fill_(-12345)
    plan.slot_keep.fill_(77)
    plan.status.fill_(55)
    ids_d, w_d = hw.dev(ids), hw.dev(w)
    B.hm_plan_mapped(ids_d, w_d, dm_d, nd, dedup, plan=plan)
    st, total = B.hm_plan_status(plan)
    n = min(total, plan.row_capacity)
    host = dict(dest_count=plan.dest_count[:nd].cpu().numpy(), dest_offset=plan.dest_offset[:nd + 1].cpu().numpy(),
                row_token=plan.row_token[:n].cpu().numpy(), row_weight=plan.row_weight[:n].cpu().numpy(),
                slot_row=plan.slot_row[:rows * K].cpu().numpy().reshape(rows, K),
                slot_keep=plan.slot_keep[:rows * K].cpu().numpy().reshape(rows, K),
                rank_mask=plan.rank_mask[:rows].cpu().numpy().view(np.uint64),
                node_mask=plan.node_mask[:rows].cpu().numpy().view(np.uint32))
    return plan, st, total, host, ids_d, w_d


def _assert_mapped_equal(host, st, total, ora, ctx=""):
    assert st == ora.status and total == ora.total_rows, ctx
    for f in ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "rank_mask"):
        assert np.array_equal(host[f], getattr(ora, f)), (ctx, f)
    assert np.array_equal(host["row_weight"].view(np.uint32), ora.row_weight.view(np.uint32)), (ctx, "row_weight")
    assert not host["node_mask"].any(), ctx


def test_recv_dest_map_parity(hw, oracle):
    rng = np.random.default_rng(21)
    cases = [(4, 8, 256), (8, 8, 256), (2, 2, 16), (1, 8, 64), (3, 5, 45), (4, 8, 3000)]
    for nodes, rpn, E in cases:
        G = nodes * rpn
        for e2r in (W.contiguous_placement(E - E % G, G) if E % G == 0 else rng.integers(0, G, E).astype(np.int32),
                    rng.integers(0, G, E).astype(np.int32)):
            e2r = np.ascontiguousarray(e2r, dtype=np.int32)
            for me in sorted({0, G - 1, int(rng.integers(0, G))}):
                for stage in (INTRA, LOCAL):
                    dm_d, nd = _gpu_dest_map(hw, e2r, nodes, rpn, me, stage)
                    dm, nd_ref = oracle.recv_dest_map(e2r, nodes, rpn, me, stage)
                    assert nd == nd_ref and np.array_equal(dm_d.cpu().numpy(), dm), (nodes, rpn, E, me, stage)
    bad = np.array([0, 9, 1, -4, 3, 3], np.int32)
    for stage in (INTRA, LOCAL):
        dm_d, nd = _gpu_dest_map(hw, bad, 2, 2, 3, stage)
        dm, nd_ref = oracle.recv_dest_map(bad, 2, 2, 3, stage)
        assert nd == nd_ref and np.array_equal(dm_d.cpu().numpy(), dm)


@pytest.mark.parametrize("rows,K,E,nd", [(0, 4, 16, 4), (1, 1, 3, 1), (700, 8, 256, 8), (1300, 5, 40, 7),
                                          (257, 64, 128, 64), (2049, 3, 12, 2)])
def test_plan_mapped_parity(hw, oracle, rows, K, E, nd):
    rng = np.random.default_rng(rows + K)
    ids = rng.integers(0, E, (rows, K), dtype=np.int32)
    w = rng.random((rows, K), dtype=np.float32) + np.float32(0.01)
    for dm in (rng.integers(-1, nd, E).astype(np.int32), rng.integers(0, nd, E).astype(np.int32),
               np.full(E, -1, np.int32)):
        for dedup in (True, False):
            ctx = "mapped rows=%d K=%d E=%d nd=%d dedup=%s" % (rows, K, E, nd, dedup)
            print("case:", ctx, flush=True)
            ora = oracle.plan_mapped(ids, w, dm, nd, dedup)
            plan, st, total, host, _, _ = _gpu_plan_mapped(hw, ids, w, hw.dev(dm), nd, dedup)
            _assert_mapped_equal(host, st, total, ora, ctx)
    if rows > 10:
        # invalid table entries / ids: dropped and flagged, the rest unchanged
        dm = rng.integers(-1, nd, E).astype(np.int32)
        dm[1] = nd + 3
        dm[2] = -2
        ids2 = ids.copy()
        ids2[3, 0] = E
        ids2[7, K - 1] = -1
        ora = oracle.plan_mapped(ids2, w, dm, nd, True)
        plan, st, total, host, _, _ = _gpu_plan_mapped(hw, ids2, w, hw.dev(dm), nd, True)
        assert st == oracle.BAD_ID
        _assert_mapped_equal(host, st, total, ora, "bad entries")


@pytest.mark.parametrize("rows,K,H", [(500, 8, 512), (300, 4, 1000), (129, 6, 100), (64, 8, 7168),
                                       (66000, 6, 520),        # enough segments and rows per token for the wide kernel
                                       (66000, 2, 520)])       # as many segments, about one row per token: the narrow one
def test_combine_mix_parity(hw, oracle, rows, K, H):
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(rows * 3 + H)
    E, nd = 48, 6
    ids = rng.integers(0, E, (rows, K), dtype=np.int32)
    w = rng.random((rows, K), dtype=np.float32) + np.float32(0.05)
    dm = rng.integers(-1, nd, E).astype(np.int32)
    dm[:20] = -1
    ids[0, :] = 3                                       # row 0 has no valid slot at this hop
    for dedup in (True, False):
        ora = oracle.plan_mapped(ids, w, dm, nd, dedup)
        plan, st, total, host, ids_d, w_d = _gpu_plan_mapped(hw, ids, w, hw.dev(dm), nd, dedup)
        _assert_mapped_equal(host, st, total, ora)
        y = W.f32_to_bf16_bits((rng.random((max(total, 1), H)) + 0.5).astype(np.float32))[:total]
        out_d = torch.full((rows, H), float("nan"), dtype=torch.bfloat16, device="cuda")
        y_d = hw.to_dev_bf16(y) if total else torch.zeros((0, H), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine_mix, y_d, w_d, plan, out_d)
        ref = oracle.combine_mix(y, w, ora.slot_row)
        got = hw.bf16_to_host(out_d)
        dist = bf16_ulp_distance(got, ref)
        assert dist.max() <= 1, (rows, K, H, dedup, int(dist.max()))
        assert (dist == 0).mean() > 0.98
        empty = (ora.slot_row < 0).all(axis=1)
        assert empty.any() and not got[empty].any()      # rows without a valid slot give zeros
        # the unnormalised merge on the same plan still matches hm_combine's oracle
        hw.combine_forms(B.hm_combine, y_d, w_d, plan, out_d)
        assert bf16_ulp_distance(hw.bf16_to_host(out_d), oracle.combine(y, w, ora.slot_row)).max() <= 1


@pytest.mark.parametrize("name,T,H,src_local", [("tiny", 1024, 256, 0), ("qwen3", 1500, 512, 3), ("dsv3", 1200, 1024, 5),
                                                 ("skew", 900, 256, 7)])
def test_hierarchical_layer_stage_by_stage(hw, oracle, name, T, H, src_local):
    """node-level dispatch -> intra-node stage -> local experts -> normalised merges -> combine, every
    stage on the GPU through the C ABI and compared with the oracle run on that stage's inputs."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS[name]
    R, K = wl.ranks_per_node, wl.K
    r = W.make_routing(wl, T=T)
    ids, w = r.topk_ids, r.topk_weights
    e2r = r.extras.get("expert_to_rank_swapped", r.expert_to_rank)
    x = W.make_activations(wl, T=T, H=H)
    c = W.make_expert_scales(wl)
    e2r_d = hw.dev(e2r)

    def pack(plan, rows_d, total, H_units):
        out = torch.zeros((max(total, 1), H_units), dtype=torch.bfloat16, device="cuda")
        if total:
            B.hm_dispatch_pack(rows_d, plan, out[:total])
        return out[:total]

    # ---- hop 1 at the source: node-level dedup; activations, ids and weights travel together ----
    o1 = oracle.plan(ids, w, e2r, wl.nodes, R, NODE)
    g1 = hw.GpuPlan(ids, w, e2r, wl.nodes, R, NODE)
    hw.assert_plan_equal(g1, o1, "hop1")
    x_d = hw.to_dev_bf16(x)
    packed1_d = pack(g1.plan, x_d, o1.total_rows, H)
    ids1_d = pack(g1.plan, g1.ids_d.view(torch.bfloat16).view(T, 2 * K), o1.total_rows, 2 * K).contiguous().view(torch.int32).view(-1, K)
    w1_d = pack(g1.plan, g1.w_d.view(torch.bfloat16).view(T, 2 * K), o1.total_rows, 2 * K).contiguous().view(torch.float32).view(-1, K)
    assert np.array_equal(hw.bf16_to_host(packed1_d), oracle.dispatch_pack(x, o1.row_token))
    assert np.array_equal(ids1_d.cpu().numpy(), ids[o1.row_token]) and np.array_equal(w1_d.cpu().numpy(), w[o1.row_token])
    y1_d = torch.zeros_like(packed1_d)

    for d in range(wl.nodes):
        a1, b1 = int(o1.dest_offset[d]), int(o1.dest_offset[d + 1])
        if a1 == b1:
            continue
        rows1_ids, rows1_w = ids1_d[a1:b1].contiguous(), w1_d[a1:b1].contiguous()
        h_ids1, h_w1 = rows1_ids.cpu().numpy(), rows1_w.cpu().numpy()
        # ---- hop 2 on the receiving rank of node d ----
        me = d * R + src_local
        dm2_d, nd2 = _gpu_dest_map(hw, e2r, wl.nodes, R, me, INTRA)
        dm2, nd2_ref = oracle.recv_dest_map(e2r, wl.nodes, R, me, INTRA)
        assert nd2 == nd2_ref and np.array_equal(dm2_d.cpu().numpy(), dm2)
        o2 = oracle.plan_mapped(h_ids1, h_w1, dm2, nd2, True)
        plan2, st, total, host, _, _ = _gpu_plan_mapped(hw, h_ids1, h_w1, dm2_d, nd2, True)
        _assert_mapped_equal(host, st, total, o2, "hop2 node %d" % d)
        seg1 = packed1_d[a1:b1]
        packed2_d = pack(plan2, seg1, total, H)
        ids2_d = pack(plan2, rows1_ids.view(torch.bfloat16).view(-1, 2 * K), total, 2 * K).contiguous().view(torch.int32).view(-1, K)
        w2_d = pack(plan2, rows1_w.view(torch.bfloat16).view(-1, 2 * K), total, 2 * K).contiguous().view(torch.float32).view(-1, K)
        assert np.array_equal(hw.bf16_to_host(packed2_d), oracle.dispatch_pack(hw.bf16_to_host(seg1), o2.row_token))
        y2_d = torch.zeros_like(packed2_d)
        for lr in range(R):
            a2, b2 = int(o2.dest_offset[lr]), int(o2.dest_offset[lr + 1])
            if a2 == b2:
                continue
            g = d * R + lr
            rows2_ids, rows2_w = ids2_d[a2:b2].contiguous(), w2_d[a2:b2].contiguous()
            h_ids2, h_w2 = rows2_ids.cpu().numpy(), rows2_w.cpu().numpy()
            # ---- local experts on rank g: expert-contiguous expansion, experts, normalised merge ----
            dm3_d, nd3 = _gpu_dest_map(hw, e2r, wl.nodes, R, g, LOCAL)
            dm3, nd3_ref = oracle.recv_dest_map(e2r, wl.nodes, R, g, LOCAL)
            assert nd3 == nd3_ref and np.array_equal(dm3_d.cpu().numpy(), dm3)
            if nd3 == 0:
                continue
            o3 = oracle.plan_mapped(h_ids2, h_w2, dm3, nd3, False)
            plan3, st, total3, host3, _, w3_d = _gpu_plan_mapped(hw, h_ids2, h_w2, dm3_d, nd3, False)
            _assert_mapped_equal(host3, st, total3, o3, "experts rank %d" % g)
            xin_d = pack(plan3, packed2_d[a2:b2], total3, H)
            xin = hw.bf16_to_host(xin_d)
            assert np.array_equal(xin, oracle.dispatch_pack(hw.bf16_to_host(packed2_d[a2:b2]), o3.row_token))
            yexp = np.zeros_like(xin)                                  # harness: expert e returns c[e] * x
            for j, e in enumerate(np.flatnonzero(e2r == g)):
                s3 = slice(o3.dest_offset[j], o3.dest_offset[j + 1])
                yexp[s3] = W.f32_to_bf16_bits(c[e] * W.bf16_bits_to_f32(xin[s3]))
            out3_d = torch.zeros((b2 - a2, H), dtype=torch.bfloat16, device="cuda")
            hw.combine_forms(B.hm_combine_mix, hw.to_dev_bf16(yexp), w3_d, plan3, out3_d)
            assert bf16_ulp_distance(hw.bf16_to_host(out3_d), oracle.combine_mix(yexp, h_w2, o3.slot_row)).max() <= 1
            y2_d[a2:b2] = out3_d
        # ---- merge on the receiving rank before the rows go back to the source ----
        out2_d = torch.zeros((b1 - a1, H), dtype=torch.bfloat16, device="cuda")
        hw.combine_forms(B.hm_combine_mix, y2_d, hw.dev(h_w1), plan2, out2_d)
        assert bf16_ulp_distance(hw.bf16_to_host(out2_d), oracle.combine_mix(hw.bf16_to_host(y2_d), h_w1, o2.slot_row)).max() <= 1
        y1_d[a1:b1] = out2_d
    # ---- final combine at the source ----
    out_d = torch.zeros((T, H), dtype=torch.bfloat16, device="cuda")
    hw.combine_forms(B.hm_combine, y1_d, g1.w_d, g1.plan, out_d)
    out = hw.bf16_to_host(out_d)
    assert bf16_ulp_distance(out, oracle.combine(hw.bf16_to_host(y1_d), w, o1.slot_row)).max() <= 1
    expect = (w.astype(np.float64) * c[ids].astype(np.float64)).sum(1)[:, None] * W.bf16_bits_to_f64(x)
    # four bf16 roundings on the way (expert output, two merges, final combine), each <= 2^-8 relative
    assert np.all(np.abs(W.bf16_bits_to_f64(out) - expect) <= 4 * 2.0 ** -8 * np.abs(expect) + 1e-30)


def test_level_dest_map_parity(hw, oracle):
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(91)
    for _ in range(60):
        G = int(rng.choice([4, 8, 16, 32, 64, 12]))
        divs = [u for u in range(1, G + 1) if G % u == 0]
        parent = int(rng.choice(divs))
        child = int(rng.choice([u for u in divs if u % parent == 0]))
        E = int(rng.integers(1, 2500))
        e2r = rng.integers(0, G, E).astype(np.int32)
        if E > 3:
            e2r[2] = G + 4
        me = int(rng.integers(0, G))
        dm_d = torch.full((E,), -77, dtype=torch.int32, device="cuda")
        nd_d = torch.full((1,), -77, dtype=torch.int32, device="cuda")
        B.hm_level_dest_map(hw.dev(e2r), G, me, parent, child, dm_d, nd_d)
        dm, nd = oracle.level_dest_map(e2r, G, me, parent, child)
        assert int(nd_d.item()) == nd and np.array_equal(dm_d.cpu().numpy(), dm), (G, parent, child, E, me)


@pytest.mark.parametrize("name,chain,T,H", [("qwen3", [4, 8, 16, 32], 1000, 256), ("dsv3", [2, 8, 32], 800, 512)])
def test_d_dimensional_exchange_hop_by_hop(hw, oracle, name, chain, T, H):
    """The paper's 4-level hierarchy (U = [1,4,8,16] on 32 GPUs) and a 3-level one: every hop planned,
    packed and merged on the GPU through the C ABI, each compared with the oracle on the same hop
    inputs; at the end every rank holds the one-hop exchange's tokens and the output is the layer's."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS[name]
    G, K = wl.G, wl.K
    r = W.make_routing(wl, T=T)
    ids, w, e2r = r.topk_ids, r.topk_weights, r.expert_to_rank
    x = W.make_activations(wl, T=T, H=H)
    c = W.make_expert_scales(wl)
    e2r_d = hw.dev(e2r)
    delivered = {}

    def pack(plan, rows_d, total, units):
        out = torch.zeros((max(total, 1), units), dtype=torch.bfloat16, device="cuda")
        if total:
            B.hm_dispatch_pack(rows_d, plan, out[:total])
        return out[:total]

    def hop(level, rank, tokens, rows_d, ids_d, w_d):
        parent = 1 if level == 0 else chain[level - 1]
        child = chain[level]
        n = tokens.shape[0]
        dm_d = torch.empty(wl.E, dtype=torch.int32, device="cuda")
        nd_d = torch.empty(1, dtype=torch.int32, device="cuda")
        B.hm_level_dest_map(e2r_d, G, rank, parent, child, dm_d, nd_d)
        nd = int(nd_d.item())
        dm, nd_ref = oracle.level_dest_map(e2r, G, rank, parent, child)
        assert nd == nd_ref and np.array_equal(dm_d.cpu().numpy(), dm)
        h_ids, h_w = ids_d.cpu().numpy(), w_d.cpu().numpy()
        assert np.array_equal(h_ids, ids[tokens]) and np.array_equal(h_w, w[tokens])       # metadata travelled intact
        ora = oracle.plan_mapped(h_ids, h_w, dm, nd, True)
        plan, st, total, host, _, _ = _gpu_plan_mapped(hw, h_ids, h_w, dm_d, nd, True)
        _assert_mapped_equal(host, st, total, ora, "level %d rank %d" % (level, rank))
        packed_d = pack(plan, rows_d, total, H)
        assert np.array_equal(hw.bf16_to_host(packed_d), oracle.dispatch_pack(hw.bf16_to_host(rows_d), ora.row_token))
        pid_d = pack(plan, ids_d.view(torch.bfloat16).view(n, 2 * K), total, 2 * K).contiguous().view(torch.int32).view(-1, K)
        pw_d = pack(plan, w_d.view(torch.bfloat16).view(n, 2 * K), total, 2 * K).contiguous().view(torch.float32).view(-1, K)
        y_d = torch.zeros_like(packed_d)
        for j in range(nd):
            a, b = int(ora.dest_offset[j]), int(ora.dest_offset[j + 1])
            if a == b:
                continue
            sub_tokens = tokens[ora.row_token[a:b]]
            peer = (rank // (G // parent)) * (G // parent) + j * (G // child) + rank % (G // child)
            sub_rows, sub_ids, sub_w = packed_d[a:b].contiguous(), pid_d[a:b].contiguous(), pw_d[a:b].contiguous()
            if level == len(chain) - 1:
                delivered[peer] = sub_tokens
                dm3_d, nd3 = _gpu_dest_map(hw, e2r, 1, G, peer, LOCAL)
                dm3, _ = oracle.recv_dest_map(e2r, 1, G, peer, LOCAL)
                h2i, h2w = sub_ids.cpu().numpy(), sub_w.cpu().numpy()
                o3 = oracle.plan_mapped(h2i, h2w, dm3, nd3, False)
                plan3, st3, tot3, host3, _, w3_d = _gpu_plan_mapped(hw, h2i, h2w, dm3_d, nd3, False)
                _assert_mapped_equal(host3, st3, tot3, o3, "experts rank %d" % peer)
                xin = hw.bf16_to_host(pack(plan3, sub_rows, tot3, H))
                yexp = np.zeros_like(xin)
                for jj, e in enumerate(np.flatnonzero(e2r == peer)):
                    s3 = slice(o3.dest_offset[jj], o3.dest_offset[jj + 1])
                    yexp[s3] = W.f32_to_bf16_bits(c[e] * W.bf16_bits_to_f32(xin[s3]))
                res_d = torch.zeros((b - a, H), dtype=torch.bfloat16, device="cuda")
                hw.combine_forms(B.hm_combine_mix, hw.to_dev_bf16(yexp), w3_d, plan3, res_d)
                assert bf16_ulp_distance(hw.bf16_to_host(res_d), oracle.combine_mix(yexp, h2w, o3.slot_row)).max() <= 1
                y_d[a:b] = res_d
            else:
                y_d[a:b] = hop(level + 1, peer, sub_tokens, sub_rows, sub_ids, sub_w)
        out_d = torch.zeros((n, H), dtype=torch.bfloat16, device="cuda")
        if level == 0:
            hw.combine_forms(B.hm_combine, y_d, w_d, plan, out_d)
            ref = oracle.combine(hw.bf16_to_host(y_d), h_w, ora.slot_row)
        else:
            hw.combine_forms(B.hm_combine_mix, y_d, w_d, plan, out_d)
            ref = oracle.combine_mix(hw.bf16_to_host(y_d), h_w, ora.slot_row)
        assert bf16_ulp_distance(hw.bf16_to_host(out_d), ref).max() <= 1
        return out_d

    out_d = hop(0, 5, np.arange(T), hw.to_dev_bf16(x), hw.dev(ids), hw.dev(w))
    flat = oracle.plan(ids, w, e2r, wl.nodes, wl.ranks_per_node, GPU)
    for g in range(G):
        want = flat.row_token[flat.dest_offset[g]:flat.dest_offset[g + 1]]
        assert np.array_equal(delivered.get(g, np.zeros(0, np.int64)), want), g
    expect = (w.astype(np.float64) * c[ids].astype(np.float64)).sum(1)[:, None] * W.bf16_bits_to_f64(x)
    got = W.bf16_bits_to_f64(hw.bf16_to_host(out_d))
    assert np.all(np.abs(got - expect) <= (len(chain) + 2) * 2.0 ** -8 * np.abs(expect) + 1e-30)
