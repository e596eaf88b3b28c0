"""Pins for the receiver side of the two-hop exchange (HD2): destination maps, the mapped plan,
the normalised merge, and the property that makes the hierarchy correct -- two deduplicated hops
deliver exactly what the one-hop exchange delivers, and the merges on the way back reproduce
the MoE layer's output.  CPU only."""
import itertools
from fractions import Fraction

import numpy as np
import pytest

from helpers import GPU, NODE, NONE, bf16_ulp_distance, brute_plan_mapped, exact_round_to_bf16
from paper_2508_09591_amd import workloads as W

INTRA, LOCAL = 0, 1


def test_dest_maps_against_numpy(oracle):
    rng = np.random.default_rng(4)
    for _ in range(50):
        nodes, rpn = int(rng.integers(1, 5)), int(rng.integers(1, 9))
        G = nodes * rpn
        E = G * int(rng.integers(1, 5))
        e2r = rng.integers(0, G, E).astype(np.int32)
        me = int(rng.integers(0, G))
        dm, nd = oracle.recv_dest_map(e2r, nodes, rpn, me, INTRA)
        assert nd == rpn
        assert np.array_equal(dm, np.where(e2r // rpn == me // rpn, e2r % rpn, -1))
        dm, nd = oracle.recv_dest_map(e2r, nodes, rpn, me, LOCAL)
        mine = e2r == me
        assert nd == int(mine.sum())
        assert np.array_equal(dm, np.where(mine, np.cumsum(mine) - 1, -1))
    # an invalid placement entry is marked, not mapped
    dm, nd = oracle.recv_dest_map(np.array([0, 5, 1, -1], np.int32), 1, 2, 0, INTRA)
    assert dm.tolist() == [0, -2, 1, -2]


def _assert_mapped_equals_brute(oracle, ids, w, dm, nd, dedup):
    p = oracle.plan_mapped(ids, w, dm, nd, dedup)
    b = brute_plan_mapped(ids, w, dm, nd, dedup)
    ctx = (ids.tolist(), dm.tolist(), nd, dedup)
    assert p.status == 0, ctx
    assert p.dest_count.tolist() == b["dest_count"], ctx
    assert p.dest_offset.tolist() == [0] + list(itertools.accumulate(b["dest_count"])), ctx
    assert p.row_token.tolist() == b["row_token"], ctx
    assert p.slot_row.tolist() == b["slot_row"], ctx
    assert p.slot_keep.tolist() == b["slot_keep"], ctx
    assert [float(v) for v in p.row_weight] == [float(v) for v in b["row_weight"]], ctx
    assert [int(v) for v in p.rank_mask] == b["dest_mask"], ctx


def test_mapped_plan_exhaustive_and_random(oracle):
    rng = np.random.default_rng(8)
    E = 4
    maps = [(np.array([0, 0, 1, -1], np.int32), 2), (np.array([-1, 1, -1, 0], np.int32), 2),
            (np.array([2, 0, 1, 0], np.int32), 3), (np.array([-1, -1, -1, -1], np.int32), 1)]
    for T, K in ((2, 2), (2, 3)):
        for table in itertools.product(range(E), repeat=T * K):
            ids = np.array(table, np.int32).reshape(T, K)
            w = rng.random((T, K), dtype=np.float32)
            for dm, nd in maps:
                for dedup in (True, False):
                    _assert_mapped_equals_brute(oracle, ids, w, dm, nd, dedup)
    for _ in range(200):
        E = int(rng.integers(2, 40))
        nd = int(rng.integers(1, 9))
        dm = rng.integers(-1, nd, E).astype(np.int32)
        T, K = int(rng.integers(0, 10)), int(rng.integers(1, 6))
        ids = rng.integers(0, E, (T, K), dtype=np.int32)
        w = rng.random((T, K), dtype=np.float32)
        for dedup in (True, False):
            _assert_mapped_equals_brute(oracle, ids, w, dm, nd, dedup)
    # invalid table entries and ids are dropped and flagged; -1 entries are dropped silently
    ids = np.array([[0, 1, 2], [3, 7, 1]], np.int32)
    w = np.ones((2, 3), np.float32)
    p = oracle.plan_mapped(ids, w, np.array([0, -1, 5, 1], np.int32), 2, True)
    assert p.status == oracle.BAD_ID and p.slot_row.tolist() == [[0, -1, -1], [1, -1, -1]]
    p = oracle.plan_mapped(ids[:1], w[:1], np.array([0, -1, 1, 1], np.int32), 2, True)
    assert p.status == 0 and p.slot_row.tolist() == [[0, -1, 1]]


@pytest.mark.parametrize("name", ["tiny", "qwen3", "dsv3"])
def test_sender_plans_are_mapped_plans(oracle, name):
    """hmo_plan at the three levels == hmo_plan_mapped with the corresponding table (two functions
    written separately)."""
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=700)
    e2r = r.expert_to_rank
    for level, dm, nd, dedup in ((NONE, e2r, wl.G, False), (GPU, e2r, wl.G, True),
                                 (NODE, e2r // wl.ranks_per_node, wl.nodes, True)):
        a = oracle.plan(r.topk_ids, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, level)
        b = oracle.plan_mapped(r.topk_ids, r.topk_weights, dm, nd, dedup)
        for f in ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "row_weight"):
            assert np.array_equal(getattr(a, f), getattr(b, f)), (level, f)
        want_mask = a.node_mask.astype(np.uint64) if level == NODE else a.rank_mask
        assert np.array_equal(b.rank_mask, want_mask)


def _two_hop_delivery(oracle, wl, r, src_local):
    """Token lists per (destination rank) and per (rank, expert) produced by node-level dedup, then
    the receiver's intra-node stage, then the local-expert stage."""
    ids, w, e2r = r.topk_ids, r.topk_weights, r.expert_to_rank
    R = wl.ranks_per_node
    p1 = oracle.plan(ids, w, e2r, wl.nodes, R, NODE)
    per_rank, per_expert, forwarded = {}, {}, 0
    for d in range(wl.nodes):
        tok1 = p1.row_token[p1.dest_offset[d]:p1.dest_offset[d + 1]]          # tokens behind the rows node d receives
        recv_rank = d * R + src_local                                          # same local index as the sender
        dm, nd = oracle.recv_dest_map(e2r, wl.nodes, R, recv_rank, INTRA)
        p2 = oracle.plan_mapped(ids[tok1], w[tok1], dm, nd, True)
        assert p2.status == 0
        assert (p2.slot_keep.sum(1) >= 1).all()                               # every received row is needed somewhere in the node
        forwarded += p2.total_rows - int(p2.dest_count[src_local])            # copies that leave the receiving GPU
        for lr in range(R):
            tok2 = tok1[p2.row_token[p2.dest_offset[lr]:p2.dest_offset[lr + 1]]]
            g = d * R + lr
            per_rank[g] = tok2
            dm3, nd3 = oracle.recv_dest_map(e2r, wl.nodes, R, g, LOCAL)
            p3 = oracle.plan_mapped(ids[tok2], w[tok2], dm3, nd3, False)
            experts_here = np.flatnonzero(e2r == g)
            for j, e in enumerate(experts_here):
                per_expert[int(e)] = tok2[p3.row_token[p3.dest_offset[j]:p3.dest_offset[j + 1]]]
    return p1, per_rank, per_expert, forwarded


@pytest.mark.parametrize("name", ["tiny", "qwen3", "dsv3", "skew"])
def test_two_hops_deliver_what_one_hop_delivers(oracle, name):
    """Section III-A: the hops of the hierarchical exchange together 'complete the functionality of
    the original AlltoAll' -- every rank ends up with exactly the tokens the one-hop deduplicated
    exchange gives it, and every expert with exactly its tokens."""
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=600)
    e2r = r.extras.get("expert_to_rank_swapped", r.expert_to_rank)
    r.expert_to_rank = e2r
    p1, per_rank, per_expert, forwarded = _two_hop_delivery(oracle, wl, r, src_local=1)
    flat = oracle.plan(r.topk_ids, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, GPU)
    for g in range(wl.G):
        assert np.array_equal(per_rank[g], flat.row_token[flat.dest_offset[g]:flat.dest_offset[g + 1]]), g
    for e in range(wl.E):
        want = np.flatnonzero((r.topk_ids == e).any(axis=1))                   # tokens that selected expert e, ascending
        assert np.array_equal(per_expert[e], want), e
    # traffic bookkeeping: first hop carries rows(node); the second hop carries the rest of rows(gpu)
    # except the copies that are already on the receiving GPU
    assert forwarded <= flat.total_rows
    assert p1.total_rows <= flat.total_rows


def test_fig5_two_more_intra_node_copies(oracle):
    """2 nodes x 8 GPUs, one expert per GPU.  Two tokens on node 0 pick experts on GPUs {8,9} and
    {8,10}: HD1 sends four copies across nodes, HD2 two, and HD2 then forwards 'two more' inside
    node 1 (from GPU 8, which already holds its own copy of both)."""
    class WL:  # minimal stand-in for the helper
        nodes, ranks_per_node, G, E = 2, 8, 16, 16
    ids = np.array([[8, 9], [8, 10]], np.int32)
    w = np.full((2, 2), 0.5, np.float32)
    r = W.Routing(ids, w, W.contiguous_placement(16, 16))
    p1, per_rank, per_expert, forwarded = _two_hop_delivery(oracle, WL, r, src_local=0)
    flat = oracle.plan(ids, w, r.expert_to_rank, 2, 8, GPU)
    assert int(flat.dest_count[8:].sum()) == 4 and int(p1.dest_count[1]) == 2 and forwarded == 2
    assert per_rank[8].tolist() == [0, 1] and per_rank[9].tolist() == [0] and per_rank[10].tolist() == [1]


def test_combine_mix_exact_rational(oracle):
    rng = np.random.default_rng(12)
    rows, K, H, E = 6, 4, 5, 10
    ids = rng.integers(0, E, (rows, K), dtype=np.int32)
    w = rng.random((rows, K), dtype=np.float32) + np.float32(0.1)
    dm = np.array([0, 0, 1, -1, 2, 2, -1, 1, 0, -1], np.int32)
    for dedup in (True, False):
        p = oracle.plan_mapped(ids, w, dm, 3, dedup)
        y = W.f32_to_bf16_bits((rng.random((max(p.total_rows, 1), H)) + 0.5).astype(np.float32))
        out = oracle.combine_mix(y, w, p.slot_row)
        yf = W.bf16_bits_to_f64(y)
        for i in range(rows):
            ks = [k for k in range(K) if p.slot_row[i, k] >= 0]
            for j in range(H):
                if not ks:
                    assert out[i, j] == 0
                    continue
                num = sum(Fraction(float(w[i, k])) * Fraction(float(yf[p.slot_row[i, k], j])) for k in ks)
                den = sum(Fraction(float(w[i, k])) for k in ks)
                assert bf16_ulp_distance(np.array([out[i, j]]), np.array([exact_round_to_bf16(num / den)]))[0] == 0
    # a mixture of identical rows is that row
    y = W.f32_to_bf16_bits(rng.standard_normal((1, 64)).astype(np.float32))
    sr = np.zeros((3, 4), np.int32)
    out = oracle.combine_mix(y, rng.random((3, 4), dtype=np.float32) + np.float32(0.01), sr)
    assert bf16_ulp_distance(out, np.repeat(y, 3, 0)).max() == 0


def hierarchical_layer(oracle, wl, ids, w, e2r, x, c, src_local):
    """The whole two-hop layer on the oracle: node-level dispatch -> intra-node stage -> local
    experts f_e(x) = c_e x -> normalised merges back through both hops -> final combine."""
    R = wl.ranks_per_node
    p1 = oracle.plan(ids, w, e2r, wl.nodes, R, NODE)
    packed1 = oracle.dispatch_pack(x, p1.row_token)
    y1 = np.zeros_like(packed1)
    for d in range(wl.nodes):
        seg1 = slice(p1.dest_offset[d], p1.dest_offset[d + 1])
        tok1 = p1.row_token[seg1]
        dm, nd = oracle.recv_dest_map(e2r, wl.nodes, R, d * R + src_local, INTRA)
        p2 = oracle.plan_mapped(ids[tok1], w[tok1], dm, nd, True)
        packed2 = oracle.dispatch_pack(packed1[seg1], p2.row_token)
        y2 = np.zeros_like(packed2)
        for lr in range(R):
            seg2 = slice(p2.dest_offset[lr], p2.dest_offset[lr + 1])
            tok2 = tok1[p2.row_token[seg2]]
            g = d * R + lr
            dm3, nd3 = oracle.recv_dest_map(e2r, wl.nodes, R, g, LOCAL)
            p3 = oracle.plan_mapped(ids[tok2], w[tok2], dm3, nd3, False)
            xin = oracle.dispatch_pack(packed2[seg2], p3.row_token)            # expert-contiguous inputs
            yexp = np.zeros_like(xin)
            for j, e in enumerate(np.flatnonzero(e2r == g)):
                s3 = slice(p3.dest_offset[j], p3.dest_offset[j + 1])
                yexp[s3] = W.f32_to_bf16_bits(c[e] * W.bf16_bits_to_f32(xin[s3]))
            y2[seg2] = oracle.combine_mix(yexp, w[tok2], p3.slot_row)          # one row per row received by g
        y1[seg1] = oracle.combine_mix(y2, w[tok1], p2.slot_row)                # one row per row received by the node
    return oracle.combine(y1, w, p1.slot_row)


@pytest.mark.parametrize("name,src_local", [("tiny", 0), ("qwen3", 3), ("dsv3", 5)])
def test_hierarchical_round_trip_reproduces_the_layer(oracle, name, src_local):
    """The two-hop layer with experts f_e(x) = c_e x equals (sum_k w_k c_{e_k}) x, the MoE layer's
    output, and with identity experts it returns its input."""
    wl = W.WORKLOADS[name]
    T, H = 300, 48
    r = W.make_routing(wl, T=T)
    ids, w, e2r = r.topk_ids, r.topk_weights, r.expert_to_rank
    x = W.make_activations(wl, T=T, H=H)
    c = W.make_expert_scales(wl)
    out = W.bf16_bits_to_f64(hierarchical_layer(oracle, wl, ids, w, e2r, x, c, src_local))
    expect = (w.astype(np.float64) * c[ids].astype(np.float64)).sum(1)[:, None] * W.bf16_bits_to_f64(x)
    # four bf16 roundings on the way (expert output, two merges, final combine), each at most half an
    # ulp = 2^-8 relative
    assert np.all(np.abs(out - expect) <= 4 * 2.0 ** -8 * np.abs(expect) + 1e-30)
    same = hierarchical_layer(oracle, wl, ids, w, e2r, x, np.ones_like(c), src_local)
    assert bf16_ulp_distance(same, x).max() == 0


# ---- d-dimensional exchange: any chain of group cuts ------------------------------------------------
def test_level_dest_map_against_numpy(oracle):
    rng = np.random.default_rng(31)
    for _ in range(80):
        G = int(rng.choice([4, 8, 16, 32, 64, 12]))
        divs = [u for u in range(1, G + 1) if G % u == 0]
        parent = int(rng.choice(divs))
        child = int(rng.choice([u for u in divs if u % parent == 0]))
        E = G * int(rng.integers(1, 4))
        e2r = rng.integers(0, G, E).astype(np.int32)
        me = int(rng.integers(0, G))
        dm, nd = oracle.level_dest_map(e2r, G, me, parent, child)
        in_parent = e2r // (G // parent) == me // (G // parent)
        want = np.where(in_parent, (e2r // (G // child)) % (child // parent), -1)
        assert nd == child // parent and np.array_equal(dm, want)
    # the two-level special cases are the tables of hmo_recv_dest_map and of the node-level sender plan
    e2r = W.contiguous_placement(256, 32)
    a, na = oracle.level_dest_map(e2r, 32, 13, 4, 32)
    b, nb = oracle.recv_dest_map(e2r, 4, 8, 13, INTRA)
    assert na == nb and np.array_equal(a, b)
    a, na = oracle.level_dest_map(e2r, 32, 13, 1, 4)
    assert na == 4 and np.array_equal(a, e2r // 8)


def multi_hop_layer(oracle, ids, w, e2r, G, chain, x, c, holder=0):
    """The d-dimensional exchange on the oracle for one source rank: `chain` = [U[1], .., U[d-1], G].
    Returns (per-rank token lists, layer output).  Each hop plans with the table of its cut, packs,
    hands every child group's rows to a rank of that group, and merges what comes back."""
    delivered = {}

    def hop(level, rank, tokens, rows):
        """rows: bf16 rows held by `rank` for `tokens`; returns the merged result rows."""
        parent = 1 if level == 0 else chain[level - 1]
        child = chain[level]
        dm, nd = oracle.level_dest_map(e2r, G, rank, parent, child)
        p = oracle.plan_mapped(ids[tokens], w[tokens], dm, nd, True)
        packed = oracle.dispatch_pack(rows, p.row_token)
        y = np.zeros_like(packed)
        for j in range(nd):
            seg = slice(p.dest_offset[j], p.dest_offset[j + 1])
            if seg.start == seg.stop:
                continue
            sub_tokens = tokens[p.row_token[seg]]
            # a rank of child group j (inside my parent group): same offset inside the group as mine
            first = (rank // (G // parent)) * (G // parent) + j * (G // child)
            peer = first + rank % (G // child)
            if level == len(chain) - 1:                      # child groups are single ranks: local experts
                delivered[peer] = sub_tokens
                dm3, nd3 = oracle.recv_dest_map(e2r, 1, G, peer, LOCAL)
                p3 = oracle.plan_mapped(ids[sub_tokens], w[sub_tokens], dm3, nd3, False)
                xin = oracle.dispatch_pack(packed[seg], p3.row_token)
                yexp = np.zeros_like(xin)
                for jj, e in enumerate(np.flatnonzero(e2r == peer)):
                    s3 = slice(p3.dest_offset[jj], p3.dest_offset[jj + 1])
                    yexp[s3] = W.f32_to_bf16_bits(c[e] * W.bf16_bits_to_f32(xin[s3]))
                y[seg] = oracle.combine_mix(yexp, w[sub_tokens], p3.slot_row)
            else:
                y[seg] = hop(level + 1, peer, sub_tokens, packed[seg])
        if level == 0:
            return oracle.combine(y, w[tokens], p.slot_row)
        return oracle.combine_mix(y, w[tokens], p.slot_row)

    out = hop(0, holder, np.arange(ids.shape[0]), x)
    return delivered, out


@pytest.mark.parametrize("name,chain", [("qwen3", [4, 8, 16, 32]), ("dsv3", [4, 32]), ("dsv3", [2, 8, 32]),
                                        ("tiny", [2, 4]), ("skew", [32]), ("qwen3", [8, 32])])
def test_d_dimensional_exchange_delivers_and_reproduces_the_layer(oracle, name, chain):
    """HDd for any chain of cuts (the paper's 4-level U = [1,4,8,16] on 32 GPUs included): every rank
    receives exactly the tokens of the one-hop deduplicated exchange, and the merged result is the
    MoE layer's output."""
    wl = W.WORKLOADS[name]
    T, H = 260, 40
    r = W.make_routing(wl, T=T)
    ids, w = r.topk_ids, r.topk_weights
    e2r = r.extras.get("expert_to_rank_swapped", r.expert_to_rank)
    x = W.make_activations(wl, T=T, H=H)
    c = W.make_expert_scales(wl)
    delivered, out = multi_hop_layer(oracle, ids, w, e2r, wl.G, chain, x, c, holder=wl.G - 1)
    flat = oracle.plan(ids, w, e2r, wl.nodes, wl.ranks_per_node, GPU)
    for g in range(wl.G):
        want = flat.row_token[flat.dest_offset[g]:flat.dest_offset[g + 1]]
        assert np.array_equal(delivered.get(g, np.zeros(0, np.int64)), want), (chain, g)
    expect = (w.astype(np.float64) * c[ids].astype(np.float64)).sum(1)[:, None] * W.bf16_bits_to_f64(x)
    n_roundings = len(chain) + 2                              # expert output, one merge per hop, final combine
    assert np.all(np.abs(W.bf16_bits_to_f64(out) - expect) <= n_roundings * 2.0 ** -8 * np.abs(expect) + 1e-30)
    _, same = multi_hop_layer(oracle, ids, w, e2r, wl.G, chain, x, np.ones_like(c), holder=0)
    assert bf16_ulp_distance(same, x).max() == 0
