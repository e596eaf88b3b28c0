"""Pins for the oracle's plan / load functions against what the paper and the mathematics fix.

CPU only.  Every check compares the oracle with something that is not the oracle: the set
definition of Eq.(7) by brute force, numpy's bincount / stable argsort, closed forms for
uniformly random K-subsets, the duplication rates printed in Table II, the Fig.5 narrative
and the swap counts printed for Fig.7.
"""
import itertools
import math
import os

import numpy as np
import pytest

from helpers import GPU, NODE, NONE, brute_plan, group_counts_by_sets
from paper_2508_09591_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _assert_plan_equals_brute(oracle, ids, w, e2r, nodes, rpn, level):
    p = oracle.plan(ids, w, e2r, nodes, rpn, level)
    b = brute_plan(ids, w, e2r, nodes, rpn, level)
    ctx = (ids.tolist(), e2r.tolist(), nodes, rpn, level)
    assert p.status == 0, ctx
    assert p.num_dest == b["num_dest"], ctx
    assert p.dest_count.tolist() == b["dest_count"], ctx
    assert p.dest_offset.tolist() == [0] + list(itertools.accumulate(b["dest_count"])), ctx
    assert p.row_token.tolist() == b["row_token"], ctx
    assert p.slot_row.tolist() == b["slot_row"], ctx
    assert p.slot_keep.tolist() == b["slot_keep"], ctx
    assert [float(x) for x in p.row_weight] == [float(x) for x in b["row_weight"]], ctx
    assert [int(x) for x in p.rank_mask] == b["rank_mask"], ctx
    assert [int(x) for x in p.node_mask] == b["node_mask"], ctx


# ---- Eq.(7) by exhaustive enumeration ------------------------------------------------------
@pytest.mark.parametrize("T,K", [(1, 2), (2, 2), (3, 2), (2, 3)])
def test_exhaustive_tiny_tables_match_set_definition(oracle, T, K):
    E = 4
    rng = np.random.default_rng(7)
    placements = {
        (1, 2): [np.array([0, 0, 1, 1]), np.array([1, 0, 1, 0])],
        (2, 1): [np.array([0, 0, 1, 1]), np.array([0, 1, 1, 0])],
        (2, 2): [np.array([0, 1, 2, 3]), np.array([3, 1, 0, 2]), np.array([0, 0, 3, 3])],
        (1, 4): [np.array([0, 1, 2, 3])],
    }
    n_checked = 0
    for table in itertools.product(range(E), repeat=T * K):
        ids = np.array(table, dtype=np.int32).reshape(T, K)
        w = rng.random((T, K), dtype=np.float32)
        for (nodes, rpn), e2rs in placements.items():
            for e2r in e2rs:
                for level in (NONE, GPU, NODE):
                    _assert_plan_equals_brute(oracle, ids, w, e2r.astype(np.int32), nodes, rpn, level)
                    n_checked += 1
    assert n_checked == (E ** (T * K)) * 8 * 3


def test_random_small_tables_match_set_definition(oracle):
    rng = np.random.default_rng(11)
    for _ in range(300):
        nodes = int(rng.integers(1, 5))
        rpn = int(rng.integers(1, 5))
        G = nodes * rpn
        E = G * int(rng.integers(1, 4))
        K = int(rng.integers(1, 6))
        T = int(rng.integers(0, 12))
        ids = rng.integers(0, E, size=(T, K), dtype=np.int32)     # repeated experts allowed
        w = rng.random((T, K), dtype=np.float32)
        e2r = rng.integers(0, G, size=E, dtype=np.int32)           # arbitrary, uneven placement
        for level in (NONE, GPU, NODE):
            _assert_plan_equals_brute(oracle, ids, w, e2r, nodes, rpn, level)


def test_dropped_slots_are_skipped_without_error(oracle):
    """The id -1 marks a slot a capacity-limited router dropped: it takes no part in the plan, the
    loads or the combine, and it is not an error."""
    rng = np.random.default_rng(19)
    for _ in range(200):
        nodes, rpn = int(rng.integers(1, 4)), int(rng.integers(1, 4))
        G = nodes * rpn
        E = G * int(rng.integers(1, 4))
        K, T = int(rng.integers(1, 6)), int(rng.integers(1, 10))
        ids = rng.integers(0, E, size=(T, K), dtype=np.int32)
        ids[rng.random((T, K)) < 0.3] = -1
        w = rng.random((T, K), dtype=np.float32)
        e2r = rng.integers(0, G, size=E, dtype=np.int32)
        for level in (NONE, GPU, NODE):
            _assert_plan_equals_brute(oracle, ids, w, e2r, nodes, rpn, level)
        le, lr, ln, st = oracle.expert_load(ids, e2r, nodes, rpn)
        assert st == 0 and int(le.sum()) == int((ids != -1).sum())
        assert np.array_equal(le, np.bincount(ids[ids != -1], minlength=E))
    # a token whose slots were all dropped gets no row and a zero output
    ids = np.array([[-1, -1], [0, -1]], np.int32)
    w = np.array([[.5, .5], [.25, .75]], np.float32)
    p = oracle.plan(ids, w, np.array([0, 1], np.int32), 1, 2, GPU)
    assert p.status == 0 and p.total_rows == 1 and p.slot_row.tolist() == [[-1, -1], [0, -1]]
    y = W.f32_to_bf16_bits(np.array([[2.0, -4.0]], np.float32))
    out = oracle.combine(y, w, p.slot_row)
    assert W.bf16_bits_to_f32(out).tolist() == [[0.0, 0.0], [0.5, -1.0]]


# ---- library-routine special cases ---------------------------------------------------------
@pytest.mark.parametrize("name", ["tiny", "qwen3"])
def test_plan_is_bincount_and_stable_argsort(oracle, name):
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=min(wl.T, 2048))
    ids, e2r = r.topk_ids, r.expert_to_rank
    T, K = ids.shape
    rank = e2r[ids]
    for level in (NONE, GPU, NODE):
        p = oracle.plan(ids, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, level)
        d = (rank // wl.ranks_per_node if level == NODE else rank).reshape(-1)
        kept = p.slot_keep.reshape(-1).astype(bool)
        # per-destination histogram of the kept slots == numpy bincount
        assert np.array_equal(p.dest_count, np.bincount(d[kept], minlength=p.num_dest))
        # row order == stable argsort of the destinations of the kept slots
        kept_idx = np.flatnonzero(kept)
        order = kept_idx[np.argsort(d[kept_idx], kind="stable")]
        assert np.array_equal(p.row_token, order // K)
        # slot_row is the inverse map on kept slots ...
        inv = np.empty(order.size, np.int64)
        inv[np.arange(order.size)] = order
        assert np.array_equal(p.slot_row.reshape(-1)[order], np.arange(order.size))
        # ... and on every slot it names a row of the slot's own token and destination
        row_dest = np.repeat(np.arange(p.num_dest), p.dest_count)
        sr = p.slot_row.reshape(-1)
        assert np.array_equal(p.row_token[sr], np.repeat(np.arange(T), K))
        assert np.array_equal(row_dest[sr], d)
        if level == NONE:
            assert kept.all() and p.total_rows == T * K
            assert np.array_equal(p.row_weight, r.topk_weights.reshape(-1)[order])
        # load_expert is the bincount of ids
        le, lr, ln, st = oracle.expert_load(ids, e2r, wl.nodes, wl.ranks_per_node)
        assert st == 0 and np.array_equal(le, np.bincount(ids.reshape(-1), minlength=wl.E))


# ---- invariants on the five workloads --------------------------------------------------------
def _popcount64(a):
    a = a.astype(np.uint64)
    return np.array([bin(int(v)).count("1") for v in a], dtype=np.int64)


@pytest.mark.parametrize("name", ["tiny", "qwen3", "dsv3", "skew", "stress"])
def test_level_invariants(oracle, name):
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=min(wl.T, 16384))
    ids, w, e2r = r.topk_ids, r.topk_weights, r.expert_to_rank
    T, K = ids.shape
    plans = {lv: oracle.plan(ids, w, e2r, wl.nodes, wl.ranks_per_node, lv) for lv in (NONE, GPU, NODE)}
    le, lr, ln, st = oracle.expert_load(ids, e2r, wl.nodes, wl.ranks_per_node)
    assert st == 0
    assert plans[NONE].total_rows == T * K
    assert plans[NODE].total_rows <= plans[GPU].total_rows <= T * K
    assert int(lr.sum()) == plans[GPU].total_rows
    assert int(ln.sum()) == plans[NODE].total_rows
    assert int(le.sum()) == T * K
    assert np.array_equal(lr, plans[GPU].dest_count)        # p^(1,G) of Eq.(7)
    assert np.array_equal(ln, plans[NODE].dest_count)       # p^(1,U[1]) of Eq.(7)
    rows_per_token_gpu = plans[GPU].slot_keep.sum(axis=1)
    rows_per_token_node = plans[NODE].slot_keep.sum(axis=1)
    assert np.array_equal(_popcount64(plans[GPU].rank_mask), rows_per_token_gpu)
    assert np.array_equal(_popcount64(plans[GPU].node_mask), rows_per_token_node)
    for lv in (NONE, GPU, NODE):
        p = plans[lv]
        # weights of a token's rows add up to the token's router weights
        tot = np.zeros(T)
        np.add.at(tot, p.row_token, p.row_weight.astype(np.float64))
        assert np.allclose(tot, w.astype(np.float64).sum(axis=1), rtol=0, atol=1e-6)
        # stable: tokens ascend inside each destination
        for d in range(p.num_dest):
            seg = p.row_token[p.dest_offset[d]:p.dest_offset[d + 1]]
            assert np.all(np.diff(seg) >= (0 if lv == NONE else 1))
    if wl.router == "deepseek":
        # group-limited routing keeps 4 expert groups and a group never straddles a node under
        # the contiguous placement, so a token reaches at most 4 nodes
        assert rows_per_token_node.max() <= wl.topk_groups
        assert 2.0 < plans[NODE].total_rows / T <= wl.topk_groups


def test_degenerate_topologies(oracle):
    rng = np.random.default_rng(5)
    T, K, E = 257, 4, 24
    ids, w = W.uniform_subset_routing(T, E, K, seed=3)
    w = rng.random((T, K), dtype=np.float32)
    # one node: node level gives exactly one row per token, in token order
    e2r = W.contiguous_placement(E, 8)
    p = oracle.plan(ids, w, e2r, 1, 8, NODE)
    assert p.total_rows == T and np.array_equal(p.row_token, np.arange(T))
    assert np.array_equal(p.slot_row, np.repeat(np.arange(T)[:, None], K, 1))
    # one rank per node: node level == gpu level
    a = oracle.plan(ids, w, e2r, 8, 1, NODE)
    b = oracle.plan(ids, w, e2r, 8, 1, GPU)
    for f in ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "row_weight"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    # one expert per rank and distinct experts per token: no duplicates, gpu level == none
    e2r1 = W.contiguous_placement(E, E)
    a = oracle.plan(ids, w, e2r1, 6, 4, GPU)
    b = oracle.plan(ids, w, e2r1, 6, 4, NONE)
    for f in ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "row_weight"):
        assert np.array_equal(getattr(a, f), getattr(b, f)), f
    # empty input
    p = oracle.plan(np.zeros((0, K), np.int32), np.zeros((0, K), np.float32), e2r, 2, 4, GPU)
    assert p.total_rows == 0 and p.dest_count.tolist() == [0] * 8


def test_same_rank_swap_leaves_plan_unchanged(oracle):
    wl = W.WORKLOADS["qwen3"]
    r = W.make_routing(wl, T=1024)
    e2r = r.expert_to_rank.copy()
    ids_swapped = r.topk_ids.copy()
    # experts 4 and 6 both live on rank 1: renaming one as the other changes no destination
    assert e2r[4] == e2r[6]
    ids_swapped[r.topk_ids == 4] = 6
    ids_swapped[r.topk_ids == 6] = 4
    for lv in (GPU, NODE):
        a = oracle.plan(r.topk_ids, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, lv)
        b = oracle.plan(ids_swapped, r.topk_weights, e2r, wl.nodes, wl.ranks_per_node, lv)
        for f in ("dest_count", "row_token", "slot_row", "slot_keep", "row_weight"):
            assert np.array_equal(getattr(a, f), getattr(b, f)), f


# ---- closed forms and the paper's Table II ---------------------------------------------------
def _expected_rows_per_token(E, K, g):
    """Uniform K-subset of E experts, g equal groups: g * (1 - C(E - E/g, K) / C(E, K))."""
    return g * (1.0 - math.comb(E - E // g, K) / math.comb(E, K))


@pytest.mark.parametrize("name", ["tiny", "qwen3"])
def test_expected_copies_closed_form(oracle, name):
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl)
    for lv, g in ((GPU, wl.G), (NODE, wl.nodes)):
        p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, lv)
        expect = _expected_rows_per_token(wl.E, wl.K, g)
        # rows per token is bounded by K, so its standard deviation is below K/2
        tol = 5 * (min(wl.K, g) / 2) / math.sqrt(wl.T)
        assert abs(p.total_rows / wl.T - expect) < tol, (lv, p.total_rows / wl.T, expect)

def test_table2_duplication_rates(oracle):
    rows = [tuple(int(v) for v in ln.split()) for ln in open(os.path.join(GOLDEN, "table2_duplication.txt"))
            if ln.strip() and not ln.startswith("#")]
    assert len(rows) == 16
    E, T = 256, 20000
    topo = {32: (4, 8), 16: (2, 8), 8: (1, 8), 4: (1, 4)}
    for R, K, pct in rows:
        ids, w = W.uniform_subset_routing(T, E, K, seed=100 + K)
        nodes, rpn = topo[R]
        p = oracle.plan(ids, w, W.contiguous_placement(E, R), nodes, rpn, GPU)
        dup = 100.0 * (1.0 - p.total_rows / (T * K))
        assert abs(dup - pct) <= 1.5, (R, K, dup, pct)


# ---- Fig.5: HD1 sends four tokens across nodes where HD2 sends two --------------------------
def test_fig5_two_nodes_sixteen_gpus(oracle):
    nodes, rpn, E = 2, 8, 16                      # one expert per GPU, 2 nodes x 8 GPUs
    e2r = W.contiguous_placement(E, nodes * rpn)
    # two tokens on node 0, each choosing two experts on two different GPUs of node 1
    ids = np.array([[8, 9], [10, 11]], np.int32)
    w = np.full((2, 2), 0.5, np.float32)
    gpu = oracle.plan(ids, w, e2r, nodes, rpn, GPU)
    node = oracle.plan(ids, w, e2r, nodes, rpn, NODE)
    rows_to_remote_node_gpu_level = int(gpu.dest_count[rpn:].sum())
    assert rows_to_remote_node_gpu_level == 4      # HD1: four tokens cross the node boundary
    assert int(node.dest_count[1]) == 2            # HD2: two
    # and the second hop inside the remote node needs the remaining two copies
    assert rows_to_remote_node_gpu_level - int(node.dest_count[1]) == 2


# ---- Fig.7: counts per group after swapping two experts -------------------------------------
def test_fig7_swap_counts(oracle):
    printed = {(r, c): (a, b) for r, c, a, b in
               (tuple(int(v) for v in ln.split())
                for ln in open(os.path.join(GOLDEN, "fig7_swap_counts.txt")) if ln.strip() and not ln.startswith("#"))}
    base = np.array([0, 0, 1, 1], np.int32)        # {E1,E2} -> group 0, {E3,E4} -> group 1

    def swapped(r, c):
        m = base.copy()
        m[r - 1], m[c - 1] = base[c - 1], base[r - 1]
        return m

    # search the token multisets (each token picks 2 of the 4 experts) for ones that give the
    # printed counts under the set definition; then the oracle must print the same numbers.
    pairs = list(itertools.combinations(range(4), 2))
    found = []
    for mult in itertools.product(range(4), repeat=len(pairs)):
        if not 4 <= sum(mult) <= 8:
            continue
        ids = np.array([p for p, m in zip(pairs, mult) for _ in range(m)], np.int32)
        ok = True
        for (r, c), want in printed.items():
            e2r = swapped(r, c)
            got = group_counts_by_sets(ids, e2r, lambda g: g)
            if (got.get(0, 0), got.get(1, 0)) != want:
                ok = False
                break
        if ok:
            found.append(ids)
    assert found, "no token assignment reproduces the counts printed for Fig.7"
    for ids in found[:20]:
        for (r, c), want in printed.items():
            for (rr, cc) in ((r, c), (c, r)):       # Z is symmetric in (r, c)
                _, lr, ln, st = oracle.expert_load(ids, swapped(rr, cc), 2, 1)
                assert st == 0 and tuple(lr.tolist()) == want and tuple(ln.tolist()) == want


# ---- swap recount: Z[r,c,:] is the load under the swapped placement --------------------------
def test_swapped_placement_recount(oracle):
    wl = W.WORKLOADS["skew"]
    r = W.make_routing(wl, T=512)
    ids = r.topk_ids
    for e2r in (r.expert_to_rank, r.extras["expert_to_rank_swapped"]):
        le, lr, ln, st = oracle.expert_load(ids, e2r, wl.nodes, wl.ranks_per_node)
        by_rank = group_counts_by_sets(ids, e2r, lambda g: g)
        by_node = group_counts_by_sets(ids, e2r, lambda g: g // wl.ranks_per_node)
        assert lr.tolist() == [by_rank.get(g, 0) for g in range(wl.G)]
        assert ln.tolist() == [by_node.get(n, 0) for n in range(wl.nodes)]
    # both experts selected, or neither: swapping them cannot change any count (Section IV-A)
    e2r = r.expert_to_rank
    a, b = 3, 77
    both_or_neither = np.array([((ids[t] == a).any() == (ids[t] == b).any()) for t in range(ids.shape[0])])
    sub = ids[both_or_neither]
    sw = e2r.copy()
    sw[a], sw[b] = e2r[b], e2r[a]
    assert oracle.expert_load(sub, e2r, wl.nodes, wl.ranks_per_node)[1].tolist() == \
        oracle.expert_load(sub, sw, wl.nodes, wl.ranks_per_node)[1].tolist()


# ---- invalid ids are dropped and flagged ------------------------------------------------------
def test_bad_ids_are_dropped(oracle):
    ids = np.array([[0, 99, 1], [-1, 2, 2], [3, 3, 5]], np.int32)
    w = np.array([[.5, .25, .25], [.1, .2, .7], [.3, .3, .4]], np.float32)
    e2r = np.array([0, 0, 1, 1, 2, 7], np.int32)           # expert 5 -> rank 7 does not exist (G=4)
    p = oracle.plan(ids, w, e2r, 2, 2, GPU)
    assert p.status == oracle.BAD_ID
    good = np.array([[0, 1], [2, 2], [3, 3]], np.int32)     # the same table with the bad slots removed
    q = oracle.plan(good, np.array([[.5, .25], [.2, .7], [.3, .3]], np.float32), e2r, 2, 2, GPU)
    assert np.array_equal(p.dest_count, q.dest_count) and np.array_equal(p.row_token, q.row_token)
    assert p.slot_row.tolist() == [[0, -1, 0], [-1, 1, 1], [2, 2, -1]]
    assert p.slot_keep.tolist() == [[1, 0, 0], [0, 1, 0], [1, 0, 0]]
    assert np.array_equal(p.row_weight, q.row_weight)
    le, lr, ln, st = oracle.expert_load(ids, e2r, 2, 2)
    assert st == oracle.BAD_ID and le.tolist() == [1, 1, 2, 2, 0, 0] and lr.tolist() == [1, 2, 0, 0] and ln.tolist() == [3, 0]
