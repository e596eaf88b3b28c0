"""GPU parity for the dimension-selection pieces: per-level duplicate-free counts (bit-exact) and
the fp64 time model (same operations in the same order as the oracle: bit-exact times, same d*)."""
import numpy as np
import pytest

from paper_2508_09591_amd import workloads as W

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def hw():
    import torch
    assert torch.cuda.is_available(), "these tests need the MI355X"
    import gpu_harness
    from paper_2508_09591_amd import binding
    binding.lib()
    return gpu_harness


@pytest.mark.parametrize("name,T", [("tiny", 1024), ("qwen3", 8192), ("dsv3", 3000), ("skew", 16384), ("stress", 65536)])
def test_group_counts_parity(hw, oracle, name, T):
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=T)
    e2r = r.extras.get("expert_to_rank_swapped", r.expert_to_rank)
    G = wl.G
    for groups in ([G], [G, wl.nodes], [1, wl.nodes, G // 2, G], [G, G, 1]):
        groups = [g for g in groups if g >= 1 and G % g == 0]
        ref, st = oracle.group_counts(r.topk_ids, e2r, G, groups)
        counts_d = torch.full((len(groups), 64), -5, dtype=torch.int32, device="cuda")
        st_d = torch.full((1,), 7, dtype=torch.int32, device="cuda")
        B.hm_group_counts(hw.dev(r.topk_ids), hw.dev(e2r), G, groups, counts_d, st_d)
        assert np.array_equal(counts_d.cpu().numpy(), ref) and int(st_d.item()) == st == 0, (name, groups)
    bad = r.topk_ids.copy()
    bad[T // 2, 0] = wl.E
    ref, st = oracle.group_counts(bad, e2r, G, [G, wl.nodes])
    counts_d = torch.zeros((2, 64), dtype=torch.int32, device="cuda")
    st_d = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.hm_group_counts(hw.dev(bad), hw.dev(e2r), G, [G, wl.nodes], counts_d, st_d)
    assert np.array_equal(counts_d.cpu().numpy(), ref) and int(st_d.item()) == st == B.HM_ERR_BAD_ID
    # empty table
    B.hm_group_counts(hw.dev(bad[:0]), hw.dev(e2r), G, [G], counts_d[:1], st_d)
    assert not counts_d[:1].any() and int(st_d.item()) == 0


def test_alltoall_times_parity(hw, oracle):
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(33)
    for trial in range(200):
        D = int(rng.integers(1, 5))
        G = int(rng.choice([8, 16, 32, 64]))
        U = [1]
        for _ in range(D - 1):
            choices = [u for u in (1, 2, 4, 8, 16, 32, 64) if u >= U[-1] and u % U[-1] == 0 and G % u == 0]
            U.append(int(rng.choice(choices)))
        p_inter = rng.integers(0, 5000, (D, 64)).astype(np.int32)
        p_intra = rng.integers(0, 5000, (D, 64)).astype(np.int32)
        if trial % 3 == 0:                      # small integer times: exact ties exercise Eq.(6)
            ai, bi, ba = [0.0] * D, [0.0] * D, [0.0] * D
            aa = rng.integers(1, 4, D).astype(float).tolist()
        else:
            ai, bi = rng.random(D).tolist(), (rng.random(D) * 1e-6).tolist()
            aa, ba = rng.random(D).tolist(), (rng.random(D) * 1e-6).tolist()
        M, v = float(rng.choice([2048, 7168])), 2.0
        t_ref, d_ref = oracle.alltoall_times(U, G, M, v, p_inter, p_intra, ai, bi, aa, ba)
        times_d = torch.full((4,), float("nan"), dtype=torch.float64, device="cuda")
        best_d = torch.full((1,), -1, dtype=torch.int32, device="cuda")
        B.hm_alltoall_times(U, G, M, v, hw.dev(p_inter), hw.dev(p_intra), ai, bi, aa, ba, times_d, best_d)
        got = times_d.cpu().numpy()[:D]
        assert np.array_equal(got.view(np.uint64), t_ref.view(np.uint64)), (U, G, got, t_ref)
        assert int(best_d.item()) == d_ref


def test_dimension_choice_from_plan_counts(hw, oracle):
    """End to end on the device: counts produced by hm_group_counts feed hm_alltoall_times with the
    parameters printed for Fig.9 of the paper; nothing is copied to the host in between."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["qwen3"]
    r = W.make_routing(wl)
    U, G, M, v = [1, 4, 8, 16], 32, wl.H, 2
    ai, bi = [0, 4.97e-1, 3.01e-1, 1.49e-1], [0, 5.29e-7, 1.17e-7, 2.06e-8]
    aa, ba = [7.22e-1, 5.71e-1, 1.14e-1, 2.04e-1], [5.70e-7, 1.27e-7, 2.63e-8, 1.64e-8]
    own_d = torch.zeros((4, 64), dtype=torch.int32, device="cuda")
    B.hm_group_counts(hw.dev(r.topk_ids), hw.dev(r.expert_to_rank), G, [G, 4, 8, 16], own_d)
    p_inter_d = own_d.clone()
    p_inter_d[0].zero_()
    fan_in = torch.tensor(U, dtype=torch.int32, device="cuda")[:, None]
    p_intra_d = (own_d[0:1] * fan_in).contiguous()             # per-GPU counts times the fan-in U[l] (harness arithmetic)
    times_d = torch.zeros(4, dtype=torch.float64, device="cuda")
    best_d = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.hm_alltoall_times(U, G, M, v, p_inter_d, p_intra_d, ai, bi, aa, ba, times_d, best_d)
    own, _ = oracle.group_counts(r.topk_ids, r.expert_to_rank, G, [G, 4, 8, 16])
    p_inter = own.copy()
    p_inter[0] = 0
    p_intra = own[0:1] * np.array(U, np.int32)[:, None]
    t_ref, d_ref = oracle.alltoall_times(U, G, M, v, p_inter, p_intra, ai, bi, aa, ba)
    assert np.array_equal(times_d.cpu().numpy().view(np.uint64), t_ref.view(np.uint64))
    assert int(best_d.item()) == d_ref
    print("t_d =", t_ref, "d* =", d_ref)


# ---- pins on the device formulas themselves: hand cases, the printed Fig.9 parameters in exact
# rational arithmetic and a direct statement of Eq.(6), none of them through the oracle ---------
def _pad(rows):
    out = np.zeros((len(rows), 64), np.int32)
    for i, r in enumerate(rows):
        out[i, :len(r)] = r
    return out


def _device_times(hw, U, G, M, v, p_inter, p_intra, ai, bi, aa, ba):
    import torch
    from paper_2508_09591_amd import binding as B
    times_d = torch.full((4,), float("nan"), dtype=torch.float64, device="cuda")
    best_d = torch.full((1,), -1, dtype=torch.int32, device="cuda")
    B.hm_alltoall_times(U, G, M, v, hw.dev(p_inter), hw.dev(p_intra), ai, bi, aa, ba, times_d, best_d)
    return times_d.cpu().numpy()[:len(U)], int(best_d.item())


def test_alltoall_times_hand_cases_on_the_device(hw):
    # Eq.(1)-(2): G = 4 GPUs, p = [3,5,2,7], M = 10, v = 2: n = 4 * 7 * 10 * 2 = 560 bytes
    t, d = _device_times(hw, [1], 4, 10, 2, _pad([[0]]), _pad([[3, 5, 2, 7]]), [0], [0], [0.722], [5.7e-7])
    assert d == 1 and abs(t[0] - 0.7223192) < 1e-15
    # Eq.(3)-(5): 2 nodes x 2 GPUs.  inter(1): 2 peers x max([6,4]) x (M v = 8) = 96 bytes; intra(1):
    # G/U[1] = 2 peers x max([5,2,3,4]) x 8 = 80 bytes; flat: 4 x max([3,1,2,2]) x 8 = 96 bytes
    args = ([1, 2], 4, 4, 2, _pad([[0], [6, 4]]), _pad([[3, 1, 2, 2], [5, 2, 3, 4]]))
    t, d = _device_times(hw, *args, [0, 1.0], [0, 0.5], [2.0, 0.25], [0.125, 0.0625])
    assert t.tolist() == [14.0, 54.25] and d == 1
    t, d = _device_times(hw, *args, [0, 1.0], [0, 0.01], [2.0, 0.25], [0.125, 0.0625])     # a cheap inter-node link
    assert t.tolist() == [14.0, (1.0 + 0.96) + 5.25] and d == 2


def test_alltoall_times_with_the_papers_parameters_on_the_device(hw):
    """G = 32, U = [1,4,8,16] (the paper's testbed hierarchy) with the alpha / beta printed for Fig.9:
    the device's t_d against exact rational arithmetic on the printed decimals, and d* against
    Eq.(6) stated on those exact values."""
    import os
    from fractions import Fraction
    f9 = {}
    for ln in open(os.path.join(os.path.dirname(__file__), "golden", "fig9_alpha_beta.txt")):
        if ln.strip() and not ln.startswith("#"):
            kind, a, b = ln.split()
            f9[kind] = (a, b)
    rng = np.random.default_rng(9)
    U, G, M, v = [1, 4, 8, 16], 32, 2048, 2
    for trial in range(20):
        p_inter = rng.integers(0, 9000, (4, 64)).astype(np.int32)
        p_intra = rng.integers(0, 9000 * (trial + 1), (4, 64)).astype(np.int32)
        a_i = [0] + [float(f9["inter(%d)" % i][0]) for i in (1, 2, 3)]
        b_i = [0] + [float(f9["inter(%d)" % i][1]) for i in (1, 2, 3)]
        a_a = [float(f9["a2a"][0])] + [float(f9["intra(%d)" % i][0]) for i in (1, 2, 3)]
        b_a = [float(f9["a2a"][1])] + [float(f9["intra(%d)" % i][1]) for i in (1, 2, 3)]
        t, d = _device_times(hw, U, G, M, v, p_inter, p_intra, a_i, b_i, a_a, b_a)
        exact = []
        for dim in range(1, 5):
            acc = Fraction(0)
            for i in range(1, dim):
                n = Fraction(U[i] // U[i - 1]) * int(p_inter[i, :U[i]].max()) * M * v
                acc += Fraction(f9["inter(%d)" % i][0]) + n * Fraction(f9["inter(%d)" % i][1])
            kind = "a2a" if dim == 1 else "intra(%d)" % (dim - 1)
            n = Fraction(G // U[dim - 1]) * int(p_intra[dim - 1, :G].max()) * M * v
            acc += Fraction(f9[kind][0]) + n * Fraction(f9[kind][1])
            exact.append(acc)
        for got, want in zip(t, exact):
            assert abs(Fraction(float(got)) - want) <= want * Fraction(1, 10 ** 13), (trial, float(got), float(want))
        best_hier = min(range(1, 4), key=lambda i: exact[i])
        gap = abs(exact[0] - exact[best_hier]) / exact[0]
        if gap > Fraction(1, 10 ** 10):                       # not a near-tie that rounding could flip
            assert d == (1 if exact[0] < exact[best_hier] else best_hier + 1), trial


def test_eq6_selection_rule_on_the_device(hw):
    """d* = 1 only when t_1 is strictly below every t_d, d > 1; otherwise the lowest d > 1 with the
    smallest time: times built from small integers (ties are common), rule stated directly."""
    rng = np.random.default_rng(6)
    for _ in range(100):
        D = int(rng.integers(1, 5))
        target = rng.integers(1, 4, D).astype(float)
        t, d = _device_times(hw, [1, 2, 4, 8][:D], 8, 1, 1, _pad([[0]] * D), _pad([[1] * 8] * D),
                             [0.0] * D, [0.0] * D, target.tolist(), [0.0] * D)
        assert t.tolist() == target.tolist()
        if D == 1:
            want = 1
        else:
            m = min(target[1:])
            want = 1 if target[0] < m else 2 + target[1:].tolist().index(m)
        assert d == want, (target, d)


def test_dimension_choice_from_monitored_counts(hw, oracle):
    """Alg.1 with the counts it actually monitors: for the two-dimensional exchange the per-GPU
    counts at the input of the Intra-level AlltoAll are those of the tokens a rank holds AFTER the
    inter-node hop.  Here the inter-node hop of the N same-local-index source ranks is run on the
    device (hm_plan at node level + hm_dispatch_pack of the id / weight rows), the receiver's
    intra-node plan (hm_plan_mapped) yields p^(2,G), and those dest_count vectors go into
    hm_alltoall_times without leaving the device.  Checked three ways: the oracle doing the same
    chain, an identity that needs no oracle (two deduplicated hops deliver what one hop would),
    and the fan-in proxy printed beside it."""
    import dataclasses
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["skew"]
    N, R, G, K, E = wl.nodes, wl.ranks_per_node, wl.G, wl.K, wl.E
    T = 700
    me_node, me_local = 1, 3
    me = me_node * R + me_local
    e2r = W.make_routing(wl, T=8).extras["expert_to_rank_swapped"]      # an uneven placement
    e2r_d = hw.dev(e2r)
    routing = {n: W.make_routing(dataclasses.replace(wl, seed=4000 + n * R + me_local), T=T) for n in range(N)}

    def meta_rows(plan, t_d, rows):                   # ids / weights travel as rows of 2K 2-byte units
        out = torch.empty((rows, 2 * K), dtype=torch.bfloat16, device="cuda")
        B.hm_dispatch_pack(t_d.view(torch.bfloat16).view(-1, 2 * K), plan, out)
        return out

    # ---- device chain
    recv_ids, recv_w, one_hop = [], [], np.zeros(R, np.int64)
    o_recv_ids, o_recv_w = [], []
    for n in range(N):                                # source rank (n, me_local) sends its node-me_node buffer to me
        r = routing[n]
        ids_d, w_d = hw.dev(r.topk_ids), hw.dev(r.topk_weights)
        p1 = B.hm_plan(ids_d, w_d, e2r_d, N, R, B.HM_DEDUP_NODE)
        st, tot = B.hm_plan_status(p1)
        assert st == 0
        off = p1.dest_offset[:N + 1].cpu().numpy()
        a, b = int(off[me_node]), int(off[me_node + 1])
        recv_ids.append(meta_rows(p1, ids_d, tot)[a:b].contiguous().view(torch.int32).view(-1, K))
        recv_w.append(meta_rows(p1, w_d, tot)[a:b].contiguous().view(torch.float32).view(-1, K))
        # the one-hop exchange of the same source: rows per GPU of my node
        pg = B.hm_plan(ids_d, w_d, e2r_d, N, R, B.HM_DEDUP_GPU)
        assert B.hm_plan_status(pg)[0] == 0
        one_hop += pg.dest_count[me_node * R:(me_node + 1) * R].cpu().numpy()
        o1 = oracle.plan(r.topk_ids, r.topk_weights, e2r, N, R, B.HM_DEDUP_NODE)
        rows = o1.row_token[o1.dest_offset[me_node]:o1.dest_offset[me_node + 1]]
        o_recv_ids.append(r.topk_ids[rows])
        o_recv_w.append(r.topk_weights[rows])
    rid_d, rw_d = torch.cat(recv_ids).contiguous(), torch.cat(recv_w).contiguous()
    dmA = torch.empty(E, dtype=torch.int32, device="cuda")
    ndA = torch.empty(1, dtype=torch.int32, device="cuda")
    B.hm_recv_dest_map(e2r_d, N, R, me, B.HM_RECV_INTRA_NODE, dmA, ndA)
    planA = B.hm_plan_mapped(rid_d, rw_d, dmA, R, True)
    assert B.hm_plan_status(planA)[0] == 0
    own = routing[me_node]                            # my own tokens (I am one of the sources)
    own_ids_d, own_w_d = hw.dev(own.topk_ids), hw.dev(own.topk_weights)
    plan_gpu = B.hm_plan(own_ids_d, own_w_d, e2r_d, N, R, B.HM_DEDUP_GPU)
    plan_node = B.hm_plan(own_ids_d, own_w_d, e2r_d, N, R, B.HM_DEDUP_NODE)
    p_inter_d = torch.zeros((2, 64), dtype=torch.int32, device="cuda")
    p_intra_d = torch.zeros((2, 64), dtype=torch.int32, device="cuda")
    p_inter_d[1, :N] = plan_node.dest_count[:N]       # p^(1,U[1]): device-to-device, nothing visits the host
    p_intra_d[0, :G] = plan_gpu.dest_count[:G]        # p^(1,G)
    p_intra_d[1, :R] = planA.dest_count[:R]           # p^(2,G): the monitored counts
    U, M, v = [1, N], float(wl.H), 2.0
    ai, bi, aa, ba = [0, 4.97e-1], [0, 5.29e-7], [7.22e-1, 5.71e-1], [5.70e-7, 1.27e-7]       # the paper's Fig.9 fit
    times_d = torch.zeros(4, dtype=torch.float64, device="cuda")
    best_d = torch.zeros(1, dtype=torch.int32, device="cuda")
    B.hm_alltoall_times(U, G, M, v, p_inter_d, p_intra_d, ai, bi, aa, ba, times_d, best_d)
    t_mon, d_mon = times_d.cpu().numpy()[:2].copy(), int(best_d.item())

    # ---- the identity: what the receiver forwards to local GPU j is what the sources' one-hop plans send there
    assert np.array_equal(planA.dest_count[:R].cpu().numpy().astype(np.int64), one_hop)

    # ---- the oracle doing the same chain
    o_ids, o_w = np.concatenate(o_recv_ids), np.concatenate(o_recv_w)
    assert np.array_equal(rid_d.cpu().numpy(), o_ids) and np.array_equal(rw_d.cpu().numpy(), o_w)
    dm, nd = oracle.recv_dest_map(e2r, N, R, me, B.HM_RECV_INTRA_NODE)
    oA = oracle.plan_mapped(o_ids, o_w, dm, nd, True)
    o_gpu = oracle.plan(own.topk_ids, own.topk_weights, e2r, N, R, B.HM_DEDUP_GPU)
    o_node = oracle.plan(own.topk_ids, own.topk_weights, e2r, N, R, B.HM_DEDUP_NODE)
    pi, pa = np.zeros((2, 64), np.int32), np.zeros((2, 64), np.int32)
    pi[1, :N], pa[0, :G], pa[1, :R] = o_node.dest_count, o_gpu.dest_count, oA.dest_count
    assert np.array_equal(p_inter_d.cpu().numpy(), pi) and np.array_equal(p_intra_d.cpu().numpy(), pa)
    t_ref, d_ref = oracle.alltoall_times(U, G, M, v, pi, pa, ai, bi, aa, ba)
    assert np.array_equal(t_mon.view(np.uint64), t_ref[:2].view(np.uint64)) and d_mon == d_ref

    # ---- the fan-in proxy a planner uses before the exchange has run: own per-GPU counts x N
    p_proxy_d = p_intra_d.clone()
    p_proxy_d[1, :G] = plan_gpu.dest_count[:G] * N
    B.hm_alltoall_times(U, G, M, v, p_inter_d, p_proxy_d, ai, bi, aa, ba, times_d, best_d)
    t_proxy, d_proxy = times_d.cpu().numpy()[:2], int(best_d.item())
    print("monitored: t =", t_mon, "d* =", d_mon, "| fan-in proxy: t =", t_proxy, "d* =", d_proxy,
          "| max p^(2,G): monitored %d, proxy %d" % (int(pa[1].max()), int(p_proxy_d[1].max().item())), flush=True)
    assert t_proxy[0] == t_mon[0]                       # the one-dimensional time does not involve the second hop
