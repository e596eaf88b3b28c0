"""GPU parity for the hierarchical expert swap: the swap tensor Z (bit-exact against the oracle's
definition-based recount on small inputs and against its incremental update at full size) and
the selection of Eq.(8)-(11) (bit-exact for the plain maximum, 1e-12 with the smooth maximum)."""
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


def _gpu_z(hw, ids, e2r, G, ng):
    import torch
    from paper_2508_09591_amd import binding as B
    E = e2r.shape[0]
    Z = torch.full((E, E, ng), -9, dtype=torch.int32, device="cuda")
    st = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    B.hm_swap_counts(hw.dev(ids), hw.dev(e2r), G, ng, Z, st)
    return Z, int(st.item())


def test_swap_counts_small_against_definition(hw, oracle):
    rng = np.random.default_rng(5)
    for trial in range(60):
        G = int(rng.choice([2, 4, 8, 6, 64]))
        ng = int(rng.choice([g for g in (1, 2, 3, 4, 6, 8, 32, 64) if G % g == 0 and g <= G]))
        E = int(rng.integers(2, 40))
        T, K = int(rng.integers(0, 300)), int(rng.integers(1, 7))
        ids = rng.integers(0, E, (T, K), dtype=np.int32)
        e2r = rng.integers(0, G, E).astype(np.int32)
        if trial % 5 == 0 and T:
            ids[rng.integers(0, T), 0] = -2
        if trial % 7 == 0:
            e2r[rng.integers(0, E)] = G + 1
        ref, st_ref = oracle.swap_counts(ids, e2r, G, ng, "naive")
        Z, st = _gpu_z(hw, ids, e2r, G, ng)
        assert np.array_equal(Z.cpu().numpy(), ref) and st == st_ref, (trial, G, ng, E, T, K)


@pytest.mark.parametrize("G,ng,E,T,K", [(8, 4, 200, 500, 12), (64, 64, 256, 300, 20), (8, 8, 300, 400, 5),
                                          (4, 2, 33, 1000, 64), (32, 32, 256, 5000, 8), (16, 8, 96, 4097, 3),
                                          (64, 64, 512, 700, 6)])      # the last: tables too large for LDS
def test_swap_counts_other_shapes(hw, oracle, G, ng, E, T, K):
    """K from 3 to 64 (sub-groups of 4 to 64 lanes per token), several rounds per workgroup, expert
    counts from 33 to 300, dropped slots: against the oracle's incremental update (itself pinned
    to the definition)."""
    rng = np.random.default_rng(G * 1000 + E)
    ids = rng.integers(0, E, (T, K), dtype=np.int32)
    ids[rng.random((T, K)) < 0.05] = -1                       # dropped slots
    e2r = rng.integers(0, G, E).astype(np.int32)
    ref, st_ref = oracle.swap_counts(ids, e2r, G, ng, "incremental")
    Z, st = _gpu_z(hw, ids, e2r, G, ng)
    assert st == st_ref == 0
    assert np.array_equal(Z.cpu().numpy(), ref), (G, ng, E, T, K)


@pytest.mark.parametrize("name,T,cuts", [("skew", 16384, [4, 8, 16, 32]), ("dsv3", 3000, [32, 4]), ("qwen3", 2000, [1, 2, 32]),
                                         ("stress", 1500, [64, 8, 16, 2])])
def test_swap_counts_multi_equals_separate_calls(hw, oracle, name, T, cuts):
    """Several cuts in one pass: every Z must equal the oracle's (and so the single-cut call's)."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl, T=T)
    e2r = r.extras.get("expert_to_rank_swapped", r.expert_to_rank) if hasattr(r, "extras") and r.extras else r.expert_to_rank
    ids = r.topk_ids.copy()
    ids[5, 1] = -1                                            # a dropped slot
    E, G = wl.E, wl.G
    Z = [torch.full((E, E, u), -9, dtype=torch.int32, device="cuda") for u in cuts]
    st = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    B.hm_swap_counts_multi(hw.dev(ids), hw.dev(e2r), G, cuts, Z, st)
    assert int(st.item()) == 0
    for u, z in zip(cuts, Z):
        ref, _ = oracle.swap_counts(ids, e2r, G, u, "incremental")
        assert np.array_equal(z.cpu().numpy(), ref), (name, u)
    # an invalid id and an invalid placement entry: flagged, every cut follows the single-cut rule
    ids[7, 0] = E + 3
    bad = e2r.copy()
    bad[2] = G
    B.hm_swap_counts_multi(hw.dev(ids), hw.dev(bad), G, cuts, Z, st)
    assert int(st.item()) == B.HM_ERR_BAD_ID
    for u, z in zip(cuts, Z):
        ref, st_ref = oracle.swap_counts(ids, bad, G, u, "incremental")
        assert st_ref == B.HM_ERR_BAD_ID and np.array_equal(z.cpu().numpy(), ref), (name, u, "bad")


@pytest.mark.parametrize("G,E,T,K,cuts", [(12, 48, 900, 5, [4, 6, 12]),      # cuts that do not refine one another
                                          (12, 60, 700, 4, [6, 2, 12, 3]),
                                          (16, 64, 800, 6, [8, 8]),           # the same cut twice
                                          (24, 96, 1000, 8, [12, 2, 24, 4])]) # nested, given out of order
def test_swap_counts_multi_any_set_of_cuts(hw, oracle, G, E, T, K, cuts):
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(G + E)
    ids = rng.integers(0, E, (T, K), dtype=np.int32)
    ids[rng.random((T, K)) < 0.05] = -1
    e2r = rng.integers(0, G, E).astype(np.int32)
    Z = [torch.full((E, E, u), -9, dtype=torch.int32, device="cuda") for u in cuts]
    st = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    B.hm_swap_counts_multi(hw.dev(ids), hw.dev(e2r), G, cuts, Z, st)
    assert int(st.item()) == 0
    for u, z in zip(cuts, Z):
        ref, _ = oracle.swap_counts(ids, e2r, G, u, "naive" if E <= 60 else "incremental")
        assert np.array_equal(z.cpu().numpy(), ref), (G, E, cuts, u)


@pytest.mark.parametrize("name,placement", [("qwen3", "contiguous"), ("dsv3", "contiguous"), ("skew", "swapped")])
def test_swap_counts_full_size(hw, oracle, name, placement):
    wl = W.WORKLOADS[name]
    r = W.make_routing(wl)
    e2r = r.extras["expert_to_rank_swapped"] if placement == "swapped" else r.expert_to_rank
    for ng in (wl.G, wl.nodes):
        ref, st_ref = oracle.swap_counts(r.topk_ids, e2r, wl.G, ng, "incremental")
        Z, st = _gpu_z(hw, r.topk_ids, e2r, wl.G, ng)
        assert np.array_equal(Z.cpu().numpy(), ref) and st == st_ref == 0, (name, ng)


@pytest.mark.parametrize("E,G,K,T,cuts", [(256, 64, 8, 65536, [8, 64]),       # 64 Ki-token layer: four fetch stages per chunk, four panels
                                          (128, 32, 8, 40000, [4, 32]),       # ragged: the last chunk ends inside a stage
                                          (96, 16, 3, 20000, [16]),           # four lanes per token: lanes beyond 128 tokens idle
                                          (200, 8, 24, 9000, [2, 8]),         # 32 lanes per token: four passes per tile
                                          (48, 8, 2, 523000, [4])])           # more tokens than 16 chunks of 16-bit counts hold: the path with atomics
def test_swap_counts_long_chunks(hw, oracle, E, G, K, T, cuts):
    """Token counts beyond what one fetch stage of a chunk covers (16 chunks x 1,024 slots-per-lane
    passes), so the matrix kernel's outer loop, its clamped loads at a ragged end and the
    multi-pass tiles are all exercised; the four-panel split of E > 128 too."""
    import torch
    from paper_2508_09591_amd import binding as B
    rng = np.random.default_rng(E + T)
    ids = rng.integers(0, E, (T, K), dtype=np.int32)
    ids[rng.random((T, K)) < 0.03] = -1
    ids[T - 1, 0] = ids[T - 1, K - 1]                           # a repeated expert in the very last token
    e2r = rng.integers(0, G, E).astype(np.int32)
    Z = [torch.full((E, E, u), -9, dtype=torch.int32, device="cuda") for u in cuts]
    st = torch.full((1,), 5, dtype=torch.int32, device="cuda")
    B.hm_swap_counts_multi(hw.dev(ids), hw.dev(e2r), G, cuts, Z, st)
    assert int(st.item()) == 0
    for u, z in zip(cuts, Z):
        ref, _ = oracle.swap_counts(ids, e2r, G, u, "incremental")
        assert np.array_equal(z.cpu().numpy(), ref), (E, G, K, T, u)


def test_swap_select_parity(hw, oracle):
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["skew"]
    r = W.make_routing(wl, T=4096)
    e2r = r.extras["expert_to_rank_swapped"]
    G, E = wl.G, wl.E
    cuts = {u: _gpu_z(hw, r.topk_ids, e2r, G, u)[0] for u in (4, 8, 16, 32)}
    host = {u: z.cpu().numpy() for u, z in cuts.items()}
    ai, bi = [0, 4.97e-1, 3.01e-1, 1.49e-1], [0, 5.29e-7, 1.17e-7, 2.06e-8]
    aa, ba = [7.22e-1, 5.71e-1, 1.14e-1, 2.04e-1], [5.70e-7, 1.27e-7, 2.63e-8, 1.64e-8]
    Ufull = [1, 4, 8, 16]
    for d in (1, 2, 3, 4):
        U = Ufull[:d]
        for gamma in (0.0, 10.0, 5.0):
            zi_h = [None] + [host[U[i]] for i in range(1, d)]
            zi_d = [None] + [cuts[U[i]] for i in range(1, d)]
            si = [0.0] + [float(U[i - 1]) for i in range(1, d)]              # fan-in of each inter level
            Qr, best_r, bt_r = oracle.swap_select(U, G, wl.H, 2.0, zi_h, host[32], si, float(U[d - 1]), ai[:d], bi[:d],
                                                  aa[d - 1], ba[d - 1], gamma)
            Q = torch.full((E, E), float("nan"), dtype=torch.float64, device="cuda")
            bp = torch.full((2,), -1, dtype=torch.int32, device="cuda")
            bt = torch.zeros(1, dtype=torch.float64, device="cuda")
            B.hm_swap_select(U, G, wl.H, 2.0, zi_d, cuts[32], si, float(U[d - 1]), ai[:d], bi[:d], aa[d - 1], ba[d - 1],
                             gamma, Q, bp, bt)
            Qg = Q.cpu().numpy()
            pair = tuple(int(x) for x in bp.cpu().numpy())
            if gamma <= 0:
                assert np.array_equal(Qg.view(np.uint64), Qr.view(np.uint64)), (d, gamma)
                assert pair == best_r and float(bt.item()) == bt_r
            else:
                assert np.allclose(Qg, Qr, rtol=1e-12, atol=0), (d, gamma)
                assert Qr[pair] <= bt_r * (1 + 1e-12) and abs(float(bt.item()) - bt_r) <= 1e-12 * bt_r
            assert float(bt.item()) == Qg[pair] == Qg.min()
            flat = int(np.argmin(Qg))
            assert pair == (flat // E, flat % E)                               # first minimiser in row-major order
    print("d=4 gamma=5 best pair", pair, "time", float(bt.item()), "no swap", Qg[0, 0])


def test_planner_loop_stays_on_the_device(hw, oracle):
    """(Z, select, apply) repeated on the device with no host step in between; afterwards every
    iteration is replayed on the oracle.  gamma <= 0 keeps Q bit-exact, so the chosen pairs and
    the placements must be identical."""
    import torch
    from paper_2508_09591_amd import binding as B
    wl = W.WORKLOADS["skew"]
    r = W.make_routing(wl, T=3000)
    G, E, iters = wl.G, wl.E, 5
    ids_d = hw.dev(r.topk_ids)
    e2r_d = hw.dev(r.expert_to_rank.copy())
    Zn = torch.empty((E, E, wl.nodes), dtype=torch.int32, device="cuda")
    Zg = torch.empty((E, E, G), dtype=torch.int32, device="cuda")
    st = torch.zeros(1, dtype=torch.int32, device="cuda")
    Q = torch.empty((E, E), dtype=torch.float64, device="cuda")
    pairs = torch.full((iters, 2), -1, dtype=torch.int32, device="cuda")
    times = torch.zeros(iters, dtype=torch.float64, device="cuda")
    places = torch.empty((iters, E), dtype=torch.int32, device="cuda")
    U, M, v = [1, wl.nodes], float(wl.H), 2.0
    ai, bi, aa, ba = [0, 0.497], [0, 5.29e-7], 0.571, 1.27e-7
    for it in range(iters):
        B.hm_swap_counts(ids_d, e2r_d, G, wl.nodes, Zn, st)
        B.hm_swap_counts(ids_d, e2r_d, G, G, Zg, st)
        B.hm_swap_select(U, G, M, v, [None, Zn], Zg, [0, 1.0], float(wl.nodes), ai, bi, aa, ba, 0.0, Q, pairs[it], times[it:it + 1])
        B.hm_swap_apply(e2r_d, pairs[it])
        places[it].copy_(e2r_d)
    torch.cuda.synchronize()
    assert int(st.item()) == 0
    place = r.expert_to_rank.copy()
    got_pairs, got_times, got_places = pairs.cpu().numpy(), times.cpu().numpy(), places.cpu().numpy()
    for it in range(iters):
        zn, _ = oracle.swap_counts(r.topk_ids, place, G, wl.nodes)
        zg, _ = oracle.swap_counts(r.topk_ids, place, G, G)
        _, best, bt = oracle.swap_select(U, G, M, v, [None, zn], zg, [0, 1.0], float(wl.nodes), ai, bi, aa, ba, 0.0)
        assert tuple(int(x) for x in got_pairs[it]) == best and got_times[it] == bt, it
        place = oracle.swap_apply(place, best)
        assert np.array_equal(got_places[it], place), it
    assert (np.diff(got_times) <= 0).all()
    # degenerate pairs leave the placement alone
    before = e2r_d.clone()
    for pr in ((3, 3), (-1, 2), (0, E)):
        B.hm_swap_apply(e2r_d, hw.dev(np.array(pr, np.int32)))
    assert torch.equal(e2r_d, before)


def test_swap_select_hand_cases_on_the_device(hw):
    """Eq.(8)-(11) on the device against numbers worked out by hand and against numpy -- a pin on
    the device formulas that does not pass through the oracle."""
    import torch
    from paper_2508_09591_amd import binding as B
    E, G = 3, 2
    Z = np.zeros((E, E, G), np.int32)
    Z[:] = [4, 4]
    Z[0, 1] = Z[1, 0] = [5, 2]
    Z[0, 2] = Z[2, 0] = [3, 3]
    Zd = hw.dev(Z)

    def select(U, M, v, z_inter, z_intra, si, s_intra, ai, bi, aa, ba, gamma):
        n = z_intra.shape[0]
        Q = torch.full((n, n), float("nan"), dtype=torch.float64, device="cuda")
        bp = torch.full((2,), -1, dtype=torch.int32, device="cuda")
        bt = torch.zeros(1, dtype=torch.float64, device="cuda")
        B.hm_swap_select(U, G if n == 3 else wl.G, M, v, z_inter, z_intra, si, s_intra, ai, bi, aa, ba, gamma, Q, bp, bt)
        return Q.cpu().numpy(), tuple(int(x) for x in bp.cpu().numpy()), float(bt.item())

    # one dimension, plain maximum: Q = alpha + G * max(Z[r,c,:]) * M v * beta
    Q, best, bt = select([1], 2.0, 1.0, [None], Zd, [0], 1.0, [0], [0], 10.0, 0.5, 0.0)
    assert Q[0, 1] == 10 + 2 * 5 * 2 * 0.5 and Q[0, 2] == 10 + 2 * 3 * 2 * 0.5 and Q[1, 1] == 10 + 2 * 4 * 2 * 0.5
    assert best == (0, 2) and bt == 16.0                           # first minimiser in row-major order
    # smooth maximum of Eq.(11): n equal entries m -> m * n^(1/gamma); dominated entries vanish as gamma grows
    Q10, _, _ = select([1], 1.0, 1.0, [None], Zd, [0], 1.0, [0], [0], 0.0, 1.0, 10.0)
    assert abs(Q10[1, 1] - G * 4 * 2 ** 0.1) < 1e-12
    assert abs(Q10[0, 1] - G * 5 * (1 + 0.4 ** 10) ** 0.1) < 1e-12
    Qbig, _, _ = select([1], 1.0, 1.0, [None], Zd, [0], 1.0, [0], [0], 0.0, 1.0, 400.0)
    assert abs(Qbig[0, 1] - G * 5) < 1e-9
    # two dimensions on a real routing table, gamma = 10 (the paper's default), against numpy
    wl = W.WORKLOADS["skew"]
    r = W.make_routing(wl, T=256)
    e2r = r.extras["expert_to_rank_swapped"]
    Zn_d, Zg_d = _gpu_z(hw, r.topk_ids, e2r, wl.G, wl.nodes)[0], _gpu_z(hw, r.topk_ids, e2r, wl.G, wl.G)[0]
    Zn, Zg = Zn_d.cpu().numpy(), Zg_d.cpu().numpy()
    U, M, v, gamma = [1, wl.nodes], 2048.0, 2.0, 10.0
    ai, bi, aa, ba = [0, 0.497], [0, 5.29e-7], 0.571, 1.27e-7
    Q, best, bt = select(U, M, v, [None, Zn_d], Zg_d, [0, 1.0], float(wl.nodes), ai, bi, aa, ba, gamma)

    def smax(x):
        m = x.max(axis=-1).astype(np.float64)
        s = ((x / np.maximum(m, 1)[..., None]) ** gamma).sum(-1) ** (1 / gamma)
        return np.where(m > 0, m * s, 0.0)

    ref = (wl.nodes * smax(Zn) * M * v * bi[1] + ai[1]) + ((wl.G // wl.nodes) * wl.nodes * smax(Zg) * M * v * ba + aa)
    assert np.allclose(Q, ref, rtol=1e-12, atol=0)
    assert best == tuple(int(i) for i in np.unravel_index(np.argmin(Q), Q.shape)) and bt == Q[best]
    assert bt <= Q[0, 0]
