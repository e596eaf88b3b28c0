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
