"""Pins for the dimension-selection arithmetic (Eq.(1)-(6), Alg.1): per-level duplicate-free
counts and the linear time model.  CPU only; references are set-based counting, hand-computed
numbers, exact rational arithmetic on the parameters printed for Fig.9, and a brute-force
statement of Eq.(6)."""
import os
from fractions import Fraction

import numpy as np
import pytest

from helpers import GPU, NODE, group_counts_by_sets
from paper_2508_09591_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def fig9():
    out = {}
    for ln in open(os.path.join(GOLDEN, "fig9_alpha_beta.txt")):
        if ln.strip() and not ln.startswith("#"):
            kind, a, b = ln.split()
            out[kind] = (a, b)
    return out


def test_group_counts_by_sets_and_against_plans(oracle):
    for name in ("qwen3", "dsv3", "skew"):
        wl = W.WORKLOADS[name]
        r = W.make_routing(wl, T=900)
        e2r = r.extras.get("expert_to_rank_swapped", r.expert_to_rank)
        groups = [wl.G, wl.nodes, wl.nodes * 2, 1]                       # U-style cuts: 32, 4, 8 and a single group
        counts, st = oracle.group_counts(r.topk_ids, e2r, wl.G, groups)
        assert st == 0
        for l, g in enumerate(groups):
            per = wl.G // g
            by_sets = group_counts_by_sets(r.topk_ids, e2r, lambda rank: rank // per)
            assert counts[l, :g].tolist() == [by_sets.get(j, 0) for j in range(g)]
            assert not counts[l, g:].any()
            # the same numbers as the destination counts of a deduplicated plan for that cut
            p = oracle.plan_mapped(r.topk_ids, r.topk_weights, (e2r // per).astype(np.int32), g, True)
            assert np.array_equal(counts[l, :g], p.dest_count)
        assert counts[3, 0] == 900                                        # one group: every token once
        le, lr, ln, _ = oracle.expert_load(r.topk_ids, e2r, wl.nodes, wl.ranks_per_node)
        assert np.array_equal(counts[0, :wl.G], lr) and np.array_equal(counts[1, :wl.nodes], ln)


def _pad(rows):
    out = np.zeros((len(rows), 64), np.int32)
    for i, r in enumerate(rows):
        out[i, :len(r)] = r
    return out


def test_one_dimension_is_eq1_eq2(oracle):
    # G = 4 GPUs, p = [3,5,2,7], M = 10, v = 2: n = 4 * 7 * 10 * 2 = 560 bytes; t = 0.722 + 560 * 5.7e-7
    t, d = oracle.alltoall_times([1], 4, 10, 2, _pad([[0]]), _pad([[3, 5, 2, 7]]), [0], [0], [0.722], [5.7e-7])
    assert d == 1 and abs(t[0] - 0.7223192) < 1e-15


def test_two_dimensions_by_hand(oracle):
    # 2 nodes x 2 GPUs.  inter(1): 2 peers x max([6,4]) x (M v = 8) = 96 bytes; intra(1): G/U[1] = 2
    # peers x max([5,2,3,4]) x 8 = 80 bytes; flat: 4 x max([3,1,2,2]) x 8 = 96 bytes.
    t, d = oracle.alltoall_times([1, 2], 4, 4, 2, _pad([[0], [6, 4]]), _pad([[3, 1, 2, 2], [5, 2, 3, 4]]),
                                 [0, 1.0], [0, 0.5], [2.0, 0.25], [0.125, 0.0625])
    assert t.tolist() == [2.0 + 96 * 0.125, (1.0 + 96 * 0.5) + (0.25 + 80 * 0.0625)]
    assert t.tolist() == [14.0, 54.25] and d == 1
    # make the inter-node link cheap: the two-dimensional exchange wins
    t, d = oracle.alltoall_times([1, 2], 4, 4, 2, _pad([[0], [6, 4]]), _pad([[3, 1, 2, 2], [5, 2, 3, 4]]),
                                 [0, 1.0], [0, 0.01], [2.0, 0.25], [0.125, 0.0625])
    assert t.tolist() == [14.0, (1.0 + 0.96) + 5.25] and d == 2


def test_four_dimensions_with_the_papers_parameters(oracle):
    """The paper's testbed: G = 32, U = [1, 4, 8, 16] (Section III-B), parameters of Fig.9; counts
    from a seeded routing.  Expected values in exact rational arithmetic from the printed decimals."""
    f9 = fig9()
    wl = W.WORKLOADS["qwen3"]
    r = W.make_routing(wl, T=1024)
    U, G, M, v = [1, 4, 8, 16], 32, 2048, 2
    own, _ = oracle.group_counts(r.topk_ids, r.expert_to_rank, G, [G, 4, 8, 16])
    p_inter = _pad([[0], own[1, :4], own[2, :8], own[3, :16]])
    # counts per GPU at the input of Intra-level-l: this rank's own counts times the fan-in U[l]
    p_intra = _pad([own[0, :G] * u for u in U])
    a_i = [0] + [float(f9["inter(%d)" % i][0]) for i in (1, 2, 3)]
    b_i = [0] + [float(f9["inter(%d)" % i][1]) for i in (1, 2, 3)]
    a_a = [float(f9["a2a"][0])] + [float(f9["intra(%d)" % i][0]) for i in (1, 2, 3)]
    b_a = [float(f9["a2a"][1])] + [float(f9["intra(%d)" % i][1]) for i in (1, 2, 3)]
    t, d = oracle.alltoall_times(U, G, M, v, p_inter, p_intra, a_i, b_i, a_a, b_a)
    exact = []
    for dim in range(1, 5):
        acc = Fraction(0)
        for i in range(1, dim):
            n = Fraction(U[i] // U[i - 1]) * int(p_inter[i].max()) * M * v
            acc += Fraction(f9["inter(%d)" % i][0]) + n * Fraction(f9["inter(%d)" % i][1])
        kind = "a2a" if dim == 1 else "intra(%d)" % (dim - 1)
        n = Fraction(G // U[dim - 1]) * int(p_intra[dim - 1].max()) * M * v
        acc += Fraction(f9[kind][0]) + n * Fraction(f9[kind][1])
        exact.append(acc)
    for got, want in zip(t, exact):
        assert abs(Fraction(float(got)) - want) <= want * Fraction(1, 10 ** 13)
    best_hier = min(range(1, 4), key=lambda i: exact[i])
    assert d == (1 if exact[0] < exact[best_hier] else best_hier + 1)
    # Eq.(2) with max(p): the intra-level volume of every dimension equals the flat one here
    # (fan-in times own counts), so only the link parameters separate them
    assert len({int(p_intra[l].max()) * (G // U[l]) for l in range(4)}) == 1


def test_eq6_selection_rule(oracle):
    """d* = 1 only when t_1 is strictly below every t_d, d > 1; otherwise the lowest d > 1 with the
    smallest time -- against a direct statement of Eq.(6) on times built to include ties."""
    rng = np.random.default_rng(6)
    for _ in range(300):
        D = int(rng.integers(1, 5))
        target = rng.integers(1, 4, D).astype(float)                    # small integers: ties are common
        # make t_d == target[d-1] exactly: zero betas, alphas chosen so the partial sums hit the targets
        a_intra = target.copy()
        t, d = oracle.alltoall_times([1, 2, 4, 8][:D], 8, 1, 1, _pad([[0]] * D), _pad([[1] * 8] * D),
                                     [0.0] * D, [0.0] * D, a_intra.tolist(), [0.0] * D)
        assert t.tolist() == target.tolist()
        if D == 1:
            want = 1
        else:
            m = min(target[1:])
            want = 1 if target[0] < m else 2 + target[1:].tolist().index(m)
        assert d == want, (target, d)


def test_argument_checks(oracle):
    with pytest.raises(ValueError):
        oracle.alltoall_times([2], 4, 1, 1, _pad([[0]]), _pad([[1]]), [0], [0], [0], [0])           # U[0] != 1
    with pytest.raises(ValueError):
        oracle.alltoall_times([1, 3], 4, 1, 1, _pad([[0]] * 2), _pad([[1]] * 2), [0] * 2, [0] * 2, [0] * 2, [0] * 2)
    with pytest.raises(ValueError):
        oracle.group_counts(np.zeros((1, 1), np.int32), np.zeros(4, np.int32), 4, [3])
