"""Pins for the hierarchical expert swap (HierD-ES, Section IV): the swap tensor Z from its
definition and from the paper's incremental update, and the selection of Eq.(8)-(11).  CPU only."""
import itertools
import os

import numpy as np
import pytest

from helpers import group_counts_by_sets
from paper_2508_09591_amd import workloads as W

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _swapped(e2r, r, c):
    m = e2r.copy()
    m[r], m[c] = e2r[c], e2r[r]
    return m


def test_z_definition_by_sets_and_fig7(oracle):
    """Z[r,c,:] is the per-group count under the placement with r and c exchanged -- checked by
    sets on random tables, and on the worked example printed with Fig.7."""
    rng = np.random.default_rng(2)
    for _ in range(30):
        G = int(rng.choice([2, 4, 6]))
        ng = int(rng.choice([g for g in (1, 2, 3, 4, 6) if G % g == 0 and g <= G]))
        E = G * int(rng.integers(1, 4))
        T, K = int(rng.integers(1, 10)), int(rng.integers(1, 4))
        ids = rng.integers(0, E, (T, K), dtype=np.int32)
        e2r = rng.integers(0, G, E).astype(np.int32)
        Z, st = oracle.swap_counts(ids, e2r, G, ng, "naive")
        per = G // ng
        for r in range(E):
            for c in range(E):
                by = group_counts_by_sets(ids, _swapped(e2r, r, c), lambda rank: rank // per)
                assert Z[r, c].tolist() == [by.get(j, 0) for j in range(ng)]
    printed = {(r, c): (a, b) for r, c, a, b in
               (tuple(int(v) for v in ln.split())
                for ln in open(os.path.join(GOLDEN, "fig7_swap_counts.txt")) if ln.strip() and not ln.startswith("#"))}
    base = np.array([0, 0, 1, 1], np.int32)
    pairs = list(itertools.combinations(range(4), 2))
    hits = 0
    for mult in itertools.product(range(4), repeat=len(pairs)):
        if not 4 <= sum(mult) <= 8:
            continue
        ids = np.array([p for p, m in zip(pairs, mult) for _ in range(m)], np.int32)
        Z, _ = oracle.swap_counts(ids, base, 2, 2, "naive")
        if all(tuple(Z[r - 1, c - 1]) == want for (r, c), want in printed.items()):
            hits += 1
            Zi, _ = oracle.swap_counts(ids, base, 2, 2, "incremental")
            assert np.array_equal(Z, Zi)
            for (r, c), want in printed.items():
                assert tuple(Z[c - 1, r - 1]) == want              # the paper prints Z[r,c] = Z[c,r]
    assert hits > 0, "no token assignment reproduces the counts printed for Fig.7"


def test_incremental_update_equals_definition(oracle):
    rng = np.random.default_rng(3)
    for trial in range(120):
        G = int(rng.choice([2, 4, 8, 6]))
        ng = int(rng.choice([g for g in (1, 2, 3, 4, 6, 8) if G % g == 0 and g <= G]))
        E = int(rng.integers(2, 14))
        T, K = int(rng.integers(0, 14)), int(rng.integers(1, 5))
        ids = rng.integers(0, E, (T, K), dtype=np.int32)            # repeated experts inside a token allowed
        e2r = rng.integers(0, G, E).astype(np.int32)
        if trial % 5 == 0 and T:
            ids[rng.integers(0, T), 0] = E + 3                        # an invalid id
        if trial % 7 == 0:
            e2r[rng.integers(0, E)] = G                               # an expert without a valid placement
        Zn, sn = oracle.swap_counts(ids, e2r, G, ng, "naive")
        Zi, si = oracle.swap_counts(ids, e2r, G, ng, "incremental")
        assert np.array_equal(Zn, Zi) and sn == si, (ids.tolist(), e2r.tolist(), G, ng)


def test_z_structure(oracle):
    wl = W.WORKLOADS["tiny"]
    r = W.make_routing(wl, T=400)
    ids, e2r, G = r.topk_ids, r.expert_to_rank, wl.G
    for ng in (G, wl.nodes):
        Z, st = oracle.swap_counts(ids, e2r, G, ng)
        per = G // ng
        base, _ = oracle.group_counts(ids, e2r, G, [ng])
        grp = e2r // per
        assert st == 0 and np.array_equal(Z, Z.transpose(1, 0, 2))                 # swapping r,c == swapping c,r
        same = grp[:, None] == grp[None, :]
        assert (Z[same] == base[0, :ng]).all()                                      # a swap inside one group changes nothing
        # only the two groups involved can change
        for rr, cc in [(0, 5), (3, 12), (7, 9), (15, 0)]:
            others = [j for j in range(ng) if j not in (grp[rr], grp[cc])]
            assert (Z[rr, cc, others] == base[0, others]).all()
        # tokens selecting both or neither of the pair are unaffected: restrict to them and recount
        rr, cc = 1, 14
        both_or_neither = np.array([((row == rr).any() == (row == cc).any()) for row in ids])
        Zs, _ = oracle.swap_counts(ids[both_or_neither], e2r, G, ng)
        bs, _ = oracle.group_counts(ids[both_or_neither], e2r, G, [ng])
        assert np.array_equal(Zs[rr, cc], bs[0, :ng])
        # the same numbers through the separately written per-level counter
        gc, _ = oracle.group_counts(ids, _swapped(e2r, 2, 13), G, [ng])
        assert np.array_equal(Z[2, 13], gc[0, :ng])


def test_smooth_max_and_selection(oracle):
    """Eq.(8)-(11) on a hand-sized case and against numpy."""
    E, G = 3, 2
    # one dimension: Q = alpha + G * smax(Z[r,c,:]) * M v * beta
    Z = np.zeros((E, E, G), np.int32)
    Z[:] = [4, 4]
    Z[0, 1] = Z[1, 0] = [5, 2]
    Z[0, 2] = Z[2, 0] = [3, 3]
    Q, best, bt = oracle.swap_select([1], G, 2.0, 1.0, [None], Z, [0], 1.0, [0], [0], 10.0, 0.5, 0.0)
    assert Q[0, 1] == 10 + 2 * 5 * 2 * 0.5 and Q[0, 2] == 10 + 2 * 3 * 2 * 0.5 and Q[1, 1] == 10 + 2 * 4 * 2 * 0.5
    assert best == (0, 2) and bt == 16.0                                             # first minimiser in row-major order
    # smooth maximum: n equal entries m -> m * n^(1/gamma); dominated entries vanish as gamma grows
    Q10, _, _ = oracle.swap_select([1], G, 1.0, 1.0, [None], Z, [0], 1.0, [0], [0], 0.0, 1.0, 10.0)
    assert abs(Q10[1, 1] - G * 4 * 2 ** 0.1) < 1e-12
    assert abs(Q10[0, 1] - G * 5 * (1 + 0.4 ** 10) ** 0.1) < 1e-12
    Qbig, _, _ = oracle.swap_select([1], G, 1.0, 1.0, [None], Z, [0], 1.0, [0], [0], 0.0, 1.0, 400.0)
    assert abs(Qbig[0, 1] - G * 5) < 1e-9
    # against numpy on a real workload, two dimensions, gamma = 10 (the paper's default)
    wl = W.WORKLOADS["skew"]
    r = W.make_routing(wl, T=256)
    e2r = r.extras["expert_to_rank_swapped"]
    Zn, _ = oracle.swap_counts(r.topk_ids, e2r, wl.G, wl.nodes)
    Zg, _ = oracle.swap_counts(r.topk_ids, e2r, wl.G, wl.G)
    U, M, v, gamma = [1, wl.nodes], 2048.0, 2.0, 10.0
    ai, bi, aa, ba = [0, 0.497], [0, 5.29e-7], 0.571, 1.27e-7
    Q, best, bt = oracle.swap_select(U, wl.G, M, v, [None, Zn], Zg, [0, 1.0], float(wl.nodes), ai, bi, aa, ba, gamma)

    def smax(x):
        m = x.max(axis=-1).astype(np.float64)
        s = ((x / np.maximum(m, 1)[..., None]) ** gamma).sum(-1) ** (1 / gamma)
        return np.where(m > 0, m * s, 0.0)

    ref = (wl.nodes * smax(Zn) * M * v * bi[1] + ai[1]) + ((wl.G // wl.nodes) * wl.nodes * smax(Zg) * M * v * ba + aa)
    assert np.allclose(Q, ref, rtol=1e-12, atol=0)
    assert best == tuple(int(i) for i in np.unravel_index(np.argmin(Q), Q.shape)) and bt == Q[best]
    # the chosen swap does not make things worse than no swap (r == c is always a candidate)
    assert bt <= Q[0, 0]


def test_swap_apply_and_the_planner_loop(oracle):
    """Applying the chosen pair exchanges two placement entries; the load of the new placement is
    the row Z[r,c,:] that predicted it, and a greedy loop of (Z, select, apply) never raises the
    estimated time and stops changing the placement once the diagonal wins."""
    e2r = np.array([0, 0, 1, 1, 2, 3], np.int32)
    assert oracle.swap_apply(e2r, (1, 4)).tolist() == [0, 2, 1, 1, 0, 3]
    assert oracle.swap_apply(e2r, (4, 1)).tolist() == [0, 2, 1, 1, 0, 3]
    for pair in ((2, 2), (-1, 3), (0, 6), (7, 7)):
        assert oracle.swap_apply(e2r, pair).tolist() == e2r.tolist()
    assert e2r.tolist() == [0, 0, 1, 1, 2, 3]                           # the wrapper works on a copy

    wl = W.WORKLOADS["skew"]
    r = W.make_routing(wl, T=512)
    place = r.expert_to_rank.copy()
    M, v = 2048.0, 2.0
    times = []
    for it in range(6):
        Zg, _ = oracle.swap_counts(r.topk_ids, place, wl.G, wl.G)
        Q, best, bt = oracle.swap_select([1], wl.G, M, v, [None], Zg, [0], 1.0, [0], [0], 0.3, 1e-6, 10.0)
        nxt = oracle.swap_apply(place, best)
        assert np.array_equal(nxt, _swapped(place, *best))
        # the prediction Z[r,c,:] is the duplicate-free load of the placement just produced
        _, lr, _, _ = oracle.expert_load(r.topk_ids, nxt, wl.nodes, wl.ranks_per_node)
        assert np.array_equal(lr, Zg[best[0], best[1]])
        smax = lr.max() * ((lr / lr.max()) ** 10.0).sum() ** 0.1         # Eq.(11), gamma = 10: a plain maximum
        assert abs(bt - (0.3 + wl.G * smax * M * v * 1e-6)) <= 1e-12 * bt   # cannot see past the hottest rank
        times.append(bt)
        if best[0] == best[1]:
            assert np.array_equal(nxt, place)
        place = nxt
    assert all(b <= a for a, b in zip(times, times[1:])) and times[-1] < times[0]
