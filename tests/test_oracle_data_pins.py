"""Pins for the oracle's data functions: bf16 rounding, dispatch pack, combine, transpose.

CPU only.  The references here are exact rational arithmetic (fractions), numpy library
routines for the special cases that reduce to them (plain MoE permute and weighted sum at
dedup level none), algebraic identities (round trip, adjoint) and the closed form of the
scaled-expert model.
"""
from fractions import Fraction

import numpy as np
import pytest

from helpers import GPU, NODE, NONE, bf16_ulp_distance, exact_round_to_bf16, exact_round_to_f32
from paper_2508_09591_amd import workloads as W


# ---- rounding binary64 -> bf16 --------------------------------------------------------------
def test_bf16_rounding_is_identity_on_bf16_values(oracle):
    for enc in list(range(0, 0x7F80, 97)) + [0x0001, 0x007F, 0x0080, 0x7F7F]:
        for sign in (0, 0x8000):
            v = float(W.bf16_bits_to_f64(np.array([enc | sign], np.uint16))[0])
            assert oracle.f64_to_bf16(v) == (enc | sign)


def test_bf16_rounding_against_exact_rationals(oracle):
    rng = np.random.default_rng(0)
    vals = list(rng.standard_normal(400) * np.exp(rng.uniform(-90, 90, 400)))
    # exact midpoints between neighbouring bf16 values (ties) and their two double neighbours
    for enc in (0x3F80, 0x3F81, 0x4000, 0x0001, 0x007F, 0x0080, 0x7F7E, 0x3EFF, 0x0000):
        lo = float(W.bf16_bits_to_f64(np.array([enc], np.uint16))[0])
        hi = float(W.bf16_bits_to_f64(np.array([enc + 1], np.uint16))[0])
        mid = (lo + hi) / 2                       # exact in binary64
        vals += [mid, np.nextafter(mid, 0.0), np.nextafter(mid, np.inf), -mid]
    # a double that rounds differently when it is first rounded to binary32 (double rounding)
    vals.append(1.0 + 2.0 ** -8 + 2.0 ** -40)      # just above the tie 1 + 2^-8 -> must round up
    vals.append(1.0 + 2.0 ** -8 - 2.0 ** -40)      # just below -> must round down
    vals += [3.4e38, -3.4e38, 3.3895e38, 1e-45, 4.6e-41, 9.2e-41, 0.0, -0.0]
    for v in vals:
        v = float(v)
        got = oracle.f64_to_bf16(v)
        if v == 0.0:                      # a rational has no signed zero
            assert got == (0x8000 if np.signbit(v) else 0), v
        else:
            assert got == exact_round_to_bf16(Fraction(v)), v
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8 + 2.0 ** -40) == 0x3F81
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8 - 2.0 ** -40) == 0x3F80
    assert oracle.f64_to_bf16(1.0 + 2.0 ** -8) == 0x3F80           # tie -> even
    assert oracle.f64_to_bf16(1.0 + 3 * 2.0 ** -8) == 0x3F82       # tie -> even (up)


# ---- dispatch pack ----------------------------------------------------------------------------
@pytest.mark.parametrize("name,level", [("tiny", NONE), ("tiny", GPU), ("tiny", NODE), ("qwen3", GPU), ("qwen3", NODE)])
def test_dispatch_pack_rows(oracle, name, level):
    wl = W.WORKLOADS[name]
    T = min(wl.T, 1024)
    r = W.make_routing(wl, T=T)
    x = W.make_activations(wl, T=T, H=min(wl.H, 512))
    p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
    packed = oracle.dispatch_pack(x, p.row_token)
    assert packed.shape == (p.total_rows, x.shape[1])
    # every slot finds its token's row in the destination's buffer
    assert np.array_equal(packed[p.slot_row.reshape(-1)], np.repeat(x, wl.K, axis=0))
    # every packed row is reached by some slot: nothing else was written
    assert np.array_equal(np.unique(p.slot_row), np.arange(p.total_rows))
    if level == NONE:
        # the standard MoE permute: rows sorted by destination, stable
        d = r.expert_to_rank[r.topk_ids].reshape(-1)
        order = np.argsort(d, kind="stable")
        assert np.array_equal(packed, x[order // wl.K])


# ---- combine ------------------------------------------------------------------------------------
def test_combine_exact_rational_small(oracle):
    rng = np.random.default_rng(3)
    T, K, H, E = 5, 3, 7, 6
    ids = rng.integers(0, E, (T, K), dtype=np.int32)
    w = rng.random((T, K), dtype=np.float32)
    e2r = np.array([0, 0, 1, 1, 2, 3], np.int32)
    for level in (NONE, GPU, NODE):
        p = oracle.plan(ids, w, e2r, 2, 2, level)
        y = W.f32_to_bf16_bits(rng.standard_normal((p.total_rows, H)).astype(np.float32) * 3)
        out = oracle.combine(y, w, p.slot_row)
        yf = W.bf16_bits_to_f64(y)
        for t in range(T):
            for j in range(H):
                q = sum(Fraction(float(w[t, k])) * Fraction(float(yf[p.slot_row[t, k], j])) for k in range(K))
                assert int(out[t, j]) == exact_round_to_bf16(q), (level, t, j)


def test_combine_accumulates_beyond_binary32(oracle):
    """Sums that sit 2^-30 above a bf16 rounding tie: a binary32 accumulator would land on the tie
    and round to even (down); the binary64 sum rounded once must round up."""
    ids = np.array([[0, 2]], np.int32)
    e2r = np.array([0, 0, 1, 1], np.int32)
    one = W.f32_to_bf16_bits(np.array([1.0], np.float32))[0]
    for bump, want in ((2.0 ** -30, 0x3F81), (-2.0 ** -30, 0x3F80), (0.0, 0x3F80)):
        w = np.array([[1.0, 2.0 ** -8 + bump]], np.float32)
        assert float(w[0, 1]) == 2.0 ** -8 + bump                       # representable in binary32
        p = oracle.plan(ids, w, e2r, 2, 1, GPU)
        y = np.full((p.total_rows, 3), one, np.uint16)
        out = oracle.combine(y, w, p.slot_row)
        q = Fraction(1) + Fraction(float(w[0, 1]))
        assert exact_round_to_bf16(q) == want
        assert out.tolist() == [[want] * 3], (bump, out)


def test_combine_level_none_is_plain_moe_weighted_sum(oracle):
    wl = W.WORKLOADS["tiny"]
    r = W.make_routing(wl, T=256)
    rng = np.random.default_rng(9)
    p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, NONE)
    y = W.f32_to_bf16_bits(rng.standard_normal((p.total_rows, 64)).astype(np.float32))
    out = oracle.combine(y, r.topk_weights, p.slot_row)
    # out[t] = sum_k w[t,k] * y_slot[t,k]  (library einsum in fp64), rounded once
    y_slot = W.bf16_bits_to_f64(y)[p.slot_row]                           # [T,K,H]
    ref = np.einsum("tk,tkh->th", r.topk_weights.astype(np.float64), y_slot)
    ref_bits = np.array([[exact_round_to_bf16(Fraction(float(v))) for v in row] for row in ref[:16]], np.uint16)
    # einsum's fp64 summation order may differ in the last bit of the double: allow 1 ulp there
    assert bf16_ulp_distance(out[:16], ref_bits).max() <= 1
    assert np.abs(W.bf16_bits_to_f64(out) - ref).max() <= 2.0 ** -8 * np.abs(ref).max()


# ---- combine on binary32 rows ---------------------------------------------------------------------
def test_exact_f32_rounding_helper():
    assert exact_round_to_f32(Fraction(1, 3)) == float(np.float32(1.0) / np.float32(3.0))
    assert exact_round_to_f32(Fraction(1) + Fraction(1, 2 ** 24)) == 1.0                  # tie -> even
    assert exact_round_to_f32(Fraction(1) + Fraction(3, 2 ** 24)) == 1.0 + 2.0 ** -22      # tie -> even (up)
    assert exact_round_to_f32(-(Fraction(1) + Fraction(1, 2 ** 24) + Fraction(1, 2 ** 60))) == -(1.0 + 2.0 ** -23)


def test_combine_f32_exact_rational_small(oracle):
    rng = np.random.default_rng(31)
    T, K, H, E = 6, 3, 5, 6
    ids = rng.integers(0, E, (T, K), dtype=np.int32)
    w = rng.random((T, K), dtype=np.float32)
    e2r = np.array([0, 0, 1, 1, 2, 3], np.int32)
    for level in (NONE, GPU, NODE):
        p = oracle.plan(ids, w, e2r, 2, 2, level)
        y = (rng.standard_normal((p.total_rows, H)) * 3).astype(np.float32)
        out = oracle.combine_f32(y, w, p.slot_row)
        assert out.dtype == np.float32 and out.shape == (T, H)
        for t in range(T):
            for j in range(H):
                q = sum(Fraction(float(w[t, k])) * Fraction(float(y[p.slot_row[t, k], j])) for k in range(K))
                assert float(out[t, j]) == exact_round_to_f32(q), (level, t, j)


def test_combine_f32_accumulates_beyond_binary32(oracle):
    """1 + 2^-24 + 2^-30: a binary32 accumulator stops at the tie 1 + 2^-24 -> 1 and then loses the
    last term; the exact sum lies above the tie and rounds up."""
    ids = np.array([[0, 1, 2]], np.int32)
    e2r = np.array([0, 1, 2], np.int32)
    w = np.array([[1.0, 2.0 ** -24, 2.0 ** -30]], np.float32)
    p = oracle.plan(ids, w, e2r, 3, 1, GPU)
    assert p.total_rows == 3
    y = np.ones((3, 4), np.float32)
    out = oracle.combine_f32(y, w, p.slot_row)
    assert out.tolist() == [[1.0 + 2.0 ** -23] * 4]
    w[0, 2] = 0.0                                       # the exact tie: to even, down
    assert oracle.combine_f32(y, w, p.slot_row).tolist() == [[1.0] * 4]
    w[0, 1] = -(2.0 ** -25)                             # 1 - 2^-25: a tie below 1 (spacing 2^-24), to even = 1
    assert oracle.combine_f32(y, w, p.slot_row).tolist() == [[1.0] * 4]


def test_combine_f32_is_plain_weighted_sum_and_agrees_with_bf16_combine(oracle):
    wl = W.WORKLOADS["qwen3"]
    r = W.make_routing(wl, T=200)
    rng = np.random.default_rng(19)
    for level in (NONE, NODE):
        p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        yb = W.f32_to_bf16_bits(rng.standard_normal((p.total_rows, 48)).astype(np.float32))
        y = W.bf16_bits_to_f32(yb)
        out = oracle.combine_f32(y, r.topk_weights, p.slot_row)
        ref = np.einsum("tk,tkh->th", r.topk_weights.astype(np.float64), y.astype(np.float64)[p.slot_row])
        assert np.abs(out.astype(np.float64) - ref).max() <= 2.0 ** -23 * np.abs(ref).max()
        # the same rows through the bf16 path: its result is this one rounded once more to bf16
        ob = oracle.combine(yb, r.topk_weights, p.slot_row)
        assert bf16_ulp_distance(ob, W.f32_to_bf16_bits(out)).max() <= 1
    # dropped slots contribute nothing
    sr = p.slot_row.copy()
    sr[:, 1:] = -1
    out = oracle.combine_f32(y, r.topk_weights, sr)
    want = (r.topk_weights[:, :1].astype(np.float64) * y.astype(np.float64)[sr[:, 0]]).astype(np.float32)
    assert np.array_equal(out, want)


@pytest.mark.parametrize("name", ["tiny", "dsv3"])
def test_identity_expert_round_trip_is_exact(oracle, name):
    wl = W.WORKLOADS[name]
    T, H = 512, 128
    r = W.make_routing(wl, T=T)
    x = W.make_activations(wl, T=T, H=H)
    assert np.abs(r.topk_weights.astype(np.float64).sum(1) - 1).max() < 4 * 2.0 ** -24
    for level in (NONE, GPU, NODE):
        p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        packed = oracle.dispatch_pack(x, p.row_token)
        out = oracle.combine(packed, r.topk_weights, p.slot_row)
        # equal as values: the only bit difference allowed is -0.0 coming back as +0.0
        assert bf16_ulp_distance(out, x).max() == 0, level
        assert np.array_equal(out[x != 0x8000], x[x != 0x8000]), level


def test_scaled_experts_closed_form_all_levels(oracle):
    """Expert e returns c[e] * x.  A row that serves several experts of one destination carries
    their weight-normalised mixture, so the layer output is (sum_k w_k c[e_k]) * x at every level."""
    wl = W.WORKLOADS["qwen3"]
    T, H = 384, 96
    r = W.make_routing(wl, T=T)
    x = W.make_activations(wl, T=T, H=H)
    c = W.make_expert_scales(wl)
    xf = W.bf16_bits_to_f64(x)
    coef = (r.topk_weights.astype(np.float64) * c[r.topk_ids].astype(np.float64)).sum(1)
    expect = coef[:, None] * xf
    for level in (NONE, GPU, NODE):
        p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        packed = oracle.dispatch_pack(x, p.row_token)
        num = np.zeros(p.total_rows)
        np.add.at(num, p.slot_row.reshape(-1), (r.topk_weights * c[r.topk_ids]).astype(np.float64).reshape(-1))
        s = num / p.row_weight.astype(np.float64)
        y = W.f32_to_bf16_bits((s[:, None] * W.bf16_bits_to_f64(packed)).astype(np.float32))
        out = W.bf16_bits_to_f64(oracle.combine(y, r.topk_weights, p.slot_row))
        # Y is rounded to bf16 once (rel 2^-9), the output once more (rel 2^-9)
        assert np.all(np.abs(out - expect) <= 2.0 ** -7 * np.abs(expect) + 1e-30), level


# ---- transpose ----------------------------------------------------------------------------------
@pytest.mark.parametrize("level", [NONE, GPU, NODE])
def test_transpose_is_adjoint_and_one_multiply(oracle, level):
    wl = W.WORKLOADS["stress"]
    T, H = 300, 40
    r = W.make_routing(wl, T=T)
    rng = np.random.default_rng(17)
    p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
    gout = W.make_output_grads(wl, T=T, H=H)
    gy = oracle.combine_transpose(gout, p.row_token, p.row_weight)
    # one IEEE binary32 multiply per element
    assert np.array_equal(gy, p.row_weight[:, None] * gout[p.row_token])
    # <combine(Y), g> == <Y, combine^T(g)> with the linear (unrounded) combine in fp64
    y = rng.standard_normal((p.total_rows, H))
    lin = np.zeros((T, H))
    for k in range(wl.K):
        lin += r.topk_weights[:, k].astype(np.float64)[:, None] * y[p.slot_row[:, k]]
    lhs = float((lin * gout.astype(np.float64)).sum())
    # exact adjoint uses the exact per-row weight sums; row_weight is their fp32 rounding
    rhs = float((y * gy.astype(np.float64)).sum())
    scale = float(np.abs(lin * gout).sum())
    assert abs(lhs - rhs) <= 4e-7 * scale
    # with the exact (fp64) row weights the identity holds to rounding of the dot products
    rw64 = np.zeros(p.total_rows)
    np.add.at(rw64, p.slot_row.reshape(-1), r.topk_weights.astype(np.float64).reshape(-1))
    rhs64 = float((y * (rw64[:, None] * gout.astype(np.float64)[p.row_token])).sum())
    assert abs(lhs - rhs64) <= 1e-12 * scale


def test_transpose_bf16_exact_products_and_double_rounding_trap(oracle):
    """Gradients in bf16: the product is rounded ONCE to bf16.  Checked against exact rational
    arithmetic on a plan with merged rows, on a weight of one (bit copy), and on a product whose
    binary32 rounding lands on a bf16 tie, so that rounding twice gives the other neighbour."""
    wl = W.WORKLOADS["qwen3"]
    T, H = 40, 9
    r = W.make_routing(wl, T=T)
    rng = np.random.default_rng(23)
    for level in (NONE, NODE):
        p = oracle.plan(r.topk_ids, r.topk_weights, r.expert_to_rank, wl.nodes, wl.ranks_per_node, level)
        g = W.f32_to_bf16_bits((rng.standard_normal((T, H)) * 1e-2).astype(np.float32))
        gy = oracle.combine_transpose_bf16(g, p.row_token, p.row_weight)
        assert gy.shape == (p.total_rows, H) and gy.dtype == np.uint16
        gf = W.bf16_bits_to_f64(g)
        for row in range(0, p.total_rows, 7):
            for j in range(H):
                q = Fraction(float(p.row_weight[row])) * Fraction(float(gf[p.row_token[row], j]))
                assert int(gy[row, j]) == exact_round_to_bf16(q), (level, row, j)
    # weight one: the row comes back bit for bit
    ones = np.ones(p.total_rows, np.float32)
    assert np.array_equal(oracle.combine_transpose_bf16(g, p.row_token, ones), g[p.row_token])
    # w = 1 + 2^-8 + 2^-17 (24 significant bits), g = 1 + 2^-7: the product is
    # 1 + 2^-7 + 2^-8 + 2^-15 + 2^-17 + 2^-24, above the bf16 tie 1 + 2^-7 + 2^-8 -> rounds up to
    # 1 + 2^-6; with w = 1 + 2^-8 exactly the product is 1 + 2^-7 + 2^-8 + 2^-15: still above the tie.
    # Below the tie: w = 1 + 2^-8 - 2^-14 gives 1 + 2^-7 + 2^-8 - 2^-14 + ... -> rounds down.
    one_p = W.f32_to_bf16_bits(np.array([[1.0 + 2.0 ** -7]], np.float32))
    for w, want in ((1.0 + 2.0 ** -8 + 2.0 ** -17, 1.0 + 2.0 ** -6), (1.0 + 2.0 ** -8 - 2.0 ** -14, 1.0 + 2.0 ** -7)):
        wv = np.array([w], np.float32)
        assert float(wv[0]) == w
        out = oracle.combine_transpose_bf16(one_p, np.array([0], np.int32), wv)
        q = Fraction(w) * Fraction(1.0 + 2.0 ** -7)
        assert exact_round_to_bf16(q) == int(W.f32_to_bf16_bits(np.array([want], np.float32))[0])
        assert int(out[0, 0]) == exact_round_to_bf16(q)
    # the double-rounding trap proper: the exact product lies just above a bf16 tie but its
    # binary32 rounding lands ON the tie, whose even neighbour is the lower one
    # (around w * g = 1 + 2^-6 + 2^-8, the tie between an even and an odd bf16 value)
    found = 0
    gb = W.f32_to_bf16_bits(np.array([[1.0 + 2.0 ** -7]], np.float32))
    for n in range(97000, 98100):
        w = np.float32(1.0 + n * 2.0 ** -23)
        q = Fraction(float(w)) * Fraction(1.0 + 2.0 ** -7)
        once = exact_round_to_bf16(q)
        twice = int(W.f32_to_bf16_bits(np.array([np.float32(float(w) * (1.0 + 2.0 ** -7))], np.float32))[0])
        if once != twice:
            found += 1
            out = oracle.combine_transpose_bf16(gb, np.array([0], np.int32), np.array([w], np.float32))
            assert int(out[0, 0]) == once
    assert found > 0
