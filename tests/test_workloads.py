"""The seeded input generators: shapes, determinism and the routing rules they promise."""
import numpy as np
import pytest

from paper_2508_09591_amd import workloads as W


@pytest.mark.parametrize("name", list(W.WORKLOADS))
def test_routing_shapes_and_rules(name):
    wl = W.WORKLOADS[name]
    T = min(wl.T, 2048)
    r = W.make_routing(wl, T=T)
    r2 = W.make_routing(wl, T=T)
    assert np.array_equal(r.topk_ids, r2.topk_ids) and np.array_equal(r.topk_weights, r2.topk_weights)
    assert r.topk_ids.shape == (T, wl.K) and r.topk_ids.dtype == np.int32
    assert r.topk_weights.shape == (T, wl.K) and r.topk_weights.dtype == np.float32
    assert r.topk_ids.min() >= 0 and r.topk_ids.max() < wl.E
    # distinct experts per token, positive weights that sum to one, slots in descending weight order
    assert all(len(set(row)) == wl.K for row in r.topk_ids.tolist())
    assert (r.topk_weights > 0).all()
    assert np.abs(r.topk_weights.astype(np.float64).sum(1) - 1).max() < 1e-6
    assert (np.diff(r.topk_weights, axis=1) <= 0).all()
    assert np.array_equal(r.expert_to_rank, np.arange(wl.E) // (wl.E // wl.G))
    if wl.router == "deepseek":
        groups = r.topk_ids // (wl.E // wl.n_groups)
        assert max(len(set(g)) for g in groups.tolist()) <= wl.topk_groups
    if wl.router == "softmax_zipf":
        sw = r.extras["expert_to_rank_swapped"]
        assert sorted(sw.tolist()) == sorted(r.expert_to_rank.tolist())        # same experts per rank count
        load = np.bincount(r.topk_ids.reshape(-1), minlength=wl.E)
        assert load.max() > 5 * load.mean()                                     # skewed


def test_activations_and_bf16_helpers():
    wl = W.WORKLOADS["tiny"]
    x = W.make_activations(wl)
    assert x.shape == (wl.T, wl.H) and x.dtype == np.uint16
    assert np.array_equal(x, W.make_activations(wl))
    xf = W.bf16_bits_to_f32(x)
    assert abs(float(xf.mean())) < 0.01 and abs(float(xf.std()) - 1) < 0.01
    assert np.array_equal(W.f32_to_bf16_bits(xf), x)                            # bf16 values round-trip
    # round to nearest even on the dropped 16 bits
    cases = np.array([0x3F800000, 0x3F808000, 0x3F818000, 0x3F808001, 0x3F807FFF], np.uint32).view(np.float32)
    assert W.f32_to_bf16_bits(cases).tolist() == [0x3F80, 0x3F80, 0x3F82, 0x3F81, 0x3F80]
    g = W.make_output_grads(W.WORKLOADS["stress"], T=64, H=128)
    assert g.dtype == np.float32 and abs(float(g.std()) - 1e-2) < 1e-3
