"""Seeded synthetic MoE-layer inputs (routing tables, weights, activations).

This module only *produces inputs* for the dedup dispatch/combine path: top-k
expert ids, router weights, the expert->rank placement and bf16 activations.
It holds none of the method's arithmetic (no dedup, no plan, no packing, no
combine), so both the CPU oracle's tests and the HIP path's tests may draw
their inputs from it.  Everything is numpy on the CPU and a pure function of
the seed.

The paper trains DeepSeek-V3 (halved dims) and Qwen3-30B-A3B with micro-batch
1, sequence 1024 and EP=32 (Section V-A, "Real-World MoE Models"); no routing
traces are published, so the five workloads below use the models' layer shapes
with random routers.

bf16 tensors are carried as numpy uint16 arrays holding the raw encodings.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Dict, Optional, Tuple

import numpy as np

LEVEL_NONE, LEVEL_GPU, LEVEL_NODE = 0, 1, 2
LEVEL_NAMES = {LEVEL_NONE: "none", LEVEL_GPU: "gpu", LEVEL_NODE: "node"}


# --------------------------------------------------------------------------
# bf16 <-> fp32 encodings (input preparation / test read-back only)
# --------------------------------------------------------------------------
def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round fp32 to bf16 (nearest even); returns the uint16 encodings."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def bf16_bits_to_f64(b: np.ndarray) -> np.ndarray:
    return bf16_bits_to_f32(b).astype(np.float64)


# --------------------------------------------------------------------------
# workload description
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    H: int
    E: int
    K: int
    nodes: int
    ranks_per_node: int
    router: str            # "softmax" | "deepseek" | "softmax_zipf"
    levels: Tuple[int, ...]
    seed: int
    expert_model: str      # "identity" | "scaled"
    n_groups: int = 1      # DeepSeek group-limited routing
    topk_groups: int = 1

    @property
    def G(self) -> int:
        return self.nodes * self.ranks_per_node


WORKLOADS: Dict[str, Workload] = {
    # configs[0]: tiny reference layer
    "tiny": Workload("tiny", T=1024, H=256, E=16, K=2, nodes=2, ranks_per_node=2,
                     router="softmax", levels=(LEVEL_NONE, LEVEL_GPU, LEVEL_NODE), seed=0,
                     expert_model="identity"),
    # configs[1]: Qwen3-30B-A3B-shaped layer
    "qwen3": Workload("qwen3", T=8192, H=2048, E=128, K=8, nodes=4, ranks_per_node=8,
                      router="softmax", levels=(LEVEL_GPU, LEVEL_NODE), seed=1,
                      expert_model="scaled"),
    # configs[2]: DeepSeek-V3-shaped layer (headline)
    "dsv3": Workload("dsv3", T=8192, H=7168, E=256, K=8, nodes=4, ranks_per_node=8,
                     router="deepseek", levels=(LEVEL_NODE,), seed=2,
                     expert_model="identity", n_groups=8, topk_groups=4),
    # configs[3]: skewed-load layer for the expert swap
    "skew": Workload("skew", T=16384, H=2048, E=128, K=8, nodes=4, ranks_per_node=8,
                     router="softmax_zipf", levels=(LEVEL_GPU, LEVEL_NODE), seed=3,
                     expert_model="scaled"),
    # configs[4]: large-token stress layer
    "stress": Workload("stress", T=65536, H=7168, E=256, K=8, nodes=8, ranks_per_node=8,
                       router="deepseek", levels=(LEVEL_NODE, LEVEL_GPU), seed=4,
                       expert_model="identity", n_groups=8, topk_groups=4),
}


def table4_variants():
    """The K / E / G grid of the paper's Table IV (one parameter varied at a time around the
    defaults K=8, E=128, G=32) on the Qwen3-30B-A3B-shaped layer; 8 ranks per node."""
    import dataclasses
    base = WORKLOADS["qwen3"]
    out = []
    for K in (6, 8, 10):
        out.append(dataclasses.replace(base, name="K%d" % K, K=K, seed=40 + K))
    for E in (64, 256):
        out.append(dataclasses.replace(base, name="E%d" % E, E=E, seed=50 + E))
    for G in (8, 16):
        out.append(dataclasses.replace(base, name="G%d" % G, nodes=G // 8, seed=60 + G))
    return out


@dataclass
class Routing:
    topk_ids: np.ndarray        # [T,K] int32, slot order = descending score
    topk_weights: np.ndarray    # [T,K] float32
    expert_to_rank: np.ndarray  # [E] int32
    extras: dict = field(default_factory=dict)


# --------------------------------------------------------------------------
# routers (they make inputs; the library never sees logits)
# --------------------------------------------------------------------------
def _topk_desc(scores: np.ndarray, K: int) -> np.ndarray:
    """Indices of the K largest entries per row, descending, ties to the lower index."""
    order = np.argsort(-scores, axis=1, kind="stable")
    return np.ascontiguousarray(order[:, :K])


def softmax_topk(logits: np.ndarray, K: int):
    ids = _topk_desc(logits, K)
    sel = np.take_along_axis(logits, ids, axis=1).astype(np.float32)
    sel = sel - sel.max(axis=1, keepdims=True)
    ex = np.exp(sel, dtype=np.float32)
    w = (ex / ex.sum(axis=1, keepdims=True, dtype=np.float32)).astype(np.float32)
    return ids.astype(np.int32), w


def deepseek_group_limited_topk(logits: np.ndarray, K: int, n_groups: int, topk_groups: int):
    """Sigmoid scores; rank groups by the sum of their two best scores; keep the best
    `topk_groups` groups; take the K best experts inside them; weights are the
    selected scores normalised to sum to one."""
    T, E = logits.shape
    per = E // n_groups
    scores = (1.0 / (1.0 + np.exp(-logits.astype(np.float32)))).astype(np.float32)
    g = scores.reshape(T, n_groups, per)
    top2 = -np.sort(-g, axis=2)[:, :, :2]
    gscore = top2.sum(axis=2, dtype=np.float32)
    keep_groups = _topk_desc(gscore, topk_groups)                      # [T, topk_groups]
    gmask = np.zeros((T, n_groups), dtype=bool)
    np.put_along_axis(gmask, keep_groups, True, axis=1)
    masked = np.where(np.repeat(gmask, per, axis=1), scores, np.float32(-1.0))
    ids = _topk_desc(masked, K)
    sel = np.take_along_axis(scores, ids, axis=1)
    w = (sel / sel.sum(axis=1, keepdims=True, dtype=np.float32)).astype(np.float32)
    return ids.astype(np.int32), w


def contiguous_placement(E: int, G: int) -> np.ndarray:
    """Expert e lives on rank e // (E/G): the contiguous blocks of Eq.(7)."""
    return (np.arange(E, dtype=np.int64) // (E // G)).astype(np.int32)


def zipf_log_bias(E: int, rng: np.random.Generator, s: float = 1.2) -> np.ndarray:
    """log of a Zipf(s) pmf over expert popularity ranks, assigned through a random permutation."""
    ranks = np.arange(1, E + 1, dtype=np.float64)
    pmf = ranks ** (-s)
    pmf /= pmf.sum()
    perm = rng.permutation(E)              # perm[e] = popularity rank (0-based) of expert e
    return np.log(pmf[perm]).astype(np.float32)


def make_routing(wl: Workload, T: Optional[int] = None) -> Routing:
    """Routing tables for a workload; `T` overrides the token count (reduced-size tests)."""
    T = wl.T if T is None else T
    rng = np.random.default_rng(wl.seed)
    extras = {}
    logits = rng.standard_normal((T, wl.E), dtype=np.float32)
    if wl.router == "softmax":
        ids, w = softmax_topk(logits, wl.K)
    elif wl.router == "softmax_zipf":
        bias = zipf_log_bias(wl.E, rng)
        extras["bias"] = bias
        ids, w = softmax_topk(logits + bias[None, :], wl.K)
        # a second placement: the contiguous map composed with a random expert permutation
        extras["expert_to_rank_swapped"] = contiguous_placement(wl.E, wl.G)[rng.permutation(wl.E)].astype(np.int32)
    elif wl.router == "deepseek":
        ids, w = deepseek_group_limited_topk(logits, wl.K, wl.n_groups, wl.topk_groups)
    else:
        raise ValueError(wl.router)
    return Routing(ids, w, contiguous_placement(wl.E, wl.G), extras)


def make_activations(wl: Workload, T: Optional[int] = None, H: Optional[int] = None,
                     chunk_tokens: int = 4096) -> np.ndarray:
    """X ~ N(0,1) fp32 rounded to bf16; returns uint16 encodings [T,H]."""
    T = wl.T if T is None else T
    H = wl.H if H is None else H
    rng = np.random.default_rng([wl.seed, 0x5EED])
    out = np.empty((T, H), dtype=np.uint16)
    for t0 in range(0, T, chunk_tokens):
        t1 = min(T, t0 + chunk_tokens)
        out[t0:t1] = f32_to_bf16_bits(rng.standard_normal((t1 - t0, H), dtype=np.float32))
    return out


def make_expert_scales(wl: Workload) -> np.ndarray:
    """Per-expert output scale ~ U(0.5,1.5) (the 'scaled' expert model of the test harness)."""
    rng = np.random.default_rng([wl.seed, 0xE5CA1E])
    return rng.uniform(0.5, 1.5, size=wl.E).astype(np.float32)


def make_output_grads(wl: Workload, T: Optional[int] = None, H: Optional[int] = None,
                      sigma: float = 1e-2, chunk_tokens: int = 4096) -> np.ndarray:
    """fp32 output gradients ~ N(0, sigma^2) [T,H] for the combine transpose (sigma = 1e-2)."""
    T = wl.T if T is None else T
    H = wl.H if H is None else H
    rng = np.random.default_rng([wl.seed, 0x6BAD])
    out = np.empty((T, H), dtype=np.float32)
    for t0 in range(0, T, chunk_tokens):
        t1 = min(T, t0 + chunk_tokens)
        out[t0:t1] = rng.standard_normal((t1 - t0, H), dtype=np.float32) * np.float32(sigma)
    return out


def uniform_subset_routing(T: int, E: int, K: int, seed: int):
    """Each token picks a uniformly random K-subset of the E experts (Table II style)."""
    rng = np.random.default_rng(seed)
    keys = rng.random((T, E))
    ids = np.argsort(keys, axis=1, kind="stable")[:, :K].astype(np.int32)
    w = np.full((T, K), 1.0 / K, dtype=np.float32)
    return np.ascontiguousarray(ids), w
