"""CPU oracle for the dedup dispatch/combine path -- TEST INFRASTRUCTURE ONLY.

A ctypes front end to ``hmo.c`` (plain single-threaded C, written from the paper:
HierMoE Eq.(7) and Sections II-A/B, III-A, IV).  Only tests, the smoke check and the
benchmark's CPU-baseline leg may import this package; the product path never does and
shares no code with it.  Arrays are numpy, on the host.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass
from typing import Optional

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "hmo.c")
_LIB = os.path.join(_HERE, "libhmo.so")

LEVEL_NONE, LEVEL_GPU, LEVEL_NODE = 0, 1, 2
RECV_INTRA_NODE, RECV_LOCAL_EXPERTS = 0, 1
BAD_ID = -7

# No -ffast-math, no contraction: the float adds and the single float multiply must be IEEE.
CFLAGS = ["-O2", "-std=c99", "-ffp-contract=off", "-fno-fast-math", "-shared", "-fPIC"]


def build(force: bool = False) -> str:
    """Compile hmo.c with gcc into libhmo.so next to it."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        tmp = _LIB + ".tmp.%d" % os.getpid()
        subprocess.check_call(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"])
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        _lib = ctypes.CDLL(build())
        _lib.hmo_f64_to_bf16.restype = ctypes.c_uint16
        _lib.hmo_f64_to_bf16.argtypes = [ctypes.c_double]
    return _lib


def _p(a: Optional[np.ndarray]):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _c(a, dtype):
    a = np.ascontiguousarray(a, dtype=dtype)
    return a


@dataclass
class Plan:
    level: int
    num_dest: int
    dest_count: np.ndarray    # [num_dest] int32
    dest_offset: np.ndarray   # [num_dest+1] int32
    row_token: np.ndarray     # [total_rows] int32
    slot_row: np.ndarray      # [T,K] int32
    slot_keep: np.ndarray     # [T,K] uint8
    row_weight: np.ndarray    # [total_rows] float32
    rank_mask: np.ndarray     # [T] uint64
    node_mask: np.ndarray     # [T] uint32
    status: int

    @property
    def total_rows(self) -> int:
        return int(self.dest_offset[-1])


def plan(topk_ids, topk_weights, expert_to_rank, nodes: int, ranks_per_node: int, level: int) -> Plan:
    lib = _load()
    ids = _c(topk_ids, np.int32)
    w = _c(topk_weights, np.float32)
    e2r = _c(expert_to_rank, np.int32)
    T, K = ids.shape
    E = e2r.shape[0]
    G = nodes * ranks_per_node
    Dn = nodes if level == LEVEL_NODE else G
    dest_count = np.zeros(max(Dn, 1), np.int32)
    dest_offset = np.zeros(max(Dn, 1) + 1, np.int32)
    row_token = np.full(max(T * K, 1), -1, np.int32)
    slot_row = np.full((T, K), -1, np.int32)
    slot_keep = np.zeros((T, K), np.uint8)
    row_weight = np.zeros(max(T * K, 1), np.float32)
    rank_mask = np.zeros(max(T, 1), np.uint64)
    node_mask = np.zeros(max(T, 1), np.uint32)
    status = np.zeros(1, np.int32)
    rc = lib.hmo_plan(_p(ids), _p(w), _p(e2r), ctypes.c_int32(T), ctypes.c_int32(K), ctypes.c_int32(E),
                      ctypes.c_int32(nodes), ctypes.c_int32(ranks_per_node), ctypes.c_int32(level),
                      _p(dest_count), _p(dest_offset), _p(row_token), _p(slot_row), _p(slot_keep),
                      _p(row_weight), _p(rank_mask), _p(node_mask), _p(status))
    if rc != 0:
        raise ValueError("hmo_plan: argument error %d" % rc)
    total = int(dest_offset[Dn])
    return Plan(level, Dn, dest_count[:Dn], dest_offset[:Dn + 1], row_token[:total].copy(), slot_row, slot_keep,
                row_weight[:total].copy(), rank_mask[:T], node_mask[:T], int(status[0]))


def dispatch_pack(x_rows: np.ndarray, row_token: np.ndarray) -> np.ndarray:
    """packed[row] = x[row_token[row]]; x is [T, ...] of any fixed-size dtype, rows are copied as bytes."""
    lib = _load()
    x = np.ascontiguousarray(x_rows)
    rt = _c(row_token, np.int32)
    T = x.shape[0]
    row_bytes = x.strides[0] if x.ndim > 1 else x.itemsize
    out = np.empty((rt.shape[0],) + x.shape[1:], dtype=x.dtype)
    if out.size == 0:
        return out
    rc = lib.hmo_dispatch_pack(_p(x), ctypes.c_int64(T), ctypes.c_int64(row_bytes), _p(rt),
                               ctypes.c_int64(rt.shape[0]), _p(out))
    if rc != 0:
        raise ValueError("hmo_dispatch_pack: argument error %d" % rc)
    return out


def combine(y_bf16: np.ndarray, topk_weights, slot_row) -> np.ndarray:
    """out[t] = bf16(sum_k w[t,k] * Y[slot_row[t,k]]) in binary64; y and out are uint16 bf16 encodings."""
    lib = _load()
    y = _c(y_bf16, np.uint16)
    w = _c(topk_weights, np.float32)
    sr = _c(slot_row, np.int32)
    T, K = sr.shape
    H = y.shape[1]
    out = np.empty((T, H), np.uint16)
    if out.size == 0:
        return out
    if y.shape[0] == 0:
        y = np.zeros((1, H), np.uint16)      # never read: every slot_row is negative
    rc = lib.hmo_combine(_p(y), ctypes.c_int64(y.shape[0]), _p(w), _p(sr), ctypes.c_int64(T), ctypes.c_int32(K),
                         ctypes.c_int64(H), _p(out))
    if rc != 0:
        raise ValueError("hmo_combine: argument error %d" % rc)
    return out


def combine_f32(y_f32: np.ndarray, topk_weights, slot_row) -> np.ndarray:
    """out[t] = float32(sum_k w[t,k] * Y[slot_row[t,k]]) in binary64; y and out are float32."""
    lib = _load()
    y = _c(y_f32, np.float32)
    w = _c(topk_weights, np.float32)
    sr = _c(slot_row, np.int32)
    T, K = sr.shape
    H = y.shape[1]
    out = np.empty((T, H), np.float32)
    if out.size == 0:
        return out
    if y.shape[0] == 0:
        y = np.zeros((1, H), np.float32)     # never read: every slot_row is negative
    rc = lib.hmo_combine_f32(_p(y), ctypes.c_int64(y.shape[0]), _p(w), _p(sr), ctypes.c_int64(T), ctypes.c_int32(K),
                             ctypes.c_int64(H), _p(out))
    if rc != 0:
        raise ValueError("hmo_combine_f32: argument error %d" % rc)
    return out


def combine_transpose(gout: np.ndarray, row_token, row_weight) -> np.ndarray:
    """gy[row] = row_weight[row] * gout[row_token[row]] (fp32)."""
    lib = _load()
    g = _c(gout, np.float32)
    rt = _c(row_token, np.int32)
    rw = _c(row_weight, np.float32)
    T, H = g.shape
    gy = np.empty((rt.shape[0], H), np.float32)
    if gy.size == 0:
        return gy
    rc = lib.hmo_combine_transpose(_p(g), ctypes.c_int64(T), ctypes.c_int64(H), _p(rt), _p(rw),
                                   ctypes.c_int64(rt.shape[0]), _p(gy))
    if rc != 0:
        raise ValueError("hmo_combine_transpose: argument error %d" % rc)
    return gy


def combine_transpose_bf16(gout_bf16: np.ndarray, row_token, row_weight) -> np.ndarray:
    """gy[row] = bf16(row_weight[row] * gout[row_token[row]]), one rounding; uint16 bf16 encodings."""
    lib = _load()
    g = _c(gout_bf16, np.uint16)
    rt = _c(row_token, np.int32)
    rw = _c(row_weight, np.float32)
    T, H = g.shape
    gy = np.empty((rt.shape[0], H), np.uint16)
    if gy.size == 0:
        return gy
    rc = lib.hmo_combine_transpose_bf16(_p(g), ctypes.c_int64(T), ctypes.c_int64(H), _p(rt), _p(rw),
                                        ctypes.c_int64(rt.shape[0]), _p(gy))
    if rc != 0:
        raise ValueError("hmo_combine_transpose_bf16: argument error %d" % rc)
    return gy


def expert_load(topk_ids, expert_to_rank, nodes: int, ranks_per_node: int):
    """(load_expert[E], load_rank[G], load_node[nodes], status)."""
    lib = _load()
    ids = _c(topk_ids, np.int32)
    e2r = _c(expert_to_rank, np.int32)
    T, K = ids.shape
    E = e2r.shape[0]
    G = nodes * ranks_per_node
    le = np.zeros(E, np.int32)
    lr = np.zeros(G, np.int32)
    ln = np.zeros(nodes, np.int32)
    status = np.zeros(1, np.int32)
    rc = lib.hmo_expert_load(_p(ids), _p(e2r), ctypes.c_int32(T), ctypes.c_int32(K), ctypes.c_int32(E),
                             ctypes.c_int32(nodes), ctypes.c_int32(ranks_per_node), _p(le), _p(lr), _p(ln),
                             _p(status))
    if rc != 0:
        raise ValueError("hmo_expert_load: argument error %d" % rc)
    return le, lr, ln, int(status[0])


def recv_dest_map(expert_to_rank, nodes: int, ranks_per_node: int, my_rank: int, stage: int):
    """(dest_map[E], num_dest): destination of each expert as seen by `my_rank` at a receiver stage."""
    lib = _load()
    e2r = _c(expert_to_rank, np.int32)
    E = e2r.shape[0]
    dm = np.full(E, -9, np.int32)
    nd = ctypes.c_int32(0)
    rc = lib.hmo_recv_dest_map(_p(e2r), ctypes.c_int32(E), ctypes.c_int32(nodes), ctypes.c_int32(ranks_per_node),
                               ctypes.c_int32(my_rank), ctypes.c_int32(stage), _p(dm), ctypes.byref(nd))
    if rc != 0:
        raise ValueError("hmo_recv_dest_map: argument error %d" % rc)
    return dm, int(nd.value)


def level_dest_map(expert_to_rank, G: int, my_rank: int, parent_groups: int, child_groups: int):
    """(dest_map[E], num_dest) of one hop of the d-dimensional exchange (see hmo.c)."""
    lib = _load()
    e2r = _c(expert_to_rank, np.int32)
    E = e2r.shape[0]
    dm = np.full(E, -9, np.int32)
    nd = ctypes.c_int32(0)
    rc = lib.hmo_level_dest_map(_p(e2r), ctypes.c_int32(E), ctypes.c_int32(G), ctypes.c_int32(my_rank),
                                ctypes.c_int32(parent_groups), ctypes.c_int32(child_groups), _p(dm), ctypes.byref(nd))
    if rc != 0:
        raise ValueError("hmo_level_dest_map: argument error %d" % rc)
    return dm, int(nd.value)


def plan_mapped(ids, weights, dest_map, num_dest: int, dedup: bool) -> Plan:
    """Plan for an arbitrary expert -> destination table; Plan.rank_mask holds the destination mask."""
    lib = _load()
    ids = _c(ids, np.int32)
    w = _c(weights, np.float32)
    dm = _c(dest_map, np.int32)
    rows, K = ids.shape
    E = dm.shape[0]
    dest_count = np.zeros(num_dest, np.int32)
    dest_offset = np.zeros(num_dest + 1, np.int32)
    row_token = np.full(max(rows * K, 1), -1, np.int32)
    slot_row = np.full((rows, K), -1, np.int32)
    slot_keep = np.zeros((rows, K), np.uint8)
    row_weight = np.zeros(max(rows * K, 1), np.float32)
    dest_mask = np.zeros(max(rows, 1), np.uint64)
    status = np.zeros(1, np.int32)
    # numpy hands out a null pointer for empty arrays; the C side wants real ones
    ids_p = ids if ids.size else np.zeros((1, K), np.int32)
    w_p = w if w.size else np.zeros((1, K), np.float32)
    sr_p = slot_row if slot_row.size else np.zeros((1, K), np.int32)
    sk_p = slot_keep if slot_keep.size else np.zeros((1, K), np.uint8)
    rc = lib.hmo_plan_mapped(_p(ids_p), _p(w_p), _p(dm), ctypes.c_int32(rows), ctypes.c_int32(K), ctypes.c_int32(E),
                             ctypes.c_int32(num_dest), ctypes.c_int32(1 if dedup else 0), _p(dest_count),
                             _p(dest_offset), _p(row_token), _p(sr_p), _p(sk_p), _p(row_weight), _p(dest_mask),
                             _p(status))
    if rc != 0:
        raise ValueError("hmo_plan_mapped: argument error %d" % rc)
    total = int(dest_offset[num_dest])
    return Plan(LEVEL_GPU if dedup else LEVEL_NONE, num_dest, dest_count, dest_offset, row_token[:total].copy(),
                slot_row, slot_keep, row_weight[:total].copy(), dest_mask[:rows], np.zeros(rows, np.uint32),
                int(status[0]))


def combine_mix(y_bf16: np.ndarray, weights, slot_row) -> np.ndarray:
    """out[i] = bf16(sum_k w[i,k] Y[slot_row[i,k]] / sum_k w[i,k]) over the valid slots, binary64."""
    lib = _load()
    y = _c(y_bf16, np.uint16)
    w = _c(weights, np.float32)
    sr = _c(slot_row, np.int32)
    rows, K = sr.shape
    H = y.shape[1]
    out = np.empty((rows, H), np.uint16)
    if out.size == 0:
        return out
    if y.shape[0] == 0:
        y = np.zeros((1, H), np.uint16)
    rc = lib.hmo_combine_mix(_p(y), ctypes.c_int64(y.shape[0]), _p(w), _p(sr), ctypes.c_int64(rows), ctypes.c_int32(K),
                             ctypes.c_int64(H), _p(out))
    if rc != 0:
        raise ValueError("hmo_combine_mix: argument error %d" % rc)
    return out


def group_counts(topk_ids, expert_to_rank, G: int, groups):
    """counts[l][j]: tokens with a slot in group j when the G ranks are cut into groups[l] groups."""
    lib = _load()
    ids = _c(topk_ids, np.int32)
    e2r = _c(expert_to_rank, np.int32)
    T, K = ids.shape
    gr = np.asarray(groups, np.int32)
    counts = np.zeros((len(gr), 64), np.int32)
    status = np.zeros(1, np.int32)
    ids_p = ids if ids.size else np.zeros((1, K), np.int32)
    rc = lib.hmo_group_counts(_p(ids_p), _p(e2r), ctypes.c_int32(T), ctypes.c_int32(K), ctypes.c_int32(e2r.shape[0]),
                              ctypes.c_int32(G), ctypes.c_int32(len(gr)), _p(gr), _p(counts), _p(status))
    if rc != 0:
        raise ValueError("hmo_group_counts: argument error %d" % rc)
    return counts, int(status[0])


def alltoall_times(U, G: int, M: float, v: float, p_inter, p_intra, alpha_inter, beta_inter, alpha_intra, beta_intra):
    """(times[D], d*) from Eq.(1)-(6); p_inter / p_intra are int32 [D,64] (see hmo.c)."""
    lib = _load()
    U = np.asarray(U, np.int32)
    D = len(U)
    pi = _c(p_inter, np.int32).reshape(-1)
    pa = _c(p_intra, np.int32).reshape(-1)
    arrs = [np.zeros(4) for _ in range(4)]
    for a, src in zip(arrs, (alpha_inter, beta_inter, alpha_intra, beta_intra)):
        a[:len(src)] = src
    times = np.zeros(4)
    best = ctypes.c_int32(0)
    rc = lib.hmo_alltoall_times(ctypes.c_int32(D), _p(U), ctypes.c_int32(G), ctypes.c_double(M), ctypes.c_double(v),
                                _p(pi), _p(pa), _p(arrs[0]), _p(arrs[1]), _p(arrs[2]), _p(arrs[3]), _p(times),
                                ctypes.byref(best))
    if rc != 0:
        raise ValueError("hmo_alltoall_times: argument error %d" % rc)
    return times[:D].copy(), int(best.value)


def swap_counts(topk_ids, expert_to_rank, G: int, ng: int, method: str = "incremental"):
    """(Z[E,E,ng], status): duplicate-free tokens per group after swapping experts r and c.
    method "naive" recounts every pair from the definition; "incremental" is the paper's update."""
    lib = _load()
    ids = _c(topk_ids, np.int32)
    e2r = _c(expert_to_rank, np.int32)
    T, K = ids.shape
    E = e2r.shape[0]
    Z = np.zeros((E, E, ng), np.int32)
    status = np.zeros(1, np.int32)
    ids_p = ids if ids.size else np.zeros((1, K), np.int32)
    fn = lib.hmo_swap_counts_naive if method == "naive" else lib.hmo_swap_counts_incremental
    rc = fn(_p(ids_p), _p(e2r), ctypes.c_int32(T), ctypes.c_int32(K), ctypes.c_int32(E), ctypes.c_int32(G),
            ctypes.c_int32(ng), _p(Z), _p(status))
    if rc != 0:
        raise ValueError("hmo_swap_counts: argument error %d" % rc)
    return Z, int(status[0])


def swap_select(U, G: int, M: float, v: float, z_inter, z_intra, scale_inter, scale_intra, alpha_inter, beta_inter,
                alpha_intra: float, beta_intra: float, gamma: float):
    """(Q[E,E], (r*,c*), best time) for dimension d = len(U); z_inter[i] is Z of the U[i] cut (None at 0)."""
    lib = _load()
    U = np.asarray(U, np.int32)
    d = len(U)
    zi = [None if z is None else _c(z, np.int32) for z in z_inter]
    za = _c(z_intra, np.int32)
    E = za.shape[0]
    ptrs = (ctypes.c_void_p * 4)()
    for i in range(1, d):
        ptrs[i] = zi[i].ctypes.data
    pad = lambda a: np.asarray(list(a) + [0.0] * (4 - len(a)), np.float64)
    si, ai, bi = pad(scale_inter), pad(alpha_inter), pad(beta_inter)
    Q = np.zeros((E, E), np.float64)
    best = np.zeros(2, np.int32)
    bt = ctypes.c_double(0.0)
    rc = lib.hmo_swap_select(ctypes.c_int32(d), _p(U), ctypes.c_int32(G), ctypes.c_int32(E), ctypes.c_double(M),
                             ctypes.c_double(v), ptrs, _p(za), _p(si), ctypes.c_double(scale_intra), _p(ai), _p(bi),
                             ctypes.c_double(alpha_intra), ctypes.c_double(beta_intra), ctypes.c_double(gamma),
                             _p(Q), _p(best), ctypes.byref(bt))
    if rc != 0:
        raise ValueError("hmo_swap_select: argument error %d" % rc)
    return Q, (int(best[0]), int(best[1])), float(bt.value)


def swap_apply(expert_to_rank, pair) -> np.ndarray:
    """A copy of the placement with the entries of experts pair[0] and pair[1] exchanged."""
    lib = _load()
    e2r = np.array(expert_to_rank, dtype=np.int32, copy=True)
    pr = _c(pair, np.int32)
    rc = lib.hmo_swap_apply(_p(e2r), ctypes.c_int32(e2r.shape[0]), _p(pr))
    if rc != 0:
        raise ValueError("hmo_swap_apply: argument error %d" % rc)
    return e2r


def f64_to_bf16(v: float) -> int:
    return int(_load().hmo_f64_to_bf16(float(v)))
