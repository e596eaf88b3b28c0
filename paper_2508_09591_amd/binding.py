"""Thin ctypes binding over libhiermoe.so: argument marshalling only.

Function names and arguments mirror ``include/hiermoe.h``.  Tensors are torch tensors on the
GPU (torch supplies device memory and the current stream, nothing else); every step of the path
runs in the library's HIP kernels.  There is no CPU fallback: if the library is missing or a
tensor is not on the GPU the call raises.
"""
from __future__ import annotations

import ctypes
import os
from dataclasses import dataclass
from typing import Optional

import torch  # must be imported before the library so both share one HIP runtime

HM_DEDUP_NONE, HM_DEDUP_GPU, HM_DEDUP_NODE = 0, 1, 2
HM_RECV_INTRA_NODE, HM_RECV_LOCAL_EXPERTS = 0, 1
HM_OK = 0
HM_ERR_NULL, HM_ERR_SHAPE, HM_ERR_TOPOLOGY, HM_ERR_LEVEL = -1, -2, -3, -4
HM_ERR_WORKSPACE, HM_ERR_CAPACITY, HM_ERR_BAD_ID, HM_ERR_HIP = -5, -6, -7, -8

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libhiermoe.so")

EXPORTS = ("hm_plan_workspace_bytes", "hm_plan", "hm_plan_status", "hm_dispatch_pack", "hm_combine",
           "hm_combine_transpose", "hm_expert_load", "hm_status_string", "hm_recv_dest_map",
           "hm_plan_mapped_workspace_bytes", "hm_plan_mapped", "hm_combine_mix", "hm_group_counts",
           "hm_alltoall_times", "hm_swap_workspace_bytes", "hm_swap_counts", "hm_swap_select_workspace_bytes",
           "hm_swap_select", "hm_level_dest_map", "hm_combine_f32", "hm_swap_apply",
           "hm_swap_counts_multi", "hm_swap_multi_workspace_bytes", "hm_combine_transpose_bf16", "hm_plan_one_launch_limit", "hm_plan_one_launch_capacity",
           "hm_plan_static", "hm_plan_static_max_bytes", "hm_combine_launch_shape")


class hm_topology(ctypes.Structure):
    _fields_ = [("nodes", ctypes.c_int32), ("ranks_per_node", ctypes.c_int32)]


class hm_plan_out(ctypes.Structure):
    _fields_ = [("num_dest", ctypes.c_int32), ("row_capacity", ctypes.c_int64),
                ("dest_count", ctypes.c_void_p), ("dest_offset", ctypes.c_void_p),
                ("row_token", ctypes.c_void_p), ("slot_row", ctypes.c_void_p),
                ("slot_keep", ctypes.c_void_p), ("row_weight", ctypes.c_void_p),
                ("rank_mask", ctypes.c_void_p), ("node_mask", ctypes.c_void_p),
                ("status", ctypes.c_void_p), ("load_expert", ctypes.c_void_p),
                ("load_rank", ctypes.c_void_p), ("load_node", ctypes.c_void_p),
                ("max_rows_per_token", ctypes.c_int32), ("expected_rows", ctypes.c_int64)]


class HierMoEError(RuntimeError):
    def __init__(self, fn: str, code: int):
        self.code = code
        super().__init__("%s failed: %s (%d)" % (fn, status_string(code), code))


_lib = None


def lib():
    """The loaded C library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise RuntimeError("libhiermoe.so is not built (run __graft_entry__.build()); "
                               "there is no fallback path")
        L = ctypes.CDLL(_LIB_PATH)
        vp, i32, i64 = ctypes.c_void_p, ctypes.c_int32, ctypes.c_int64
        L.hm_plan_workspace_bytes.restype = ctypes.c_size_t
        L.hm_plan_workspace_bytes.argtypes = [i32, i32, i32, hm_topology, ctypes.c_int]
        L.hm_plan.restype = ctypes.c_int
        L.hm_plan.argtypes = [vp, vp, vp, i32, i32, i32, hm_topology, ctypes.c_int,
                              ctypes.POINTER(hm_plan_out), vp, ctypes.c_size_t, vp]
        L.hm_plan_static_max_bytes.restype = ctypes.c_size_t
        L.hm_plan_static_max_bytes.argtypes = []
        L.hm_plan_one_launch_limit.restype = ctypes.c_int32
        L.hm_plan_one_launch_limit.argtypes = [ctypes.c_int32]
        L.hm_plan_one_launch_capacity.restype = ctypes.c_int32
        L.hm_plan_one_launch_capacity.argtypes = []
        L.hm_plan_static.restype = ctypes.c_int
        L.hm_plan_static.argtypes = [vp, vp, vp, i32, i32, i32, hm_topology, ctypes.c_int,
                                     ctypes.POINTER(hm_plan_out), vp]
        L.hm_plan_status.restype = ctypes.c_int
        L.hm_plan_status.argtypes = [ctypes.POINTER(hm_plan_out), ctypes.POINTER(i64), vp]
        L.hm_dispatch_pack.restype = ctypes.c_int
        L.hm_dispatch_pack.argtypes = [vp, i32, i32, i32, ctypes.POINTER(hm_plan_out), vp, i64, vp]
        L.hm_combine.restype = ctypes.c_int
        L.hm_combine.argtypes = [vp, i64, vp, i32, i32, i32, ctypes.POINTER(hm_plan_out), vp, vp]
        L.hm_combine_launch_shape.restype = ctypes.c_int
        L.hm_combine_launch_shape.argtypes = [i32, i32, i32, ctypes.POINTER(hm_plan_out), i32, ctypes.POINTER(i32),
                                              ctypes.POINTER(i32), ctypes.POINTER(i32)]
        L.hm_swap_multi_workspace_bytes.restype = ctypes.c_size_t
        L.hm_swap_multi_workspace_bytes.argtypes = [i32, i32, i32, i32, i32, vp]
        L.hm_swap_counts_multi.restype = ctypes.c_int
        L.hm_swap_counts_multi.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.hm_swap_apply.restype = ctypes.c_int
        L.hm_swap_apply.argtypes = [vp, i32, vp, vp]
        L.hm_combine_f32.restype = ctypes.c_int
        L.hm_combine_f32.argtypes = [vp, i64, vp, i32, i32, i32, ctypes.POINTER(hm_plan_out), vp, vp]
        L.hm_combine_transpose.restype = ctypes.c_int
        L.hm_combine_transpose.argtypes = [vp, i32, i32, i32, ctypes.POINTER(hm_plan_out), vp, i64, vp]
        L.hm_combine_transpose_bf16.restype = ctypes.c_int
        L.hm_combine_transpose_bf16.argtypes = [vp, i32, i32, i32, ctypes.POINTER(hm_plan_out), vp, i64, vp]
        L.hm_expert_load.restype = ctypes.c_int
        L.hm_expert_load.argtypes = [vp, vp, i32, i32, i32, hm_topology, vp, vp, vp, vp, vp]
        L.hm_recv_dest_map.restype = ctypes.c_int
        L.hm_recv_dest_map.argtypes = [vp, i32, hm_topology, i32, ctypes.c_int, vp, vp, vp]
        L.hm_plan_mapped_workspace_bytes.restype = ctypes.c_size_t
        L.hm_plan_mapped_workspace_bytes.argtypes = [i32, i32, i32]
        L.hm_plan_mapped.restype = ctypes.c_int
        L.hm_plan_mapped.argtypes = [vp, vp, vp, i32, i32, i32, i32, i32, ctypes.POINTER(hm_plan_out), vp,
                                     ctypes.c_size_t, vp]
        L.hm_combine_mix.restype = ctypes.c_int
        L.hm_combine_mix.argtypes = [vp, i64, vp, i32, i32, i32, ctypes.POINTER(hm_plan_out), vp, vp]
        L.hm_group_counts.restype = ctypes.c_int
        L.hm_group_counts.argtypes = [vp, vp, i32, i32, i32, i32, i32, ctypes.POINTER(i32), vp, vp, vp]
        dp = ctypes.POINTER(ctypes.c_double)
        L.hm_alltoall_times.restype = ctypes.c_int
        L.hm_alltoall_times.argtypes = [i32, ctypes.POINTER(i32), i32, ctypes.c_double, ctypes.c_double, vp, vp,
                                        dp, dp, dp, dp, vp, vp, vp]
        L.hm_swap_workspace_bytes.restype = ctypes.c_size_t
        L.hm_swap_workspace_bytes.argtypes = [i32, i32, i32, i32]
        L.hm_swap_counts.restype = ctypes.c_int
        L.hm_swap_counts.argtypes = [vp, vp, i32, i32, i32, i32, i32, vp, vp, vp, ctypes.c_size_t, vp]
        L.hm_swap_select_workspace_bytes.restype = ctypes.c_size_t
        L.hm_swap_select_workspace_bytes.argtypes = [i32]
        L.hm_swap_select.restype = ctypes.c_int
        L.hm_swap_select.argtypes = [i32, ctypes.POINTER(i32), i32, i32, ctypes.c_double, ctypes.c_double,
                                     ctypes.POINTER(vp), vp, dp, ctypes.c_double, dp, dp, ctypes.c_double,
                                     ctypes.c_double, ctypes.c_double, vp, vp, vp, vp, ctypes.c_size_t, vp]
        L.hm_level_dest_map.restype = ctypes.c_int
        L.hm_level_dest_map.argtypes = [vp, i32, i32, i32, i32, i32, vp, vp, vp]
        L.hm_status_string.restype = ctypes.c_char_p
        L.hm_status_string.argtypes = [ctypes.c_int]
        _lib = L
    return _lib


def status_string(code: int) -> str:
    return lib().hm_status_string(int(code)).decode()


def _dev(t: Optional[torch.Tensor], dtype: torch.dtype, name: str) -> Optional[int]:
    if t is None:
        return None
    if not t.is_cuda:
        raise TypeError("%s must be a GPU tensor (no CPU path exists)" % name)
    if t.dtype != dtype:
        raise TypeError("%s must be %s, got %s" % (name, dtype, t.dtype))
    if not t.is_contiguous():
        raise TypeError("%s must be contiguous" % name)
    return t.data_ptr()


def _stream(stream) -> Optional[int]:
    s = torch.cuda.current_stream() if stream is None else stream
    return s.cuda_stream or None


def _check(fn: str, rc: int):
    if rc != HM_OK:
        raise HierMoEError(fn, rc)


@dataclass
class Plan:
    """Device buffers of one plan plus the host struct the C calls take."""
    T: int
    K: int
    level: int
    num_dest: int
    row_capacity: int
    dest_count: torch.Tensor
    dest_offset: torch.Tensor
    row_token: torch.Tensor
    slot_row: torch.Tensor
    slot_keep: torch.Tensor
    row_weight: torch.Tensor
    rank_mask: Optional[torch.Tensor]
    node_mask: Optional[torch.Tensor]
    status: torch.Tensor
    workspace: torch.Tensor
    c: hm_plan_out
    load_expert: Optional[torch.Tensor] = None
    load_rank: Optional[torch.Tensor] = None
    load_node: Optional[torch.Tensor] = None

    def ref(self):
        return ctypes.byref(self.c)


def hm_plan_workspace_bytes(T: int, K: int, E: int, nodes: int, ranks_per_node: int, level: int) -> int:
    return int(lib().hm_plan_workspace_bytes(T, K, E, hm_topology(nodes, ranks_per_node), level))


def alloc_plan(T: int, K: int, E: int, nodes: int, ranks_per_node: int, level: int, device="cuda",
               row_capacity: Optional[int] = None, masks: bool = True, num_dest: Optional[int] = None,
               loads: bool = False) -> Plan:
    """Allocate (uninitialised) plan buffers; row_capacity defaults to the worst case.  With
    num_dest given the buffers are sized for hm_plan_mapped (level none = no dedup); with loads
    hm_plan also fills load_expert / load_rank / load_node."""
    G = nodes * ranks_per_node
    Dn = num_dest if num_dest is not None else (nodes if level == HM_DEDUP_NODE else G)
    if row_capacity is None:
        row_capacity = T * (K if level == HM_DEDUP_NONE else min(K, Dn))
    e = lambda n, dt: torch.empty(max(int(n), 1), dtype=dt, device=device)
    if num_dest is not None:
        ws_bytes = int(lib().hm_plan_mapped_workspace_bytes(T, K, num_dest))
    else:
        ws_bytes = hm_plan_workspace_bytes(T, K, E, nodes, ranks_per_node, level)
    bufs = dict(dest_count=e(Dn, torch.int32), dest_offset=e(Dn + 1, torch.int32),
                row_token=e(row_capacity, torch.int32), slot_row=e(T * K, torch.int32),
                slot_keep=e(T * K, torch.uint8), row_weight=e(row_capacity, torch.float32),
                rank_mask=e(T, torch.int64) if masks else None,
                node_mask=e(T, torch.int32) if masks else None,
                status=e(1, torch.int32), workspace=e(max(ws_bytes, 16) // 4 + 4, torch.int32),
                load_expert=e(E, torch.int32) if loads else None, load_rank=e(G, torch.int32) if loads else None,
                load_node=e(nodes, torch.int32) if loads else None)
    c = hm_plan_out()
    c.num_dest = Dn
    c.row_capacity = int(row_capacity)
    for name in ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "row_weight",
                 "rank_mask", "node_mask", "status", "load_expert", "load_rank", "load_node"):
        t = bufs[name]
        setattr(c, name, t.data_ptr() if t is not None else None)
    return Plan(T=T, K=K, level=level, num_dest=Dn, row_capacity=int(row_capacity), c=c, **bufs)


def _adopt_table(plan: Plan, T: int, K: int, weights: torch.Tensor):
    """A plan's buffers may be reused for another routing table if they are large enough; the
    plan then describes that table (the row calls check their tensors against plan.T / plan.K)."""
    if weights.numel() != T * K:
        raise ValueError("weights hold %d values for %d x %d slots" % (weights.numel(), T, K))
    if T * K > plan.slot_row.numel() or T * K > plan.slot_keep.numel():
        raise ValueError("plan buffers hold %d slots, the table has %d x %d" % (plan.slot_row.numel(), T, K))
    for m in (plan.rank_mask, plan.node_mask):
        if m is not None and T > m.numel():
            raise ValueError("plan mask buffers hold %d tokens, the table has %d" % (m.numel(), T))
    plan.T, plan.K = T, K


def hm_plan(topk_ids: torch.Tensor, topk_weights: torch.Tensor, expert_to_rank: torch.Tensor,
            nodes: int, ranks_per_node: int, level: int, plan: Optional[Plan] = None, stream=None) -> Plan:
    T, K = topk_ids.shape
    E = expert_to_rank.shape[0]
    if plan is None:
        plan = alloc_plan(T, K, E, nodes, ranks_per_node, level, device=topk_ids.device)
    _adopt_table(plan, T, K, topk_weights)
    rc = lib().hm_plan(_dev(topk_ids, torch.int32, "topk_ids"), _dev(topk_weights, torch.float32, "topk_weights"),
                       _dev(expert_to_rank, torch.int32, "expert_to_rank"), T, K, E,
                       hm_topology(nodes, ranks_per_node), level, plan.ref(),
                       plan.workspace.data_ptr(), plan.workspace.numel() * 4, _stream(stream))
    _check("hm_plan", rc)
    plan.num_dest = int(plan.c.num_dest)
    return plan


def hm_plan_static(topk_ids: torch.Tensor, topk_weights: torch.Tensor, expert_to_rank: torch.Tensor,
                   nodes: int, ranks_per_node: int, level: int, plan: Plan, stream=None) -> Plan:
    """hm_plan on the library's static scratch: `plan` must be allocated by the caller beforehand
    (alloc_plan); the call itself allocates nothing."""
    T, K = topk_ids.shape
    E = expert_to_rank.shape[0]
    _adopt_table(plan, T, K, topk_weights)
    rc = lib().hm_plan_static(_dev(topk_ids, torch.int32, "topk_ids"), _dev(topk_weights, torch.float32, "topk_weights"),
                              _dev(expert_to_rank, torch.int32, "expert_to_rank"), T, K, E,
                              hm_topology(nodes, ranks_per_node), level, plan.ref(), _stream(stream))
    _check("hm_plan_static", rc)
    plan.num_dest = int(plan.c.num_dest)
    return plan


def hm_plan_one_launch_limit(workgroups: int) -> int:
    """Largest plan (workgroups of 1,024 slots) that runs as one launch; returns the previous limit."""
    return int(lib().hm_plan_one_launch_limit(int(workgroups)))


def hm_plan_status(plan: Plan, stream=None):
    """(status code, total_rows); synchronises the stream."""
    total = ctypes.c_int64(0)
    rc = lib().hm_plan_status(plan.ref(), ctypes.byref(total), _stream(stream))
    return int(rc), int(total.value)


def _rows_call_shape(plan: Plan, tokens: int, weights: Optional[torch.Tensor], what: str):
    """The C calls take T and K beside the plan and trust them: a tensor with more tokens than the
    plan was built for would make the kernels read the slot tables past their end."""
    if tokens != plan.T:
        raise ValueError("%s has %d rows but the plan was built for %d tokens" % (what, tokens, plan.T))
    if weights is not None and weights.numel() != plan.T * plan.K:
        raise ValueError("weights hold %d values, the plan has %d x %d slots" % (weights.numel(), plan.T, plan.K))


def hm_dispatch_pack(x: torch.Tensor, plan: Plan, packed: torch.Tensor, stream=None) -> torch.Tensor:
    T, H = x.shape
    _rows_call_shape(plan, T, None, "x")
    rc = lib().hm_dispatch_pack(_dev(x, torch.bfloat16, "x"), T, plan.K, H, plan.ref(),
                                _dev(packed, torch.bfloat16, "packed"), packed.shape[0], _stream(stream))
    _check("hm_dispatch_pack", rc)
    return packed


def hm_combine(y: torch.Tensor, topk_weights: Optional[torch.Tensor], plan: Plan, out: torch.Tensor, stream=None) -> torch.Tensor:
    """topk_weights None: the weights the plan merged (plan.row_weight) are used, the faster form."""
    T, H = out.shape
    _rows_call_shape(plan, T, topk_weights, "out")
    rc = lib().hm_combine(_dev(y, torch.bfloat16, "y"), y.shape[0], _dev(topk_weights, torch.float32, "topk_weights"),
                          T, plan.K, H, plan.ref(), _dev(out, torch.bfloat16, "out"), _stream(stream))
    _check("hm_combine", rc)
    return out


def hm_combine_f32(y: torch.Tensor, topk_weights: Optional[torch.Tensor], plan: Plan, out: torch.Tensor, stream=None) -> torch.Tensor:
    T, H = out.shape
    _rows_call_shape(plan, T, topk_weights, "out")
    rc = lib().hm_combine_f32(_dev(y, torch.float32, "y"), y.shape[0], _dev(topk_weights, torch.float32, "topk_weights"),
                              T, plan.K, H, plan.ref(), _dev(out, torch.float32, "out"), _stream(stream))
    _check("hm_combine_f32", rc)
    return out


def hm_combine_launch_shape(plan: Plan, H: int, weights_from_plan: bool = True):
    """(16-byte vectors per lane, rows in flight per wave, waves per CU) the combine calls would use."""
    v, r, w = ctypes.c_int32(0), ctypes.c_int32(0), ctypes.c_int32(0)
    rc = lib().hm_combine_launch_shape(plan.T, plan.K, H, plan.ref(), 1 if weights_from_plan else 0,
                                       ctypes.byref(v), ctypes.byref(r), ctypes.byref(w))
    _check("hm_combine_launch_shape", rc)
    return int(v.value), int(r.value), int(w.value)


def hm_combine_transpose(gout: torch.Tensor, plan: Plan, gy: torch.Tensor, stream=None) -> torch.Tensor:
    T, H = gout.shape
    _rows_call_shape(plan, T, None, "gout")
    rc = lib().hm_combine_transpose(_dev(gout, torch.float32, "gout"), T, plan.K, H, plan.ref(),
                                    _dev(gy, torch.float32, "gy"), gy.shape[0], _stream(stream))
    _check("hm_combine_transpose", rc)
    return gy


def hm_combine_transpose_bf16(gout: torch.Tensor, plan: Plan, gy: torch.Tensor, stream=None) -> torch.Tensor:
    T, H = gout.shape
    _rows_call_shape(plan, T, None, "gout")
    rc = lib().hm_combine_transpose_bf16(_dev(gout, torch.bfloat16, "gout"), T, plan.K, H, plan.ref(),
                                         _dev(gy, torch.bfloat16, "gy"), gy.shape[0], _stream(stream))
    _check("hm_combine_transpose_bf16", rc)
    return gy


def hm_expert_load(topk_ids: torch.Tensor, expert_to_rank: torch.Tensor, nodes: int, ranks_per_node: int,
                   load_expert: torch.Tensor, load_rank: torch.Tensor, load_node: torch.Tensor,
                   status: Optional[torch.Tensor] = None, stream=None):
    T, K = topk_ids.shape
    E = expert_to_rank.shape[0]
    rc = lib().hm_expert_load(_dev(topk_ids, torch.int32, "topk_ids"), _dev(expert_to_rank, torch.int32, "expert_to_rank"),
                              T, K, E, hm_topology(nodes, ranks_per_node), _dev(load_expert, torch.int32, "load_expert"),
                              _dev(load_rank, torch.int32, "load_rank"), _dev(load_node, torch.int32, "load_node"),
                              _dev(status, torch.int32, "status"), _stream(stream))
    _check("hm_expert_load", rc)
    return load_expert, load_rank, load_node


def hm_recv_dest_map(expert_to_rank: torch.Tensor, nodes: int, ranks_per_node: int, my_rank: int, stage: int,
                     dest_map: torch.Tensor, num_dest: torch.Tensor, stream=None):
    E = expert_to_rank.shape[0]
    rc = lib().hm_recv_dest_map(_dev(expert_to_rank, torch.int32, "expert_to_rank"), E,
                                hm_topology(nodes, ranks_per_node), my_rank, stage,
                                _dev(dest_map, torch.int32, "dest_map"), _dev(num_dest, torch.int32, "num_dest"),
                                _stream(stream))
    _check("hm_recv_dest_map", rc)
    return dest_map, num_dest


def hm_plan_mapped(row_ids: torch.Tensor, row_weights: torch.Tensor, dest_map: torch.Tensor, num_dest: int,
                   dedup: bool, plan: Optional[Plan] = None, stream=None) -> Plan:
    rows, K = row_ids.shape
    E = dest_map.shape[0]
    if plan is None:
        plan = alloc_plan(rows, K, E, 1, 1, HM_DEDUP_GPU if dedup else HM_DEDUP_NONE, device=dest_map.device,
                          num_dest=num_dest)
    _adopt_table(plan, rows, K, row_weights)
    rc = lib().hm_plan_mapped(_dev(row_ids, torch.int32, "row_ids"), _dev(row_weights, torch.float32, "row_weights"),
                              _dev(dest_map, torch.int32, "dest_map"), rows, K, E, num_dest, 1 if dedup else 0,
                              plan.ref(), plan.workspace.data_ptr(), plan.workspace.numel() * 4, _stream(stream))
    _check("hm_plan_mapped", rc)
    plan.num_dest = int(plan.c.num_dest)
    return plan


def hm_combine_mix(y: torch.Tensor, row_weights: Optional[torch.Tensor], plan: Plan, out: torch.Tensor, stream=None) -> torch.Tensor:
    T, H = out.shape
    _rows_call_shape(plan, T, row_weights, "out")
    rc = lib().hm_combine_mix(_dev(y, torch.bfloat16, "y"), y.shape[0], _dev(row_weights, torch.float32, "row_weights"),
                              T, plan.K, H, plan.ref(), _dev(out, torch.bfloat16, "out"), _stream(stream))
    _check("hm_combine_mix", rc)
    return out


def hm_group_counts(topk_ids: torch.Tensor, expert_to_rank: torch.Tensor, G: int, groups, counts: torch.Tensor,
                    status: Optional[torch.Tensor] = None, stream=None) -> torch.Tensor:
    """counts: int32 [len(groups), 64] on the GPU."""
    T, K = topk_ids.shape
    E = expert_to_rank.shape[0]
    arr = (ctypes.c_int32 * len(groups))(*[int(g) for g in groups])
    rc = lib().hm_group_counts(_dev(topk_ids, torch.int32, "topk_ids"), _dev(expert_to_rank, torch.int32, "expert_to_rank"),
                               T, K, E, G, len(groups), arr, _dev(counts, torch.int32, "counts"),
                               _dev(status, torch.int32, "status"), _stream(stream))
    _check("hm_group_counts", rc)
    return counts


def hm_alltoall_times(U, G: int, M: float, v: float, p_inter: torch.Tensor, p_intra: torch.Tensor, alpha_inter,
                      beta_inter, alpha_intra, beta_intra, times: torch.Tensor, best: torch.Tensor, stream=None):
    """times: float64 [4], best: int32 [1] on the GPU; p_inter / p_intra: int32 [D,64] on the GPU."""
    D = len(U)
    ua = (ctypes.c_int32 * D)(*[int(u) for u in U])
    dbl = lambda a: (ctypes.c_double * D)(*[float(x) for x in a])
    rc = lib().hm_alltoall_times(D, ua, G, float(M), float(v), _dev(p_inter, torch.int32, "p_inter"),
                                 _dev(p_intra, torch.int32, "p_intra"), dbl(alpha_inter), dbl(beta_inter),
                                 dbl(alpha_intra), dbl(beta_intra), _dev(times, torch.float64, "times"),
                                 _dev(best, torch.int32, "best"), _stream(stream))
    _check("hm_alltoall_times", rc)
    return times, best


def hm_swap_counts(topk_ids: torch.Tensor, expert_to_rank: torch.Tensor, G: int, ng: int, Z: torch.Tensor,
                   status: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """Z: int32 [E,E,ng] on the GPU."""
    T, K = topk_ids.shape
    E = expert_to_rank.shape[0]
    need = int(lib().hm_swap_workspace_bytes(T, K, E, ng))
    if workspace is None:
        workspace = torch.empty(need // 4 + 4, dtype=torch.int32, device=Z.device)
    rc = lib().hm_swap_counts(_dev(topk_ids, torch.int32, "topk_ids"), _dev(expert_to_rank, torch.int32, "expert_to_rank"),
                              T, K, E, G, ng, _dev(Z, torch.int32, "Z"), _dev(status, torch.int32, "status"),
                              workspace.data_ptr(), workspace.numel() * 4, _stream(stream))
    _check("hm_swap_counts", rc)
    return Z


def hm_swap_counts_multi(topk_ids: torch.Tensor, expert_to_rank: torch.Tensor, G: int, ng, Z,
                         status: Optional[torch.Tensor] = None, workspace: Optional[torch.Tensor] = None, stream=None):
    """ng: up to 4 group counts; Z: list of int32 [E,E,ng[c]] GPU tensors, one per cut."""
    T, K = topk_ids.shape
    E = expert_to_rank.shape[0]
    n = len(ng)
    if len(Z) != n:
        raise ValueError("one Z tensor per cut")
    nga = (ctypes.c_int32 * n)(*[int(u) for u in ng])
    zp = (ctypes.c_void_p * n)(*[_dev(z, torch.int32, "Z") for z in Z])
    need = int(lib().hm_swap_multi_workspace_bytes(T, K, E, G, n, nga))
    if workspace is None:
        workspace = torch.empty(need // 4 + 4, dtype=torch.int32, device=Z[0].device)
    rc = lib().hm_swap_counts_multi(_dev(topk_ids, torch.int32, "topk_ids"), _dev(expert_to_rank, torch.int32, "expert_to_rank"),
                                    T, K, E, G, n, nga, zp, _dev(status, torch.int32, "status"),
                                    workspace.data_ptr(), workspace.numel() * 4, _stream(stream))
    _check("hm_swap_counts_multi", rc)
    return Z


def hm_swap_select(U, G: int, M: float, v: float, z_inter, z_intra: torch.Tensor, scale_inter, scale_intra: float,
                   alpha_inter, beta_inter, alpha_intra: float, beta_intra: float, gamma: float, Q: torch.Tensor,
                   best_pair: torch.Tensor, best_time: torch.Tensor, workspace: Optional[torch.Tensor] = None, stream=None):
    """z_inter: list of d entries (entry 0 None), each an int32 [E,E,U[i]] GPU tensor."""
    d = len(U)
    E = z_intra.shape[0]
    ua = (ctypes.c_int32 * d)(*[int(u) for u in U])
    ptrs = (ctypes.c_void_p * d)()
    for i in range(1, d):
        ptrs[i] = _dev(z_inter[i], torch.int32, "z_inter")
    dbl = lambda a: (ctypes.c_double * d)(*[float(x) for x in a])
    need = int(lib().hm_swap_select_workspace_bytes(E))
    if workspace is None:
        workspace = torch.empty(need // 8 + 2, dtype=torch.float64, device=Q.device)
    rc = lib().hm_swap_select(d, ua, G, E, float(M), float(v), ptrs, _dev(z_intra, torch.int32, "z_intra"),
                              dbl(scale_inter), float(scale_intra), dbl(alpha_inter), dbl(beta_inter), float(alpha_intra),
                              float(beta_intra), float(gamma), _dev(Q, torch.float64, "Q"),
                              _dev(best_pair, torch.int32, "best_pair"), _dev(best_time, torch.float64, "best_time"),
                              workspace.data_ptr(), workspace.numel() * 8, _stream(stream))
    _check("hm_swap_select", rc)
    return Q, best_pair, best_time


def hm_swap_apply(expert_to_rank: torch.Tensor, best_pair: torch.Tensor, stream=None) -> torch.Tensor:
    rc = lib().hm_swap_apply(_dev(expert_to_rank, torch.int32, "expert_to_rank"), expert_to_rank.shape[0],
                             _dev(best_pair, torch.int32, "best_pair"), _stream(stream))
    _check("hm_swap_apply", rc)
    return expert_to_rank


def hm_level_dest_map(expert_to_rank: torch.Tensor, G: int, my_rank: int, parent_groups: int, child_groups: int,
                      dest_map: torch.Tensor, num_dest: torch.Tensor, stream=None):
    E = expert_to_rank.shape[0]
    rc = lib().hm_level_dest_map(_dev(expert_to_rank, torch.int32, "expert_to_rank"), E, G, my_rank, parent_groups,
                                 child_groups, _dev(dest_map, torch.int32, "dest_map"),
                                 _dev(num_dest, torch.int32, "num_dest"), _stream(stream))
    _check("hm_level_dest_map", rc)
    return dest_map, num_dest
