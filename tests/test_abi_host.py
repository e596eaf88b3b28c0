"""Host-side checks of the C ABI that need no GPU: the library loads, exports every function the
header declares, and rejects bad arguments before launching anything."""
import ctypes
import os
import re

import pytest

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def B():
    from paper_2508_09591_amd import binding, build
    if not os.path.exists(build.LIB):
        build.build_library()
    binding.lib()
    return binding


def _declared_functions():
    text = open(os.path.join(ROOT, "include", "hiermoe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(hm_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_function(B):
    declared = _declared_functions()
    assert set(declared) == set(B.EXPORTS)
    L = B.lib()
    for name in declared:
        assert getattr(L, name) is not None, name


def test_status_strings(B):
    seen = {B.status_string(c) for c in range(0, -9, -1)}
    assert len(seen) == 9 and "unknown status" not in seen
    assert B.status_string(-99) == "unknown status"


def _workspace(workgroups, dests):
    """Count matrix [workgroups + 1][dests] int32, padded to 8 bytes, then, for plans the one-launch
    kernel takes (at most 256 workgroups of 1024 slots), its matrix of 8-byte words and one
    8-byte flag per workgroup."""
    counts = ((workgroups + 1) * dests * 4 + 7) // 8 * 8
    return counts + (8 * (workgroups * dests + workgroups) if workgroups <= 256 else 0)


def test_workspace_query(B):
    assert B.hm_plan_workspace_bytes(8192, 8, 256, 4, 8, B.HM_DEDUP_NODE) == _workspace(64, 4)
    assert B.hm_plan_workspace_bytes(8192, 8, 256, 4, 8, B.HM_DEDUP_GPU) == _workspace(64, 32)
    assert B.hm_plan_workspace_bytes(0, 8, 256, 4, 8, B.HM_DEDUP_GPU) == _workspace(1, 32)
    assert B.hm_plan_workspace_bytes(8191, 3, 256, 1, 3, B.HM_DEDUP_GPU) == _workspace(24, 3)   # odd entry count: padded
    assert B.hm_plan_workspace_bytes(32768, 8, 256, 8, 8, B.HM_DEDUP_GPU) == _workspace(256, 64)
    assert B.hm_plan_workspace_bytes(32769, 8, 256, 8, 8, B.HM_DEDUP_GPU) == _workspace(257, 64)  # several launches: no flags
    assert B.hm_plan_workspace_bytes(8192, 8, 256, 9, 8, B.HM_DEDUP_GPU) == 0      # 72 ranks
    assert B.hm_plan_workspace_bytes(8192, 65, 256, 4, 8, B.HM_DEDUP_GPU) == 0     # K too large
    assert B.hm_plan_workspace_bytes(8192, 8, 256, 4, 8, 3) == 0                   # bad level


def _plan_struct(B, fake=0x1000, capacity=16):
    c = B.hm_plan_out()
    c.num_dest = 4
    c.row_capacity = capacity
    for f in ("dest_count", "dest_offset", "row_token", "slot_row", "slot_keep", "row_weight", "status"):
        setattr(c, f, fake)
    return c


def _no_gpu_here():
    import torch
    return not torch.cuda.is_available()


# Tests that hand the library made-up device addresses run only where no GPU is visible: should a
# host-side check ever regress, the call then fails with a HIP error instead of launching a kernel
# on such an address.
fake_pointers = pytest.mark.skipif(not _no_gpu_here(), reason="passes made-up device pointers: CPU-only by design")


@fake_pointers
def test_argument_errors_are_reported_before_any_launch(B):
    """Every call below must return from the host-side checks; the fake pointers are never used."""
    L = B.lib()
    topo = B.hm_topology(2, 2)
    fake = ctypes.c_void_p(0x1000)
    c = _plan_struct(B)
    ref = ctypes.byref(c)

    def plan(ids=fake, w=fake, e2r=fake, T=4, K=2, E=8, topo=topo, level=B.HM_DEDUP_GPU, out=ref, ws=fake, ws_bytes=1 << 20):
        return L.hm_plan(ids, w, e2r, T, K, E, topo, level, out, ws, ws_bytes, None)

    assert plan(out=None) == B.HM_ERR_NULL
    assert plan(e2r=None) == B.HM_ERR_NULL
    assert plan(ids=None) == B.HM_ERR_NULL
    assert plan(ws=None) == B.HM_ERR_NULL
    assert plan(T=-1) == B.HM_ERR_SHAPE
    assert plan(K=0) == B.HM_ERR_SHAPE
    assert plan(K=65) == B.HM_ERR_SHAPE
    assert plan(E=0) == B.HM_ERR_SHAPE
    assert plan(T=1 << 30, K=8) == B.HM_ERR_SHAPE
    assert plan(topo=B.hm_topology(0, 2)) == B.HM_ERR_TOPOLOGY
    assert plan(topo=B.hm_topology(9, 8)) == B.HM_ERR_TOPOLOGY
    assert plan(topo=B.hm_topology(33, 1)) == B.HM_ERR_TOPOLOGY
    assert plan(level=7) == B.HM_ERR_LEVEL
    assert plan(ws_bytes=8) == B.HM_ERR_WORKSPACE
    broken = _plan_struct(B)
    broken.slot_row = None
    assert plan(out=ctypes.byref(broken)) == B.HM_ERR_NULL

    # the variant on the library's static scratch: same checks, and a size limit instead of a workspace
    def static(ids=fake, w=fake, e2r=fake, T=4, K=2, E=8, topo=topo, level=B.HM_DEDUP_GPU, out=ref):
        return L.hm_plan_static(ids, w, e2r, T, K, E, topo, level, out, None)

    assert L.hm_plan_static_max_bytes() == 1 << 20
    assert static(out=None) == B.HM_ERR_NULL
    assert static(w=None) == B.HM_ERR_NULL
    assert static(K=65) == B.HM_ERR_SHAPE
    assert static(topo=B.hm_topology(9, 8)) == B.HM_ERR_TOPOLOGY
    assert static(level=-1) == B.HM_ERR_LEVEL
    assert static(out=ctypes.byref(broken)) == B.HM_ERR_NULL
    big = B.hm_topology(8, 8)
    assert L.hm_plan_workspace_bytes(600000, 8, 256, big, B.HM_DEDUP_GPU) > 1 << 20
    assert static(T=600000, K=8, E=256, topo=big) == B.HM_ERR_WORKSPACE

    assert L.hm_dispatch_pack(fake, 4, 2, 64, None, fake, 8, None) == B.HM_ERR_NULL
    assert L.hm_dispatch_pack(None, 4, 2, 64, ref, fake, 8, None) == B.HM_ERR_NULL
    assert L.hm_dispatch_pack(fake, 4, 2, 0, ref, fake, 8, None) == B.HM_ERR_SHAPE
    assert L.hm_dispatch_pack(fake, 4, 2, 64, ref, fake, -1, None) == B.HM_ERR_SHAPE
    assert L.hm_dispatch_pack(fake, 0, 2, 64, ref, fake, 8, None) == B.HM_OK          # nothing to do
    # weights = NULL selects the plan's merged weights: the plan must then carry row_weight and slot_keep
    no_rw = _plan_struct(B)
    no_rw.row_weight = None
    no_keep = _plan_struct(B)
    no_keep.slot_keep = None
    assert L.hm_combine(fake, 8, None, 4, 2, 64, ctypes.byref(no_rw), fake, None) == B.HM_ERR_NULL
    assert L.hm_combine(fake, 8, None, 4, 2, 64, ctypes.byref(no_keep), fake, None) == B.HM_ERR_NULL
    assert L.hm_combine(fake, 8, fake, 4, 2, 64, ctypes.byref(no_keep), None, None) == B.HM_ERR_NULL   # out missing
    assert L.hm_combine(fake, 8, fake, 4, 0, 64, ref, fake, None) == B.HM_ERR_SHAPE
    assert L.hm_combine(fake, 8, fake, 4, 2, 64, ref, None, None) == B.HM_ERR_NULL
    assert L.hm_combine_f32(fake, 8, None, 4, 2, 64, ctypes.byref(no_rw), fake, None) == B.HM_ERR_NULL
    assert L.hm_combine_f32(fake, -2, fake, 4, 2, 64, ref, fake, None) == B.HM_ERR_SHAPE
    assert L.hm_combine_f32(fake, 8, fake, 0, 2, 64, ref, fake, None) == B.HM_OK          # T = 0: nothing to do
    assert L.hm_combine_transpose(None, 4, 2, 64, ref, fake, 8, None) == B.HM_ERR_NULL
    assert L.hm_combine_transpose(fake, 4, 2, -5, ref, fake, 8, None) == B.HM_ERR_SHAPE
    assert L.hm_combine_transpose_bf16(None, 4, 2, 64, ref, fake, 8, None) == B.HM_ERR_NULL
    assert L.hm_combine_transpose_bf16(fake, 4, 2, 64, ref, fake, -1, None) == B.HM_ERR_SHAPE
    assert L.hm_expert_load(fake, None, 4, 2, 8, topo, fake, fake, fake, None, None) == B.HM_ERR_NULL
    assert L.hm_expert_load(fake, fake, 4, 2, 8, B.hm_topology(8, 9), fake, fake, fake, None, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_expert_load(fake, fake, 4, 99, 8, topo, fake, fake, fake, None, None) == B.HM_ERR_SHAPE
    assert L.hm_plan_status(None, None, None) == B.HM_ERR_NULL

    # receiver-side entry points
    assert L.hm_recv_dest_map(None, 8, topo, 0, 0, fake, fake, None) == B.HM_ERR_NULL
    assert L.hm_recv_dest_map(fake, 0, topo, 0, 0, fake, fake, None) == B.HM_ERR_SHAPE
    assert L.hm_recv_dest_map(fake, 8, topo, 4, 0, fake, fake, None) == B.HM_ERR_TOPOLOGY     # rank 4 of 4
    assert L.hm_recv_dest_map(fake, 8, topo, 0, 2, fake, fake, None) == B.HM_ERR_LEVEL
    assert L.hm_plan_mapped_workspace_bytes(8192, 8, 8) == _workspace(64, 8)
    assert L.hm_plan_mapped_workspace_bytes(8192, 8, 65) == 0

    def mapped(ids=fake, w=fake, dm=fake, rows=4, K=2, E=8, nd=4, out=ref, ws=fake, ws_bytes=1 << 20):
        return L.hm_plan_mapped(ids, w, dm, rows, K, E, nd, 1, out, ws, ws_bytes, None)

    assert mapped(dm=None) == B.HM_ERR_NULL
    assert mapped(ids=None) == B.HM_ERR_NULL
    assert mapped(rows=-2) == B.HM_ERR_SHAPE
    assert mapped(nd=0) == B.HM_ERR_TOPOLOGY
    assert mapped(nd=65) == B.HM_ERR_TOPOLOGY
    assert mapped(ws_bytes=4) == B.HM_ERR_WORKSPACE
    assert L.hm_combine_mix(fake, 8, None, 4, 2, 64, ctypes.byref(no_rw), fake, None) == B.HM_ERR_NULL
    assert L.hm_combine_mix(fake, -1, fake, 4, 2, 64, ref, fake, None) == B.HM_ERR_SHAPE

    assert L.hm_level_dest_map(fake, 8, 8, 0, 2, 3, fake, fake, None) == B.HM_ERR_TOPOLOGY      # 2 does not divide 3
    assert L.hm_level_dest_map(fake, 8, 8, 0, 4, 2, fake, fake, None) == B.HM_ERR_TOPOLOGY      # child coarser than parent
    assert L.hm_level_dest_map(fake, 8, 8, 8, 1, 2, fake, fake, None) == B.HM_ERR_TOPOLOGY      # rank 8 of 8
    assert L.hm_level_dest_map(fake, 8, 8, 0, 1, 2, None, fake, None) == B.HM_ERR_NULL

    # dimension selection
    i32x = lambda *a: (ctypes.c_int32 * len(a))(*a)
    dbl = lambda *a: (ctypes.c_double * len(a))(*a)
    assert L.hm_group_counts(fake, fake, 4, 2, 8, 4, 1, i32x(3), fake, None, None) == B.HM_ERR_TOPOLOGY   # 3 does not divide 4
    assert L.hm_group_counts(fake, fake, 4, 2, 8, 65, 1, i32x(1), fake, None, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_group_counts(fake, fake, 4, 2, 8, 4, 5, i32x(1, 1, 1, 1, 1), fake, None, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_group_counts(fake, None, 4, 2, 8, 4, 1, i32x(4), fake, None, None) == B.HM_ERR_NULL
    z = dbl(0, 0)
    assert L.hm_alltoall_times(2, i32x(2, 4), 4, 1.0, 1.0, fake, fake, z, z, z, z, fake, fake, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_alltoall_times(2, i32x(1, 3), 4, 1.0, 1.0, fake, fake, z, z, z, z, fake, fake, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_alltoall_times(5, i32x(1, 1, 1, 1, 1), 4, 1.0, 1.0, fake, fake, z, z, z, z, fake, fake, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_alltoall_times(2, i32x(1, 2), 4, 1.0, 1.0, None, fake, z, z, z, z, fake, fake, None) == B.HM_ERR_NULL

    # expert swap
    # E <= 256: one summed set of tables with transposes, 16 chunks' partial tables (C, CG, base as 16-bit
    # values), a byte per slot; larger E: private copies of C
    part_words = (256 * 256 + 256 * 32 + 64 + 1) // 2
    assert L.hm_swap_workspace_bytes(1000, 6, 256, 32) == (64 + 2 * 256 + 2 * (256 * 256 + 256 * 32) + 16 * part_words + 1500) * 4
    assert L.hm_swap_workspace_bytes(1000, 6, 512, 32) == (64 + 2 * 512 + 512 * 32 + 2 * 512 * 512) * 4
    # more tokens than 16 chunks of 16-bit counts can hold: the path with atomics, 8 private copies of C
    assert L.hm_swap_workspace_bytes(2000000, 1, 256, 4) == (64 + 2 * 256 + 256 * 4 + 8 * 256 * 256) * 4
    assert L.hm_swap_workspace_bytes(10, 2, 0, 4) == 0 and L.hm_swap_workspace_bytes(-1, 2, 8, 4) == 0
    big = 1 << 30
    assert L.hm_swap_counts(fake, fake, 4, 2, 8, 4, 3, fake, None, fake, big, None) == B.HM_ERR_TOPOLOGY     # 3 does not divide 4
    assert L.hm_swap_counts(fake, fake, 4, 2, 8, 4, 2, None, None, fake, big, None) == B.HM_ERR_NULL
    assert L.hm_swap_counts(fake, fake, 4, 2, 8, 4, 2, fake, None, fake, 16, None) == B.HM_ERR_WORKSPACE
    assert L.hm_swap_counts(fake, fake, 4, 2, 10000, 4, 2, fake, None, fake, big, None) == B.HM_ERR_SHAPE    # E*E*64 overflows
    zp = (ctypes.c_void_p * 2)(None, 0x1000)
    assert L.hm_swap_select(2, i32x(1, 2), 4, 8, 1.0, 1.0, zp, fake, z, 1.0, z, z, 0.0, 0.0, 10.0, fake, fake, fake, fake, 8, None) == B.HM_ERR_WORKSPACE
    assert L.hm_swap_select(2, i32x(1, 3), 4, 8, 1.0, 1.0, zp, fake, z, 1.0, z, z, 0.0, 0.0, 10.0, fake, fake, fake, fake, big, None) == B.HM_ERR_TOPOLOGY
    zn = (ctypes.c_void_p * 2)(None, None)
    assert L.hm_swap_select(2, i32x(1, 2), 4, 8, 1.0, 1.0, zn, fake, z, 1.0, z, z, 0.0, 0.0, 10.0, fake, fake, fake, fake, big, None) == B.HM_ERR_NULL
    ng2 = i32x(2, 4)
    zz = (ctypes.c_void_p * 2)(fake, fake)
    assert L.hm_swap_multi_workspace_bytes(7, 3, 16, 4, 2, ng2) == (16 + 6 + sum(64 + 16 + 2 * (16 * g + 256) + 16 * ((256 + 16 * g + 64 + 1) // 2) for g in (2, 4))) * 4
    assert L.hm_swap_multi_workspace_bytes(7, 3, 16, 4, 5, ng2) == 0 and L.hm_swap_multi_workspace_bytes(7, 3, 16, 6, 2, ng2) == 0
    assert L.hm_swap_counts_multi(fake, fake, 4, 2, 16, 4, 2, ng2, zz, None, fake, 8, None) == B.HM_ERR_WORKSPACE
    assert L.hm_swap_counts_multi(fake, fake, 4, 2, 16, 6, 2, ng2, zz, None, fake, big, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_swap_counts_multi(fake, fake, 4, 2, 16, 4, 0, ng2, zz, None, fake, big, None) == B.HM_ERR_TOPOLOGY
    assert L.hm_swap_counts_multi(fake, fake, 4, 2, 16, 4, 2, None, zz, None, fake, big, None) == B.HM_ERR_NULL
    zn2 = (ctypes.c_void_p * 2)(fake, None)
    assert L.hm_swap_counts_multi(fake, fake, 4, 2, 16, 4, 2, ng2, zn2, None, fake, big, None) == B.HM_ERR_NULL
    assert L.hm_swap_apply(None, 8, fake, None) == B.HM_ERR_NULL
    assert L.hm_swap_apply(fake, 8, None, None) == B.HM_ERR_NULL
    assert L.hm_swap_apply(fake, 0, fake, None) == B.HM_ERR_SHAPE
    assert L.hm_swap_select(1, i32x(1), 4, 8, 1.0, 1.0, None, None, None, 1.0, None, None, 0.0, 0.0, 10.0, fake, fake, fake, fake, big, None) == B.HM_ERR_NULL


def test_combine_launch_shape_follows_the_plan_not_the_buffers(B):
    """The row kernels size their launches from what the plan struct says about rows per token
    (expected_rows, else the bound hm_plan left), never from the caller's buffer sizes -- which is
    why the query takes no buffer size at all.  Host logic only: nothing is launched."""
    L = B.lib()
    T, K, H = 8192, 8, 7168

    def shape(bound, expected, from_plan=1, tokens=T):
        c = _plan_struct(B)
        c.max_rows_per_token = bound
        c.expected_rows = expected
        v, r, w = ctypes.c_int32(-1), ctypes.c_int32(-1), ctypes.c_int32(-1)
        rc = L.hm_combine_launch_shape(tokens, K, H, ctypes.byref(c), from_plan, ctypes.byref(v), ctypes.byref(r), ctypes.byref(w))
        assert rc == B.HM_OK
        return v.value, r.value, w.value

    assert shape(4, 0) == (1, 8, 32)                    # node level on 4 nodes: at most 4 rows per token
    assert shape(8, 0) == (1, 8, 16)                    # rank level / no dedup, K = 8: eight 1 KiB loads per wave
    assert shape(0, 0) == (4, 4, 32)                    # a mapped plan that was never synchronised: unknown, assume few
    assert shape(8, int(1.16 * T)) == (4, 2, 32)        # the count wins over the bound (local-expert stage of a receiver)
    assert shape(0, int(2.2 * T)) == (1, 8, 32)         # the intra-node stage of a receiver
    assert shape(0, int(6.0 * T)) == (1, 8, 20)         # 128 KiB / 6 KiB = 21 waves -> whole workgroups of four
    assert shape(4, int(7.49 * T)) == (1, 8, 16)
    assert shape(8, 64 * T) == (1, 8, 16)               # never below 16 waves per CU
    assert shape(8, int(7.49 * T), from_plan=0) == (4, 4, 32)   # caller's weights: the merging kernel, no cap
    assert shape(8, 0, tokens=0) == (1, 8, 16)
    assert L.hm_combine_launch_shape(T, K, H, None, 1, None, None, None) == B.HM_ERR_NULL
    assert L.hm_combine_launch_shape(T, 0, H, ctypes.byref(_plan_struct(B)), 1, None, None, None) == B.HM_ERR_SHAPE


def test_binding_checks_tensors_against_the_plan(B):
    """The C calls take T and K beside the plan; the binding refuses tensors that do not match
    the table the plan was built for before anything reaches the library."""
    import torch
    from types import SimpleNamespace
    plan = SimpleNamespace(T=16, K=2)
    B._rows_call_shape(plan, 16, torch.zeros(32), "x")
    with pytest.raises(ValueError):
        B._rows_call_shape(plan, 17, None, "x")
    with pytest.raises(ValueError):
        B._rows_call_shape(plan, 16, torch.zeros(33), "x")
    small = SimpleNamespace(T=4, K=2, slot_row=torch.zeros(8), slot_keep=torch.zeros(8), rank_mask=torch.zeros(4),
                            node_mask=None)
    B._adopt_table(small, 3, 2, torch.zeros(6))
    assert (small.T, small.K) == (3, 2)
    with pytest.raises(ValueError):
        B._adopt_table(small, 5, 2, torch.zeros(10))      # more slots than the buffers hold
    with pytest.raises(ValueError):
        B._adopt_table(small, 4, 2, torch.zeros(7))       # weights do not match the table


def test_binding_refuses_cpu_tensors(B):
    import torch
    ids = torch.zeros((4, 2), dtype=torch.int32)
    with pytest.raises(TypeError):
        B._dev(ids, torch.int32, "topk_ids")


def test_bench_refuses_more_than_one_gpu():
    import subprocess
    import sys
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout == ""


def test_header_is_plain_c(tmp_path):
    """include/hiermoe.h must compile as C99 on its own (the boundary is a C ABI, not C++)."""
    import subprocess
    src = tmp_path / "use_header.c"
    src.write_text('#include "hiermoe.h"\n'
                   "int main(void) { hm_plan_out p; hm_topology t = {1, 1}; (void)p; (void)t;\n"
                   "  return (int)sizeof(hm_status) > 0 ? 0 : 1; }\n")
    subprocess.check_call(["gcc", "-std=c99", "-Wall", "-Wextra", "-Werror", "-pedantic", "-fsyntax-only",
                           "-I", os.path.join(ROOT, "include"), str(src)])
