// Device-side helpers shared by the gfx950 kernels of libhiermoe (wave64 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include "hiermoe.h"

namespace hm {

constexpr int kWave = 64;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ int lane_id() { return (int)(threadIdx.x & (kWave - 1)); }

// Sticky error word: codes are negative and the most negative one wins, so the result does not
// depend on the order in which waves report.
__device__ __forceinline__ void flag(int32_t *status, int32_t code) {
  if (status) atomicMin(status, code);
}

// Rank of an expert id; -1 when the id or the placement entry is out of range (an error), -2 for
// the id -1, the marker of a slot the router dropped (skipped everywhere, not an error).
__device__ __forceinline__ int rank_of(const int32_t *__restrict__ expert_to_rank, int E, int G, int id) {
  if (id == -1) return -2;
  if ((unsigned)id >= (unsigned)E) return -1;
  const int g = expert_to_rank[id];
  return ((unsigned)g >= (unsigned)G) ? -1 : g;
}

// Value held by lane `src` (src must be wave-uniform).
__device__ __forceinline__ int read_lane(int v, int src) { return __builtin_amdgcn_readlane(v, src); }
__device__ __forceinline__ float read_lane(float v, int src) {
  return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), src));
}

// bf16 pair packed in one 32-bit word -> two floats (low half first).
__device__ __forceinline__ float bf16_lo(uint32_t w) { return __builtin_bit_cast(float, w << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t w) { return __builtin_bit_cast(float, w & 0xFFFF0000u); }

// float -> bf16 encoding, round to nearest even; NaN maps to the quiet NaN 0x7FC0.
__device__ __forceinline__ uint32_t f32_to_bf16(float f) {
  const uint32_t u = __builtin_bit_cast(uint32_t, f);
  if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;
  return (u + 0x7FFFu + ((u >> 16) & 1u)) >> 16;
}
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  return f32_to_bf16(lo) | (f32_to_bf16(hi) << 16);
}

// Streaming 16-byte accesses: packed rows are written once and read by a later kernel (or, in a
// real deployment, by the network), so they should not displace useful lines.
__device__ __forceinline__ void store_stream(u32x4 *p, u32x4 v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ void store_stream(f32x4 *p, f32x4 v) { __builtin_nontemporal_store(v, p); }
__device__ __forceinline__ u32x4 load_stream(const u32x4 *p) { return __builtin_nontemporal_load(p); }
__device__ __forceinline__ f32x4 load_stream(const f32x4 *p) { return __builtin_nontemporal_load(p); }

}  // namespace hm

// Host-side argument checks shared by the entry points.
static inline hm_status hm_check_topology(hm_topology topo) {
  if (topo.nodes < 1 || topo.ranks_per_node < 1) return HM_ERR_TOPOLOGY;
  if (topo.nodes > 32 || topo.ranks_per_node > 64) return HM_ERR_TOPOLOGY;
  if ((int64_t)topo.nodes * topo.ranks_per_node > 64) return HM_ERR_TOPOLOGY;
  return HM_OK;
}
static inline hm_status hm_check_tk(int32_t T, int32_t K) {
  if (T < 0 || K < 1 || K > 64) return HM_ERR_SHAPE;
  if ((int64_t)T * K > 2147483647LL) return HM_ERR_SHAPE;
  return HM_OK;
}
// Launch errors.  HIP keeps the last error of a thread until somebody reads it, so an error the
// host program left behind before calling into this library must not be reported as a failed
// launch of ours (nor cleared: it is the host program's to find).  Every entry point notes what
// was pending when it was entered; a launch counts as failed only if a new error appears.
static thread_local hipError_t hm_pending_at_entry = hipSuccess;
struct hm_entry_scope {
  hm_entry_scope() { hm_pending_at_entry = hipPeekAtLastError(); }
};
#define HM_ENTRY_SCOPE const hm_entry_scope hm_entry_scope_here
static inline hm_status hm_launch_status() {
  const hipError_t now = hipPeekAtLastError();
  if (now == hipSuccess || now == hm_pending_at_entry) return HM_OK;
  (void)hipGetLastError();   // ours: reported through the return code, not left for the next caller
  return HM_ERR_HIP;
}
