// hm_plan: routing -> deduplicated, stable per-destination send lists (HierMoE Eq.(7)).
//
// One lane owns one routing slot s = t*K + k; a wave owns 64 consecutive slots, a workgroup 1024.
// Rows of a destination are numbered in ascending slot order, so a lane's row is
//     dest_offset[d] + (kept slots of d in earlier workgroups) + (in earlier waves of this
//     workgroup) + (in lower lanes of this wave),
// and the last term is a popcount over a wavefront ballot.  No atomics decide positions, so the
// plan is deterministic and stable.  A workgroup first stages the rank and destination of its
// 1024 slots, plus a halo of K-1 slots on either side (the rest of the first and last token), in
// LDS: each expert id is looked up once and all "same destination as an earlier / later slot of
// my token" questions become LDS reads.
//
// Every workgroup needs the counts of all the others (the destination totals give dest_offset),
// so the plan has a grid-wide dependency in the middle.  Two ways through it:
//   * plans of at most 256 workgroups (262,144 slots) run as ONE launch, plan_fused_kernel: the
//     workgroups publish their counts, meet at a grid barrier and go on to write the maps from
//     what they staged.  At these sizes the work is a few microseconds and a second launch (its
//     gap, and staging everything again) cost more than the kernels themselves.  All workgroups
//     are resident together (the launcher checks the device's capacity), the barrier spins on
//     per-workgroup flags holding a value unique to the launch, so the caller's workspace needs
//     no initialisation, and every wait is bounded: a wave that gives up flags HM_ERR_HIP and
//     exits.
//   * larger plans take separate launches: plan_count_kernel (per-workgroup counts ->
//     workspace), plan_scan_kernel once the matrix has kPlanScanMinEntries entries (one
//     workgroup per destination turns it into exclusive prefixes plus a row of totals; below
//     that every workgroup re-reads the small matrix itself), and plan_write_kernel: the body of
//     the one-launch kernel without its grid-wide wait (the counts are complete when it starts).
//     Linear in the number of slots at any size.
#include "hm_device.h"

#include <unistd.h>

#include <atomic>
#include <chrono>
#include <mutex>

namespace hm {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kPlanHalo = 63;                              // K - 1 <= 63
constexpr int kPlanStaged = kPlanThreads + 2 * kPlanHalo;
constexpr int64_t kPlanScanMinEntries = 16384;             // count-matrix entries from which the scan launch pays
constexpr int kPlanFusedMaxBlocks = 256;                   // largest plan (in workgroups) the one-launch kernel takes
constexpr int kPlanSpinLimit = 1 << 18;                    // polls of the grid barrier before a wave gives up
constexpr int kPlanStagedExperts = 4096;                   // one-launch kernel: largest expert table staged in LDS

struct PlanParams {
  const int32_t *ids;
  const float *weights;
  const int32_t *expert_to_rank;
  const int32_t *dest_map;  // non-null: destinations come from this table (hm_plan_mapped)
  int32_t T, K, E, G, R, Dn, level;
  int32_t nslots, nblocks;
  int32_t scanned;  // counts holds exclusive prefixes over workgroups and the totals in row nblocks
  int64_t row_capacity;
  int32_t *counts;  // workspace [nblocks + 1][Dn]
  int32_t *dest_count, *dest_offset, *row_token, *slot_row;
  uint8_t *slot_keep;
  float *row_weight;
  uint64_t *rank_mask;
  uint32_t *node_mask;
  int32_t *status;
  int32_t *load_expert, *load_rank, *load_node;  // optional: the counts of hm_expert_load, fused
};

// What one lane knows about its slot after staging.
struct Slot {
  bool live;   // inside the table
  int t, k;    // token and position in the token
  int tok0;    // LDS index of the token's slot 0
  int rank;    // -1: invalid expert id or table entry; -2: valid, but no copy at this hop
  int dest;    // destination at the chosen level, -1 if there is none
  bool keep;   // owns the row of (token, dest)
};

// Stage rank / destination of slots [first - halo, first + 1024 + halo) and classify this lane's
// slot.  A slot owns its (token, destination) row at level none always, else iff no earlier slot
// of the token has the same destination: the OR over a group's experts in Eq.(7) leaves one copy
// per group, and the lowest k keeps it.
__device__ __forceinline__ Slot stage_and_classify(const PlanParams &p, int8_t *s_rank, int8_t *s_dest) {
  const int halo = p.K - 1;
  const int64_t first = (int64_t)blockIdx.x * kPlanThreads;
  for (int i = threadIdx.x; i < kPlanThreads + 2 * halo; i += kPlanThreads) {
    const int64_t s = first - halo + i;
    int r = -1, d = -1;
    if (s >= 0 && s < p.nslots) {
      if (p.dest_map) {
        const int id = p.ids[s];
        if (id == -1) {
          r = -2;   // slot dropped by the router
        } else if ((unsigned)id < (unsigned)p.E) {
          const int v = p.dest_map[id];
          if (v >= 0 && v < p.Dn) r = d = v;
          else if (v == -1) r = -2;
        }
      } else {
        r = rank_of(p.expert_to_rank, p.E, p.G, p.ids[s]);
        if (r >= 0) d = p.level == HM_DEDUP_NODE ? r / p.R : r;
      }
    }
    s_rank[i] = (int8_t)r;
    s_dest[i] = (int8_t)d;
  }
  __syncthreads();
  Slot me;
  const int64_t s = first + threadIdx.x;
  me.live = s < p.nslots;
  me.t = me.k = me.tok0 = 0;
  me.rank = me.dest = -1;
  me.keep = false;
  if (me.live) {
    me.t = (int)(s / p.K);
    me.k = (int)(s - (int64_t)me.t * p.K);
    const int own = halo + (int)threadIdx.x;
    me.tok0 = own - me.k;
    me.rank = s_rank[own];
    me.dest = s_dest[own];
    me.keep = me.dest >= 0;
    if (me.keep && p.level != HM_DEDUP_NONE)
      for (int k1 = 0; k1 < me.k; ++k1)
        if (s_dest[me.tok0 + k1] == me.dest) me.keep = false;
  }
  return me;
}

__global__ __launch_bounds__(kPlanThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void plan_count_kernel(PlanParams p) {
  __shared__ int8_t s_rank[kPlanStaged];
  __shared__ int8_t s_dest[kPlanStaged];
  __shared__ int32_t wave_cnt[kPlanWaves][kWave];
  const int lane = lane_id(), wv = (int)(threadIdx.x >> 6);
  const Slot me = stage_and_classify(p, s_rank, s_dest);
  const int kept_dest = me.keep ? me.dest : -1;
  int mine = 0;  // lane d ends up with the wave's count for destination d
  for (int d = 0; d < p.Dn; ++d) {
    const uint64_t b = __ballot(kept_dest == d);
    if (lane == d) mine = __popcll(b);
  }
  wave_cnt[wv][lane] = mine;
  __syncthreads();
  if ((int)threadIdx.x < p.Dn) {
    int sum = 0;
    for (int w = 0; w < kPlanWaves; ++w) sum += wave_cnt[w][threadIdx.x];
    p.counts[(int64_t)blockIdx.x * p.Dn + threadIdx.x] = sum;
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) *p.status = 0;
  if (p.load_expert) {   // the write kernel accumulates into these with atomics
    const int64_t stride = (int64_t)gridDim.x * kPlanThreads;
    for (int64_t i = (int64_t)blockIdx.x * kPlanThreads + threadIdx.x; i < p.E; i += stride) p.load_expert[i] = 0;
    if (blockIdx.x == 0 && (int)threadIdx.x < p.G) p.load_rank[threadIdx.x] = 0;
    if (blockIdx.x == 0 && (int)threadIdx.x < p.G / p.R) p.load_node[threadIdx.x] = 0;
  }
}

// Column d of the count matrix -> exclusive prefix over the workgroups, in place; total -> row nblocks.
__global__ __launch_bounds__(kPlanThreads) void plan_scan_kernel(PlanParams p) {
  __shared__ int32_t wave_tot[kPlanWaves];
  __shared__ int32_t carry;
  const int lane = lane_id(), wv = (int)(threadIdx.x >> 6);
  const int d = blockIdx.x;
  if (threadIdx.x == 0) carry = 0;
  __syncthreads();
  for (int b0 = 0; b0 < p.nblocks; b0 += kPlanThreads) {
    const int b = b0 + (int)threadIdx.x;
    const int v = b < p.nblocks ? p.counts[(int64_t)b * p.Dn + d] : 0;
    int incl = v;
    for (int off = 1; off < kWave; off <<= 1) {
      const int u = __shfl_up(incl, off, kWave);
      if (lane >= off) incl += u;
    }
    if (lane == kWave - 1) wave_tot[wv] = incl;
    __syncthreads();
    int base = carry;
    for (int w = 0; w < wv; ++w) base += wave_tot[w];
    if (b < p.nblocks) p.counts[(int64_t)b * p.Dn + d] = base + incl - v;
    __syncthreads();
    if (threadIdx.x == 0) {
      int tot = 0;
      for (int w = 0; w < kPlanWaves; ++w) tot += wave_tot[w];
      carry += tot;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) p.counts[(int64_t)p.nblocks * p.Dn + d] = carry;
}

// ---- one-launch plan ---------------------------------------------------------------------------
// Words that another workgroup of the same launch reads or writes are accessed with device-scope
// atomic loads and stores (the workgroups sit on different dies with caches of their own).
__device__ __forceinline__ void st_device(int32_t *a, int32_t v) {
  __hip_atomic_store(a, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ uint64_t ld_device(const uint64_t *a) {
  return __hip_atomic_load(a, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ void st_device(uint64_t *a, uint64_t v) {
  __hip_atomic_store(a, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// The calling wave's earlier device-scope stores have been acknowledged when this returns.
__device__ __forceinline__ void wait_for_own_stores() { __asm__ volatile("s_waitcnt vmcnt(0)" ::: "memory"); }

constexpr int kTagShift = 11;   // a workgroup keeps at most 1024 slots per destination: the count takes 11 bits

// Rank (or hop-table destination) of an expert id from the table staged in LDS; the codes of
// stage_and_classify: -1 invalid, -2 no copy at this hop / slot dropped by the router.
__device__ __forceinline__ int lookup_staged(const PlanParams &p, const int8_t *s_map, int id) {
  if (id == -1) return -2;
  if ((unsigned)id >= (unsigned)p.E) return -1;
  return s_map[id];
}
// The same from global memory, for tables too large to stage.
__device__ __forceinline__ int lookup_global(const PlanParams &p, int id) {
  if (p.dest_map) {
    if (id == -1) return -2;
    if ((unsigned)id >= (unsigned)p.E) return -1;
    const int v = p.dest_map[id];
    return (v >= 0 && v < p.Dn) ? v : (v == -1 ? -2 : -1);
  }
  return rank_of(p.expert_to_rank, p.E, p.G, id);
}

// The grid-wide step without a separate barrier: a workgroup publishes its per-destination
// counts as 64-bit words (launch tag << 11 | count), one atomic store each, and every workgroup
// reads the whole matrix, waiting on each word until it carries the tag of this launch -- the
// count and its "ready" flag arrive in one word, so no fence orders them.  The tag is 53 bits
// of a value unique to the launch, so what an uninitialised workspace holds cannot pass for it.
// passed[b] is set once workgroup b has read the matrix; workgroup 0 finally waits for all of
// passed and zeroes matrix and flags, so a replay of a captured launch (same tag) starts clean.
// Every wait is bounded by kPlanSpinLimit polls; a wave that gives up makes the workgroup skip
// its writes, flags HM_ERR_HIP and exits.
//
// The kernel is a chain of dependent memory round trips, so it is ordered to keep that chain
// short: the expert -> rank table is staged in LDS while the ids are in flight (no dependent
// lookup, and the division by ranks_per_node is done once per expert, not per slot), the halo
// slots are fetched in the same round as the workgroup's own, and everything that does not need
// the other workgroups' counts -- slot_keep, the masks, the LDS partials of the load counts --
// is done while the counts are on their way.
template <bool FUSED>
__device__ __forceinline__ void plan_body(const PlanParams &p, uint64_t *matrix, uint64_t *passed, uint64_t tag,
                                          int staged_table) {
  __shared__ int8_t s_rank[kPlanStaged];
  __shared__ int8_t s_node[kPlanStaged];
  __shared__ int8_t s_dest[kPlanStaged];
  __shared__ float s_weight[kPlanStaged];
  __shared__ uint64_t ballots[kPlanWaves][kWave];
  __shared__ int32_t wave_base[kPlanWaves][kWave];
  __shared__ int32_t part_tot[kPlanWaves][kWave];
  __shared__ int32_t part_pre[kPlanWaves][kWave];
  __shared__ int32_t block_base[kWave];
  __shared__ int32_t blk_rank[kWave], blk_node[kWave];
  __shared__ int32_t gave_up;
  extern __shared__ int32_t dyn_lds[];   // if staged_table: [hist: E int32 if the load arrays are asked for][rank: E int8][node: E int8]
  const int lane = lane_id(), wv = (int)(threadIdx.x >> 6);
  const int bid = (int)blockIdx.x;
  const bool loads = p.load_expert != nullptr;
  int32_t *hist = dyn_lds;
  int8_t *s_map = (int8_t *)(dyn_lds + (loads ? p.E : 0));
  int8_t *s_nmap = s_map + p.E;
  const int halo = p.K - 1;
  const int first = bid * kPlanThreads;   // slot indices fit 31 bits

  // ---- phase 1a: everything that comes from memory, issued in one round
  const int s = first + (int)threadIdx.x;                     // own slot, LDS entry halo + threadIdx.x
  const bool has2 = (int)threadIdx.x < 2 * halo;              // a halo slot as well:
  const int i2 = (int)threadIdx.x < halo ? (int)threadIdx.x : kPlanThreads + (int)threadIdx.x;   // its LDS entry
  const int64_t s2 = (int64_t)first - halo + i2;
  const bool live = s < p.nslots, live2 = has2 && s2 >= 0 && s2 < p.nslots;
  int id = -1, id2 = -1;
  float w = 0.0f, w2 = 0.0f;
  if (live) {
    id = p.ids[s];
    w = p.weights[s];
  }
  if (live2) {
    id2 = p.ids[s2];
    w2 = p.weights[s2];
  }
  if (staged_table) {
    for (int e = threadIdx.x; e < p.E; e += kPlanThreads) {
      int v, n = -1;
      if (p.dest_map) {
        const int m = p.dest_map[e];
        v = (m >= 0 && m < p.Dn) ? m : (m == -1 ? -2 : -1);
      } else {
        const int g = p.expert_to_rank[e];
        v = ((unsigned)g >= (unsigned)p.G) ? -1 : g;
        if (v >= 0) n = v / p.R;
      }
      s_map[e] = (int8_t)v;
      s_nmap[e] = (int8_t)n;
    }
    if (loads)
      for (int e = threadIdx.x; e < p.E; e += kPlanThreads) hist[e] = 0;
  }
  if (threadIdx.x < kWave) blk_rank[threadIdx.x] = blk_node[threadIdx.x] = 0;
  if (threadIdx.x == 0) gave_up = 0;
  if (FUSED && bid == 0) {   // what the atomics of the other workgroups add to: out before this workgroup's counts are
    if (threadIdx.x == 0) st_device(p.status, 0);
    if (loads) {
      for (int i = threadIdx.x; i < p.E; i += kPlanThreads) st_device(p.load_expert + i, 0);
      if ((int)threadIdx.x < p.G) st_device(p.load_rank + threadIdx.x, 0);
      if ((int)threadIdx.x < p.G / p.R) st_device(p.load_node + threadIdx.x, 0);
    }
    wait_for_own_stores();
  }
  __syncthreads();

  // ---- phase 1b: ranks, nodes and destinations of the staged slots into LDS
  {
    int r = -1, n = -1;
    if (live) {
      if (staged_table) {
        r = lookup_staged(p, s_map, id);
        if (r >= 0) n = s_nmap[id];
      } else {
        r = lookup_global(p, id);
        if (r >= 0 && !p.dest_map) n = r / p.R;
      }
    }
    const int own = halo + (int)threadIdx.x;
    s_rank[own] = (int8_t)r;
    s_node[own] = (int8_t)n;
    s_dest[own] = (int8_t)(r < 0 ? -1 : (p.level == HM_DEDUP_NODE && !p.dest_map ? n : r));
    s_weight[own] = w;
    if (has2) {
      int r2 = -1, n2 = -1;
      if (live2) {
        if (staged_table) {
          r2 = lookup_staged(p, s_map, id2);
          if (r2 >= 0) n2 = s_nmap[id2];
        } else {
          r2 = lookup_global(p, id2);
          if (r2 >= 0 && !p.dest_map) n2 = r2 / p.R;
        }
      }
      s_rank[i2] = (int8_t)r2;
      s_node[i2] = (int8_t)n2;
      s_dest[i2] = (int8_t)(r2 < 0 ? -1 : (p.level == HM_DEDUP_NODE && !p.dest_map ? n2 : r2));
      s_weight[i2] = w2;
    }
  }
  __syncthreads();
  Slot me;
  me.live = live;
  me.t = me.k = me.tok0 = 0;
  me.rank = me.dest = -1;
  me.keep = false;
  if (live) {
    // s / K without a per-lane division: the workgroup's first slot is divided once (uniform),
    // the rest is a numerator below 1024 + K, for which a 22-bit reciprocal is exact (K <= 64)
    const unsigned t0 = (unsigned)first / (unsigned)p.K, r0 = (unsigned)first - t0 * (unsigned)p.K;
    const unsigned recip = ((1u << 22) + (unsigned)p.K - 1u) / (unsigned)p.K;
    me.t = (int)(t0 + (((r0 + threadIdx.x) * recip) >> 22));
    me.k = s - me.t * p.K;
    const int own = halo + (int)threadIdx.x;
    me.tok0 = own - me.k;
    me.rank = s_rank[own];
    me.dest = s_dest[own];
    me.keep = me.dest >= 0;
    if (me.keep && p.level != HM_DEDUP_NONE)
      for (int k1 = 0; k1 < me.k; ++k1)
        if (s_dest[me.tok0 + k1] == me.dest) me.keep = false;
  }
  const int kept_dest = me.keep ? me.dest : -1;
  for (int d = 0; d < p.Dn; ++d) {
    const uint64_t b = __ballot(kept_dest == d);
    if (lane == d) ballots[wv][d] = b;
  }
  __syncthreads();
  if (lane < p.Dn) {
    int a = 0;
    for (int w1 = 0; w1 < wv; ++w1) a += __popcll(ballots[w1][lane]);
    wave_base[wv][lane] = a;
    if (FUSED && wv == kPlanWaves - 1)   // the last wave's base plus its own count is the workgroup's count
      st_device(matrix + (int64_t)bid * p.Dn + lane, (tag << kTagShift) | (uint64_t)(a + __popcll(ballots[wv][lane])));
  }

  // ---- while the counts travel: what needs no other workgroup
  uint64_t rm = 0;
  uint32_t nm = 0;
  if (me.live) {
    if (me.dest < 0) {
      p.slot_row[s] = -1;
      p.slot_keep[s] = 0;
    } else {
      p.slot_keep[s] = me.keep ? 1 : 0;
    }
    if (me.k == 0 && (p.rank_mask || p.node_mask || loads)) {   // per-token masks, owned by the token's slot 0
      for (int k2 = 0; k2 < p.K; ++k2) {
        const int r2 = s_rank[me.tok0 + k2];
        if (r2 >= 0) {
          // the first slot that sets a bit also counts the token for that rank / node: the
          // duplicate-free loads of hm_expert_load, as LDS partials (the wave-wide ballots per
          // group this replaces were a third of the kernel's vector instructions)
          if (loads && !((rm >> r2) & 1ull)) atomicAdd(&blk_rank[r2], 1);
          rm |= 1ull << r2;
          if (!p.dest_map) {
            const int n2 = s_node[me.tok0 + k2];
            if (loads && !((nm >> n2) & 1u)) atomicAdd(&blk_node[n2], 1);
            nm |= 1u << n2;
          }
        }
      }
      if (p.rank_mask) p.rank_mask[me.t] = rm;
      if (p.node_mask) p.node_mask[me.t] = nm;
    }
  }
  if (loads && me.live && me.rank >= 0 && staged_table) atomicAdd(&hist[id], 1);   // slots per expert, LDS partial

  // ---- the count matrix: wave wv reads rows wv, wv+16, ..., lane = destination
  if (FUSED) {   // ... and reads them again, as a whole wave, until every word carries this launch's tag
    int tot = 0, pre = 0;
    bool ready = false;
    for (int spin = 0; spin < kPlanSpinLimit; ++spin) {
      tot = pre = 0;
      bool mine = true;
      if (lane < p.Dn) {
        for (int b0 = wv; b0 < p.nblocks; b0 += 4 * kPlanWaves) {   // four rows in flight
          uint64_t v[4];
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            const int b = b0 + j * kPlanWaves;
            v[j] = b < p.nblocks ? ld_device(matrix + (int64_t)b * p.Dn + lane) : (tag << kTagShift);
          }
#pragma unroll
          for (int j = 0; j < 4; ++j) {
            mine = mine && (v[j] >> kTagShift) == tag;
            const int c = (int)(v[j] & ((1u << kTagShift) - 1u));
            tot += c;
            if (b0 + j * kPlanWaves < bid) pre += c;
          }
        }
      }
      ready = __ballot(!mine) == 0ull;
      if (ready) break;
      __builtin_amdgcn_s_sleep(2);
    }
    part_tot[wv][lane] = tot;
    part_pre[wv][lane] = pre;
    if (!ready && lane == 0) gave_up = 1;
  } else {   // an earlier launch left the counts (or, scanned, their prefixes and a row of totals) in p.counts
    int tot = 0, pre = 0;
    if (p.scanned) {
      if (wv == 0 && lane < p.Dn) {
        tot = p.counts[(int64_t)p.nblocks * p.Dn + lane];
        pre = p.counts[(int64_t)bid * p.Dn + lane];
      }
    } else if (lane < p.Dn) {
      for (int b0 = wv; b0 < p.nblocks; b0 += 8 * kPlanWaves) {   // eight rows in flight
        int c[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int b = b0 + j * kPlanWaves;
          c[j] = b < p.nblocks ? p.counts[(int64_t)b * p.Dn + lane] : 0;
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          tot += c[j];
          if (b0 + j * kPlanWaves < bid) pre += c[j];
        }
      }
    }
    part_tot[wv][lane] = tot;
    part_pre[wv][lane] = pre;
  }
  __syncthreads();
  const bool go = gave_up == 0;   // uniform over the workgroup
  if (go) {
    if (FUSED && threadIdx.x == 0) st_device(passed + bid, tag);
    if (loads) {   // global atomics first: they complete in the shadow of the map stores
      const int nodes = p.G / p.R;
      if (staged_table) {
        for (int e = threadIdx.x; e < p.E; e += kPlanThreads)
          if (hist[e]) atomicAdd(&p.load_expert[e], hist[e]);
      } else if (me.live && me.rank >= 0) {
        atomicAdd(&p.load_expert[id], 1);
      }
      if ((int)threadIdx.x < p.G && blk_rank[threadIdx.x]) atomicAdd(&p.load_rank[threadIdx.x], blk_rank[threadIdx.x]);
      if ((int)threadIdx.x < nodes && blk_node[threadIdx.x]) atomicAdd(&p.load_node[threadIdx.x], blk_node[threadIdx.x]);
    }
    if (me.live && me.rank == -1) flag(p.status, HM_ERR_BAD_ID);
    if (wv == 0) {
      int tot = 0, pre = 0;
      if (lane < p.Dn)
        for (int w1 = 0; w1 < kPlanWaves; ++w1) {
          tot += part_tot[w1][lane];
          pre += part_pre[w1][lane];
        }
      int incl = tot;  // inclusive scan over destinations (lanes >= Dn hold 0)
      for (int off = 1; off < kWave; off <<= 1) {
        const int v = __shfl_up(incl, off, kWave);
        if (lane >= off) incl += v;
      }
      const int offset = incl - tot;
      block_base[lane] = offset + pre;
      if (bid == 0 && lane < p.Dn) {
        p.dest_count[lane] = tot;
        p.dest_offset[lane] = offset;
        if (lane == p.Dn - 1) p.dest_offset[p.Dn] = incl;
      }
    }
  } else if (threadIdx.x == 0) {
    flag(p.status, HM_ERR_HIP);
  }
  __syncthreads();

  // ---- rows: the slot that owns a row numbers it and serves the later slots that share it
  if (go && me.live && me.keep) {
    const uint64_t b = ballots[wv][me.dest];
    const int pos = __popcll(b & ((1ull << lane) - 1ull));
    const int row = block_base[me.dest] + wave_base[wv][me.dest] + pos;
    p.slot_row[s] = row;
    float wsum = s_weight[me.tok0 + me.k];
    if (p.level != HM_DEDUP_NONE) {
      for (int k2 = me.k + 1; k2 < p.K; ++k2) {
        if (s_dest[me.tok0 + k2] == me.dest) {
          p.slot_row[s + (k2 - me.k)] = row;
          wsum = wsum + s_weight[me.tok0 + k2];  // ascending k, fp32
        }
      }
    }
    if (row < p.row_capacity) {
      p.row_token[row] = me.t;
      p.row_weight[row] = wsum;
    } else {
      flag(p.status, HM_ERR_CAPACITY);
    }
  }

  // ---- workgroup 0 leaves matrix and flags clean (also when a wait gave up: the status word says so)
  if (FUSED && bid == 0) {
    if (wv == 0 && go) {
      bool ok = true;
      for (int spin = 0; spin < kPlanSpinLimit; ++spin) {
        ok = true;
        for (int b = lane; b < p.nblocks; b += kWave) ok = ok && ld_device(passed + b) == tag;
        if (__ballot(!ok) == 0ull) break;
        __builtin_amdgcn_s_sleep(2);
      }
      if (__ballot(!ok) != 0ull && lane == 0) flag(p.status, HM_ERR_HIP);
    }
    __syncthreads();
    for (int i = threadIdx.x; i < p.nblocks * p.Dn; i += kPlanThreads) st_device(matrix + i, 0ull);
    for (int b = threadIdx.x; b < p.nblocks; b += kPlanThreads) st_device(passed + b, 0ull);
  }
}

// The one-launch plan.  It runs one workgroup per CU at the sizes it is used for, so it takes the
// scalar registers the compiler wants (106: the many pointers of PlanParams).
__global__ __launch_bounds__(kPlanThreads) void plan_fused_kernel(PlanParams p, uint64_t *matrix, uint64_t *passed,
                                                                  uint64_t tag, int staged_table) {
  plan_body<true>(p, matrix, passed, tag, staged_table);
}

// The last launch of a large plan: the same body without the grid-wide wait.  Held to 96 scalar
// registers, i.e. eight waves per SIMD, so that two workgroups fit a CU and the 512 workgroups of a
// 64 Ki-token layer run in one round (thirty-odd scalars then live in vector lanes, which is
// cheaper than a second round).
__global__ __launch_bounds__(kPlanThreads) __attribute__((amdgpu_waves_per_eu(8, 8))) void plan_write_kernel(PlanParams p,
                                                                                                      int staged_table) {
  plan_body<false>(p, nullptr, nullptr, 0, staged_table);
}

// Table of one hop for a (parent, child) pair of group cuts: purely elementwise.
__global__ __launch_bounds__(kPlanThreads) void level_dest_map_kernel(const int32_t *__restrict__ expert_to_rank, int E,
                                                                       int G, int my_rank, int ranks_per_parent,
                                                                       int ranks_per_child, int children_per_parent,
                                                                       int32_t *__restrict__ dest_map,
                                                                       int32_t *__restrict__ num_dest) {
  const int e = blockIdx.x * kPlanThreads + threadIdx.x;
  if (e == 0) *num_dest = children_per_parent;
  if (e >= E) return;
  const int g = expert_to_rank[e];
  int v;
  if ((unsigned)g >= (unsigned)G) v = -2;
  else if (g / ranks_per_parent != my_rank / ranks_per_parent) v = -1;
  else v = (g / ranks_per_child) % children_per_parent;
  dest_map[e] = v;
}

// Destination table of a receiver stage: one workgroup walks the E experts in chunks of 1024 and
// numbers the experts placed on `my_rank` with a ballot scan, so local indices ascend with the
// expert id.
__global__ __launch_bounds__(kPlanThreads) void recv_dest_map_kernel(const int32_t *__restrict__ expert_to_rank, int E,
                                                                      int G, int R, int my_rank, int stage,
                                                                      int32_t *__restrict__ dest_map,
                                                                      int32_t *__restrict__ num_dest) {
  __shared__ int32_t wave_cnt[kPlanWaves];
  __shared__ int32_t base;
  const int lane = lane_id(), wv = (int)(threadIdx.x >> 6);
  if (threadIdx.x == 0) base = 0;
  __syncthreads();
  for (int e0 = 0; e0 < E; e0 += kPlanThreads) {
    const int e = e0 + (int)threadIdx.x;
    int g = -1;
    if (e < E) {
      g = expert_to_rank[e];
      if ((unsigned)g >= (unsigned)G) g = -2;
    }
    const bool mine = g == my_rank;
    const uint64_t b = __ballot(mine);
    if (lane == 0) wave_cnt[wv] = __popcll(b);
    __syncthreads();
    int before = base;
    for (int w = 0; w < wv; ++w) before += wave_cnt[w];
    if (e < E) {
      int v;
      if (g == -2) v = -2;
      else if (stage == HM_RECV_INTRA_NODE) v = (g / R == my_rank / R) ? g % R : -1;
      else v = mine ? before + __popcll(b & ((1ull << lane) - 1ull)) : -1;
      dest_map[e] = v;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
      int tot = 0;
      for (int w = 0; w < kPlanWaves; ++w) tot += wave_cnt[w];
      base += tot;
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) *num_dest = stage == HM_RECV_INTRA_NODE ? R : base;
}

static inline int32_t plan_blocks(int64_t nslots) {
  const int64_t b = (nslots + kPlanThreads - 1) / kPlanThreads;
  return (int32_t)(b < 1 ? 1 : b);
}

// Workspace: the count matrix [workgroups + 1][Dn] int32 of the multi-launch kernels, then
// (8-byte aligned) what the one-launch kernel uses instead: a matrix of [workgroups][Dn] tagged
// 64-bit words and one 64-bit flag per workgroup.
static inline size_t plan_counts_bytes(int64_t nslots, int Dn) {
  const size_t b = ((size_t)plan_blocks(nslots) + 1) * (size_t)Dn * sizeof(int32_t);
  return (b + 7) & ~(size_t)7;
}
static inline size_t plan_workspace(int64_t nslots, int Dn) {
  const int32_t nb = plan_blocks(nslots);
  const size_t fused = nb <= kPlanFusedMaxBlocks ? ((size_t)nb * (size_t)Dn + (size_t)nb) * sizeof(uint64_t) : 0;
  return plan_counts_bytes(nslots, Dn) + fused;
}

// Workgroups of plan_fused_kernel that can be resident together on the current device (0 if that
// cannot be established: the multi-launch path is always available).
static inline int fused_capacity() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  int v = cached[dev].load(std::memory_order_relaxed);
  if (v == 0) {
    int cus = 0, per_cu = 0;
    v = -1;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) == hipSuccess &&
        hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, plan_fused_kernel, kPlanThreads,
                                                     kPlanStagedExperts * 6) == hipSuccess &&
        cus > 0 && per_cu > 0)
      v = cus * per_cu;
    cached[dev].store(v, std::memory_order_relaxed);
  }
  return v > 0 ? v : 0;
}

// 53 bits no earlier launch of this process has used and stale memory is unlikely to hold; never 0.
static inline uint64_t next_tag() {
  static std::atomic<uint64_t> counter{0};
  static std::once_flag seeded;
  std::call_once(seeded, [] {
    uint64_t z = (uint64_t)std::chrono::steady_clock::now().time_since_epoch().count() ^ ((uint64_t)getpid() << 40);
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    counter.store(z ^ (z >> 31), std::memory_order_relaxed);
  });
  const uint64_t mask = (1ull << 53) - 1ull;
  uint64_t e = (counter.fetch_add(1, std::memory_order_relaxed) + 1) & mask;
  if (e == 0) e = (counter.fetch_add(1, std::memory_order_relaxed) + 1) & mask;
  return e;
}

// Largest plan, in workgroups, that takes the one-launch kernel (hm_plan_one_launch_limit).
static std::atomic<int> one_launch_limit{kPlanFusedMaxBlocks};

// One launch when the plan is small enough, else count -> (scan) -> write, on `stream`;
// p.nblocks, p.Dn and p.counts are set.
static inline hm_status launch_plan(PlanParams &p, hipStream_t stream) {
  const bool loads = p.load_expert != nullptr;
  const int staged = p.E <= kPlanStagedExperts ? 1 : 0;   // tables (and histogram) in LDS
  const unsigned lds = staged ? ((loads ? (unsigned)p.E * sizeof(int32_t) : 0u) + ((2u * (unsigned)p.E + 15u) & ~15u)) : 0u;
  if (p.nblocks <= one_launch_limit.load(std::memory_order_relaxed) && p.nblocks <= fused_capacity()) {
    p.scanned = 0;
    uint64_t *matrix = (uint64_t *)((char *)p.counts + plan_counts_bytes(p.nslots, p.Dn));
    hipLaunchKernelGGL(plan_fused_kernel, dim3(p.nblocks), dim3(kPlanThreads), lds, stream, p, matrix,
                       matrix + (size_t)p.nblocks * p.Dn, next_tag(), staged);
    return hm_launch_status();
  }
  p.scanned = (int64_t)p.nblocks * p.Dn >= kPlanScanMinEntries ? 1 : 0;
  hipLaunchKernelGGL(plan_count_kernel, dim3(p.nblocks), dim3(kPlanThreads), 0, stream, p);
  if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  if (p.scanned) {
    hipLaunchKernelGGL(plan_scan_kernel, dim3(p.Dn), dim3(kPlanThreads), 0, stream, p);
    if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  }
  // the same kernel without its grid-wide wait: the counts are complete
  hipLaunchKernelGGL(plan_write_kernel, dim3(p.nblocks), dim3(kPlanThreads), lds, stream, p, staged);
  return hm_launch_status();
}

}  // namespace hm

extern "C" int32_t hm_plan_one_launch_capacity(void) { return hm::fused_capacity(); }

extern "C" int32_t hm_plan_one_launch_limit(int32_t workgroups) {
  const int v = workgroups < 0 ? 0 : workgroups > hm::kPlanFusedMaxBlocks ? hm::kPlanFusedMaxBlocks : workgroups;
  return hm::one_launch_limit.exchange(v, std::memory_order_relaxed);
}

extern "C" size_t hm_plan_workspace_bytes(int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level) {
  if (E < 1 || hm_check_tk(T, K) != HM_OK || hm_check_topology(topo) != HM_OK) return 0;
  if (level != HM_DEDUP_NONE && level != HM_DEDUP_GPU && level != HM_DEDUP_NODE) return 0;
  const int Dn = level == HM_DEDUP_NODE ? topo.nodes : topo.nodes * topo.ranks_per_node;
  return hm::plan_workspace((int64_t)T * K, Dn);
}

// Argument checks and launches of hm_plan; `counts` is the count matrix (caller's workspace or the
// library's static scratch), already known to be large enough.
static hm_status plan_on_counts(const int32_t *topk_ids, const float *topk_weights, const int32_t *expert_to_rank,
                                int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level, hm_plan_out *out,
                                int32_t *counts, void *hip_stream) {
  hm::PlanParams p;
  p.ids = topk_ids;
  p.weights = topk_weights;
  p.expert_to_rank = expert_to_rank;
  p.dest_map = nullptr;
  p.T = T;
  p.K = K;
  p.E = E;
  p.R = topo.ranks_per_node;
  p.G = topo.nodes * topo.ranks_per_node;
  p.Dn = level == HM_DEDUP_NODE ? topo.nodes : p.G;
  p.level = (int32_t)level;
  p.nslots = (int32_t)((int64_t)T * K);
  p.nblocks = hm::plan_blocks(p.nslots);
  p.row_capacity = out->row_capacity;
  p.counts = counts;
  p.dest_count = out->dest_count;
  p.dest_offset = out->dest_offset;
  p.row_token = out->row_token;
  p.slot_row = out->slot_row;
  p.slot_keep = out->slot_keep;
  p.row_weight = out->row_weight;
  p.rank_mask = out->rank_mask;
  p.node_mask = out->node_mask;
  p.status = out->status;
  p.load_expert = out->load_expert;
  p.load_rank = out->load_rank;
  p.load_node = out->load_node;
  out->num_dest = p.Dn;
  out->max_rows_per_token = level == HM_DEDUP_NONE ? K : (K < p.Dn ? K : p.Dn);
  return hm::launch_plan(p, (hipStream_t)hip_stream);
}

static hm_status check_plan_args(const int32_t *topk_ids, const float *topk_weights, const int32_t *expert_to_rank,
                                 int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level,
                                 const hm_plan_out *out) {
  if (!out || !expert_to_rank) return HM_ERR_NULL;
  if (!out->dest_count || !out->dest_offset || !out->row_token || !out->slot_row || !out->slot_keep ||
      !out->row_weight || !out->status)
    return HM_ERR_NULL;
  hm_status st = hm_check_tk(T, K);
  if (st != HM_OK) return st;
  if (E < 1 || out->row_capacity < 0) return HM_ERR_SHAPE;
  if (T > 0 && (!topk_ids || !topk_weights)) return HM_ERR_NULL;
  if (out->load_expert && (!out->load_rank || !out->load_node)) return HM_ERR_NULL;
  if (!out->load_expert && (out->load_rank || out->load_node)) return HM_ERR_NULL;
  st = hm_check_topology(topo);
  if (st != HM_OK) return st;
  if (level != HM_DEDUP_NONE && level != HM_DEDUP_GPU && level != HM_DEDUP_NODE) return HM_ERR_LEVEL;
  return HM_OK;
}

extern "C" hm_status hm_plan(const int32_t *topk_ids, const float *topk_weights, const int32_t *expert_to_rank,
                             int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level,
                             hm_plan_out *out, void *workspace, size_t workspace_bytes, void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!workspace) return HM_ERR_NULL;
  hm_status st = check_plan_args(topk_ids, topk_weights, expert_to_rank, T, K, E, topo, level, out);
  if (st != HM_OK) return st;
  if (workspace_bytes < hm_plan_workspace_bytes(T, K, E, topo, level)) return HM_ERR_WORKSPACE;
  return plan_on_counts(topk_ids, topk_weights, expert_to_rank, T, K, E, topo, level, out, (int32_t *)workspace,
                        hip_stream);
}

// ---- hm_plan_static: hm_plan for callers that cannot hand over (or allocate) a workspace ----------
// The count matrix lives in a file-scope device array.  In host code the array's name is only a
// stand-in for the symbol: its device address is looked up once per device and that pointer is
// what the kernels receive.
namespace hm {
constexpr size_t kPlanStaticBytes = (size_t)1 << 20;   // 1 MiB per GPU, held until the process ends
constexpr int kPlanStaticDevices = 64;
static __device__ __align__(256) unsigned char plan_static_scratch[kPlanStaticBytes];
static std::mutex plan_static_lock;
static void *plan_static_ptr[kPlanStaticDevices];   // device address of the array on each GPU, 0 = not asked yet

// Device address of the current GPU's copy of the scratch array (nullptr on a HIP error).
static void *plan_static_address() {
  int dev = -1;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kPlanStaticDevices) return nullptr;
  std::lock_guard<std::mutex> hold(plan_static_lock);
  if (!plan_static_ptr[dev]) {
    void *ptr = nullptr;
    if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(plan_static_scratch)) != hipSuccess) return nullptr;
    plan_static_ptr[dev] = ptr;
  }
  return plan_static_ptr[dev];
}
}  // namespace hm

extern "C" size_t hm_plan_static_max_bytes(void) { return hm::kPlanStaticBytes; }

extern "C" hm_status hm_plan_static(const int32_t *topk_ids, const float *topk_weights, const int32_t *expert_to_rank,
                                    int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level,
                                    hm_plan_out *out, void *hip_stream) {
  HM_ENTRY_SCOPE;
  hm_status st = check_plan_args(topk_ids, topk_weights, expert_to_rank, T, K, E, topo, level, out);
  if (st != HM_OK) return st;
  if (hm_plan_workspace_bytes(T, K, E, topo, level) > hm::kPlanStaticBytes) return HM_ERR_WORKSPACE;
  void *counts = hm::plan_static_address();
  if (!counts) return HM_ERR_HIP;
  // Nothing in the matrix has to start at zero: the count kernel overwrites every entry the later
  // kernels read, so the previous call's contents are harmless.
  return plan_on_counts(topk_ids, topk_weights, expert_to_rank, T, K, E, topo, level, out, (int32_t *)counts,
                        hip_stream);
}

extern "C" size_t hm_plan_mapped_workspace_bytes(int32_t rows, int32_t K, int32_t num_dest) {
  if (hm_check_tk(rows, K) != HM_OK || num_dest < 1 || num_dest > 64) return 0;
  return hm::plan_workspace((int64_t)rows * K, num_dest);
}

extern "C" hm_status hm_plan_mapped(const int32_t *row_ids, const float *row_weights, const int32_t *dest_map,
                                    int32_t rows, int32_t K, int32_t E, int32_t num_dest, int32_t dedup, hm_plan_out *out,
                                    void *workspace, size_t workspace_bytes, void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!out || !dest_map || !workspace) return HM_ERR_NULL;
  if (!out->dest_count || !out->dest_offset || !out->row_token || !out->slot_row || !out->slot_keep ||
      !out->row_weight || !out->status)
    return HM_ERR_NULL;
  hm_status st = hm_check_tk(rows, K);
  if (st != HM_OK) return st;
  if (E < 1 || out->row_capacity < 0) return HM_ERR_SHAPE;
  if (num_dest < 1 || num_dest > 64) return HM_ERR_TOPOLOGY;
  if (rows > 0 && (!row_ids || !row_weights)) return HM_ERR_NULL;
  if (workspace_bytes < hm_plan_mapped_workspace_bytes(rows, K, num_dest)) return HM_ERR_WORKSPACE;

  hm::PlanParams p;
  p.ids = row_ids;
  p.weights = row_weights;
  p.expert_to_rank = nullptr;
  p.dest_map = dest_map;
  p.T = rows;
  p.K = K;
  p.E = E;
  p.R = 1;
  p.G = num_dest;
  p.Dn = num_dest;
  p.level = dedup ? (int32_t)HM_DEDUP_GPU : (int32_t)HM_DEDUP_NONE;
  p.nslots = (int32_t)((int64_t)rows * K);
  p.nblocks = hm::plan_blocks(p.nslots);
  p.row_capacity = out->row_capacity;
  p.counts = (int32_t *)workspace;
  p.dest_count = out->dest_count;
  p.dest_offset = out->dest_offset;
  p.row_token = out->row_token;
  p.slot_row = out->slot_row;
  p.slot_keep = out->slot_keep;
  p.row_weight = out->row_weight;
  p.rank_mask = out->rank_mask;
  p.node_mask = out->node_mask;
  p.status = out->status;
  p.load_expert = p.load_rank = p.load_node = nullptr;   // the fused loads need the rank placement
  out->num_dest = num_dest;
  out->max_rows_per_token = 0;   // a hop table may leave most slots without a copy: no useful bound

  return hm::launch_plan(p, (hipStream_t)hip_stream);
}

extern "C" hm_status hm_recv_dest_map(const int32_t *expert_to_rank, int32_t E, hm_topology topo, int32_t my_rank,
                                      hm_recv_stage stage, int32_t *dest_map, int32_t *num_dest, void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!expert_to_rank || !dest_map || !num_dest) return HM_ERR_NULL;
  if (E < 1) return HM_ERR_SHAPE;
  hm_status st = hm_check_topology(topo);
  if (st != HM_OK) return st;
  const int G = topo.nodes * topo.ranks_per_node;
  if (my_rank < 0 || my_rank >= G) return HM_ERR_TOPOLOGY;
  if (stage != HM_RECV_INTRA_NODE && stage != HM_RECV_LOCAL_EXPERTS) return HM_ERR_LEVEL;
  hipLaunchKernelGGL(hm::recv_dest_map_kernel, dim3(1), dim3(hm::kPlanThreads), 0, (hipStream_t)hip_stream,
                     expert_to_rank, E, G, topo.ranks_per_node, my_rank, (int)stage, dest_map, num_dest);
  return hm_launch_status();
}

extern "C" hm_status hm_level_dest_map(const int32_t *expert_to_rank, int32_t E, int32_t G, int32_t my_rank,
                                       int32_t parent_groups, int32_t child_groups, int32_t *dest_map, int32_t *num_dest,
                                       void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!expert_to_rank || !dest_map || !num_dest) return HM_ERR_NULL;
  if (E < 1) return HM_ERR_SHAPE;
  if (G < 1 || G > 64 || my_rank < 0 || my_rank >= G) return HM_ERR_TOPOLOGY;
  if (parent_groups < 1 || child_groups < parent_groups || child_groups > G) return HM_ERR_TOPOLOGY;
  if (child_groups % parent_groups != 0 || G % child_groups != 0) return HM_ERR_TOPOLOGY;
  const int blocks = (E + hm::kPlanThreads - 1) / hm::kPlanThreads;
  hipLaunchKernelGGL(hm::level_dest_map_kernel, dim3(blocks), dim3(hm::kPlanThreads), 0, (hipStream_t)hip_stream,
                     expert_to_rank, E, G, my_rank, G / parent_groups, G / child_groups, child_groups / parent_groups,
                     dest_map, num_dest);
  return hm_launch_status();
}

extern "C" hm_status hm_plan_status(hm_plan_out *plan, int64_t *total_rows, void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!plan || !plan->status || !plan->dest_offset) return HM_ERR_NULL;
  if (plan->num_dest < 1 || plan->num_dest > 64) return HM_ERR_SHAPE;
  hipStream_t stream = (hipStream_t)hip_stream;
  int32_t host[2] = {0, 0};
  if (hipMemcpyAsync(&host[0], plan->status, sizeof(int32_t), hipMemcpyDeviceToHost, stream) != hipSuccess)
    return HM_ERR_HIP;
  if (hipMemcpyAsync(&host[1], plan->dest_offset + plan->num_dest, sizeof(int32_t), hipMemcpyDeviceToHost,
                     stream) != hipSuccess)
    return HM_ERR_HIP;
  if (hipStreamSynchronize(stream) != hipSuccess) return HM_ERR_HIP;
  if (total_rows) *total_rows = host[1];
  plan->expected_rows = host[1];   // what the row kernels size their launches by
  return (hm_status)host[0];
}

extern "C" const char *hm_status_string(hm_status s) {
  switch (s) {
    case HM_OK: return "ok";
    case HM_ERR_NULL: return "null pointer";
    case HM_ERR_SHAPE: return "bad shape";
    case HM_ERR_TOPOLOGY: return "bad topology (need 1..32 nodes, at most 64 ranks)";
    case HM_ERR_LEVEL: return "bad dedup level";
    case HM_ERR_WORKSPACE: return "workspace too small (hm_plan_static: sizes beyond its static scratch)";
    case HM_ERR_CAPACITY: return "row index beyond the caller's row buffers";
    case HM_ERR_BAD_ID: return "expert id or rank out of range";
    case HM_ERR_HIP: return "HIP runtime error";
  }
  return "unknown status";
}
