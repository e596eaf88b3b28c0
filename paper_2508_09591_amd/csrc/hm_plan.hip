// hm_plan: routing -> deduplicated, stable per-destination send lists (HierMoE Eq.(7)).
//
// One lane owns one routing slot s = t*K + k; a wave owns 64 consecutive slots, a workgroup 1024.
// Rows of a destination are numbered in ascending slot order, so a lane's row is
//     dest_offset[d] + (kept slots of d in earlier workgroups) + (in earlier waves of this
//     workgroup) + (in lower lanes of this wave),
// and the last term is a popcount over a wavefront ballot.  No atomics decide positions, so the
// plan is deterministic and stable.  Two launches:
//   plan_count_kernel  per-workgroup, per-destination counts of kept slots -> workspace
//   plan_write_kernel  every workgroup re-reads the (small) count matrix to get its own base
//                      rows and the destination totals, then writes the index maps.
// Re-reading the matrix costs workgroups^2 * destinations loads in total, so beyond
// kPlanScanMinEntries entries a third launch in between (plan_scan_kernel, one workgroup per
// destination) turns the matrix into exclusive prefixes plus a row of totals and the write
// kernel reads just its own row: linear in the number of slots at any size.
// Both first stage the rank and destination of their 1024 slots, plus a halo of K-1 slots on
// either side (the rest of the first and last token), in LDS: each expert id is looked up once
// and all "same destination as an earlier / later slot of my token" questions become LDS reads.
#include "hm_device.h"

#include <mutex>

namespace hm {

constexpr int kPlanThreads = 1024;
constexpr int kPlanWaves = kPlanThreads / kWave;
constexpr int kPlanHalo = 63;                              // K - 1 <= 63
constexpr int kPlanStaged = kPlanThreads + 2 * kPlanHalo;
constexpr int kPlanHist = 8192;                            // experts histogrammed in LDS for the fused loads
constexpr int64_t kPlanScanMinEntries = 16384;             // count-matrix entries from which the scan launch pays

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
__device__ __forceinline__ Slot stage_and_classify(const PlanParams &p, int8_t *s_rank, int8_t *s_dest,
                                                   float *s_weight = nullptr) {
  const int halo = p.K - 1;
  const int64_t first = (int64_t)blockIdx.x * kPlanThreads;
  for (int i = threadIdx.x; i < kPlanThreads + 2 * halo; i += kPlanThreads) {
    const int64_t s = first - halo + i;
    int r = -1, d = -1;
    if (s_weight) s_weight[i] = (s >= 0 && s < p.nslots) ? p.weights[s] : 0.0f;   // in flight with the id lookups
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

__global__ __launch_bounds__(kPlanThreads) void plan_count_kernel(PlanParams p) {
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

__global__ __launch_bounds__(kPlanThreads) void plan_write_kernel(PlanParams p) {
  __shared__ int8_t s_rank[kPlanStaged];
  __shared__ int8_t s_dest[kPlanStaged];
  __shared__ int32_t part_tot[kPlanWaves][kWave];
  __shared__ int32_t part_pre[kPlanWaves][kWave];
  __shared__ int32_t block_base[kWave];             // first row of this workgroup per destination
  __shared__ uint64_t ballots[kPlanWaves][kWave];   // [wave][destination] -> lanes that keep a slot
  __shared__ int32_t wave_base[kPlanWaves][kWave];  // kept slots in earlier waves of the workgroup
  __shared__ int32_t hist[kPlanHist];               // fused expert load: slots per expert
  __shared__ int32_t blk_rank[kWave], blk_node[kWave];
  __shared__ float s_weight[kPlanStaged];           // router weights of the staged slots
  const int lane = lane_id(), wv = (int)(threadIdx.x >> 6);
  const bool loads = p.load_expert != nullptr;
  const bool lds_hist = p.E <= kPlanHist;
  if (loads) {
    if (lds_hist)
      for (int e = threadIdx.x; e < p.E; e += kPlanThreads) hist[e] = 0;
    if (threadIdx.x < kWave) blk_rank[threadIdx.x] = blk_node[threadIdx.x] = 0;
  }

  // Column sums of the count matrix: over all workgroups (destination total) and over the
  // earlier ones (this workgroup's base).  Wave wv takes rows wv, wv+16, ...
  {
    int tot = 0, pre = 0;
    if (p.scanned) {
      if (wv == 0 && lane < p.Dn) {
        tot = p.counts[(int64_t)p.nblocks * p.Dn + lane];
        pre = p.counts[(int64_t)blockIdx.x * p.Dn + lane];
      }
    } else if (lane < p.Dn) {
      for (int b = wv; b < p.nblocks; b += kPlanWaves) {
        const int c = p.counts[(int64_t)b * p.Dn + lane];
        tot += c;
        if (b < (int)blockIdx.x) pre += c;
      }
    }
    part_tot[wv][lane] = tot;
    part_pre[wv][lane] = pre;
  }

  const int64_t s = (int64_t)blockIdx.x * kPlanThreads + threadIdx.x;
  int my_id = -1;   // for the expert histogram; fetched now so that it does not cost a round trip later
  if (loads && s < p.nslots) my_id = p.ids[s];
  const Slot me = stage_and_classify(p, s_rank, s_dest, s_weight);   // contains a barrier
  const int kept_dest = me.keep ? me.dest : -1;
  for (int d = 0; d < p.Dn; ++d) {
    const uint64_t b = __ballot(kept_dest == d);
    if (lane == d) ballots[wv][d] = b;
  }
  __syncthreads();

  if (lane < p.Dn) {
    int a = 0;
    for (int w = 0; w < wv; ++w) a += __popcll(ballots[w][lane]);
    wave_base[wv][lane] = a;
  }
  if (wv == 0) {
    int tot = 0, pre = 0;
    if (lane < p.Dn)
      for (int w = 0; w < kPlanWaves; ++w) {
        tot += part_tot[w][lane];
        pre += part_pre[w][lane];
      }
    int incl = tot;  // inclusive scan over destinations (lanes >= Dn hold 0)
    for (int off = 1; off < kWave; off <<= 1) {
      const int v = __shfl_up(incl, off, kWave);
      if (lane >= off) incl += v;
    }
    const int offset = incl - tot;
    block_base[lane] = offset + pre;
    if (blockIdx.x == 0 && lane < p.Dn) {
      p.dest_count[lane] = tot;
      p.dest_offset[lane] = offset;
      if (lane == p.Dn - 1) p.dest_offset[p.Dn] = incl;
    }
  }
  __syncthreads();

  if (me.live) {
    if (me.dest < 0) {
      p.slot_row[s] = -1;
      p.slot_keep[s] = 0;
      if (me.rank == -1) flag(p.status, HM_ERR_BAD_ID);
    } else if (!me.keep) {
      p.slot_keep[s] = 0;  // its slot_row is written by the slot that owns the row
    } else {
      const uint64_t b = ballots[wv][me.dest];
      const int pos = __popcll(b & ((1ull << lane) - 1ull));
      const int row = block_base[me.dest] + wave_base[wv][me.dest] + pos;
      p.slot_keep[s] = 1;
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
  }
  // Per-token masks, owned by the lane of the token's slot 0.
  uint64_t rm = 0;
  uint32_t nm = 0;
  if (me.live && me.k == 0 && (p.rank_mask || p.node_mask || loads)) {
    for (int k2 = 0; k2 < p.K; ++k2) {
      const int r2 = s_rank[me.tok0 + k2];
      if (r2 >= 0) {
        rm |= 1ull << r2;
        if (!p.dest_map) nm |= 1u << (r2 / p.R);
      }
    }
    if (p.rank_mask) p.rank_mask[me.t] = rm;
    if (p.node_mask) p.node_mask[me.t] = nm;
  }
  if (!loads) return;

  // Fused hm_expert_load: slots per expert, and tokens per rank / node counted once each from the
  // masks above (a ballot per group; lane g keeps the count of group g).
  if (me.live && me.rank >= 0) {
    if (lds_hist) atomicAdd(&hist[my_id], 1);
    else atomicAdd(&p.load_expert[my_id], 1);
  }
  int my_rank_cnt = 0, my_node_cnt = 0;
  const int nodes = p.G / p.R;
  for (int g = 0; g < p.G; ++g) {
    const uint64_t b = __ballot((rm >> g) & 1ull);
    if (lane == g) my_rank_cnt = __popcll(b);
  }
  for (int n = 0; n < nodes; ++n) {
    const uint64_t b = __ballot((nm >> n) & 1u);
    if (lane == n) my_node_cnt = __popcll(b);
  }
  if (my_rank_cnt) atomicAdd(&blk_rank[lane], my_rank_cnt);
  if (my_node_cnt) atomicAdd(&blk_node[lane], my_node_cnt);
  __syncthreads();
  if (lds_hist)
    for (int e = threadIdx.x; e < p.E; e += kPlanThreads)
      if (hist[e]) atomicAdd(&p.load_expert[e], hist[e]);
  if ((int)threadIdx.x < p.G && blk_rank[threadIdx.x]) atomicAdd(&p.load_rank[threadIdx.x], blk_rank[threadIdx.x]);
  if ((int)threadIdx.x < nodes && blk_node[threadIdx.x]) atomicAdd(&p.load_node[threadIdx.x], blk_node[threadIdx.x]);
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

static inline size_t plan_workspace(int64_t nslots, int Dn) {
  return ((size_t)plan_blocks(nslots) + 1) * (size_t)Dn * sizeof(int32_t);
}

// count -> (scan) -> write on `stream`; p.nblocks, p.Dn and p.counts are set.
static inline hm_status launch_plan(PlanParams &p, hipStream_t stream) {
  p.scanned = (int64_t)p.nblocks * p.Dn >= kPlanScanMinEntries ? 1 : 0;
  hipLaunchKernelGGL(plan_count_kernel, dim3(p.nblocks), dim3(kPlanThreads), 0, stream, p);
  if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  if (p.scanned) {
    hipLaunchKernelGGL(plan_scan_kernel, dim3(p.Dn), dim3(kPlanThreads), 0, stream, p);
    if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  }
  hipLaunchKernelGGL(plan_write_kernel, dim3(p.nblocks), dim3(kPlanThreads), 0, stream, p);
  return hm_launch_status();
}

}  // namespace hm

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
