// hm_expert_load: per-expert slot counts and duplicate-free per-rank / per-node token counts
// (the p^(1,G) and p^(1,U[1]) vectors of HierMoE Eq.(7)) for the expert-swap planner of Section IV.
//
// One lane owns one token.  Expert counts go through an LDS histogram; rank and node counts come
// from ballots over the per-token bit masks (lane g accumulates the popcount for group g), so a
// token is counted once per group however many of its experts live there.  A first tiny launch
// clears the outputs, then integer atomics merge the workgroups, which keeps the result exact and
// order-independent.  The call is launch-latency bound (two launches, ~11 us on T=8192, K=8);
// two single-launch designs were measured and dropped: one 1024-lane workgroup doing everything
// (56 us) and 64 workgroups that each scan the whole table but own a slice of the outputs
// (44 us) -- both serialise dependent id -> placement loads that the token-split version spreads
// over the chip.
#include "hm_device.h"

namespace hm {

struct LoadParams {
  const int32_t *ids;
  const int32_t *expert_to_rank;
  int32_t T, K, E, G, R, N;
  int32_t *load_expert, *load_rank, *load_node, *status;
};

constexpr int kLoadThreads = 256;
constexpr int kLdsExperts = 8192;  // experts histogrammed in LDS; beyond that, global atomics

__global__ __launch_bounds__(kLoadThreads) void load_clear_kernel(LoadParams p) {
  const int i = blockIdx.x * kLoadThreads + threadIdx.x;
  if (i < p.E) p.load_expert[i] = 0;
  if (i < p.G) p.load_rank[i] = 0;
  if (i < p.N) p.load_node[i] = 0;
  if (i == 0 && p.status) *p.status = 0;
}

__global__ __launch_bounds__(kLoadThreads) void load_count_kernel(LoadParams p) {
  __shared__ int32_t hist[kLdsExperts];
  __shared__ int32_t rank_cnt[kWave];
  __shared__ int32_t node_cnt[kWave];
  const bool lds_hist = p.E <= kLdsExperts;
  if (lds_hist)
    for (int e = threadIdx.x; e < p.E; e += kLoadThreads) hist[e] = 0;
  if (threadIdx.x < kWave) {
    rank_cnt[threadIdx.x] = 0;
    node_cnt[threadIdx.x] = 0;
  }
  __syncthreads();

  const int lane = lane_id();
  int my_rank_cnt = 0, my_node_cnt = 0;  // lane g: tokens of this wave's share that reach group g
  const int64_t stride = (int64_t)gridDim.x * kLoadThreads;
  // every lane of a wave runs the same number of rounds so the ballots stay convergent
  const int64_t rounds = ((int64_t)p.T + stride - 1) / stride;
  for (int64_t it = 0; it < rounds; ++it) {
    const int64_t t = it * stride + (int64_t)blockIdx.x * kLoadThreads + threadIdx.x;
    uint64_t rm = 0;
    uint32_t nm = 0;
    if (t < p.T) {
      const int32_t *tok = p.ids + t * p.K;
      for (int k = 0; k < p.K; ++k) {
        const int id = tok[k];
        const int g = rank_of(p.expert_to_rank, p.E, p.G, id);
        if (g < 0) {
          if (g == -1) flag(p.status, HM_ERR_BAD_ID);
          continue;
        }
        if (lds_hist) atomicAdd(&hist[id], 1);
        else atomicAdd(&p.load_expert[id], 1);
        rm |= 1ull << g;
        nm |= 1u << (g / p.R);
      }
    }
    for (int g = 0; g < p.G; ++g) {
      const uint64_t bal = __ballot((rm >> g) & 1ull);
      if (lane == g) my_rank_cnt += __popcll(bal);
    }
    for (int n = 0; n < p.N; ++n) {
      const uint64_t bal = __ballot((nm >> n) & 1u);
      if (lane == n) my_node_cnt += __popcll(bal);
    }
  }
  if (lane < p.G && my_rank_cnt) atomicAdd(&rank_cnt[lane], my_rank_cnt);
  if (lane < p.N && my_node_cnt) atomicAdd(&node_cnt[lane], my_node_cnt);
  __syncthreads();
  if (lds_hist)
    for (int e = threadIdx.x; e < p.E; e += kLoadThreads)
      if (hist[e]) atomicAdd(&p.load_expert[e], hist[e]);
  if ((int)threadIdx.x < p.G && rank_cnt[threadIdx.x]) atomicAdd(&p.load_rank[threadIdx.x], rank_cnt[threadIdx.x]);
  if ((int)threadIdx.x < p.N && node_cnt[threadIdx.x]) atomicAdd(&p.load_node[threadIdx.x], node_cnt[threadIdx.x]);
}

}  // namespace hm

extern "C" hm_status hm_expert_load(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K,
                                    int32_t E, hm_topology topo, int32_t *load_expert, int32_t *load_rank,
                                    int32_t *load_node, int32_t *status, void *hip_stream) {
  HM_ENTRY_SCOPE;
  using namespace hm;
  if (!expert_to_rank || !load_expert || !load_rank || !load_node) return HM_ERR_NULL;
  hm_status st = hm_check_tk(T, K);
  if (st != HM_OK) return st;
  if (E < 1) return HM_ERR_SHAPE;
  if (T > 0 && !topk_ids) return HM_ERR_NULL;
  st = hm_check_topology(topo);
  if (st != HM_OK) return st;
  hipStream_t stream = (hipStream_t)hip_stream;
  LoadParams p;
  p.ids = topk_ids;
  p.expert_to_rank = expert_to_rank;
  p.T = T;
  p.K = K;
  p.E = E;
  p.R = topo.ranks_per_node;
  p.G = topo.nodes * topo.ranks_per_node;
  p.N = topo.nodes;
  p.load_expert = load_expert;
  p.load_rank = load_rank;
  p.load_node = load_node;
  p.status = status;
  const int most = E > kWave ? E : kWave;
  hipLaunchKernelGGL(load_clear_kernel, dim3((most + kLoadThreads - 1) / kLoadThreads), dim3(kLoadThreads), 0, stream, p);
  if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  if (T == 0) return HM_OK;
  int64_t blocks = ((int64_t)T + kLoadThreads - 1) / kLoadThreads;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(load_count_kernel, dim3((unsigned)blocks), dim3(kLoadThreads), 0, stream, p);
  return hm_launch_status();
}
