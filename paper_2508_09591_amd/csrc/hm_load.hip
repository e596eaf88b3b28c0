// hm_expert_load: per-expert slot counts and duplicate-free per-rank / per-node token counts
// (the p^(1,G) and p^(1,U[1]) vectors of HierMoE Eq.(7)) for the expert-swap planner of Section IV.
//
// One lane owns one token.  Expert counts go through an LDS histogram; rank and node counts come
// from ballots over the per-token bit masks (lane g accumulates the popcount for group g), so a
// token is counted once per group however many of its experts live there.  A first tiny launch
// clears the outputs, then integer atomics merge the workgroups, which keeps the result exact and
// order-independent.  (One 1024-lane workgroup doing everything in a single launch was measured
// at 56 us on T=8192, K=8 against 11 us for this pair of launches.)
#include "hm_device.h"

namespace hm {

constexpr int kLoadThreads = 256;
constexpr int kLdsExperts = 8192;  // experts histogrammed in LDS; beyond that, global atomics

__global__ __launch_bounds__(kLoadThreads) void load_clear_kernel(int32_t *load_expert, int E, int32_t *load_rank, int G,
                                                                  int32_t *load_node, int N, int32_t *status) {
  const int i = blockIdx.x * kLoadThreads + threadIdx.x;
  if (i < E) load_expert[i] = 0;
  if (i < G) load_rank[i] = 0;
  if (i < N) load_node[i] = 0;
  if (i == 0 && status) *status = 0;
}

__global__ __launch_bounds__(kLoadThreads) void load_count_kernel(const int32_t *__restrict__ ids,
                                                                  const int32_t *__restrict__ expert_to_rank, int T, int K,
                                                                  int E, int G, int R, int N, int32_t *load_expert,
                                                                  int32_t *load_rank, int32_t *load_node, int32_t *status) {
  __shared__ int32_t hist[kLdsExperts];
  __shared__ int32_t rank_cnt[kWave];
  __shared__ int32_t node_cnt[kWave];
  const bool lds_hist = E <= kLdsExperts;
  if (lds_hist)
    for (int e = threadIdx.x; e < E; e += kLoadThreads) hist[e] = 0;
  if (threadIdx.x < kWave) {
    rank_cnt[threadIdx.x] = 0;
    node_cnt[threadIdx.x] = 0;
  }
  __syncthreads();

  const int lane = lane_id();
  int my_rank_cnt = 0, my_node_cnt = 0;  // lane g: tokens of this wave's share that reach group g
  const int64_t stride = (int64_t)gridDim.x * kLoadThreads;
  // every lane of a wave runs the same number of rounds so the ballots stay convergent
  const int64_t rounds = ((int64_t)T + stride - 1) / stride;
  for (int64_t it = 0; it < rounds; ++it) {
    const int64_t t = it * stride + (int64_t)blockIdx.x * kLoadThreads + threadIdx.x;
    uint64_t rm = 0;
    uint32_t nm = 0;
    if (t < T) {
      const int32_t *tok = ids + t * K;
      for (int k = 0; k < K; ++k) {
        const int id = tok[k];
        const int g = rank_of(expert_to_rank, E, G, id);
        if (g < 0) {
          flag(status, HM_ERR_BAD_ID);
          continue;
        }
        if (lds_hist) atomicAdd(&hist[id], 1);
        else atomicAdd(&load_expert[id], 1);
        rm |= 1ull << g;
        nm |= 1u << (g / R);
      }
    }
    for (int g = 0; g < G; ++g) {
      const uint64_t b = __ballot((rm >> g) & 1ull);
      if (lane == g) my_rank_cnt += __popcll(b);
    }
    for (int n = 0; n < N; ++n) {
      const uint64_t b = __ballot((nm >> n) & 1u);
      if (lane == n) my_node_cnt += __popcll(b);
    }
  }
  if (lane < G && my_rank_cnt) atomicAdd(&rank_cnt[lane], my_rank_cnt);
  if (lane < N && my_node_cnt) atomicAdd(&node_cnt[lane], my_node_cnt);
  __syncthreads();
  if (lds_hist)
    for (int e = threadIdx.x; e < E; e += kLoadThreads)
      if (hist[e]) atomicAdd(&load_expert[e], hist[e]);
  if ((int)threadIdx.x < G && rank_cnt[threadIdx.x]) atomicAdd(&load_rank[threadIdx.x], rank_cnt[threadIdx.x]);
  if ((int)threadIdx.x < N && node_cnt[threadIdx.x]) atomicAdd(&load_node[threadIdx.x], node_cnt[threadIdx.x]);
}

}  // namespace hm

extern "C" hm_status hm_expert_load(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K,
                                    int32_t E, hm_topology topo, int32_t *load_expert, int32_t *load_rank,
                                    int32_t *load_node, int32_t *status, void *hip_stream) {
  using namespace hm;
  if (!expert_to_rank || !load_expert || !load_rank || !load_node) return HM_ERR_NULL;
  hm_status st = hm_check_tk(T, K);
  if (st != HM_OK) return st;
  if (E < 1) return HM_ERR_SHAPE;
  if (T > 0 && !topk_ids) return HM_ERR_NULL;
  st = hm_check_topology(topo);
  if (st != HM_OK) return st;
  const int G = topo.nodes * topo.ranks_per_node, N = topo.nodes;
  hipStream_t stream = (hipStream_t)hip_stream;
  const int clear_blocks = ((E > kWave ? E : kWave) + kLoadThreads - 1) / kLoadThreads;
  hipLaunchKernelGGL(load_clear_kernel, dim3(clear_blocks), dim3(kLoadThreads), 0, stream, load_expert, E, load_rank, G,
                     load_node, N, status);
  if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  if (T == 0) return HM_OK;
  int64_t blocks = ((int64_t)T + kLoadThreads - 1) / kLoadThreads;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(load_count_kernel, dim3((unsigned)blocks), dim3(kLoadThreads), 0, stream,
                     topk_ids, expert_to_rank, T, K, E, G, topo.ranks_per_node, N, load_expert, load_rank, load_node, status);
  return hm_launch_status();
}
