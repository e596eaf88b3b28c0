// Dimension selection for the hierarchical exchange (HierMoE Section III-B/C, Eq.(1)-(6), Alg.1):
// per-level duplicate-free counts in one pass over the routing table, and the linear time model
// evaluated on the device so that the counts never travel to the host.
#include "hm_device.h"

namespace hm {

constexpr int kGroupThreads = 256;
constexpr int kMaxDepth = 4;

struct GroupParams {
  const int32_t *ids;
  const int32_t *expert_to_rank;
  int32_t T, K, E, G, depth;
  int32_t groups[kMaxDepth];
  int32_t *counts;   // [depth][64]
  int32_t *status;
};

__global__ __launch_bounds__(kGroupThreads) void group_clear_kernel(GroupParams p) {
  const int i = blockIdx.x * kGroupThreads + threadIdx.x;
  if (i < p.depth * kWave) p.counts[i] = 0;
  if (i == 0 && p.status) *p.status = 0;
}

// One lane per token: its rank mask is folded to one bit per group for every level, and lane j
// accumulates the popcount of the ballot over bit j (a token counts once per group).
__global__ __launch_bounds__(kGroupThreads) void group_count_kernel(GroupParams p) {
  __shared__ int32_t block_cnt[kMaxDepth][kWave];
  if (threadIdx.x < kMaxDepth * kWave) (&block_cnt[0][0])[threadIdx.x] = 0;
  __syncthreads();
  const int lane = lane_id();
  int mine[kMaxDepth] = {0, 0, 0, 0};
  const int64_t stride = (int64_t)gridDim.x * kGroupThreads;
  const int64_t rounds = ((int64_t)p.T + stride - 1) / stride;   // same for every lane: ballots stay convergent
  for (int64_t it = 0; it < rounds; ++it) {
    const int64_t t = it * stride + (int64_t)blockIdx.x * kGroupThreads + threadIdx.x;
    uint64_t rm = 0;
    if (t < p.T) {
      const int32_t *tok = p.ids + t * p.K;
      for (int k = 0; k < p.K; ++k) {
        const int g = rank_of(p.expert_to_rank, p.E, p.G, tok[k]);
        if (g >= 0) rm |= 1ull << g;
        else if (g == -1) flag(p.status, HM_ERR_BAD_ID);
      }
    }
    for (int l = 0; l < p.depth; ++l) {
      const int per = p.G / p.groups[l];
      const uint64_t field = per >= 64 ? ~0ull : ((1ull << per) - 1ull);
      for (int j = 0; j < p.groups[l]; ++j) {
        const uint64_t b = __ballot(((rm >> (j * per)) & field) != 0);
        if (lane == j) mine[l] += __popcll(b);
      }
    }
  }
  for (int l = 0; l < p.depth; ++l)
    if (lane < p.groups[l] && mine[l]) atomicAdd(&block_cnt[l][lane], mine[l]);
  __syncthreads();
  if (threadIdx.x < kMaxDepth * kWave) {
    const int l = threadIdx.x / kWave, j = threadIdx.x % kWave;
    if (l < p.depth && j < p.groups[l] && block_cnt[l][j]) atomicAdd(&p.counts[l * kWave + j], block_cnt[l][j]);
  }
}

struct TimeParams {
  int32_t D, G;
  int32_t U[kMaxDepth];
  double M, v;
  double alpha_inter[kMaxDepth], beta_inter[kMaxDepth], alpha_intra[kMaxDepth], beta_intra[kMaxDepth];
  const int32_t *p_inter, *p_intra;
  double *times;
  int32_t *best;
};

__device__ __forceinline__ int wave_max(int v) {
  for (int off = 32; off > 0; off >>= 1) v = max(v, __shfl_xor(v, off, kWave));
  return v;
}

// One wave: lane j holds entry j of each count vector; the maxima are wave reductions, the few
// fp64 operations run on lane 0 in the order the model is written (no contraction).
__global__ __launch_bounds__(kWave) void alltoall_times_kernel(TimeParams p) {
#pragma clang fp contract(off)
  const int lane = lane_id();
  double max_inter[kMaxDepth], max_intra[kMaxDepth];
  for (int l = 0; l < p.D; ++l) {
    const int vi = (l >= 1 && lane < p.U[l]) ? p.p_inter[l * kWave + lane] : 0;
    const int va = lane < p.G ? p.p_intra[l * kWave + lane] : 0;
    max_inter[l] = (double)max(wave_max(vi), 0);
    max_intra[l] = (double)max(wave_max(va), 0);
  }
  if (lane != 0) return;
  double t[kMaxDepth];
  for (int d = 1; d <= p.D; ++d) {
    double acc = 0.0;
    for (int i = 1; i <= d - 1; ++i) {
      const double n = (double)(p.U[i] / p.U[i - 1]) * max_inter[i] * p.M * p.v;
      acc = acc + (p.alpha_inter[i] + n * p.beta_inter[i]);
    }
    const double n = (double)(p.G / p.U[d - 1]) * max_intra[d - 1] * p.M * p.v;
    acc = acc + (p.alpha_intra[d - 1] + n * p.beta_intra[d - 1]);
    t[d - 1] = acc;
    p.times[d - 1] = acc;
  }
  int arg = 1;
  if (p.D > 1) {
    arg = 2;
    for (int d = 3; d <= p.D; ++d)
      if (t[d - 1] < t[arg - 1]) arg = d;
    if (t[0] < t[arg - 1]) arg = 1;
  }
  *p.best = arg;
}

}  // namespace hm

extern "C" hm_status hm_group_counts(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K,
                                     int32_t E, int32_t G, int32_t depth, const int32_t *groups, int32_t *counts,
                                     int32_t *status, void *hip_stream) {
  HM_ENTRY_SCOPE;
  using namespace hm;
  if (!expert_to_rank || !groups || !counts) return HM_ERR_NULL;
  hm_status st = hm_check_tk(T, K);
  if (st != HM_OK) return st;
  if (E < 1) return HM_ERR_SHAPE;
  if (T > 0 && !topk_ids) return HM_ERR_NULL;
  if (G < 1 || G > 64 || depth < 1 || depth > kMaxDepth) return HM_ERR_TOPOLOGY;
  GroupParams p;
  for (int l = 0; l < kMaxDepth; ++l) p.groups[l] = 1;
  for (int l = 0; l < depth; ++l) {
    if (groups[l] < 1 || groups[l] > G || G % groups[l] != 0) return HM_ERR_TOPOLOGY;
    p.groups[l] = groups[l];
  }
  p.ids = topk_ids;
  p.expert_to_rank = expert_to_rank;
  p.T = T;
  p.K = K;
  p.E = E;
  p.G = G;
  p.depth = depth;
  p.counts = counts;
  p.status = status;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(group_clear_kernel, dim3(1), dim3(kGroupThreads), 0, stream, p);
  if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  if (T == 0) return HM_OK;
  int64_t blocks = ((int64_t)T + kGroupThreads - 1) / kGroupThreads;
  if (blocks > 1024) blocks = 1024;
  hipLaunchKernelGGL(group_count_kernel, dim3((unsigned)blocks), dim3(kGroupThreads), 0, stream, p);
  return hm_launch_status();
}

extern "C" hm_status hm_alltoall_times(int32_t D, const int32_t *U, int32_t G, double M, double v,
                                       const int32_t *p_inter, const int32_t *p_intra, const double *alpha_inter,
                                       const double *beta_inter, const double *alpha_intra, const double *beta_intra,
                                       double *times, int32_t *best, void *hip_stream) {
  HM_ENTRY_SCOPE;
  using namespace hm;
  if (!U || !p_inter || !p_intra || !alpha_inter || !beta_inter || !alpha_intra || !beta_intra || !times || !best)
    return HM_ERR_NULL;
  if (D < 1 || D > kMaxDepth || G < 1 || G > 64 || U[0] != 1) return HM_ERR_TOPOLOGY;
  for (int i = 1; i < D; ++i)
    if (U[i] < U[i - 1] || U[i] > G || U[i] % U[i - 1] != 0 || G % U[i] != 0) return HM_ERR_TOPOLOGY;
  TimeParams p;
  p.D = D;
  p.G = G;
  p.M = M;
  p.v = v;
  for (int l = 0; l < kMaxDepth; ++l) {
    const bool in = l < D;
    p.U[l] = in ? U[l] : 1;
    p.alpha_inter[l] = in ? alpha_inter[l] : 0.0;
    p.beta_inter[l] = in ? beta_inter[l] : 0.0;
    p.alpha_intra[l] = in ? alpha_intra[l] : 0.0;
    p.beta_intra[l] = in ? beta_intra[l] : 0.0;
  }
  p.p_inter = p_inter;
  p.p_intra = p_intra;
  p.times = times;
  p.best = best;
  hipLaunchKernelGGL(alltoall_times_kernel, dim3(1), dim3(kWave), 0, (hipStream_t)hip_stream, p);
  return hm_launch_status();
}
