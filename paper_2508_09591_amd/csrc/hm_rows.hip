// Row-streaming kernels: hm_dispatch_pack, hm_combine, hm_combine_transpose.
//
// All three are HBM-bound and token-centric: a wave owns (token, segment of the row), reads the
// token-side data once and touches each of the token's distinct packed rows once, which is the
// algorithmic minimum of (1 + c) rows of traffic per token (c = packed rows per token).  The
// token's row list is wave-uniform: lanes 0..K-1 fetch slot_row[t,:], a ballot marks the rows to
// visit and readlane broadcasts each row index into a scalar register, so every global access
// is a base + lane*16 B coalesced stream of 16-byte vectors.
//
// Segments are 64 consecutive 16-byte vectors (1 KiB, one vector per lane).  Work items this
// small matter on MI355X: a kernel here lasts well under 100 us on the DeepSeek-V3 shape, so with
// multi-KiB items the last round of waves leaves most of the chip idle.  Every row-sized stream
// is read and written with non-temporal accesses: rows are touched once per kernel, and output
// lines left dirty in the caches were measured to slow the next kernel down by about 10 %.
//
// Waves per CU are capped on purpose.  With every wave slot filled, a kernel that writes (or
// reads) seven or eight 1 KiB pieces per wave has several hundred KiB per CU queued at the
// memory system, and the rate drops (a flat 1-read + 7-write stream: 64 % of peak with 32 waves
// per CU, 78 % with 8); with too few waves the index lookups are no longer hidden.  The cap is
// set with an unused dynamic LDS allocation: dispatch and the fp32 transpose run 24 waves per CU
// (-5 % on the 64 Ki-token layer at node level, -9 % at rank level, neutral elsewhere; the bf16
// transpose does more arithmetic per byte and is faster uncapped); combine keeps about 128 KiB
// of row loads in flight per CU (32 waves up to four rows per token, 16 at eight).
//
// Combine has two forms.  With the caller's weights (topk_weights != NULL) every wave merges the
// K slots of its token itself (2K readlanes) and handles 4 KiB of the row, four rows in flight.
// With the plan's merged weights (topk_weights == NULL) the first slot of each row is the one
// slot_keep marks and its weight is one gathered load from row_weight, so the prologue is short
// enough for 1 KiB segments with all of a token's rows (up to eight) in flight: 3-9 % faster.
// Tokens with about one row each (the local-expert stage of a receiver) keep 4 KiB segments, two
// rows in flight: a 1 KiB segment would be mostly prologue there (0.36 vs 0.28 ms on that stage).
#include "hm_device.h"

#include <atomic>

namespace hm {

constexpr int kElemThreads = 256;     // element-wise fallback kernels
constexpr int kCopyThreads = 128;     // dispatch / transpose: two waves per workgroup ...
constexpr int kCopyWavesPerCu = 24;   // ... and this many waves resident per CU (dispatch, fp32 transpose)
constexpr int kCombineThreads = 256;
constexpr int kCombineVecs = 4;       // combine with the caller's weights: 16-byte vectors per lane (4 KiB segments),
constexpr int kCombineRows = 4;       //   rows whose loads are in flight together
constexpr int kCombineRowsFew = 2;    //   ... or two, when the tokens are known to have fewer than two rows
constexpr int kCombineRowsPlan = 8;   // combine with the plan's weights, two rows per token or more: 1 KiB segments,
                                      //   up to eight rows in flight
constexpr int kCombineBytesInFlight = 128 * 1024;   // per CU, what the cap on resident waves aims at

struct RowParams {
  int32_t T, K;
  int32_t nvec;   // 16-byte vectors per row
  int32_t nseg;   // segments per row
  int64_t nunits; // T * nseg
  const int32_t *slot_row;
  const uint8_t *slot_keep;
  int32_t *status;
};

// Wave-uniform (token, segment) of this wave, or false when past the end.
template <int BLOCK>
__device__ __forceinline__ bool unit_of_wave(const RowParams &p, int &t, int &seg) {
  const int64_t unit = (int64_t)blockIdx.x * (BLOCK / kWave) + (threadIdx.x >> 6);
  if (unit >= p.nunits) return false;
  t = (int)(unit / p.nseg);
  seg = (int)(unit - (int64_t)t * p.nseg);
  return true;
}

// ---------------------------------------------------------------------------------------------
// dispatch: packed[slot_row[t,k], :] = x[t, :] for kept slots
// ---------------------------------------------------------------------------------------------
__global__ __launch_bounds__(kCopyThreads) void dispatch_rows_kernel(RowParams p, const u32x4 *__restrict__ x,
                                                                     u32x4 *__restrict__ packed, int64_t packed_rows) {
  int t, seg;
  if (!unit_of_wave<kCopyThreads>(p, t, seg)) return;
  const int lane = lane_id();
  const int v = seg * kWave + lane;
  const bool in_row = v < p.nvec;
  u32x4 r = {0u, 0u, 0u, 0u};
  if (in_row) r = x[(int64_t)t * p.nvec + v];   // does not wait for the row list below
  int my_row = -1;
  if (lane < p.K) {
    const int64_t s = (int64_t)t * p.K + lane;
    const int row = p.slot_row[s];
    if (p.slot_keep[s] && row >= 0) {
      if (row < packed_rows) my_row = row;
      else if (seg == 0) flag(p.status, HM_ERR_CAPACITY);
    }
  }
  uint64_t todo = __ballot(my_row >= 0);
  while (todo) {
    const int k = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int row = read_lane(my_row, k);
    if (in_row) store_stream(packed + (int64_t)row * p.nvec + v, r);
  }
}

// Any H / any alignment: one thread per (token, element), 2-byte accesses.
__global__ __launch_bounds__(kElemThreads) void dispatch_elems_kernel(RowParams p, int32_t H, const uint16_t *__restrict__ x,
                                                                     uint16_t *__restrict__ packed, int64_t packed_rows) {
  const int64_t i = (int64_t)blockIdx.x * kElemThreads + threadIdx.x;
  if (i >= (int64_t)p.T * H) return;
  const int t = (int)(i / H), j = (int)(i - (int64_t)t * H);
  const uint16_t v = x[i];
  for (int k = 0; k < p.K; ++k) {
    const int64_t s = (int64_t)t * p.K + k;
    const int row = p.slot_row[s];
    if (!p.slot_keep[s] || row < 0) continue;
    if (row < packed_rows) packed[(int64_t)row * H + j] = v;
    else if (j == 0) flag(p.status, HM_ERR_CAPACITY);
  }
}

// ---------------------------------------------------------------------------------------------
// combine: out[t,:] = bf16( sum over the token's distinct rows of (sum of their slots' weights) * y[row,:] )
// ---------------------------------------------------------------------------------------------
// Lane k < K holds slot k of the token.  On return `agg` is the fp32 sum, in ascending k, of the
// weights of all slots that share lane k's row, and the returned mask has bit k set for the
// lowest slot of each distinct valid row.
__device__ __forceinline__ uint64_t merge_slots(int K, int my_row, float my_w, float &agg) {
  const int lane = lane_id();
  agg = 0.0f;
  bool first = my_row >= 0;
  for (int k1 = 0; k1 < K; ++k1) {
    const int r1 = read_lane(my_row, k1);
    const float w1 = read_lane(my_w, k1);
    if (r1 == my_row && my_row >= 0) {
      agg = agg + w1;
      if (k1 < lane) first = false;
    }
  }
  return __ballot(first);
}

// Element type of a row as the combine kernels see it: how many values a 16-byte vector holds,
// how they enter the fp32 fma chain and how the fp32 sums are stored.
struct RowBf16 {
  typedef uint16_t elem;
  static constexpr int kPerVec = 8;
  static __device__ __forceinline__ void fma_into(float *acc, float a, u32x4 r) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      acc[2 * e] = __builtin_fmaf(a, bf16_lo(r[e]), acc[2 * e]);
      acc[2 * e + 1] = __builtin_fmaf(a, bf16_hi(r[e]), acc[2 * e + 1]);
    }
  }
  static __device__ __forceinline__ u32x4 pack(const float *acc) {
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = pack_bf16x2(acc[2 * e], acc[2 * e + 1]);
    return o;
  }
  static __device__ __forceinline__ float widen(elem v) { return __builtin_bit_cast(float, (uint32_t)v << 16); }
  static __device__ __forceinline__ elem narrow(float f) { return (elem)f32_to_bf16(f); }
  // bf16(a * g) with ONE rounding.  The fp32 product p is already rounded; a second rounding to
  // bf16 differs from the exact one only when p sits exactly on a bf16 tie, and there the sign of
  // the product's rounding error e = fma(a, g, -p) says on which side the true value lies.  e is
  // exact as long as it does not underflow, i.e. for |a * g| >= 2^-102 or so; for smaller products
  // (gradients of that size do not occur in practice) a tie may be broken to even instead.
  static __device__ __forceinline__ uint32_t scale1(float a, float g) {
    const float p = a * g;
    const float e = __builtin_fmaf(a, g, -p);
    const uint32_t u = __builtin_bit_cast(uint32_t, p);
    if ((u & 0x7FFFFFFFu) > 0x7F800000u) return 0x7FC0u;   // NaN
    // round to nearest: add 0x7FFF plus a tie bit -- the kept lsb (ties to even) in general, but on
    // an exact tie of p with e != 0 the side the true product lies on
    const bool tie = (u & 0xFFFFu) == 0x8000u && e != 0.0f;
    const uint32_t away = ((__builtin_bit_cast(uint32_t, e) ^ u) >> 31) ^ 1u;   // e and p have the same sign
    const uint32_t tie_bit = tie ? away : ((u >> 16) & 1u);
    return (u + 0x7FFFu + tie_bit) >> 16;
  }
  static __device__ __forceinline__ elem scale(float a, elem g) { return (elem)scale1(a, widen(g)); }
  // Eight at once: the common path rounds the fp32 products to nearest even (add 0x7FFF plus the
  // kept lsb; the upper halves of two such sums are one output word, picked by a byte permute) and
  // only notes whether any product is a NaN or sits on a bf16 tie (1 in 65536); the exact
  // treatment runs for those vectors alone.
  static __device__ __forceinline__ u32x4 scale(float a, u32x4 r) {
    float g[8];
    uint32_t sum[8];
    bool special = false;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t w = r[e];
      g[2 * e] = bf16_lo(w);
      g[2 * e + 1] = bf16_hi(w);
    }
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const float p = a * g[i];
      const uint32_t u = __builtin_bit_cast(uint32_t, p);
      sum[i] = u + 0x7FFFu + ((u >> 16) & 1u);
      special = special || (u & 0xFFFFu) == 0x8000u || __builtin_isnan(p);
    }
    u32x4 o;
    if (__builtin_expect(special, 0)) {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = scale1(a, g[2 * e]) | (scale1(a, g[2 * e + 1]) << 16);
    } else {
#pragma unroll
      for (int e = 0; e < 4; ++e) o[e] = __builtin_amdgcn_perm(sum[2 * e + 1], sum[2 * e], 0x07060302u);
    }
    return o;
  }
};
struct RowF32 {
  typedef float elem;
  static constexpr int kPerVec = 4;
  static __device__ __forceinline__ void fma_into(float *acc, float a, u32x4 r) {
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t w = r[e];   // a copy first: a bit cast applied to the vector element itself reads element 0
      acc[e] = __builtin_fmaf(a, __builtin_bit_cast(float, w), acc[e]);
    }
  }
  static __device__ __forceinline__ u32x4 pack(const float *acc) {
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) o[e] = __builtin_bit_cast(uint32_t, acc[e]);
    return o;
  }
  static __device__ __forceinline__ float widen(elem v) { return v; }
  static __device__ __forceinline__ elem narrow(float f) { return f; }
  static __device__ __forceinline__ elem scale(float a, elem g) { return a * g; }   // one IEEE multiply
  static __device__ __forceinline__ u32x4 scale(float a, u32x4 r) {
    u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      const uint32_t w = r[e];
      o[e] = __builtin_bit_cast(uint32_t, a * __builtin_bit_cast(float, w));
    }
    return o;
  }
};

// MIX = false: hm_combine.  MIX = true: hm_combine_mix, the sum times the reciprocal of the sum of
// the merged weights (added in ascending k of each row's first slot); zero for a row without a
// valid slot.  (A true division per element made the kernel ALU-bound: 8 divisions per 16 bytes.)
template <bool MIX, int U, int R, typename ROW>
__global__ __launch_bounds__(kCombineThreads) void combine_rows_kernel(RowParams p, const u32x4 *__restrict__ y,
                                                                       int64_t y_rows, const float *__restrict__ topk_weights,
                                                                       u32x4 *__restrict__ out) {
  int t, seg;
  if (!unit_of_wave<kCombineThreads>(p, t, seg)) return;
  const int lane = lane_id();
  int my_row = -1;
  float my_w = 0.0f;
  if (lane < p.K) {
    const int64_t s = (int64_t)t * p.K + lane;
    const int row = p.slot_row[s];
    if (row >= 0) {
      if (row < y_rows) {
        my_row = row;
        my_w = topk_weights[s];
      } else if (seg == 0) {
        flag(p.status, HM_ERR_CAPACITY);
      }
    }
  }
  float agg;
  uint64_t todo = merge_slots(p.K, my_row, my_w, agg);
  float inv_wsum = 0.0f;   // MIX: one division per wave, then a multiply per element
  if (MIX) {
    float wsum = 0.0f;
    for (uint64_t m = todo; m; m &= m - 1) wsum = wsum + read_lane(agg, __builtin_ctzll(m));
    inv_wsum = wsum != 0.0f ? 1.0f / wsum : 0.0f;
  }

  const int v0 = seg * (kWave * U) + lane;   // this lane's vectors: v0, v0+64, ...
  constexpr int E = ROW::kPerVec;
  float acc[U][E];
#pragma unroll
  for (int i = 0; i < U; ++i)
#pragma unroll
    for (int e = 0; e < E; ++e) acc[i][e] = 0.0f;

  while (todo) {
    // issue the loads of up to R rows, then consume them in the same (ascending k) order
    u32x4 r[R][U];
    float a[R];
    bool have[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      have[j] = todo != 0;
      a[j] = 0.0f;
#pragma unroll
      for (int i = 0; i < U; ++i) r[j][i] = (u32x4){0u, 0u, 0u, 0u};
      if (have[j]) {
        const int k = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int row = read_lane(my_row, k);
        a[j] = read_lane(agg, k);
        const u32x4 *src = y + (int64_t)row * p.nvec;
#pragma unroll
        for (int i = 0; i < U; ++i)
          if (v0 + i * kWave < p.nvec) r[j][i] = load_stream(src + v0 + i * kWave);
      }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
      if (have[j]) {
#pragma unroll
        for (int i = 0; i < U; ++i) ROW::fma_into(acc[i], a[j], r[j][i]);
      }
    }
  }
  u32x4 *dst = out + (int64_t)t * p.nvec;
#pragma unroll
  for (int i = 0; i < U; ++i) {
    if (v0 + i * kWave < p.nvec) {
      if (MIX) {
#pragma unroll
        for (int e = 0; e < E; ++e) acc[i][e] = acc[i][e] * inv_wsum;
      }
      store_stream(dst + v0 + i * kWave, ROW::pack(acc[i]));
    }
  }
}

// The same sum with the weights the plan merged: lane k < K holds slot k; the slot slot_keep marks
// is the first of its row, and row_weight[row] is the fp32 sum, in ascending k, of the weights of
// the slots that share the row -- the number merge_slots computes.  A wave owns U KiB of the row;
// the loads of up to R rows are issued before the first fma.
template <bool MIX, int U, int R, typename ROW>
__global__ __launch_bounds__(kCombineThreads) void combine_plan_rows_kernel(RowParams p, const u32x4 *__restrict__ y,
                                                                            int64_t y_rows,
                                                                            const float *__restrict__ row_weight,
                                                                            u32x4 *__restrict__ out) {
  int t, seg;
  if (!unit_of_wave<kCombineThreads>(p, t, seg)) return;
  const int lane = lane_id();
  int my_row = -1;
  float agg = 0.0f;
  if (lane < p.K) {
    const int64_t s = (int64_t)t * p.K + lane;
    const int row = p.slot_row[s];
    if (p.slot_keep[s] && row >= 0) {
      if (row < y_rows) my_row = row;
      else if (seg == 0) flag(p.status, HM_ERR_CAPACITY);
    }
  }
  uint64_t todo = __ballot(my_row >= 0);
  if (my_row >= 0) agg = row_weight[my_row];   // in flight together with the first rows
  float inv_wsum = 0.0f;
  if (MIX) {
    float wsum = 0.0f;
    for (uint64_t m = todo; m; m &= m - 1) wsum = wsum + read_lane(agg, __builtin_ctzll(m));
    inv_wsum = wsum != 0.0f ? 1.0f / wsum : 0.0f;
  }
  const int v0 = seg * (kWave * U) + lane;   // this lane's vectors: v0, v0+64, ...
  constexpr int E = ROW::kPerVec;
  float acc[U][E];
#pragma unroll
  for (int i = 0; i < U; ++i)
#pragma unroll
    for (int e = 0; e < E; ++e) acc[i][e] = 0.0f;
  while (todo) {
    u32x4 r[R][U];
    float a[R];
    bool have[R];
#pragma unroll
    for (int j = 0; j < R; ++j) {
      have[j] = todo != 0;
      a[j] = 0.0f;
#pragma unroll
      for (int i = 0; i < U; ++i) r[j][i] = (u32x4){0u, 0u, 0u, 0u};
      if (have[j]) {
        const int k = __builtin_ctzll(todo);
        todo &= todo - 1;
        const int row = read_lane(my_row, k);
        a[j] = read_lane(agg, k);
        const u32x4 *src = y + (int64_t)row * p.nvec;
#pragma unroll
        for (int i = 0; i < U; ++i)
          if (v0 + i * kWave < p.nvec) r[j][i] = load_stream(src + v0 + i * kWave);
      }
    }
#pragma unroll
    for (int j = 0; j < R; ++j) {
      if (have[j]) {
#pragma unroll
        for (int i = 0; i < U; ++i) ROW::fma_into(acc[i], a[j], r[j][i]);
      }
    }
  }
  u32x4 *dst = out + (int64_t)t * p.nvec;
#pragma unroll
  for (int i = 0; i < U; ++i) {
    if (v0 + i * kWave < p.nvec) {
      if (MIX) {
#pragma unroll
        for (int e = 0; e < E; ++e) acc[i][e] = acc[i][e] * inv_wsum;
      }
      store_stream(dst + v0 + i * kWave, ROW::pack(acc[i]));
    }
  }
}

// Any H / alignment: one thread per (token, element); same merge order and the same fma chain
// as the vector kernel, so both give identical bits.
template <bool MIX, typename ROW>
__global__ __launch_bounds__(kElemThreads) void combine_elems_kernel(RowParams p, int32_t H,
                                                                    const typename ROW::elem *__restrict__ y,
                                                                    int64_t y_rows, const float *__restrict__ topk_weights,
                                                                    const float *__restrict__ row_weight,
                                                                    typename ROW::elem *__restrict__ out) {
  const int64_t i = (int64_t)blockIdx.x * kElemThreads + threadIdx.x;
  if (i >= (int64_t)p.T * H) return;
  const int t = (int)(i / H), j = (int)(i - (int64_t)t * H);
  const int32_t *rows = p.slot_row + (int64_t)t * p.K;
  float acc = 0.0f, wsum = 0.0f;
  for (int k = 0; k < p.K; ++k) {
    const int row = rows[k];
    if (row < 0) continue;
    bool first = true;
    for (int k1 = 0; k1 < k; ++k1) first = first && rows[k1] != row;
    if (!first) continue;
    if (row >= y_rows) {
      if (j == 0) flag(p.status, HM_ERR_CAPACITY);
      continue;
    }
    float agg = 0.0f;
    if (row_weight) {   // the plan's merged weight: the same additions in the same order
      agg = row_weight[row];
    } else {
      const float *w = topk_weights + (int64_t)t * p.K;
      for (int k1 = 0; k1 < p.K; ++k1)
        if (rows[k1] == row) agg = agg + w[k1];
    }
    acc = __builtin_fmaf(agg, ROW::widen(y[(int64_t)row * H + j]), acc);
    wsum = wsum + agg;
  }
  if (MIX) acc = acc * (wsum != 0.0f ? 1.0f / wsum : 0.0f);   // same reciprocal-multiply as the vector kernel
  out[i] = ROW::narrow(acc);
}

// ---------------------------------------------------------------------------------------------
// transpose: gy[slot_row[t,k], :] = row_weight[row] * gout[t, :] for kept slots (fp32)
// ---------------------------------------------------------------------------------------------
template <typename ROW>
__global__ __launch_bounds__(kCopyThreads) void transpose_rows_kernel(RowParams p, const u32x4 *__restrict__ gout,
                                                                      const float *__restrict__ row_weight,
                                                                      int64_t weight_rows, u32x4 *__restrict__ gy,
                                                                      int64_t gy_rows) {
  int t, seg;
  if (!unit_of_wave<kCopyThreads>(p, t, seg)) return;
  const int lane = lane_id();
  const int v = seg * kWave + lane;
  const bool in_row = v < p.nvec;
  u32x4 r = {0u, 0u, 0u, 0u};
  if (in_row) r = gout[(int64_t)t * p.nvec + v];
  int my_row = -1;
  float my_w = 0.0f;
  if (lane < p.K) {
    const int64_t s = (int64_t)t * p.K + lane;
    const int row = p.slot_row[s];
    if (p.slot_keep[s] && row >= 0) {
      if (row < gy_rows && row < weight_rows) {
        my_row = row;
        my_w = row_weight[row];
      } else if (seg == 0) {
        flag(p.status, HM_ERR_CAPACITY);
      }
    }
  }
  uint64_t todo = __ballot(my_row >= 0);
  while (todo) {
    const int k = __builtin_ctzll(todo);
    todo &= todo - 1;
    const int row = read_lane(my_row, k);
    const float a = read_lane(my_w, k);
    if (in_row) store_stream(gy + (int64_t)row * p.nvec + v, ROW::scale(a, r));
  }
}

template <typename ROW>
__global__ __launch_bounds__(kElemThreads) void transpose_elems_kernel(RowParams p, int32_t H,
                                                                      const typename ROW::elem *__restrict__ gout,
                                                                      const float *__restrict__ row_weight,
                                                                      int64_t weight_rows, typename ROW::elem *__restrict__ gy,
                                                                      int64_t gy_rows) {
  const int64_t i = (int64_t)blockIdx.x * kElemThreads + threadIdx.x;
  if (i >= (int64_t)p.T * H) return;
  const int t = (int)(i / H), j = (int)(i - (int64_t)t * H);
  const typename ROW::elem g = gout[i];
  for (int k = 0; k < p.K; ++k) {
    const int64_t s = (int64_t)t * p.K + k;
    const int row = p.slot_row[s];
    if (!p.slot_keep[s] || row < 0) continue;
    if (row < gy_rows && row < weight_rows) gy[(int64_t)row * H + j] = ROW::scale(row_weight[row], g);
    else if (j == 0) flag(p.status, HM_ERR_CAPACITY);
  }
}

static inline bool aligned16(const void *p) { return ((uintptr_t)p & 15u) == 0; }

// Fills nvec / nseg / nunits for rows of `nvec` 16-byte vectors and sizes the grid.
static inline bool grid_for_units(RowParams &p, int nvec, int vecs_per_lane, int block, dim3 &grid) {
  p.nvec = nvec;
  p.nseg = (nvec + kWave * vecs_per_lane - 1) / (kWave * vecs_per_lane);
  p.nunits = (int64_t)p.T * p.nseg;
  const int waves = block / kWave;
  const int64_t blocks = (p.nunits + waves - 1) / waves;
  if (blocks > 2147483647LL) return false;
  grid = dim3((unsigned)blocks);
  return true;
}

static inline bool grid_for_elems(RowParams &p, int64_t n, dim3 &grid) {
  p.nvec = p.nseg = 0;
  p.nunits = 0;
  const int64_t blocks = (n + kElemThreads - 1) / kElemThreads;
  if (blocks > 2147483647LL) return false;
  grid = dim3((unsigned)blocks);
  return true;
}

// Bytes of (unused) dynamic LDS per workgroup that leave room for `waves_per_cu` waves of
// `block`-thread workgroups on a CU; 0 = no cap.  The CU's LDS size is read from the device once.
static inline int lds_per_cu() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 0;
  int v = cached[dev].load(std::memory_order_relaxed);
  if (v == 0) {
    int bytes = 0;
    if (hipDeviceGetAttribute(&bytes, hipDeviceAttributeMaxSharedMemoryPerMultiprocessor, dev) != hipSuccess) bytes = 0;
    v = bytes >= 65536 ? bytes : -1;
    cached[dev].store(v, std::memory_order_relaxed);
  }
  return v > 0 ? v : 0;
}
static inline unsigned lds_cap_bytes(int waves_per_cu, int block) {
  const int per_cu = lds_per_cu();
  const int blocks = waves_per_cu / (block / kWave);
  if (per_cu == 0 || blocks < 1 || waves_per_cu >= 32) return 0;
  const int bytes = (per_cu / blocks) & ~511;
  return bytes > 65536 ? 65536u : (unsigned)bytes;
}

// Rows a token is expected to own: from the caller's (or hm_plan_status's) row count if there is
// one, else from the bound hm_plan left in the struct, else unknown (0).
static inline double rows_per_token(const hm_plan_out *plan, int32_t T) {
  if (plan->expected_rows > 0 && T > 0) return (double)plan->expected_rows / (double)T;
  if (plan->max_rows_per_token > 0) return (double)plan->max_rows_per_token;
  return 0.0;
}

// Launch shape of the combine kernels: 16-byte vectors per lane, rows in flight per wave, and the
// cap on resident waves per CU (32 = none).  Kept in one place so that the launcher and
// hm_combine_launch_shape agree.
struct CombineShape {
  int vecs, rows, waves_per_cu;
};
static inline CombineShape combine_shape(const hm_plan_out *plan, int32_t T, bool weights_from_plan) {
  CombineShape sh;
  if (!weights_from_plan) {
    sh.vecs = kCombineVecs;
    sh.rows = kCombineRows;
    sh.waves_per_cu = 32;
    return sh;
  }
  const double c = rows_per_token(plan, T);
  sh.waves_per_cu = 32;
  if (c <= 0.0) {   // unknown (a hop-table plan that was never synchronised): such plans have few rows per token
    sh.vecs = kCombineVecs;
    sh.rows = kCombineRows;
    return sh;
  }
  if (c < 2.0) {    // about one row per token: 1 KiB segments would be mostly prologue
    sh.vecs = kCombineVecs;
    sh.rows = kCombineRowsFew;
    return sh;
  }
  sh.vecs = 1;
  sh.rows = kCombineRowsPlan;
  int waves = 32;
  if (c > 4.0) {   // c KiB of loads per wave: keep about kCombineBytesInFlight per CU
    waves = (int)((double)kCombineBytesInFlight / (c * 1024.0));
    waves &= ~3;   // whole workgroups of four waves
    if (waves < 16) waves = 16;
    if (waves > 32) waves = 32;
  }
  sh.waves_per_cu = waves;
  return sh;
}

}  // namespace hm

static hm_status check_rows_args(int32_t T, int32_t K, int32_t H, const hm_plan_out *plan, bool need_keep) {
  if (!plan) return HM_ERR_NULL;
  if (!plan->slot_row || !plan->status || (need_keep && !plan->slot_keep)) return HM_ERR_NULL;
  hm_status st = hm_check_tk(T, K);
  if (st != HM_OK) return st;
  if (H < 1) return HM_ERR_SHAPE;
  return HM_OK;
}

extern "C" hm_status hm_dispatch_pack(const void *x_bf16, int32_t T, int32_t K, int32_t H, const hm_plan_out *plan,
                                      void *packed_bf16, int64_t packed_rows, void *hip_stream) {
  HM_ENTRY_SCOPE;
  using namespace hm;
  hm_status st = check_rows_args(T, K, H, plan, true);
  if (st != HM_OK) return st;
  if (packed_rows < 0) return HM_ERR_SHAPE;
  if (T == 0) return HM_OK;
  if (!x_bf16 || (!packed_bf16 && packed_rows > 0)) return HM_ERR_NULL;
  hipStream_t stream = (hipStream_t)hip_stream;
  RowParams p;
  p.T = T;
  p.K = K;
  p.slot_row = plan->slot_row;
  p.slot_keep = plan->slot_keep;
  p.status = plan->status;
  dim3 grid;
  if (H % 8 == 0 && aligned16(x_bf16) && aligned16(packed_bf16)) {
    if (!grid_for_units(p, H / 8, 1, kCopyThreads, grid)) return HM_ERR_SHAPE;
    hipLaunchKernelGGL(dispatch_rows_kernel, grid, dim3(kCopyThreads), lds_cap_bytes(kCopyWavesPerCu, kCopyThreads),
                       stream, p, (const u32x4 *)x_bf16, (u32x4 *)packed_bf16, packed_rows);
  } else {
    if (!grid_for_elems(p, (int64_t)T * H, grid)) return HM_ERR_SHAPE;
    hipLaunchKernelGGL(dispatch_elems_kernel, grid, dim3(kElemThreads), 0, stream, p, H, (const uint16_t *)x_bf16,
                       (uint16_t *)packed_bf16, packed_rows);
  }
  return hm_launch_status();
}

template <bool MIX, typename ROW>
static hm_status launch_combine(const void *y, int64_t y_rows, const float *topk_weights, int32_t T, int32_t K,
                                int32_t H, const hm_plan_out *plan, void *out, void *hip_stream) {
  using namespace hm;
  typedef typename ROW::elem elem;
  const bool from_plan = topk_weights == nullptr;   // merged weights and first-slot marks of the plan
  hm_status st = check_rows_args(T, K, H, plan, from_plan);
  if (st != HM_OK) return st;
  if (from_plan && !plan->row_weight) return HM_ERR_NULL;
  if (y_rows < 0 || (from_plan && plan->row_capacity < 0)) return HM_ERR_SHAPE;
  if (T == 0) return HM_OK;
  if (!out || (!y && y_rows > 0)) return HM_ERR_NULL;
  hipStream_t stream = (hipStream_t)hip_stream;
  RowParams p;
  p.T = T;
  p.K = K;
  p.slot_row = plan->slot_row;
  p.slot_keep = plan->slot_keep;
  p.status = plan->status;
  dim3 grid;
  if (H % ROW::kPerVec == 0 && aligned16(y) && aligned16(out)) {
    const int nvec = H / ROW::kPerVec;
    const CombineShape sh = combine_shape(plan, T, from_plan);
    if (!grid_for_units(p, nvec, sh.vecs, kCombineThreads, grid)) return HM_ERR_SHAPE;
    if (from_plan) {
      // rows the plan's weight array does not cover are treated like rows beyond y
      const int64_t rows = y_rows < plan->row_capacity ? y_rows : plan->row_capacity;
      if (sh.vecs == 1)
        hipLaunchKernelGGL((combine_plan_rows_kernel<MIX, 1, kCombineRowsPlan, ROW>), grid, dim3(kCombineThreads),
                           lds_cap_bytes(sh.waves_per_cu, kCombineThreads), stream, p, (const u32x4 *)y, rows,
                           plan->row_weight, (u32x4 *)out);
      else if (sh.rows == kCombineRowsFew)
        hipLaunchKernelGGL((combine_plan_rows_kernel<MIX, kCombineVecs, kCombineRowsFew, ROW>), grid, dim3(kCombineThreads), 0,
                           stream, p, (const u32x4 *)y, rows, plan->row_weight, (u32x4 *)out);
      else
        hipLaunchKernelGGL((combine_plan_rows_kernel<MIX, kCombineVecs, kCombineRows, ROW>), grid, dim3(kCombineThreads), 0,
                           stream, p, (const u32x4 *)y, rows, plan->row_weight, (u32x4 *)out);
    } else {
      hipLaunchKernelGGL((combine_rows_kernel<MIX, kCombineVecs, kCombineRows, ROW>), grid, dim3(kCombineThreads), 0,
                         stream, p, (const u32x4 *)y, y_rows, topk_weights, (u32x4 *)out);
    }
  } else {
    if (!grid_for_elems(p, (int64_t)T * H, grid)) return HM_ERR_SHAPE;
    // the element-wise kernel finds the first slot of each row itself and takes the row's merged
    // weight from the plan when the caller passed none
    hipLaunchKernelGGL((combine_elems_kernel<MIX, ROW>), grid, dim3(kElemThreads), 0, stream, p, H, (const elem *)y,
                       from_plan && plan->row_capacity < y_rows ? plan->row_capacity : y_rows, topk_weights,
                       from_plan ? plan->row_weight : nullptr, (elem *)out);
  }
  return hm_launch_status();
}

extern "C" hm_status hm_combine_launch_shape(int32_t T, int32_t K, int32_t H, const hm_plan_out *plan,
                                             int32_t weights_from_plan, int32_t *vectors_per_lane,
                                             int32_t *rows_in_flight, int32_t *waves_per_cu) {
  HM_ENTRY_SCOPE;
  hm_status st = check_rows_args(T, K, H, plan, false);
  if (st != HM_OK) return st;
  const hm::CombineShape sh = hm::combine_shape(plan, T, weights_from_plan != 0);
  if (vectors_per_lane) *vectors_per_lane = sh.vecs;
  if (rows_in_flight) *rows_in_flight = sh.rows;
  if (waves_per_cu) *waves_per_cu = sh.waves_per_cu;
  return HM_OK;
}

extern "C" hm_status hm_combine(const void *y_bf16, int64_t y_rows, const float *topk_weights, int32_t T, int32_t K,
                                int32_t H, const hm_plan_out *plan, void *out_bf16, void *hip_stream) {
  HM_ENTRY_SCOPE;
  return launch_combine<false, hm::RowBf16>(y_bf16, y_rows, topk_weights, T, K, H, plan, out_bf16, hip_stream);
}

extern "C" hm_status hm_combine_f32(const float *y, int64_t y_rows, const float *topk_weights, int32_t T, int32_t K,
                                    int32_t H, const hm_plan_out *plan, float *out, void *hip_stream) {
  HM_ENTRY_SCOPE;
  return launch_combine<false, hm::RowF32>(y, y_rows, topk_weights, T, K, H, plan, out, hip_stream);
}

extern "C" hm_status hm_combine_mix(const void *y_bf16, int64_t y_rows, const float *row_weights, int32_t T, int32_t K,
                                    int32_t H, const hm_plan_out *plan, void *out_bf16, void *hip_stream) {
  HM_ENTRY_SCOPE;
  return launch_combine<true, hm::RowBf16>(y_bf16, y_rows, row_weights, T, K, H, plan, out_bf16, hip_stream);
}

template <typename ROW>
static hm_status launch_transpose(const void *gout, int32_t T, int32_t K, int32_t H, const hm_plan_out *plan, void *gy,
                                  int64_t gy_rows, void *hip_stream) {
  using namespace hm;
  typedef typename ROW::elem elem;
  hm_status st = check_rows_args(T, K, H, plan, true);
  if (st != HM_OK) return st;
  if (!plan->row_weight) return HM_ERR_NULL;
  if (gy_rows < 0 || plan->row_capacity < 0) return HM_ERR_SHAPE;
  if (T == 0) return HM_OK;
  if (!gout || (!gy && gy_rows > 0)) return HM_ERR_NULL;
  hipStream_t stream = (hipStream_t)hip_stream;
  RowParams p;
  p.T = T;
  p.K = K;
  p.slot_row = plan->slot_row;
  p.slot_keep = plan->slot_keep;
  p.status = plan->status;
  dim3 grid;
  if (H % ROW::kPerVec == 0 && aligned16(gout) && aligned16(gy)) {
    if (!grid_for_units(p, H / ROW::kPerVec, 1, kCopyThreads, grid)) return HM_ERR_SHAPE;
    const unsigned lds = ROW::kPerVec == 4 ? lds_cap_bytes(kCopyWavesPerCu, kCopyThreads) : 0u;   // fp32 rows only
    hipLaunchKernelGGL((transpose_rows_kernel<ROW>), grid, dim3(kCopyThreads), lds, stream, p, (const u32x4 *)gout,
                       plan->row_weight, plan->row_capacity, (u32x4 *)gy, gy_rows);
  } else {
    if (!grid_for_elems(p, (int64_t)T * H, grid)) return HM_ERR_SHAPE;
    hipLaunchKernelGGL((transpose_elems_kernel<ROW>), grid, dim3(kElemThreads), 0, stream, p, H, (const elem *)gout,
                       plan->row_weight, plan->row_capacity, (elem *)gy, gy_rows);
  }
  return hm_launch_status();
}

extern "C" hm_status hm_combine_transpose(const float *gout, int32_t T, int32_t K, int32_t H, const hm_plan_out *plan,
                                          float *gy, int64_t gy_rows, void *hip_stream) {
  HM_ENTRY_SCOPE;
  return launch_transpose<hm::RowF32>(gout, T, K, H, plan, gy, gy_rows, hip_stream);
}

extern "C" hm_status hm_combine_transpose_bf16(const void *gout_bf16, int32_t T, int32_t K, int32_t H,
                                               const hm_plan_out *plan, void *gy_bf16, int64_t gy_rows, void *hip_stream) {
  HM_ENTRY_SCOPE;
  return launch_transpose<hm::RowBf16>(gout_bf16, T, K, H, plan, gy_bf16, gy_rows, hip_stream);
}
