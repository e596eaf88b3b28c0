// Hierarchical expert swap (HierMoE Section IV): the swap tensor Z and the selection of Eq.(8)-(11).
//
// Z[r][c][:] is the vector of duplicate-free per-group token counts after experts r and c trade
// places.  A swap can only change the two groups involved, and by how much follows from three
// small co-occurrence tables over the tokens:
//   L0[a]    tokens selecting a                      CG[a][g]  ... that also select something in g
//   L[a]     tokens where a is alone in its group    C[a][b]   ... that also select b
// For g_r != g_c:  Z[r][c][g_c] = base[g_c] + (L0[r] - CG[r][g_c]) - (L[c] - C[c][r])   and the same
// with r and c exchanged for g_r: no O(T K E) walk over all unselected experts, and the per-pair
// work is an embarrassingly parallel E^2 ng kernel.  The tables come from int8 matrix products on
// the matrix cores for E <= 256 (further down), from O(T K (K + ng)) atomic updates, one lane per
// routing slot, beyond that.
#include "hm_device.h"

namespace hm {

constexpr int kSwapThreads = 256;
constexpr int kSelectThreads = 256;    // Q per pair: fp64 pow-heavy, one lane per term of Eq.(8)
constexpr int kPairLanes = 4, kSelectPairs = kSelectThreads / kPairLanes;
constexpr int kFactorThreads = 1024;   // the co-occurrence pass: 16 waves share one set of LDS tables
constexpr int kSwapLds = 30720;   // most ints of LDS for L0 and every cut's L + CG (120 KiB); larger sets stay in global memory
constexpr int kSwapCopiesMax = 32;   // private copies of C: popular expert pairs would otherwise serialise on one address
constexpr int kMaxCuts = 4;       // group cuts handled by one pass over the tokens

// One pass serves up to kMaxCuts cuts of the ranks into groups: everything that does not depend on
// the cut (ids, placement lookups, which slots repeat an expert) is done once.
struct SwapParams {
  const int32_t *ids;
  const int32_t *expert_to_rank;
  int32_t T, K, E, G;
  int32_t sub;      // lanes per token in the co-occurrence pass: the power of two >= K
  int32_t ncuts;
  int32_t use_lds;  // L0 / L / CG of all cuts accumulate in LDS
  int32_t copies;   // private copies of each C
  int32_t ng[kMaxCuts], per[kMaxCuts];
  uint32_t ng_reciprocal[kMaxCuts];   // ceil(2^32 / ng), for the division by ng in swap_build_kernel (unused when ng = 1)
  uint32_t per_reciprocal[kMaxCuts];  // ceil(2^32 / per), 0 when per = 1
  int32_t build_blocks[kMaxCuts];     // column blocks of swap_build_kernel per cut
  int32_t lds_off[kMaxCuts];   // ints: where cut c's [L (E) | CG (E * ng)] starts in LDS; L0 is at 0
  int32_t *L0;                 // [E]                                  (workspace, shared by the cuts)
  int32_t *base[kMaxCuts];     // [64]                                 (workspace, per cut)
  int32_t *L[kMaxCuts];        // [E]
  int32_t *CG[kMaxCuts];       // [E][ng]
  int32_t *C[kMaxCuts];        // [copies][E][E]
  int32_t *CT[kMaxCuts];       // [E][E]   C transposed   } matrix path only: swap_build_kernel then reads
  int32_t *CGT[kMaxCuts];      // [ng][E]  CG transposed  } along rows whichever expert of a pair a lane needs
  int32_t transposed;
  int32_t *Z[kMaxCuts];
  int32_t *ws;                 // start of the workspace and its size in ints (cleared first)
  int64_t ws_ints;
  int32_t *status;
};

__global__ __launch_bounds__(kSwapThreads) void swap_clear_kernel(SwapParams p) {
  const int64_t i = (int64_t)blockIdx.x * kSwapThreads + threadIdx.x;
  if (i < p.ws_ints) p.ws[i] = 0;
  if (i == 0 && p.status) *p.status = 0;
}

// One lane per routing slot: the K slots of a token sit in a sub-group of `sub` = 2^ceil(log2 K)
// consecutive lanes (64 / sub tokens per wave) and learn about each other through shuffles, so the
// per-token work -- K expert updates, K * groups and up to K * K co-occurrence updates -- is spread
// over K lanes instead of being a serial loop of one lane.
__global__ __launch_bounds__(kFactorThreads) void swap_factors_kernel(SwapParams p) {
  extern __shared__ int32_t lds[];   // L0 and every cut's L + CG, sized by the launch
  __shared__ int32_t base_cnt[kMaxCuts][kWave];
  __shared__ uint8_t group_of[kMaxCuts][kWave];   // rank -> group under each cut
  if (p.use_lds) {
    const int used = p.lds_off[p.ncuts - 1] + p.E * (p.ng[p.ncuts - 1] + 1);
    for (int i = threadIdx.x; i < used; i += kFactorThreads) lds[i] = 0;
  }
  if (threadIdx.x < kMaxCuts * kWave) {
    const int c = threadIdx.x / kWave, r = threadIdx.x % kWave;
    base_cnt[c][r] = 0;
    group_of[c][r] = (uint8_t)(c < p.ncuts ? r / p.per[c] : 0);
  }
  __syncthreads();

  const int lane = lane_id();
  const int k = lane & (p.sub - 1);        // my slot in the token
  const int sub0 = lane & ~(p.sub - 1);    // first lane of my token's sub-group
  const int tokens_per_wave = kWave / p.sub;
  const int64_t wave = (int64_t)blockIdx.x * (kFactorThreads / kWave) + (threadIdx.x >> 6);
  const int64_t nwaves = (int64_t)gridDim.x * (kFactorThreads / kWave);
  const int64_t per_round = nwaves * tokens_per_wave;
  const int64_t rounds = ((int64_t)p.T + per_round - 1) / per_round;
  const int64_t copy_off = (int64_t)(blockIdx.x & (p.copies - 1)) * p.E * p.E;
  int my_base[kMaxCuts] = {0, 0, 0, 0};
  for (int64_t it = 0; it < rounds; ++it) {
    const int64_t t = (it * nwaves + wave) * tokens_per_wave + lane / p.sub;
    int a = -1, g = -1;   // my expert and its rank; -1 when the slot is empty, dropped or invalid
    if (t < p.T && k < p.K) {
      const int id = p.ids[t * p.K + k];
      const int r = rank_of(p.expert_to_rank, p.E, p.G, id);
      if (r == -1) flag(p.status, HM_ERR_BAD_ID);
      if (r >= 0) {
        a = id;
        g = r;
      }
    }
    // the selected experts form a set: `first` marks the first valid occurrence of each
    bool first = a >= 0;
    uint64_t gm[kMaxCuts] = {0, 0, 0, 0};   // groups the token touches, per cut
    for (int k1 = 0; k1 < p.K; ++k1) {
      const int a1 = __shfl(a, sub0 + k1, kWave);
      const int g1 = __shfl(g, sub0 + k1, kWave);
      if (k1 < k && a1 == a) first = false;
      if (g1 >= 0) {
#pragma unroll
        for (int c = 0; c < kMaxCuts; ++c)
          if (c < p.ncuts) gm[c] |= 1ull << group_of[c][g1];
      }
    }
    int in_group[kMaxCuts] = {0, 0, 0, 0};   // distinct selected experts in my expert's group
    for (int k1 = 0; k1 < p.K; ++k1) {
      const int f1 = __shfl((int)first, sub0 + k1, kWave);
      const int g1 = __shfl(g, sub0 + k1, kWave);
      if (f1 && g >= 0) {
#pragma unroll
        for (int c = 0; c < kMaxCuts; ++c)
          if (c < p.ncuts) in_group[c] += group_of[c][g1] == group_of[c][g] ? 1 : 0;
      }
    }
    bool alone[kMaxCuts];
#pragma unroll
    for (int c = 0; c < kMaxCuts; ++c) alone[c] = c < p.ncuts && first && in_group[c] == 1;
    if (first) {
      if (p.use_lds) atomicAdd(&lds[a], 1);
      else atomicAdd(&p.L0[a], 1);
#pragma unroll
      for (int c = 0; c < kMaxCuts; ++c) {
        if (c < p.ncuts) {
          int32_t *tL = p.use_lds ? lds + p.lds_off[c] : p.L[c];
          int32_t *tCG = p.use_lds ? lds + p.lds_off[c] + p.E : p.CG[c];
          if (alone[c]) atomicAdd(&tL[a], 1);
          for (uint64_t m = gm[c]; m; m &= m - 1) atomicAdd(&tCG[a * p.ng[c] + __builtin_ctzll(m)], 1);
        }
      }
    }
    // C[a1][b] += 1 for every expert a1 of the token that is alone in its group and every other
    // selected expert b.  The lane of b issues the update, so the lanes of a token hit one row of
    // C per step (a few cache lines) rather than one column (a line per lane).
    int alone_mask = 0;
#pragma unroll
    for (int c = 0; c < kMaxCuts; ++c) alone_mask |= alone[c] ? 1 << c : 0;
    for (int k1 = 0; k1 < p.K; ++k1) {
      const int a1 = __shfl(a, sub0 + k1, kWave);
      const int m1 = __shfl(alone_mask, sub0 + k1, kWave);
      if (first && m1 && a1 != a) {
#pragma unroll
        for (int c = 0; c < kMaxCuts; ++c)
          if (m1 & (1 << c)) atomicAdd(&p.C[c][copy_off + (int64_t)a1 * p.E + a], 1);
      }
    }
    const bool leader = k == 0 && t < p.T;   // one lane per token counts the token's groups
#pragma unroll
    for (int c = 0; c < kMaxCuts; ++c) {
      if (c < p.ncuts) {
        for (int j = 0; j < p.ng[c]; ++j) {
          const uint64_t b = __ballot(leader && ((gm[c] >> j) & 1ull));
          if (lane == j) my_base[c] += __popcll(b);
        }
      }
    }
  }
#pragma unroll
  for (int c = 0; c < kMaxCuts; ++c)
    if (c < p.ncuts && lane < p.ng[c] && my_base[c]) atomicAdd(&base_cnt[c][lane], my_base[c]);
  __syncthreads();
  for (int c = 0; c < p.ncuts; ++c) {
    if ((int)threadIdx.x < p.ng[c] && base_cnt[c][threadIdx.x]) atomicAdd(&p.base[c][threadIdx.x], base_cnt[c][threadIdx.x]);
    if (p.use_lds) {
      const int32_t *sL = lds + p.lds_off[c], *sCG = sL + p.E;
      for (int i = threadIdx.x; i < p.E; i += kFactorThreads)
        if (sL[i]) atomicAdd(&p.L[c][i], sL[i]);
      for (int i = threadIdx.x; i < p.E * p.ng[c]; i += kFactorThreads)
        if (sCG[i]) atomicAdd(&p.CG[c][i], sCG[i]);
    }
  }
  if (p.use_lds)
    for (int i = threadIdx.x; i < p.E; i += kFactorThreads)
      if (lds[i]) atomicAdd(&p.L0[i], lds[i]);
}

// ---------------------------------------------------------------------------------------------
// The same tables as contractions over the tokens (E <= 256).
//
// With S[t][a] = 1 when token t selects expert a, A[t][a] = 1 when a is moreover the only selected
// expert of its group, and M[t][g] = 1 when t selects something in group g (all 0/1 bytes):
//   C  = A^T S   (its diagonal is L)        CG = S^T M   (L0[a] = CG[a][group of a])
// so the read-modify-write updates of popular expert pairs, which serialise on one address, become
// int8 matrix products with int32 accumulators held in registers.  A first kernel, one lane per
// routing slot over the whole chip, works out what only the token's other slots can tell (is this
// the first occurrence of the expert, is it alone in its group under each cut) and leaves one byte
// per slot.  In the second a workgroup takes one cut and a contiguous chunk of the tokens, builds
// the three indicator tiles for 128 tokens at a time in LDS (expert-major, so that a lane's MFMA
// operand is 16 contiguous bytes), and stores its partial tables with plain stores; a third kernel
// sums the chunks.  No table is touched by an atomic.
// ---------------------------------------------------------------------------------------------
constexpr int kCoocThreads = 1024;
constexpr int kCoocWaves = kCoocThreads / kWave;
constexpr int kCoocTokens = 128;     // tokens per tile: four k-steps of the 32x32x32 int8 MFMA
constexpr int kCoocStride = 144;     // bytes per tile row: 128 tokens + 16, which spreads 32 rows over all banks
constexpr int kCoocGroups = 64;      // rows of the group tile
constexpr int kCoocChunksMax = 16;   // partial tables per cut
constexpr int kCoocChunkTokensMax = 32640;   // a chunk's counts are stored as 16-bit values
constexpr int kCoocMaxE = 256;
constexpr int kCoocStaged = 8;       // passes whose slots are fetched together (16 KiB of LDS)
constexpr int kCoocTokensPerChunkMin = 512;   // below this a chunk is not worth a workgroup of its own

typedef int32_t i32x4 __attribute__((ext_vector_type(4)));
typedef int32_t i32x16 __attribute__((ext_vector_type(16)));

struct CoocParams {
  const int32_t *ids;
  const int32_t *expert_to_rank;
  int32_t T, K, E, G;
  int32_t sub_log2;            // lanes per token: 2^sub_log2 >= K
  int32_t ncuts;
  int32_t chunks;              // gridDim.x of the matrix kernel
  int32_t tokens_per_chunk;    // a multiple of kCoocTokens
  int32_t ng[kMaxCuts], per[kMaxCuts];
  uint8_t *slot_bits;          // [T * K]: bit 0 first valid occurrence, bit 1 + c alone in its group under cut c
  uint16_t *part[kMaxCuts];    // [chunks][E*E + E*ng + 64 (+1)]: C, CG and base of one chunk; a chunk has < 2^15 tokens
  int32_t *status;
};

__host__ __device__ static inline int64_t cooc_part_ints(int64_t E, int64_t ng) { return E * E + E * ng + 64; }   // values per chunk
__host__ __device__ static inline int64_t cooc_part_words(int64_t E, int64_t ng) { return (cooc_part_ints(E, ng) + 1) / 2; }   // 32-bit words they take

// One lane per routing slot; the K slots of a token sit in 2^sub_log2 consecutive lanes and learn
// about each other through shuffles, eight in flight at a time.
__global__ __launch_bounds__(kSwapThreads) void swap_slots_kernel(CoocParams p) {
  const int sub = 1 << p.sub_log2;
  const int lane = lane_id();
  const int k = lane & (sub - 1);
  const int sub0 = lane & ~(sub - 1);
  const int64_t t = ((int64_t)blockIdx.x * kSwapThreads + threadIdx.x) >> p.sub_log2;
  const bool live = t < p.T && k < p.K;
  int a = -1, r = -1;   // my expert and its rank; -1 when the slot is empty, dropped or invalid
  if (live) {
    const int id = p.ids[t * p.K + k];
    const int rk = rank_of(p.expert_to_rank, p.E, p.G, id);
    if (rk == -1) flag(p.status, HM_ERR_BAD_ID);
    if (rk >= 0) {
      a = id;
      r = rk;
    }
  }
  bool first = a >= 0;   // the selected experts form a set: the first occurrence stands for it
  for (int k0 = 0; k0 < p.K; k0 += 8) {
    int a1[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) a1[j] = __shfl(a, sub0 + ((k0 + j) & (sub - 1)), kWave);
#pragma unroll
    for (int j = 0; j < 8; ++j)
      if (k0 + j < k && a1[j] == a) first = false;
  }
  // The group of my rank under each cut, one byte per cut; equal bytes of two such words are counted
  // four cuts at a time (a zero byte of the exclusive or, found without a carry between bytes).
  __shared__ uint32_t groups_of_rank[kWave];
  if (threadIdx.x < kWave) {
    uint32_t packed = 0;
#pragma unroll
    for (int c = 0; c < kMaxCuts; ++c) packed |= (uint32_t)(threadIdx.x / p.per[c]) << (8 * c);
    groups_of_rank[threadIdx.x] = packed;
  }
  __syncthreads();
  const uint32_t pg = r >= 0 ? groups_of_rank[r] : 0u;
  const uint32_t mine = first ? pg : 0xFFFFFFFFu;   // no group has the number 255
  uint32_t in_group = 0;   // distinct selected experts in my expert's group, one byte per cut (at most 64)
  for (int k0 = 0; k0 < p.K; k0 += 8) {
    uint32_t g1[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) g1[j] = (uint32_t)__shfl((int)mine, sub0 + ((k0 + j) & (sub - 1)), kWave);
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      const uint32_t x = g1[j] ^ pg;
      const uint32_t nonzero = (((x & 0x7F7F7F7Fu) + 0x7F7F7F7Fu) | x) & 0x80808080u;
      if (k0 + j < p.K) in_group += (nonzero ^ 0x80808080u) >> 7;
    }
  }
  if (live) {
    int bits = 0;
    if (first) {
      bits = 1;
#pragma unroll
      for (int c = 0; c < kMaxCuts; ++c)
        if (c < p.ncuts && ((in_group >> (8 * c)) & 0xFFu) == 1u) bits |= 2 << c;
    }
    p.slot_bits[t * p.K + k] = (uint8_t)bits;
  }
}

// D += A B for one 32x32 tile over 32 tokens; a lane's operand: 16 token bytes of row (lane % 32).
__device__ __forceinline__ i32x16 mfma_i8(i32x4 a, i32x4 b, i32x16 acc) {
  return __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc, 0, 0, 0);
}

// Workgroup (chunk, cut, panel).  Every wave holds one 32x32 tile of C, so a workgroup covers 16 of
// them: all of C for E <= 128, and for E <= 256 one of four panels of two tile columns (the panels
// repeat the cheap filling of the tiles and split the products, which is what E = 256 is bound by).
template <int NE>   // experts padded to 32 * NE
__global__ __launch_bounds__(kCoocThreads) void swap_cooc_kernel(CoocParams p) {
  constexpr int kPanels = NE * NE > kCoocWaves ? NE * NE / kCoocWaves : 1;   // gridDim.z
  constexpr int kCols = NE / kPanels;                                         // tile columns of a panel
  constexpr int kVecs = (2 * 32 * NE + kCoocGroups) * kCoocStride / 16;
  extern __shared__ __align__(16) uint8_t tiles[];
  uint8_t *const s_tile = tiles;                                        // [32 NE][stride]  S
  uint8_t *const a_tile = s_tile + 32 * NE * kCoocStride;               // [32 NE][stride]  A
  uint8_t *const m_tile = a_tile + 32 * NE * kCoocStride;               // [64][stride]     M
  __shared__ uint8_t group_of_expert[32 * NE];
  __shared__ uint16_t staged[kCoocStaged][kCoocThreads];

  const int cut = blockIdx.y, panel = blockIdx.z;
  const int ng = p.ng[cut], per = p.per[cut];
  const int tid = threadIdx.x, lane = lane_id(), w = tid >> 6;
  {
    i32x4 *z = (i32x4 *)tiles;
    for (int i = tid; i < kVecs; i += kCoocThreads) z[i] = i32x4{0, 0, 0, 0};
    if (tid < 32 * NE) {
      int g = 0;   // an expert with no valid placement is never marked first, so its entry is not read
      if (tid < p.E) {
        const int r = p.expert_to_rank[tid];
        if ((unsigned)r < (unsigned)p.G) g = r / per;
      }
      group_of_expert[tid] = (uint8_t)g;
    }
  }
  __syncthreads();

  // A pass: every lane looks at one routing slot, 2^sub_log2 lanes per token.  A tile takes `passes`
  // passes; kCoocStaged passes are fetched at a time, so that the latency of global memory is paid
  // once per kCoocStaged passes and not once per tile.
  const int sub = 1 << p.sub_log2;
  const int k = min(tid & (sub - 1), p.K - 1);                        // my slot in the token (clamped: see `mine`)
  const int tp1 = tid >> p.sub_log2;                                  // my token within a pass
  const int tok_pass = min(kCoocThreads >> p.sub_log2, kCoocTokens);  // tokens one pass covers
  const int passes = kCoocTokens / tok_pass;
  const bool mine = tp1 < tok_pass && (tid & (sub - 1)) < p.K;
  const int alone_bit = 2 << cut;
  const int64_t t_begin = (int64_t)blockIdx.x * p.tokens_per_chunk;
  const int64_t t_end = min((int64_t)p.T, t_begin + p.tokens_per_chunk);

  // What this wave accumulates: one tile of C and, counted from the last wave down and dealt round
  // the panels, at most one tile of CG.
  const bool has_c = w < NE * kCols;
  const int c_row = has_c ? w / kCols : 0, c_col = has_c ? panel * kCols + w % kCols : 0;
  const int ngt = (ng + 31) / 32;
  const int g_job = (kCoocWaves - 1 - w) * kPanels + panel;
  const bool has_g = g_job < NE * ngt;
  const int g_row = has_g ? g_job / ngt : 0, g_col = has_g ? g_job % ngt : 0;
  const bool counts_base = panel == 0 && w == kCoocWaves / 2;   // lane g: tokens of this chunk that touch group g
  i32x16 acc, acc_g;
#pragma unroll
  for (int r = 0; r < 16; ++r) acc[r] = acc_g[r] = 0;
  int my_base = 0;

  const int op_at = (lane & 31) * kCoocStride + (lane >> 5) * 16;
  const uint8_t *const c_a = a_tile + 32 * c_row * kCoocStride + op_at;
  const uint8_t *const c_b = s_tile + 32 * c_col * kCoocStride + op_at;
  const uint8_t *const g_a = s_tile + 32 * g_row * kCoocStride + op_at;
  const uint8_t *const g_b = m_tile + 32 * g_col * kCoocStride + op_at;

  for (int64_t stage0 = t_begin; stage0 < t_end; stage0 += (int64_t)kCoocStaged * tok_pass) {
    // My slots of the next kCoocStaged passes: expert | bits << 8, 0 for a slot that marks nothing.
    // The loads are unconditional (clamped to the chunk) so that all of them are in flight at once.
    // A lane reads back only what it wrote itself, so this needs no barrier.
    {
      int id[kCoocStaged], bits[kCoocStaged];
#pragma unroll
      for (int j = 0; j < kCoocStaged; ++j) {
        const int64_t t = min(stage0 + (int64_t)j * tok_pass + tp1, t_end - 1);
        id[j] = p.ids[t * p.K + k];
        bits[j] = p.slot_bits[t * p.K + k];
      }
#pragma unroll
      for (int j = 0; j < kCoocStaged; ++j) {
        const bool in = mine && stage0 + (int64_t)j * tok_pass + tp1 < t_end && (bits[j] & 1);
        staged[j][tid] = (uint16_t)(in ? ((id[j] & 0xFF) | (bits[j] << 8)) : 0);
      }
    }
    int entry = staged[0][tid];
    int group_row = group_of_expert[entry & 0xFF] * kCoocStride;
    for (int tile = 0; tile < kCoocStaged / passes && stage0 + (int64_t)tile * kCoocTokens < t_end; ++tile) {
      int wrote_s = -1, wrote_a = -1, wrote_m = -1;   // LDS offsets to clear again
      for (int pass = 0; pass < passes; ++pass) {
        const int tp = pass * tok_pass + tp1;
        if (entry) {   // a valid expert with a valid placement, first time in this token
          wrote_s = (entry & 0xFF) * kCoocStride + tp;
          wrote_m = group_row + tp;
          s_tile[wrote_s] = 1;
          m_tile[wrote_m] = 1;
          if ((entry >> 8) & alone_bit) {
            wrote_a = wrote_s;
            a_tile[wrote_a] = 1;
          }
        }
        // the next pass's entry and its group: fetched here, off the path between the barriers
        const int next = tile * passes + pass + 1;
        entry = next < kCoocStaged ? staged[next][tid] : 0;
        group_row = group_of_expert[entry & 0xFF] * kCoocStride;
      }
      __syncthreads();

      {
        i32x4 a_op[kCoocTokens / 32], b_op[kCoocTokens / 32];
#pragma unroll
        for (int step = 0; step < kCoocTokens / 32; ++step) {
          a_op[step] = *(const i32x4 *)(c_a + 32 * step);
          b_op[step] = *(const i32x4 *)(c_b + 32 * step);
        }
#pragma unroll
        for (int step = 0; step < kCoocTokens / 32; ++step) acc = mfma_i8(a_op[step], b_op[step], acc);
      }
      if (has_g) {
        i32x4 a_op[kCoocTokens / 32], b_op[kCoocTokens / 32];
#pragma unroll
        for (int step = 0; step < kCoocTokens / 32; ++step) {
          a_op[step] = *(const i32x4 *)(g_a + 32 * step);
          b_op[step] = *(const i32x4 *)(g_b + 32 * step);
        }
#pragma unroll
        for (int step = 0; step < kCoocTokens / 32; ++step) acc_g = mfma_i8(a_op[step], b_op[step], acc_g);
      }
      if (counts_base) {   // bytes are 0 / 1, so a word's population count is its number of tokens
        const i32x4 *row = (const i32x4 *)(m_tile + lane * kCoocStride);
#pragma unroll
        for (int i = 0; i < kCoocTokens / 16; ++i) {
          const i32x4 v = row[i];
          my_base += __popc(v[0]) + __popc(v[1]) + __popc(v[2]) + __popc(v[3]);
        }
      }
      __syncthreads();

      // Leave the tiles clean for the next 128 tokens.  A token's column is written by the lanes of
      // one wave only, so clearing it and filling it again need no barrier in between.
      if (passes == 1) {
        if (wrote_s >= 0) {
          s_tile[wrote_s] = 0;
          m_tile[wrote_m] = 0;
          if (wrote_a >= 0) a_tile[wrote_a] = 0;
        }
      } else {
        i32x4 *z = (i32x4 *)tiles;
        for (int i = tid; i < kVecs; i += kCoocThreads) z[i] = i32x4{0, 0, 0, 0};
        __syncthreads();
      }
    }
  }

  // Accumulator layout of a 32x32 tile: register r of lane l holds row 8 (r / 4) + 4 (l / 32) + r % 4,
  // column l % 32.
  uint16_t *const part = p.part[cut] + (int64_t)blockIdx.x * 2 * cooc_part_words(p.E, ng);
  uint16_t *const part_c = part, *const part_cg = part + (int64_t)p.E * p.E, *const part_base = part_cg + (int64_t)p.E * ng;
  const int col = lane & 31, row_hi = (lane >> 5) * 4;
  if (has_c) {
    const int b = 32 * c_col + col;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int a = 32 * c_row + 8 * (r / 4) + row_hi + (r % 4);
      if (a < p.E && b < p.E) part_c[(int64_t)a * p.E + b] = (uint16_t)acc[r];
    }
  }
  if (has_g) {
    const int g = 32 * g_col + col;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int a = 32 * g_row + 8 * (r / 4) + row_hi + (r % 4);
      if (a < p.E && g < ng) part_cg[(int64_t)a * ng + g] = (uint16_t)acc_g[r];
    }
  }
  if (counts_base) part_base[lane] = (uint16_t)my_base;
}

// Sums the chunks' partial tables into the tables swap_build_kernel reads; blockIdx.y is the cut.
// L is the diagonal of C and L0[a] the entry of CG in a's own group (every token that selects a
// selects something there), so neither needs a table of its own upstream.
__global__ __launch_bounds__(kSwapThreads) void swap_reduce_kernel(SwapParams p, CoocParams cp) {
  const int cut = blockIdx.y;
  const int ng = p.ng[cut];
  const int64_t n = cooc_part_ints(p.E, ng), words = cooc_part_words(p.E, ng);
  const int64_t word = (int64_t)blockIdx.x * kSwapThreads + threadIdx.x;   // two 16-bit values of every chunk
  if (word >= words) return;
  const uint32_t *const part = (const uint32_t *)cp.part[cut];
  int sums[2] = {0, 0};
#pragma unroll
  for (int c = 0; c < kCoocChunksMax; ++c) {
    if (c < cp.chunks) {
      const uint32_t v = part[c * words + word];
      sums[0] += (int)(v & 0xFFFFu);
      sums[1] += (int)(v >> 16);
    }
  }
  const int64_t ee = (int64_t)p.E * p.E;
#pragma unroll
  for (int h = 0; h < 2; ++h) {
    const int64_t i = 2 * word + h;
    const int sum = sums[h];
    if (i >= n) break;
    if (i < ee) {
      p.C[cut][i] = sum;
      const int a = (int)(i / p.E), b = (int)(i % p.E);
      p.CT[cut][(int64_t)b * p.E + a] = sum;
      if (b == a) p.L[cut][a] = sum;
    } else if (i < ee + (int64_t)p.E * ng) {
      const int64_t j = i - ee;
      p.CG[cut][j] = sum;
      p.CGT[cut][(j % ng) * p.E + j / ng] = sum;
      if (cut == 0) {
        const int a = (int)(j / ng), g = (int)(j % ng);
        const int r = p.expert_to_rank[a];
        if ((unsigned)r < (unsigned)p.G ? r / p.per[0] == g : g == 0) p.L0[a] = (unsigned)r < (unsigned)p.G ? sum : 0;
      }
    } else {
      p.base[cut][i - ee - (int64_t)p.E * ng] = sum;
    }
  }
}

// One lane per (c, j) of a cut and kBuildRows row experts r: blockIdx.y is the block of rows and
// blockIdx.x runs over the column blocks (256 consecutive (c, j)) of all cuts, one cut after the
// other.  The loads of all rows are issued before the first value is put together, so a lane
// waits for memory once, and the waves are long enough for the chip not to be bound by starting
// them.  The two divisions a lane needs are multiplications by rounded-up reciprocals: c = l / ng
// (exact for l < 2^32 / ng, and l < 64 E < 2^19) and group = rank / per (rank < 64).
constexpr int kBuildRows = 4;
__global__ __launch_bounds__(kSwapThreads) void swap_build_kernel(SwapParams p) {
  int cut = 0, block = blockIdx.x;
  while (cut + 1 < p.ncuts && block >= p.build_blocks[cut]) block -= p.build_blocks[cut++];
  const int ng = p.ng[cut], r0 = blockIdx.y * kBuildRows;
  const int l = block * kSwapThreads + threadIdx.x;
  if (l >= p.E * ng) return;
  const int32_t *__restrict__ const C = p.C[cut];
  const int32_t *__restrict__ const CT = p.CT[cut];
  const int32_t *__restrict__ const CG = p.CG[cut];
  const int32_t *__restrict__ const CGT = p.CGT[cut];
  const int32_t *__restrict__ const L = p.L[cut];
  const int32_t *__restrict__ const L0 = p.L0;
  int32_t *__restrict__ const Z = p.Z[cut];
  const unsigned per_reciprocal = p.per_reciprocal[cut];
  const int c = ng == 1 ? l : (int)__umulhi((unsigned)l, p.ng_reciprocal[cut]);
  const int j = l - c * ng;
  const int rk = p.expert_to_rank[c];
  const bool c_ok = (unsigned)rk < (unsigned)p.G;
  const int gc = !c_ok ? -1 : per_reciprocal ? (int)__umulhi((unsigned)rk, per_reciprocal) : rk;
  const int base = p.base[cut][j];
  int add[kBuildRows], sub_[kBuildRows];   // val = base + add - sub
  bool bad = false;
#pragma unroll
  for (int i = 0; i < kBuildRows; ++i) {
    const int r = min(r0 + i, p.E - 1);
    const int rr = p.expert_to_rank[r];
    const bool r_ok = (unsigned)rr < (unsigned)p.G;
    const int gr = !r_ok ? -1 : per_reciprocal ? (int)__umulhi((unsigned)rr, per_reciprocal) : rr;
    add[i] = sub_[i] = 0;
    if (!r_ok || !c_ok) {
      bad = true;
    } else if (gr != gc && (j == gc || j == gr)) {
      const int a = j == gc ? r : c, b = j == gc ? c : r;   // group j gains tokens of a, loses tokens of b
      int cba = 0, cg;
      if (p.transposed) {   // every read runs along row r of a table, or along c
        cba = j == gc ? CT[(int64_t)r * p.E + c] : C[(int64_t)r * p.E + c];
        cg = j == gc ? CG[(int64_t)r * ng + j] : CGT[(int64_t)j * p.E + c];
      } else {
#pragma unroll 8
        for (int k = 0; k < p.copies; ++k) cba += C[((int64_t)k * p.E + b) * p.E + a];
        cg = CG[(int64_t)a * ng + j];
      }
      add[i] = L0[a] - cg;
      sub_[i] = L[b] - cba;
    }
  }
  if (bad && j == 0) flag(p.status, HM_ERR_BAD_ID);
#pragma unroll
  for (int i = 0; i < kBuildRows; ++i)
    if (r0 + i < p.E) Z[((int64_t)(r0 + i) * p.E) * ng + l] = base + (add[i] - sub_[i]);
}

// ---------------------------------------------------------------------------------------------
// selection
// ---------------------------------------------------------------------------------------------
constexpr int kMaxDim = 4;

struct SelectParams {
  int32_t d, G, E;
  int32_t U[kMaxDim];
  double M, v, gamma;
  const int32_t *z_inter[kMaxDim];
  const int32_t *z_intra;
  double scale_inter[kMaxDim], alpha_inter[kMaxDim], beta_inter[kMaxDim];
  double scale_intra, alpha_intra, beta_intra;
  double *Q;
  double *block_min;    // workspace [nblocks]
  int32_t *block_arg;   // workspace [nblocks]
  int32_t nblocks;
  int32_t *best_pair;
  double *best_time;
};

// x[i0 .. i0+16) of a term's counts, 0 beyond n: sixteen loads in flight instead of a wait per
// entry (counts are >= 0, so the padding changes neither the maximum nor, skipped, the sum).
__device__ __forceinline__ void load16(const int32_t *x, int n, int i0, int (&v)[16]) {
  if ((n & 3) == 0) {   // rows of n ints start 16-byte aligned
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      i32x4 w = {0, 0, 0, 0};
      if (i0 + 4 * j < n) w = *(const i32x4 *)(x + i0 + 4 * j);
#pragma unroll
      for (int e = 0; e < 4; ++e) v[4 * j + e] = w[e];
    }
  } else {
#pragma unroll
    for (int j = 0; j < 16; ++j) v[j] = i0 + j < n ? x[i0 + j] : 0;
  }
}

__device__ __forceinline__ double smooth_max(const int32_t *x, int n, double gamma) {
  int mi = 0;
  for (int i0 = 0; i0 < n; i0 += 16) {
    int v[16];
    load16(x, n, i0, v);
#pragma unroll
    for (int j = 0; j < 16; ++j) mi = max(mi, v[j]);
  }
  const double m = (double)mi;
  if (gamma <= 0.0 || m == 0.0) return m;
  // A small whole gamma (the paper uses 10) needs no pow per entry: square-and-multiply gives the
  // same power to a few ulp, and a lane is otherwise a serial chain of up to 64 pow calls.
  const int whole = (gamma <= 64.0 && gamma == (double)(int)gamma) ? (int)gamma : 0;
  const double inv_m = 1.0 / m;
  double sum = 0.0;
  if (whole) {
    for (int i0 = 0; i0 < n; i0 += 16) {
      int v[16];
      load16(x, n, i0, v);
#pragma unroll
      for (int j = 0; j < 16; ++j) {
        if (i0 + j < n) {
          const double ratio = (double)v[j] * inv_m;   // within an ulp of the quotient
          double acc = 1.0, sq = ratio;
          for (int e = whole; e; e >>= 1) {
            if (e & 1) acc *= sq;
            sq *= sq;
          }
          sum += acc;
        }
      }
    }
  } else {
    for (int i = 0; i < n; ++i) sum += pow((double)x[i] / m, gamma);
  }
  return m * pow(sum, 1.0 / gamma);
}

// Q of one pair by four lanes: the terms of Eq.(8) (the Inter levels 1 .. d-1, then the Intra
// level) side by side, one lane each, through one code path (a term is a pointer, a length and
// four factors).  The terms are then added in the order of the levels, so Q has the bits of a
// serial evaluation.
__global__ __launch_bounds__(kSelectThreads) void swap_q_kernel(SelectParams p) {
#pragma clang fp contract(off)
  __shared__ double s_val[kSelectPairs];
  __shared__ int32_t s_arg[kSelectPairs];
  const int lane = lane_id();
  const int term = lane & (kPairLanes - 1);
  const int pair_in_block = threadIdx.x / kPairLanes;
  const int64_t rc = (int64_t)blockIdx.x * kSelectPairs + pair_in_block;
  const int64_t pairs = (int64_t)p.E * p.E;
  const bool live = rc < pairs;
  const int64_t at = live ? rc : 0;
  double mine = 0.0;
  if (term < p.d) {
    const bool intra = term == p.d - 1;
    const int i = intra ? 0 : term + 1;
    const int n = intra ? p.G : p.U[i];
    const int32_t *x = (intra ? p.z_intra : p.z_inter[i]) + at * n;
    const double fan = intra ? (double)(p.G / p.U[p.d - 1]) : (double)(p.U[i] / p.U[intra ? 0 : i - 1]);
    const double scale = intra ? p.scale_intra : p.scale_inter[i];
    const double beta = intra ? p.beta_intra : p.beta_inter[i], alpha = intra ? p.alpha_intra : p.alpha_inter[i];
    const double volume = fan * scale * smooth_max(x, n, p.gamma) * p.M * p.v;
    mine = volume * beta + alpha;
  }
  double q = 0.0;
  const int lane0 = lane & ~(kPairLanes - 1);
  for (int j = 0; j < p.d; ++j) q = q + __shfl(mine, lane0 + j, kWave);
  if (term == 0) {
    if (live) p.Q[rc] = q;
    s_val[pair_in_block] = q;
    s_arg[pair_in_block] = live ? (int32_t)rc : -1;
  }
  __syncthreads();
  for (int off = kSelectPairs / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      const int o = threadIdx.x + off;
      const bool take = s_arg[o] >= 0 && (s_arg[threadIdx.x] < 0 || s_val[o] < s_val[threadIdx.x] ||
                                          (s_val[o] == s_val[threadIdx.x] && s_arg[o] < s_arg[threadIdx.x]));
      if (take) {   // among equal times the lower pair index survives
        s_val[threadIdx.x] = s_val[o];
        s_arg[threadIdx.x] = s_arg[o];
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    p.block_min[blockIdx.x] = s_val[0];
    p.block_arg[blockIdx.x] = s_arg[0];
  }
}

__global__ __launch_bounds__(kSwapThreads) void swap_argmin_kernel(SelectParams p) {
  __shared__ double s_val[kSwapThreads];
  __shared__ int32_t s_arg[kSwapThreads];
  double best = 0.0;
  int32_t arg = -1;
  for (int b = threadIdx.x; b < p.nblocks; b += kSwapThreads) {   // ascending blocks: first minimum wins
    const int32_t a = p.block_arg[b];
    if (a >= 0 && (arg < 0 || p.block_min[b] < best)) {
      best = p.block_min[b];
      arg = a;
    }
  }
  s_val[threadIdx.x] = best;
  s_arg[threadIdx.x] = arg;
  __syncthreads();
  for (int off = kSwapThreads / 2; off > 0; off >>= 1) {
    if ((int)threadIdx.x < off) {
      const int o = threadIdx.x + off;
      const bool better = s_arg[o] >= 0 && (s_arg[threadIdx.x] < 0 || s_val[o] < s_val[threadIdx.x] ||
                                            (s_val[o] == s_val[threadIdx.x] && s_arg[o] < s_arg[threadIdx.x]));
      if (better) {
        s_val[threadIdx.x] = s_val[o];
        s_arg[threadIdx.x] = s_arg[o];
      }
    }
    __syncthreads();
  }
  if (threadIdx.x == 0) {
    p.best_pair[0] = s_arg[0] / p.E;
    p.best_pair[1] = s_arg[0] % p.E;
    *p.best_time = s_val[0];
  }
}

// The chosen swap (Section IV): the two placement entries trade places; the diagonal (no swap won
// Eq.(10)) and out-of-range indices change nothing.
__global__ void swap_apply_kernel(int32_t *__restrict__ expert_to_rank, int32_t E, const int32_t *__restrict__ pair) {
  if (blockIdx.x != 0 || threadIdx.x != 0) return;
  const int32_t r = pair[0], c = pair[1];
  if (r < 0 || r >= E || c < 0 || c >= E || r == c) return;
  const int32_t g = expert_to_rank[r];
  expert_to_rank[r] = expert_to_rank[c];
  expert_to_rank[c] = g;
}

// The co-occurrence kernel may use more dynamic LDS than a kernel gets by default (64 KiB); ask
// once.  False: the tables stay in global memory.
static bool swap_factors_lds_ready() {
  static const bool ok = [] {
    const hipError_t e = hipFuncSetAttribute((const void *)swap_factors_kernel, hipFuncAttributeMaxDynamicSharedMemorySize,
                                             kSwapLds * (int)sizeof(int32_t));
    if (e != hipSuccess) (void)hipGetLastError();   // not sticky: do not let it fail the next launch check
    return e == hipSuccess;
  }();
  return ok;
}

// Private copies of C on the path with atomics: as many as fit 2 MiB per cut, at most
// kSwapCopiesMax (32 for E <= 128, 8 for E = 256): more copies spread the atomics of popular pairs,
// but each is cleared and summed again.  The matrix path keeps one summed C.
// The matrix path: E <= 256 and chunks short enough for 16-bit counts.
static inline bool swap_by_matrices(int64_t E, int64_t T) { return E <= kCoocMaxE && T <= (int64_t)kCoocChunksMax * kCoocChunkTokensMax; }
static inline int64_t swap_copies(int64_t E, int64_t T) {
  if (swap_by_matrices(E, T)) return 1;
  int64_t n = kSwapCopiesMax;   // a power of two, so that a workgroup finds its copy with a mask
  while (n > 1 && n * E * E > (int64_t)(1 << 19)) n /= 2;
  return n;
}

// Workspace, in ints: L0 [E], then per cut base [64] | L [E] | CG [E * ng] | C [copies * E * E], and on the
// matrix path the partial tables of kCoocChunksMax chunks and the transposes of C and CG after that.
static inline int64_t swap_cut_ints(int64_t E, int64_t ng, int64_t T) {
  return 64 + E + E * ng + swap_copies(E, T) * E * E +
         (swap_by_matrices(E, T) ? kCoocChunksMax * cooc_part_words(E, ng) + E * E + E * ng : 0);
}
// ... and, on the matrix path, one byte per routing slot at the very end.
static inline int64_t swap_slot_ints(int64_t T, int64_t K, int64_t E) { return swap_by_matrices(E, T) ? (T * K + 3) / 4 : 0; }

// The matrix kernel for E experts, its dynamic LDS, and whether the device grants that much.
typedef void (*cooc_kernel_t)(CoocParams);
static inline cooc_kernel_t cooc_kernel(int E, size_t *lds_bytes) {
  const int ne = E <= 32 ? 1 : E <= 64 ? 2 : E <= 128 ? 4 : 8;
  *lds_bytes = (size_t)(2 * 32 * ne + kCoocGroups) * kCoocStride;
  return ne == 1 ? swap_cooc_kernel<1> : ne == 2 ? swap_cooc_kernel<2> : ne == 4 ? swap_cooc_kernel<4> : swap_cooc_kernel<8>;
}
static bool cooc_lds_ready() {
  static const bool ok = [] {
    size_t bytes = 0;
    const cooc_kernel_t k = cooc_kernel(kCoocMaxE, &bytes);   // only the largest needs more than the default
    const hipError_t e = hipFuncSetAttribute((const void *)k, hipFuncAttributeMaxDynamicSharedMemorySize, (int)bytes);
    if (e != hipSuccess) (void)hipGetLastError();
    return e == hipSuccess;
  }();
  return ok;
}

static inline bool swap_cuts_ok(int32_t G, int32_t ncuts, const int32_t *ng) {
  if (G < 1 || G > 64 || ncuts < 1 || ncuts > kMaxCuts || !ng) return false;
  for (int c = 0; c < ncuts; ++c)
    if (ng[c] < 1 || ng[c] > G || G % ng[c] != 0) return false;
  return true;
}

static hm_status swap_counts_launch(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                                    int32_t G, int32_t ncuts, const int32_t *ng, int32_t *const *Z, int32_t *status,
                                    void *workspace, hipStream_t stream) {
  SwapParams p;
  p.ids = topk_ids;
  p.expert_to_rank = expert_to_rank;
  p.T = T;
  p.K = K;
  p.E = E;
  p.G = G;
  p.ncuts = ncuts;
  p.copies = (int32_t)swap_copies(E, T);
  p.sub = 1;
  while (p.sub < K) p.sub *= 2;
  p.ws = (int32_t *)workspace;
  p.L0 = p.ws;
  int64_t at = E, lds_at = E;
  for (int c = 0; c < kMaxCuts; ++c) {
    const int cc = c < ncuts ? c : 0;   // unused entries repeat cut 0 so that no pointer is left dangling
    p.ng[c] = ng[cc];
    p.per[c] = G / ng[cc];
    p.ng_reciprocal[c] = ng[cc] > 1 ? (uint32_t)((0x100000000ull + ng[cc] - 1) / ng[cc]) : 0u;
    p.per_reciprocal[c] = p.per[c] > 1 ? (uint32_t)((0x100000000ull + p.per[c] - 1) / p.per[c]) : 0u;
    p.Z[c] = Z[cc];
    if (c < ncuts) {
      p.base[c] = p.ws + at;
      p.L[c] = p.base[c] + 64;
      p.CG[c] = p.L[c] + E;
      p.C[c] = p.CG[c] + (int64_t)E * ng[c];
      at += swap_cut_ints(E, ng[c], T);
      p.lds_off[c] = (int32_t)lds_at;
      lds_at += (int64_t)E * (ng[c] + 1);
    } else {
      p.base[c] = p.base[0];
      p.L[c] = p.L[0];
      p.CG[c] = p.CG[0];
      p.C[c] = p.C[0];
      p.lds_off[c] = p.lds_off[0];
    }
  }
  p.status = status;
  size_t cooc_lds = 0;
  const cooc_kernel_t cooc = swap_by_matrices(E, T) ? cooc_kernel(E, &cooc_lds) : nullptr;
  if (cooc && (cooc_lds <= 65536 || cooc_lds_ready())) {
    // Every table is written in full by the kernels below: only the status word needs clearing.
    p.ws_ints = 0;
    p.use_lds = 0;
    p.transposed = 1;
    hipLaunchKernelGGL(swap_clear_kernel, dim3(1), dim3(kSwapThreads), 0, stream, p);
    if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
    CoocParams cp;
    cp.ids = topk_ids;
    cp.expert_to_rank = expert_to_rank;
    cp.T = T;
    cp.K = K;
    cp.E = E;
    cp.G = G;
    cp.sub_log2 = 0;
    while ((1 << cp.sub_log2) < K) ++cp.sub_log2;
    cp.ncuts = ncuts;
    cp.slot_bits = (uint8_t *)(p.ws + at);
    int64_t chunks = ((int64_t)T + kCoocTokensPerChunkMin - 1) / kCoocTokensPerChunkMin;
    chunks = chunks < 1 ? 1 : chunks > kCoocChunksMax ? kCoocChunksMax : chunks;
    const int64_t per_chunk = ((int64_t)T + chunks - 1) / chunks;
    cp.chunks = (int32_t)chunks;
    cp.tokens_per_chunk = (int32_t)((per_chunk + kCoocTokens - 1) / kCoocTokens * kCoocTokens);
    if (cp.tokens_per_chunk < kCoocTokens) cp.tokens_per_chunk = kCoocTokens;
    int64_t max_part = 0;
    for (int c = 0; c < kMaxCuts; ++c) {
      cp.ng[c] = p.ng[c];
      cp.per[c] = p.per[c];
      cp.part[c] = (uint16_t *)(p.C[c] + (int64_t)E * E);   // behind the summed C of the cut
      p.CT[c] = p.C[c] + (int64_t)E * E + kCoocChunksMax * cooc_part_words(E, p.ng[c]);
      p.CGT[c] = p.CT[c] + (int64_t)E * E;
      if (c < ncuts && cooc_part_words(E, ng[c]) > max_part) max_part = cooc_part_words(E, ng[c]);
    }
    cp.status = status;
    if (T > 0) {
      const int64_t lanes = (int64_t)T << cp.sub_log2;
      hipLaunchKernelGGL(swap_slots_kernel, dim3((unsigned)((lanes + kSwapThreads - 1) / kSwapThreads)), dim3(kSwapThreads), 0,
                         stream, cp);
      if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
    }
    hipLaunchKernelGGL(cooc, dim3((unsigned)chunks, (unsigned)ncuts, E > 128 ? 4u : 1u), dim3(kCoocThreads), cooc_lds, stream, cp);
    if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
    hipLaunchKernelGGL(swap_reduce_kernel, dim3((unsigned)((max_part + kSwapThreads - 1) / kSwapThreads), (unsigned)ncuts),
                       dim3(kSwapThreads), 0, stream, p, cp);
    if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  } else {
    p.transposed = 0;
    for (int c = 0; c < kMaxCuts; ++c) p.CT[c] = p.CGT[c] = nullptr;
    p.ws_ints = at;
    p.use_lds = (lds_at <= kSwapLds && swap_factors_lds_ready()) ? 1 : 0;
    hipLaunchKernelGGL(swap_clear_kernel, dim3((unsigned)((p.ws_ints + kSwapThreads - 1) / kSwapThreads)), dim3(kSwapThreads),
                       0, stream, p);
    if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
    if (T > 0) {
      const int64_t tokens_per_block = (int64_t)(kFactorThreads / kWave) * (kWave / p.sub);
      int64_t blocks = ((int64_t)T + tokens_per_block - 1) / tokens_per_block;
      if (blocks > 256) blocks = 256;   // one per CU; every block flushes its LDS tables with atomics
      hipLaunchKernelGGL(swap_factors_kernel, dim3((unsigned)blocks), dim3(kFactorThreads),
                         p.use_lds ? (size_t)lds_at * sizeof(int32_t) : 0, stream, p);
      if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
    }
  }
  int64_t build_blocks = 0;
  for (int c = 0; c < kMaxCuts; ++c) {
    p.build_blocks[c] = c < ncuts ? (int32_t)(((int64_t)E * ng[c] + kSwapThreads - 1) / kSwapThreads) : 0;
    build_blocks += p.build_blocks[c];
  }
  hipLaunchKernelGGL(swap_build_kernel, dim3((unsigned)build_blocks, (unsigned)((E + kBuildRows - 1) / kBuildRows)),
                     dim3(kSwapThreads), 0, stream, p);
  return hm_launch_status();
}

}  // namespace hm

extern "C" size_t hm_swap_multi_workspace_bytes(int32_t T, int32_t K, int32_t E, int32_t G, int32_t ncuts, const int32_t *ng) {
  if (E < 1 || T < 0 || K < 1 || !hm::swap_cuts_ok(G, ncuts, ng)) return 0;
  int64_t ints = E + hm::swap_slot_ints(T, K, E);
  for (int c = 0; c < ncuts; ++c) ints += hm::swap_cut_ints(E, ng[c], T);
  return (size_t)ints * sizeof(int32_t);
}

extern "C" size_t hm_swap_workspace_bytes(int32_t T, int32_t K, int32_t E, int32_t ng) {
  if (E < 1 || T < 0 || K < 1 || ng < 1 || ng > 64) return 0;
  return (size_t)(E + hm::swap_cut_ints(E, ng, T) + hm::swap_slot_ints(T, K, E)) * sizeof(int32_t);
}

static hm_status swap_counts_checks(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                                    const void *workspace) {
  if (!expert_to_rank || !workspace) return HM_ERR_NULL;
  hm_status st = hm_check_tk(T, K);
  if (st != HM_OK) return st;
  if (E < 1 || (int64_t)E * E * 64 > 2147483647LL) return HM_ERR_SHAPE;
  if (T > 0 && !topk_ids) return HM_ERR_NULL;
  return HM_OK;
}

extern "C" hm_status hm_swap_counts(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K,
                                    int32_t E, int32_t G, int32_t ng, int32_t *Z, int32_t *status, void *workspace,
                                    size_t workspace_bytes, void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!Z) return HM_ERR_NULL;
  hm_status st = swap_counts_checks(topk_ids, expert_to_rank, T, K, E, workspace);
  if (st != HM_OK) return st;
  if (!hm::swap_cuts_ok(G, 1, &ng)) return HM_ERR_TOPOLOGY;
  if (workspace_bytes < hm_swap_workspace_bytes(T, K, E, ng)) return HM_ERR_WORKSPACE;
  return hm::swap_counts_launch(topk_ids, expert_to_rank, T, K, E, G, 1, &ng, &Z, status, workspace, (hipStream_t)hip_stream);
}

extern "C" hm_status hm_swap_counts_multi(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K,
                                          int32_t E, int32_t G, int32_t ncuts, const int32_t *ng, int32_t *const *Z,
                                          int32_t *status, void *workspace, size_t workspace_bytes, void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!Z || !ng) return HM_ERR_NULL;
  hm_status st = swap_counts_checks(topk_ids, expert_to_rank, T, K, E, workspace);
  if (st != HM_OK) return st;
  if (!hm::swap_cuts_ok(G, ncuts, ng)) return HM_ERR_TOPOLOGY;
  for (int c = 0; c < ncuts; ++c)
    if (!Z[c]) return HM_ERR_NULL;
  if (workspace_bytes < hm_swap_multi_workspace_bytes(T, K, E, G, ncuts, ng)) return HM_ERR_WORKSPACE;
  return hm::swap_counts_launch(topk_ids, expert_to_rank, T, K, E, G, ncuts, ng, Z, status, workspace, (hipStream_t)hip_stream);
}

extern "C" size_t hm_swap_select_workspace_bytes(int32_t E) {
  if (E < 1) return 0;
  const int64_t blocks = ((int64_t)E * E + hm::kSelectPairs - 1) / hm::kSelectPairs;
  return (size_t)blocks * (sizeof(double) + sizeof(int32_t)) + 16;
}

extern "C" hm_status hm_swap_select(int32_t d, const int32_t *U, int32_t G, int32_t E, double M, double v,
                                    const int32_t *const *z_inter, const int32_t *z_intra, const double *scale_inter,
                                    double scale_intra, const double *alpha_inter, const double *beta_inter,
                                    double alpha_intra, double beta_intra, double gamma, double *Q, int32_t *best_pair,
                                    double *best_time, void *workspace, size_t workspace_bytes, void *hip_stream) {
  HM_ENTRY_SCOPE;
  using namespace hm;
  if (!U || !z_intra || !Q || !best_pair || !best_time || !workspace) return HM_ERR_NULL;
  if (d < 1 || d > kMaxDim || G < 1 || G > 64 || U[0] != 1) return HM_ERR_TOPOLOGY;
  if (E < 1 || (int64_t)E * E > 2147483647LL) return HM_ERR_SHAPE;
  if (d > 1 && (!z_inter || !scale_inter || !alpha_inter || !beta_inter)) return HM_ERR_NULL;
  for (int i = 1; i < d; ++i) {
    if (!z_inter[i]) return HM_ERR_NULL;
    if (U[i] < U[i - 1] || U[i] > G || U[i] % U[i - 1] != 0 || G % U[i] != 0) return HM_ERR_TOPOLOGY;
  }
  if (workspace_bytes < hm_swap_select_workspace_bytes(E)) return HM_ERR_WORKSPACE;
  SelectParams p;
  p.d = d;
  p.G = G;
  p.E = E;
  p.M = M;
  p.v = v;
  p.gamma = gamma;
  for (int i = 0; i < kMaxDim; ++i) {
    const bool in = i >= 1 && i < d;
    p.U[i] = i < d ? U[i] : 1;
    p.z_inter[i] = in ? z_inter[i] : nullptr;
    p.scale_inter[i] = in ? scale_inter[i] : 0.0;
    p.alpha_inter[i] = in ? alpha_inter[i] : 0.0;
    p.beta_inter[i] = in ? beta_inter[i] : 0.0;
  }
  p.z_intra = z_intra;
  p.scale_intra = scale_intra;
  p.alpha_intra = alpha_intra;
  p.beta_intra = beta_intra;
  p.Q = Q;
  p.nblocks = (int32_t)(((int64_t)E * E + kSelectPairs - 1) / kSelectPairs);
  p.block_min = (double *)workspace;
  p.block_arg = (int32_t *)(p.block_min + p.nblocks);
  p.best_pair = best_pair;
  p.best_time = best_time;
  hipStream_t stream = (hipStream_t)hip_stream;
  hipLaunchKernelGGL(swap_q_kernel, dim3(p.nblocks), dim3(kSelectThreads), 0, stream, p);
  if (hm_launch_status() != HM_OK) return HM_ERR_HIP;
  hipLaunchKernelGGL(swap_argmin_kernel, dim3(1), dim3(kSwapThreads), 0, stream, p);
  return hm_launch_status();
}

extern "C" hm_status hm_swap_apply(int32_t *expert_to_rank, int32_t E, const int32_t *best_pair, void *hip_stream) {
  HM_ENTRY_SCOPE;
  if (!expert_to_rank || !best_pair) return HM_ERR_NULL;
  if (E < 1) return HM_ERR_SHAPE;
  hipLaunchKernelGGL(hm::swap_apply_kernel, dim3(1), dim3(hm::kWave), 0, (hipStream_t)hip_stream, expert_to_rank, E,
                     best_pair);
  return hm_launch_status();
}
