/*
 * hiermoe.h -- C ABI of the MI355X (gfx950) dedup dispatch / combine library, libhiermoe.so.
 *
 * The library implements one expert-parallel rank's side of the hierarchical token
 * deduplication of HierMoE (arxiv 2508.09591): from the rank's top-K routing it builds, per
 * destination group (a GPU for HD1, a node for the inter-node hop of HD2; Section III-A), the
 * send list in which every token appears at most once (the group-OR of Eq.(7)), packs the bf16
 * token rows into per-destination send buffers, and merges expert outputs coming back in that
 * layout with the router weights ("AlltoAll Combine", Section II-B).  Destinations are index
 * partitions of one buffer; the exchange itself is not part of the library.
 *
 * Conventions
 *   - Unless marked "host", every pointer is a DEVICE pointer into memory the caller owns.
 *     The library never allocates or frees device memory.
 *   - Every call only enqueues work on `hip_stream` (a hipStream_t passed as void*, NULL = the
 *     default stream) and returns; only hm_plan_status synchronises.
 *   - The return value reports host-checkable argument errors, detected before anything is
 *     launched (so nothing was written), or a HIP launch failure.  Data errors found by the
 *     kernels (an expert id outside [0,E), a rank outside [0,G), a row index outside the
 *     caller's buffer) never fault: the offending slot / row is skipped and the code is stored
 *     in the plan's device status word, which hm_plan_status returns.
 *   - The expert id -1 marks a slot the router dropped (capacity-limited routing): every entry
 *     point skips such a slot (slot_row = -1, slot_keep = 0, not counted, weight ignored) without
 *     reporting an error.
 *   - Row and token indices are int32; byte offsets inside the kernels are 64-bit.
 *   - Limits: nodes*ranks_per_node <= 64, nodes <= 32 (bit masks), 1 <= K <= 64,
 *     T*K <= 2^31-1.
 *   - Re-entrant per (plan buffers, workspace, stream); the only global state is what is named
 *     where it is declared: hm_plan_one_launch_limit, the scratch of hm_plan_static, and kernel
 *     attributes (dynamic LDS limits) that hm_swap_counts sets the first time it runs.
 */
#ifndef HIERMOE_H
#define HIERMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  HM_OK = 0,
  HM_ERR_NULL = -1,      /* a required pointer is NULL                                   */
  HM_ERR_SHAPE = -2,     /* T < 0, K/E/H out of range, T*K overflows int32                */
  HM_ERR_TOPOLOGY = -3,  /* nodes or ranks_per_node < 1, more than 64 ranks or 32 nodes   */
  HM_ERR_LEVEL = -4,     /* dedup level is not one of hm_dedup_level                      */
  HM_ERR_WORKSPACE = -5, /* workspace smaller than needed (hm_plan_static: than its maximum) */
  HM_ERR_CAPACITY = -6,  /* a row index does not fit the caller's row buffers (device)    */
  HM_ERR_BAD_ID = -7,    /* expert id or rank out of range (device-detected)              */
  HM_ERR_HIP = -8        /* a HIP runtime call failed                                     */
} hm_status;

/* Where duplicates are removed (Section III-A): nowhere (plain per-rank MoE permute, the H1
 * baseline), per destination GPU (HD1), or per destination node (first hop of HD2). */
typedef enum { HM_DEDUP_NONE = 0, HM_DEDUP_GPU = 1, HM_DEDUP_NODE = 2 } hm_dedup_level;

/* Two-level hierarchy: rank g belongs to node g / ranks_per_node (contiguous, Section III-B). */
typedef struct {
  int32_t nodes;
  int32_t ranks_per_node;
} hm_topology;

/*
 * Plan buffers, allocated by the caller, filled by hm_plan.  `num_dest` (host) is written by
 * hm_plan: nodes at level node, nodes*ranks_per_node otherwise.  `row_capacity` (host, input)
 * is the number of rows row_token / row_weight can hold; T*min(K,num_dest) always suffices.
 *
 *   dest_count [num_dest]     rows destined to each group = the duplicate-free count p of Eq.(7)
 *   dest_offset[num_dest+1]   exclusive prefix sum; destination d owns packed rows
 *                             [dest_offset[d], dest_offset[d+1]); the last entry is total_rows
 *   row_token  [row_capacity] packed row -> source token.  Inside a destination rows ascend by
 *                             flat slot index t*K+k of the kept slot (i.e. by token).
 *   slot_row   [T*K]          slot (t,k) -> the packed row carrying token t to the slot's
 *                             destination (same row for all slots of t with that destination);
 *                             -1 for a dropped (invalid) slot
 *   slot_keep  [T*K]          1 for the first slot of a token with a given destination (the one
 *                             that owns the row), else 0; at level none every valid slot is 1
 *   row_weight [row_capacity] fp32 sum, in ascending k, of the router weights of the slots a row
 *                             serves
 *   rank_mask  [T]  optional  bit g set iff some valid slot of the token maps to rank g
 *   node_mask  [T]  optional  bit n set iff some valid slot maps to node n
 *   status     [1]            0, or HM_ERR_BAD_ID / HM_ERR_CAPACITY as stored by the kernels (the more
 *                             negative code wins when both occur, whatever the order of the waves)
 *   load_expert [E], load_rank [G], load_node [nodes]   optional, all three or none: when given,
 *                             hm_plan also produces the counts of hm_expert_load, in the same
 *                             launches (the planner of Section IV needs them every iteration).
 *                             hm_plan_mapped ignores them.
 *
 * Two more host fields steer launch shapes only, never results.  `max_rows_per_token` is written
 * by hm_plan (K at level none, else min(K, num_dest)) and zeroed by hm_plan_mapped (a hop table
 * may leave most slots without a copy, so there is no useful bound).  `expected_rows` is the
 * number of packed rows the caller expects the plan to hold, 0 = unknown: hm_plan_status stores
 * total_rows there, a caller that does not synchronise may store the previous iteration's count;
 * hm_plan leaves it alone.  The row kernels take rows per token from expected_rows / T if it is
 * set, else from max_rows_per_token, else assume few -- never from the sizes of the caller's row
 * buffers, which may be worst-case allocations.  Zero-initialise the struct before filling it in.
 */
typedef struct {
  int32_t num_dest;
  int64_t row_capacity;
  int32_t *dest_count;
  int32_t *dest_offset;
  int32_t *row_token;
  int32_t *slot_row;
  uint8_t *slot_keep;
  float *row_weight;
  uint64_t *rank_mask;
  uint32_t *node_mask;
  int32_t *status;
  int32_t *load_expert;
  int32_t *load_rank;
  int32_t *load_node;
  int32_t max_rows_per_token;
  int64_t expected_rows;
} hm_plan_out;

/* Bytes of device scratch hm_plan needs for these sizes (0 on invalid arguments). */
size_t hm_plan_workspace_bytes(int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level);

/*
 * hm_plan -- Eq.(7) as send lists.  For slot (t,k): rank = expert_to_rank[topk_ids[t,k]], the
 * destination is the rank (levels none, gpu) or rank / ranks_per_node (level node).  At levels
 * gpu and node a token keeps one row per destination (the OR over the group's experts); the
 * lowest k owns it.  Fills every field of *out described above and clears / sets *out->status.
 *   topk_ids [T*K] int32, topk_weights [T*K] fp32, expert_to_rank [E] int32 (any map E -> ranks;
 *   an expert swap of Section IV is an exchange of two entries).  workspace: device scratch of
 *   at least hm_plan_workspace_bytes, 16-byte aligned, private to this call until it completes.
 * Invalid slots are dropped (slot_row = -1, slot_keep = 0) and flagged HM_ERR_BAD_ID; rows beyond
 * row_capacity are not written and flagged HM_ERR_CAPACITY (counts and offsets stay exact).
 */
hm_status hm_plan(const int32_t *topk_ids, const float *topk_weights, const int32_t *expert_to_rank,
                  int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level,
                  hm_plan_out *out /* host struct */, void *workspace, size_t workspace_bytes,
                  void *hip_stream);

/*
 * hm_plan_one_launch_limit -- plans of at most `workgroups` workgroups (1,024 routing slots each;
 * default and maximum 256) run as ONE launch whose workgroups wait for one another's counts, which
 * needs all of them resident on the GPU together.  One such plan always is (the library checks
 * hm_plan_one_launch_capacity(): 256 on an MI355X, one workgroup per CU), and so are several in
 * flight on separate streams as long as together they need no more than that.  Beyond it, or on a GPU that other
 * kernels fill for longer than about 0.1 s, several plans can each hold part of the machine;
 * their waits are bounded, so nothing hangs, but such a plan ends with HM_ERR_HIP in its status
 * word and unwritten maps.  Callers that overlap that many plans lower the limit (0: always
 * separate launches, which have no such need and cost a few microseconds more on small plans).
 * Process-wide, takes effect for later calls; returns the previous limit.  The results do not
 * depend on it.
 */
int32_t hm_plan_one_launch_limit(int32_t workgroups);
/* Workgroups of the one-launch plan that the current device holds at once (0 if unknown: then
 * every plan takes separate launches).  Plans in flight together must not need more. */
int32_t hm_plan_one_launch_capacity(void);

/*
 * hm_plan_status -- waits for `hip_stream`, then returns the plan's device status word and
 * stores total_rows (= dest_offset[num_dest]) into *total_rows (host, may be NULL) and into
 * plan->expected_rows.
 */
hm_status hm_plan_status(hm_plan_out *plan /* host struct */, int64_t *total_rows /* host */, void *hip_stream);

/*
 * hm_plan_static -- hm_plan for callers that cannot allocate or pass a workspace: code recorded
 * under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments
 * and results as hm_plan without the workspace pair; the scratch (the per-workgroup count matrix)
 * is a static device array inside the library, hm_plan_static_max_bytes() = 1 MiB on every GPU
 * the library runs on, held until the process ends.  The call allocates and frees nothing (the
 * first call on a device looks the array's address up once).  Sizes that need more, i.e.
 * hm_plan_workspace_bytes(...) > hm_plan_static_max_bytes() (about 4 Mi routing slots at 64
 * destinations), are rejected with HM_ERR_WORKSPACE before anything is launched.  All calls on
 * one GPU share the array: calls that may overlap there (different streams, several threads)
 * race and must be serialised by the caller; nothing in it has to be cleared between calls.
 */
size_t hm_plan_static_max_bytes(void);
hm_status hm_plan_static(const int32_t *topk_ids, const float *topk_weights, const int32_t *expert_to_rank,
                         int32_t T, int32_t K, int32_t E, hm_topology topo, hm_dedup_level level,
                         hm_plan_out *out /* host struct */, void *hip_stream);

/*
 * hm_dispatch_pack -- the deduplicated send buffers (Section III-A, Fig.5): for every kept slot,
 * packed[slot_row[t,k], :] = x[t, :], a bit copy of H bf16 values.  x [T,H] bf16 row-major,
 * packed [packed_rows,H] bf16; rows outside [0,packed_rows) are skipped and flagged
 * HM_ERR_CAPACITY.  Uses plan->slot_row, slot_keep, status.  Fast path needs H % 8 == 0 and
 * 16-byte aligned x / packed; any other H or alignment takes a slower element-wise kernel.
 */
hm_status hm_dispatch_pack(const void *x_bf16, int32_t T, int32_t K, int32_t H, const hm_plan_out *plan,
                           void *packed_bf16, int64_t packed_rows, void *hip_stream);

/*
 * hm_combine -- weighted merge of expert outputs returned in the packed layout (Section II-A:
 * the layer output is the gate-weighted sum of the selected experts' outputs):
 *     out[t,:] = bf16( sum_k topk_weights[t,k] * y[slot_row[t,k], :] ),  fp32 accumulation.
 * Slots that share a row are merged first (their weights are added in fp32, ascending k) so each
 * distinct row is read once.  y [y_rows,H] bf16, out [T,H] bf16.  Dropped slots and rows outside
 * [0,y_rows) contribute nothing (the latter flagged HM_ERR_CAPACITY).  Uses plan->slot_row, status.
 * topk_weights may be NULL: the weights are then the ones hm_plan already merged, plan->row_weight
 * (the same additions in the same order, so the same bits when the plan was built from these
 * router weights -- the normal case), the first slot of a row is the one plan->slot_keep marks,
 * and rows at or beyond plan->row_capacity count as outside y.  This is the faster form (no
 * merge of the K slots in every wave); pass the weights only if they differ from the plan's.
 * The same holds for hm_combine_f32 and hm_combine_mix.
 */
hm_status hm_combine(const void *y_bf16, int64_t y_rows, const float *topk_weights, int32_t T, int32_t K,
                     int32_t H, const hm_plan_out *plan, void *out_bf16, void *hip_stream);

/*
 * hm_combine_launch_shape -- host only, launches nothing: the shape hm_combine / hm_combine_f32 /
 * hm_combine_mix would launch with for this plan on rows of H % 8 == 0 (H % 4 for fp32) elements:
 * 16-byte vectors per lane, rows whose loads are in flight per wave, resident waves per CU the
 * launch allows (32 = no cap).  weights_from_plan != 0 asks about the topk_weights == NULL form.
 * For tests and tuning: it shows what plan->expected_rows / max_rows_per_token select.
 */
hm_status hm_combine_launch_shape(int32_t T, int32_t K, int32_t H, const hm_plan_out *plan, int32_t weights_from_plan,
                                  int32_t *vectors_per_lane /* host */, int32_t *rows_in_flight /* host */,
                                  int32_t *waves_per_cu /* host */);

/*
 * hm_combine_f32 -- hm_combine for rows kept in binary32 (the element width is free in the paper:
 * the `v` bytes per element of the cost model in Section II-B):
 *     out[t,:] = sum_k topk_weights[t,k] * y[slot_row[t,k], :],  an fp32 fma chain over the token's
 * distinct rows in ascending k of their first slot, merged weights as in hm_combine; the result
 * differs from the exact sum by at most 2K * 2^-24 * sum_k |w y|.  y [y_rows,H] fp32, out [T,H]
 * fp32.  Fast path needs H % 4 == 0 and 16-byte aligned y / out.  Errors as hm_combine.
 */
hm_status hm_combine_f32(const float *y, int64_t y_rows, const float *topk_weights, int32_t T, int32_t K,
                         int32_t H, const hm_plan_out *plan, float *out, void *hip_stream);

/*
 * hm_combine_transpose -- adjoint of hm_combine with respect to y (the gradient that travels
 * back through the dispatch layout): for every kept slot,
 *     gy[row,:] = row_weight[row] * gout[t,:],   row = slot_row[t,k]   (one fp32 multiply).
 * gout [T,H] fp32, gy [gy_rows,H] fp32.  Uses plan->slot_row, slot_keep, row_weight, status.
 */
hm_status hm_combine_transpose(const float *gout, int32_t T, int32_t K, int32_t H, const hm_plan_out *plan,
                               float *gy, int64_t gy_rows, void *hip_stream);

/*
 * hm_combine_transpose_bf16 -- hm_combine_transpose for gradients kept in bf16 (the element
 * width of a row is free in the paper: the `v` of Section II-B):
 *     gy[row,:] = bf16( row_weight[row] * gout[t,:] ),  the exact product rounded once (the fp32
 * product's own rounding error, recovered with one fma, settles the cases where rounding twice
 * would differ; that error term underflows for |row_weight * gout| below about 2^-102, where an
 * exact tie of the fp32 product may be broken to even instead).  gout [T,H] bf16, gy [gy_rows,H]
 * bf16; fast path needs H % 8 == 0 and 16-byte aligned buffers.  Errors as hm_combine_transpose.
 */
hm_status hm_combine_transpose_bf16(const void *gout_bf16, int32_t T, int32_t K, int32_t H, const hm_plan_out *plan,
                                    void *gy_bf16, int64_t gy_rows, void *hip_stream);

/*
 * hm_expert_load -- the counts the expert-swap planner of Section IV consumes:
 *   load_expert[E]   slots per expert (duplicate-unaware, what SmartMoE-style planners count)
 *   load_rank [G]    tokens per rank after deduplication  = p^(1,G)    of Eq.(7)
 *   load_node [nodes] tokens per node after deduplication = p^(1,U[1]) of Eq.(7)
 * Invalid slots are not counted; if `status` (device int32[1], may be NULL) is given it is
 * cleared and set to HM_ERR_BAD_ID when one is met.
 */
hm_status hm_expert_load(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                         hm_topology topo, int32_t *load_expert, int32_t *load_rank, int32_t *load_node,
                         int32_t *status, void *hip_stream);

/*
 * ---- Receiver side of the two-hop exchange (HD2: an Inter-node AlltoAll, then an Intra-node
 * AlltoAll, duplicates removed in both dimensions, Section III-A; the tokens a rank received
 * become the input of the next level, Alg.1's process()) -------------------------------------
 * A received row travels with the top-K expert ids and router weights of the token behind it
 * (pack them with hm_dispatch_pack like any other row: it copies bytes, H counts 2-byte units).
 * From hop to hop only the expert -> destination table changes.
 */
typedef enum {
  HM_RECV_INTRA_NODE = 0,   /* destinations: the ranks of my node (0..ranks_per_node-1)            */
  HM_RECV_LOCAL_EXPERTS = 1 /* destinations: the experts placed on my rank, ascending expert id    */
} hm_recv_stage;

/*
 * hm_recv_dest_map -- fills dest_map[E] (device) with the destination of every expert as seen from
 * `my_rank` at `stage`: INTRA_NODE: rank index inside my node for experts on my node, -1 for experts
 * on other nodes (their copies went elsewhere; the G-group mask of Eq.(7) restricted to my node's
 * contiguous groups).  LOCAL_EXPERTS: 0,1,2.. in ascending expert id for experts on my rank, else -1.
 * Placement entries outside [0,G) become -2.  num_dest (device int32[1]) receives ranks_per_node,
 * respectively the number of experts on my rank.  One small launch; call it when the placement
 * changes, not per layer.
 */
hm_status hm_recv_dest_map(const int32_t *expert_to_rank, int32_t E, hm_topology topo, int32_t my_rank,
                           hm_recv_stage stage, int32_t *dest_map, int32_t *num_dest, void *hip_stream);

/*
 * hm_level_dest_map -- the destination table of one hop of the d-dimensional exchange (Section
 * III-A/B: Inter-level-i, or the final Intra-level hop) seen from `my_rank`.  The G ranks are cut
 * into parent_groups (= U[i-1]) and child_groups (= U[i], or G for the Intra-level hop) contiguous
 * equal groups, parent | child | G <= 64.  dest_map[e] (device int32[E]) = index of the expert's
 * child group inside my parent group (0 .. child/parent - 1, the U[i]/U[i-1] peers of Eq.(4)) when
 * its rank lies in my parent group, -1 when it lies elsewhere, -2 for an invalid placement entry;
 * num_dest (device int32[1]) = child/parent.  parent = 1, child = nodes is the node-level cut of
 * hm_plan; parent = nodes, child = G equals HM_RECV_INTRA_NODE.  Feed the table to hm_plan_mapped.
 */
hm_status hm_level_dest_map(const int32_t *expert_to_rank, int32_t E, int32_t G, int32_t my_rank,
                            int32_t parent_groups, int32_t child_groups, int32_t *dest_map, int32_t *num_dest,
                            void *hip_stream);

/*
 * hm_plan_mapped -- hm_plan for an arbitrary expert -> destination table (device int32[E]):
 * dest_map[e] in [0,num_dest) is a destination, -1 means no copy at this hop (slot skipped without
 * error: slot_row = -1, slot_keep = 0), anything else -- or an id outside [0,E) -- is invalid
 * (skipped, HM_ERR_BAD_ID).  dedup != 0 keeps one row per (row, destination), the OR of Eq.(7);
 * dedup == 0 gives every valid slot a row of its own.  `rows` tokens (received rows) of K slots
 * each; num_dest <= 64.  Fills *out as hm_plan does; out->rank_mask, if given, receives the
 * per-row destination mask and out->node_mask zeros.  Workspace: hm_plan_mapped_workspace_bytes.
 */
size_t hm_plan_mapped_workspace_bytes(int32_t rows, int32_t K, int32_t num_dest);
hm_status hm_plan_mapped(const int32_t *row_ids, const float *row_weights, const int32_t *dest_map, int32_t rows,
                         int32_t K, int32_t E, int32_t num_dest, int32_t dedup, hm_plan_out *out /* host struct */,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * hm_combine_mix -- the merge a receiving rank does before it returns results one hop back: the
 * row it returns for a received token is the weight-normalised mixture of what came back for
 * that token's slots,
 *     out[i,:] = bf16( (sum_k w[i,k] * y[slot_row[i,k], :]) / (sum_k w[i,k]) ),   valid slots only,
 * fp32 accumulation, then a multiply by the fp32 reciprocal of the weight sum.  With these mixtures as the packed-layout y of the
 * previous hop, hm_combine at the source yields sum_k w_k f_k(x) (Section II-A).  A row without
 * a valid slot gives zeros.  Arguments as hm_combine (T = number of received rows).
 */
hm_status hm_combine_mix(const void *y_bf16, int64_t y_rows, const float *row_weights, int32_t T, int32_t K,
                         int32_t H, const hm_plan_out *plan, void *out_bf16, void *hip_stream);

/*
 * ---- Choosing the dimension of the hierarchical exchange (Section III-B/C, Alg.1) -------------
 *
 * hm_group_counts -- the duplicate-free counts of Eq.(7) for up to 4 group sizes in one pass over
 * the routing table: counts[l*64 + j] (device int32[depth*64], entries beyond groups[l] zeroed) =
 * number of tokens with a valid slot whose rank lies in group j when the G ranks are cut into
 * groups[l] (host array) contiguous equal groups; groups[l] must divide G <= 64.  groups = {G}
 * gives p of Eq.(2), groups = {U[i]} gives p^(i,U[i]) on this rank's tokens.  status: optional
 * device int32[1], cleared, set to HM_ERR_BAD_ID when an invalid slot is met (it is not counted).
 */
hm_status hm_group_counts(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                          int32_t G, int32_t depth, const int32_t *groups /* host */, int32_t *counts,
                          int32_t *status, void *hip_stream);

/*
 * hm_alltoall_times -- Eq.(1)-(6) on the device (no host round trip: the counts stay where the
 * plan kernels wrote them).  D <= 4 dimensions, U[0..D-1] (host) the group counts of the Inter-level
 * AlltoAlls with U[0] = 1, each dividing the next and G.
 *   p_inter[i*64 + j]  (device) tokens per U[i]-group at the input of Inter-level-i, 1 <= i < D
 *   p_intra[l*64 + j]  (device) tokens per GPU at the input of Intra-level-l, 0 <= l < D; l = 0 is the
 *                      one-dimensional exchange (p of Eq.(2))
 *   alpha/beta_inter[i], alpha/beta_intra[l] (host, D entries each): the linear model of Eq.(1) per
 *                      kind of AlltoAll; intra index 0 is the standard AlltoAll (as in Eq.(8))
 *   n_inter(i) = U[i]/U[i-1] * max(p_inter[i]) * M * v      n_intra(l) = G/U[l] * max(p_intra[l]) * M * v
 *   t_d = sum_{i<d} (alpha_inter[i] + n_inter(i) beta_inter[i]) + alpha_intra[d-1] + n_intra(d-1) beta_intra[d-1]
 *   d*  = 1 if t_1 < min_{d>1} t_d, else the lowest d > 1 with the smallest t_d
 * times (device double[4]) receives t_1..t_D, best (device int32[1]) receives d*.  fp64, evaluated
 * in the order written above without fused multiply-adds.
 */
hm_status hm_alltoall_times(int32_t D, const int32_t *U /* host */, int32_t G, double M, double v,
                            const int32_t *p_inter, const int32_t *p_intra, const double *alpha_inter /* host */,
                            const double *beta_inter /* host */, const double *alpha_intra /* host */,
                            const double *beta_intra /* host */, double *times, int32_t *best, void *hip_stream);

/*
 * ---- Hierarchical expert swap, HierD-ES (Section IV) ------------------------------------------
 *
 * hm_swap_counts -- the swap tensor of Section IV-A: Z[(r*E + c)*ng + j] (device int32) = the
 * duplicate-free number of tokens assigned to group j (the G ranks cut into ng contiguous equal
 * groups) after the positions of experts r and c are exchanged, for every pair.  Computed from
 * per-expert / per-(expert,group) / per-(expert,expert) co-occurrence counts (for E <= 256 as int8
 * matrix products over 0/1 indicator tiles on the matrix cores, beyond that with O(T K (K + ng))
 * atomic updates) instead of the paper's O(T K E) update: only the two groups involved in a swap
 * can change, and the change is
 *   +#{tokens selecting r, nothing in c's group}  -#{tokens where c is the only
 * selected expert of its group and r is not selected}  for c's group (and symmetrically).
 * A pair in which either expert's placement entry is outside [0,G) keeps the unswapped counts;
 * invalid slots are ignored; both set *status (optional device int32[1]) to HM_ERR_BAD_ID.
 * workspace: hm_swap_workspace_bytes(T, K, E, ng) bytes of device scratch (0 for arguments out of
 * range).
 */
size_t hm_swap_workspace_bytes(int32_t T, int32_t K, int32_t E, int32_t ng);
hm_status hm_swap_counts(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                         int32_t G, int32_t ng, int32_t *Z, int32_t *status, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/*
 * hm_swap_counts_multi -- hm_swap_counts for up to 4 cuts of the ranks in one pass over the tokens
 * (Section IV needs Z of every Inter-level cut U[i] and of the G-group cut for one Q): ng (host
 * array of ncuts group counts, each dividing G) and Z (host array of ncuts device pointers,
 * Z[c] = int32 [E*E*ng[c]]).  Results, status and error rules are those of ncuts separate
 * hm_swap_counts calls; the work that does not depend on the cut is done once.
 * workspace: hm_swap_multi_workspace_bytes(T, K, E, G, ncuts, ng) bytes of device scratch.
 */
size_t hm_swap_multi_workspace_bytes(int32_t T, int32_t K, int32_t E, int32_t G, int32_t ncuts,
                                     const int32_t *ng /* host */);
hm_status hm_swap_counts_multi(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                               int32_t G, int32_t ncuts, const int32_t *ng /* host */,
                               int32_t *const *Z /* host array of device pointers */, int32_t *status, void *workspace,
                               size_t workspace_bytes, void *hip_stream);

/*
 * hm_swap_select -- Eq.(8)-(10) for dimension d (1..4): the estimated time Q[r*E + c] (device
 * double[E*E]) of the d-dimensional exchange after swapping experts r and c, and the pair with
 * the smallest time (first in row-major order among equals): best_pair (device int32[2]),
 * best_time (device double[1]).
 *   z_inter (host array of d device pointers, entry 0 unused): z_inter[i] = Z of the U[i]-group cut;
 *   z_intra = Z of the G-group cut;  U, scale_inter, alpha_inter, beta_inter: host arrays of d entries.
 *   N_inter(i) = U[i]/U[i-1] * scale_inter[i] * smax(z_inter[i][r,c,:]) * M * v                Eq.(9)
 *   N_intra    = G/U[d-1]    * scale_intra    * smax(z_intra[r,c,:])    * M * v                Eq.(9)
 *   Q = sum_{i<d} (N_inter(i) beta_inter[i] + alpha_inter[i]) + N_intra beta_intra + alpha_intra   Eq.(8)
 * smax = max(x) * (sum_i (x_i/max(x))^gamma)^(1/gamma), Eq.(11); the plain maximum if gamma <= 0.
 * workspace: hm_swap_select_workspace_bytes(E) bytes of device scratch.
 */
size_t hm_swap_select_workspace_bytes(int32_t E);
hm_status hm_swap_select(int32_t d, const int32_t *U /* host */, int32_t G, int32_t E, double M, double v,
                         const int32_t *const *z_inter /* host array of device pointers */, const int32_t *z_intra,
                         const double *scale_inter /* host */, double scale_intra, const double *alpha_inter /* host */,
                         const double *beta_inter /* host */, double alpha_intra, double beta_intra, double gamma,
                         double *Q, int32_t *best_pair, double *best_time, void *workspace, size_t workspace_bytes,
                         void *hip_stream);

/*
 * hm_swap_apply -- carries out the chosen swap (Section IV: the positions of the two selected
 * experts are exchanged, once per planner step) without a host round trip: the entries
 * expert_to_rank[best_pair[0]] and expert_to_rank[best_pair[1]] (device int32[E], updated in place;
 * best_pair device int32[2], as written by hm_swap_select) trade places.  A pair on the diagonal
 * (the unswapped placement won Eq.(10)) or with an index outside [0,E) changes nothing.  Stream
 * order makes the next hm_plan / hm_swap_counts on the same stream see the new placement.
 */
hm_status hm_swap_apply(int32_t *expert_to_rank, int32_t E, const int32_t *best_pair, void *hip_stream);

/* Static, human-readable name of a status code. */
const char *hm_status_string(hm_status s);

#ifdef __cplusplus
}
#endif
#endif /* HIERMOE_H */
