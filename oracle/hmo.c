/*
 * hmo.c -- CPU oracle for hierarchical token deduplication (dispatch plan, pack, combine).
 *
 * TEST INFRASTRUCTURE ONLY.  Plain, slow, single-threaded C; no SIMD, no threads, no blocking
 * or fusion.  It exists so the HIP path can be checked against something written directly
 * from the paper; it shares no code with that path and the product never calls it.
 *
 * What the paper fixes (HierMoE, Section III-C, Eq.(7)): an expert group's routing mask is the
 * OR of its experts' masks, so a token is sent to a group at most once, and the duplicate-free
 * count of a group is the number of tokens whose group mask is set.  Groups are the G ranks
 * ("HD1", one group per GPU) or the U[1] nodes ("HD2" inter-node hop), Section III-A/III-B.
 * What the paper leaves open (row order, which duplicate survives, combine formula) is fixed
 * by the readings listed next to each function.
 *
 * All pointers are host pointers.  Every function returns 0 on success, a negative value on
 * an argument error (nothing written).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

enum { HMO_LEVEL_NONE = 0, HMO_LEVEL_GPU = 1, HMO_LEVEL_NODE = 2 };
enum { HMO_OK = 0, HMO_ERR_ARG = -1, HMO_BAD_ID = -7 };

/* Rank of one slot's expert, -1 when the expert id or its rank is out of range, -2 when the id
 * is the drop marker -1 (a router with a capacity limit marks the slots it dropped so: such a
 * slot is skipped everywhere without being an error).
 * Rank of an expert: expert_to_rank (contiguous blocks in Eq.(7); an arbitrary map here so that
 * an expert swap of Section IV is an exchange of two entries).  Node of a rank: rank / R, ranks
 * of one node being contiguous (Section III-B, the index illustration of Fig.6). */
static int slot_rank(const int32_t *expert_to_rank, int32_t E, int32_t G, int32_t id)
{
    if (id == -1) return -2;
    if (id < 0 || id >= E) return -1;
    int32_t g = expert_to_rank[id];
    if (g < 0 || g >= G) return -1;
    return g;
}

static int slot_dest(int rank, int32_t ranks_per_node, int32_t level)
{
    if (rank < 0) return -1;
    return level == HMO_LEVEL_NODE ? rank / ranks_per_node : rank;
}

/*
 * hmo_plan -- Eq.(7) turned into per-destination send lists for one rank's T tokens.
 *
 *  step 1  d(t,k)      destination of slot (t,k) at the level (rank for none/gpu, node for node).
 *  step 2  slot_keep   none: every valid slot.  gpu/node: a slot is kept iff no earlier slot
 *                      k' < k of the same token has the same destination -- the OR of Eq.(7)
 *                      leaves one copy per (token, group); "earlier slot wins" is this build's
 *                      reading (the paper only defines the OR).
 *  step 3  dest_count  p[j] = number of kept slots with destination j (second line of Eq.(7));
 *                      dest_offset = its exclusive prefix sum, dest_offset[Dn] = total rows.
 *  step 4  rows        kept slots are numbered inside their destination in ascending flat slot
 *                      index t*K+k (so: ascending token; at level none ties inside a token by k).
 *                      row_token[row] = t.  slot_row[t,k] = the row that carries token t to
 *                      d(t,k), for kept and non-kept slots alike; -1 for invalid slots.
 *  step 5  row_weight  fp32 sum, in ascending k, of the router weights of the slots a row serves.
 *  step 6  masks       rank_mask[t] = OR_k 1<<rank, node_mask[t] = OR_k 1<<node (level-free).
 *
 * Invalid slots (expert id outside [0,E), rank outside [0,G)) are dropped everywhere and
 * *status is set to HMO_BAD_ID; the id -1 marks a slot the router dropped and is skipped the same
 * way without an error.  rank_mask / node_mask may be NULL.
 * Buffers: dest_count[Dn], dest_offset[Dn+1], row_token/row_weight[>= T*K], slot_row/slot_keep[T*K].
 */
int hmo_plan(const int32_t *topk_ids, const float *topk_weights, const int32_t *expert_to_rank,
             int32_t T, int32_t K, int32_t E, int32_t nodes, int32_t ranks_per_node, int32_t level,
             int32_t *dest_count, int32_t *dest_offset, int32_t *row_token, int32_t *slot_row,
             uint8_t *slot_keep, float *row_weight, uint64_t *rank_mask, uint32_t *node_mask,
             int32_t *status)
{
    if (!topk_ids || !topk_weights || !expert_to_rank || !dest_count || !dest_offset || !row_token ||
        !slot_row || !slot_keep || !row_weight || !status)
        return HMO_ERR_ARG;
    if (T < 0 || K <= 0 || E <= 0 || nodes <= 0 || ranks_per_node <= 0) return HMO_ERR_ARG;
    if (level != HMO_LEVEL_NONE && level != HMO_LEVEL_GPU && level != HMO_LEVEL_NODE) return HMO_ERR_ARG;
    const int32_t G = nodes * ranks_per_node;
    if (G > 64 || nodes > 32) return HMO_ERR_ARG;
    const int32_t Dn = (level == HMO_LEVEL_NODE) ? nodes : G;

    *status = HMO_OK;
    int *dest = (int *)malloc(sizeof(int) * (size_t)(T > 0 ? T : 1) * (size_t)K);
    if (!dest) return HMO_ERR_ARG;

    /* steps 1, 2, 6 */
    for (int32_t t = 0; t < T; ++t) {
        uint64_t rm = 0;
        uint32_t nm = 0;
        for (int32_t k = 0; k < K; ++k) {
            const size_t s = (size_t)t * K + k;
            const int rank = slot_rank(expert_to_rank, E, G, topk_ids[s]);
            dest[s] = slot_dest(rank, ranks_per_node, level);
            if (rank < 0) {
                if (rank == -1) *status = HMO_BAD_ID;
                slot_keep[s] = 0;
                continue;
            }
            rm |= (uint64_t)1 << rank;
            nm |= (uint32_t)1 << (rank / ranks_per_node);
            int keep = 1;
            if (level != HMO_LEVEL_NONE)
                for (int32_t k1 = 0; k1 < k; ++k1)
                    if (dest[(size_t)t * K + k1] == dest[s]) keep = 0;
            slot_keep[s] = (uint8_t)keep;
        }
        if (rank_mask) rank_mask[t] = rm;
        if (node_mask) node_mask[t] = nm;
    }

    /* step 3 */
    for (int32_t d = 0; d < Dn; ++d) dest_count[d] = 0;
    for (size_t s = 0; s < (size_t)T * K; ++s)
        if (slot_keep[s]) dest_count[dest[s]] += 1;
    dest_offset[0] = 0;
    for (int32_t d = 0; d < Dn; ++d) dest_offset[d + 1] = dest_offset[d] + dest_count[d];

    /* step 4 */
    int32_t cursor[64];
    int32_t row_of[64];
    for (int32_t d = 0; d < Dn; ++d) cursor[d] = dest_offset[d];
    for (int32_t t = 0; t < T; ++t) {
        for (int32_t d = 0; d < Dn; ++d) row_of[d] = -1;
        for (int32_t k = 0; k < K; ++k) {
            const size_t s = (size_t)t * K + k;
            if (dest[s] < 0) { slot_row[s] = -1; continue; }
            if (slot_keep[s]) {
                const int32_t row = cursor[dest[s]]++;
                row_token[row] = t;
                row_of[dest[s]] = row;      /* at level none a later slot overwrites: each slot has its own row */
                slot_row[s] = row;
            } else {
                slot_row[s] = row_of[dest[s]];
            }
        }
    }

    /* step 5 */
    const int32_t total = dest_offset[Dn];
    uint8_t *seen = (uint8_t *)calloc((size_t)(total > 0 ? total : 1), 1);
    if (!seen) { free(dest); return HMO_ERR_ARG; }
    for (int32_t t = 0; t < T; ++t)
        for (int32_t k = 0; k < K; ++k) {
            const size_t s = (size_t)t * K + k;
            const int32_t row = slot_row[s];
            if (row < 0) continue;
            if (!seen[row]) { row_weight[row] = topk_weights[s]; seen[row] = 1; }
            else            { row_weight[row] = row_weight[row] + topk_weights[s]; }
        }
    free(seen);
    free(dest);
    return HMO_OK;
}

/*
 * hmo_dispatch_pack -- the deduplicated send buffer (Section III-A, the Fig.5 example): one copy
 * of token row_token[row] per packed row; destination d owns rows [dest_offset[d], dest_offset[d+1]).
 * Rows are `row_bytes` opaque bytes (bf16: 2*H).
 */
int hmo_dispatch_pack(const void *x, int64_t T, int64_t row_bytes, const int32_t *row_token,
                      int64_t n_rows, void *packed)
{
    if (!x || !row_token || !packed || T < 0 || row_bytes <= 0 || n_rows < 0) return HMO_ERR_ARG;
    const unsigned char *src = (const unsigned char *)x;
    unsigned char *dst = (unsigned char *)packed;
    for (int64_t row = 0; row < n_rows; ++row) {
        const int32_t t = row_token[row];
        if (t < 0 || t >= T) return HMO_ERR_ARG;
        for (int64_t b = 0; b < row_bytes; ++b) dst[row * row_bytes + b] = src[(int64_t)t * row_bytes + b];
    }
    return HMO_OK;
}

/* bf16 encoding -> double (exact). */
static double bf16_to_f64(uint16_t b)
{
    uint32_t u = (uint32_t)b << 16;
    float f;
    memcpy(&f, &u, sizeof f);
    return (double)f;
}

/*
 * Round a finite double to the nearest bf16 (8 exponent bits, 7 stored fraction bits), ties to
 * even, in ONE rounding: scale so that one bf16 ulp becomes 1.0, round to an integer with the
 * default rounding mode (nearest even), scale back.  Every intermediate is exact in binary64.
 */
static uint16_t f64_to_bf16_rne(double v)
{
    if (v != v) return 0x7FC0;
    if (v == 0.0) return signbit(v) ? 0x8000 : 0x0000;
    int e;
    (void)frexp(fabs(v), &e);          /* |v| = m * 2^e, m in [0.5,1)  ->  |v| in [2^(e-1), 2^e) */
    int ulp_exp = (e - 1) - 7;         /* ulp of a bf16 normal in that binade                      */
    if (ulp_exp < -133) ulp_exp = -133; /* subnormal spacing 2^-126 * 2^-7                          */
    const double q = nearbyint(ldexp(v, -ulp_exp));
    const double r = ldexp(q, ulp_exp);
    if (fabs(r) >= ldexp(1.0, 128)) return signbit(v) ? 0xFF80 : 0x7F80;
    const float f = (float)r;          /* exact: r has at most 8 significant bits */
    uint32_t u;
    memcpy(&u, &f, sizeof u);
    return (uint16_t)(u >> 16);
}

/*
 * hmo_combine -- the weighted merge of expert outputs (Section II-A/II-B: the layer output of a
 * token is the gate-weighted sum of its K experts' outputs; "AlltoAll Combine" brings them back).
 * Y has the packed layout, one row per (token, destination); slot (t,k) reads row slot_row[t,k]:
 *     out[t][j] = bf16( sum_k  w[t,k] * Y[slot_row[t,k]][j] ),   sum in binary64, ascending k,
 * rounded once to bf16.  Slots with slot_row < 0 (dropped) contribute nothing.
 */
int hmo_combine(const uint16_t *y, int64_t y_rows, const float *topk_weights, const int32_t *slot_row,
                int64_t T, int32_t K, int64_t H, uint16_t *out)
{
    if (!y || !topk_weights || !slot_row || !out || T < 0 || K <= 0 || H <= 0) return HMO_ERR_ARG;
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < H; ++j) {
            double acc = 0.0;
            for (int32_t k = 0; k < K; ++k) {
                const int64_t row = slot_row[t * K + k];
                if (row < 0) continue;
                if (row >= y_rows) return HMO_ERR_ARG;
                acc += (double)topk_weights[t * K + k] * bf16_to_f64(y[row * H + j]);
            }
            out[t * H + j] = f64_to_bf16_rne(acc);
        }
    return HMO_OK;
}

/*
 * hmo_combine_f32 -- hmo_combine for rows kept in binary32 (the element width of a row is free in
 * the paper: its cost model carries it as the `v` bytes per element of Section II-B):
 *     out[t][j] = (float)( sum_k  w[t,k] * Y[slot_row[t,k]][j] ),   sum in binary64, ascending k.
 * Every product of two binary32 values is exact in binary64; the K-term sum carries an error of at
 * most K * 2^-53 * sum_k |w*Y| before the single rounding to binary32 (K * 2^-29 of a binary32 ulp
 * at that magnitude, far inside the kernel tolerance).
 */
int hmo_combine_f32(const float *y, int64_t y_rows, const float *topk_weights, const int32_t *slot_row,
                    int64_t T, int32_t K, int64_t H, float *out)
{
    if (!y || !topk_weights || !slot_row || !out || T < 0 || K <= 0 || H <= 0) return HMO_ERR_ARG;
    for (int64_t t = 0; t < T; ++t)
        for (int64_t j = 0; j < H; ++j) {
            double acc = 0.0;
            for (int32_t k = 0; k < K; ++k) {
                const int64_t row = slot_row[t * K + k];
                if (row < 0) continue;
                if (row >= y_rows) return HMO_ERR_ARG;
                acc += (double)topk_weights[t * K + k] * (double)y[row * H + j];
            }
            out[t * H + j] = (float)acc;
        }
    return HMO_OK;
}

/*
 * hmo_combine_transpose -- adjoint of hmo_combine with respect to Y: the gradient of packed row
 * `row` is the row's aggregated router weight times the output gradient of its token,
 *     gy[row][j] = row_weight[row] * gout[row_token[row]][j]     (one binary32 multiply).
 */
int hmo_combine_transpose(const float *gout, int64_t T, int64_t H, const int32_t *row_token,
                          const float *row_weight, int64_t n_rows, float *gy)
{
    if (!gout || !row_token || !row_weight || !gy || T < 0 || H <= 0 || n_rows < 0) return HMO_ERR_ARG;
    for (int64_t row = 0; row < n_rows; ++row) {
        const int32_t t = row_token[row];
        if (t < 0 || t >= T) return HMO_ERR_ARG;
        for (int64_t j = 0; j < H; ++j) {
            volatile float p = row_weight[row] * gout[(int64_t)t * H + j];
            gy[row * H + j] = p;
        }
    }
    return HMO_OK;
}

/*
 * hmo_combine_transpose_bf16 -- the adjoint of hmo_combine for gradients kept in bf16 (the element
 * width of a row is free in the paper, Section II-B):
 *     gy[row][j] = bf16( row_weight[row] * gout[row_token[row]][j] ),
 * the exact product (a binary32 times a bf16 value has at most 32 significant bits: exact in
 * binary64) rounded once to bf16.
 */
int hmo_combine_transpose_bf16(const uint16_t *gout, int64_t T, int64_t H, const int32_t *row_token,
                               const float *row_weight, int64_t n_rows, uint16_t *gy)
{
    if (!gout || !row_token || !row_weight || !gy || T < 0 || H <= 0 || n_rows < 0) return HMO_ERR_ARG;
    for (int64_t row = 0; row < n_rows; ++row) {
        const int32_t t = row_token[row];
        if (t < 0 || t >= T) return HMO_ERR_ARG;
        for (int64_t j = 0; j < H; ++j)
            gy[row * H + j] = f64_to_bf16_rne((double)row_weight[row] * bf16_to_f64(gout[(int64_t)t * H + j]));
    }
    return HMO_OK;
}

/*
 * hmo_expert_load -- the counts an expert-swap planner consumes (Section IV): the raw number of
 * slots per expert (what duplicate-unaware planners count) and the duplicate-free number of tokens
 * per rank, p^(1,G), and per node, p^(1,U[1]), of Eq.(7).  Written from the set definition: a
 * token counts once for a group if any of its valid slots lands in the group.
 */
int hmo_expert_load(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                    int32_t nodes, int32_t ranks_per_node, int32_t *load_expert, int32_t *load_rank,
                    int32_t *load_node, int32_t *status)
{
    if (!topk_ids || !expert_to_rank || !load_expert || !load_rank || !load_node || !status) return HMO_ERR_ARG;
    if (T < 0 || K <= 0 || E <= 0 || nodes <= 0 || ranks_per_node <= 0) return HMO_ERR_ARG;
    const int32_t G = nodes * ranks_per_node;
    if (G > 64 || nodes > 32) return HMO_ERR_ARG;
    *status = HMO_OK;
    for (int32_t e = 0; e < E; ++e) load_expert[e] = 0;
    for (int32_t g = 0; g < G; ++g) load_rank[g] = 0;
    for (int32_t n = 0; n < nodes; ++n) load_node[n] = 0;
    for (int32_t t = 0; t < T; ++t) {
        int in_rank[64] = {0};
        int in_node[32] = {0};
        for (int32_t k = 0; k < K; ++k) {
            const int32_t id = topk_ids[(size_t)t * K + k];
            const int rank = slot_rank(expert_to_rank, E, G, id);
            if (rank < 0) { if (rank == -1) *status = HMO_BAD_ID; continue; }
            load_expert[id] += 1;
            in_rank[rank] = 1;
            in_node[rank / ranks_per_node] = 1;
        }
        for (int32_t g = 0; g < G; ++g) load_rank[g] += in_rank[g];
        for (int32_t n = 0; n < nodes; ++n) load_node[n] += in_node[n];
    }
    return HMO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Receiver side of the two-hop exchange (HD2, Section III-A: an Inter-node AlltoAll followed by an
 * Intra-node AlltoAll, duplicates removed in both dimensions; Alg.1's process() step: the tokens a
 * rank received become the input of the next level).  A received row carries the top-K expert
 * ids and router weights of the token behind it; what changes from hop to hop is only the map
 * from an expert to a destination of that hop.
 * ------------------------------------------------------------------------------------------------ */
enum { HMO_RECV_INTRA_NODE = 0, HMO_RECV_LOCAL_EXPERTS = 1 };

/*
 * hmo_recv_dest_map -- destination of every expert as seen from rank `my_rank` at a stage:
 *   INTRA_NODE     experts on a rank of my node -> that rank's index inside the node (0..R-1);
 *                  experts on other nodes -> -1 (their copies travelled to other nodes).
 *                  The rank groups of one node are contiguous (Section III-B), so this is the
 *                  G-group mask of Eq.(7) restricted to the G/U[1] groups of my node.
 *   LOCAL_EXPERTS  experts placed on my rank -> 0,1,2,.. in ascending expert id; all others -> -1.
 * Placement entries outside [0,G) map to -2 (invalid).  *num_dest receives R, respectively the
 * number of experts on my rank.
 */
int hmo_recv_dest_map(const int32_t *expert_to_rank, int32_t E, int32_t nodes, int32_t ranks_per_node,
                      int32_t my_rank, int32_t stage, int32_t *dest_map, int32_t *num_dest)
{
    if (!expert_to_rank || !dest_map || !num_dest || E <= 0 || nodes <= 0 || ranks_per_node <= 0) return HMO_ERR_ARG;
    const int32_t G = nodes * ranks_per_node;
    if (my_rank < 0 || my_rank >= G) return HMO_ERR_ARG;
    if (stage != HMO_RECV_INTRA_NODE && stage != HMO_RECV_LOCAL_EXPERTS) return HMO_ERR_ARG;
    int32_t next_local = 0;
    for (int32_t e = 0; e < E; ++e) {
        const int32_t g = expert_to_rank[e];
        if (g < 0 || g >= G) { dest_map[e] = -2; continue; }
        if (stage == HMO_RECV_INTRA_NODE)
            dest_map[e] = (g / ranks_per_node == my_rank / ranks_per_node) ? g % ranks_per_node : -1;
        else
            dest_map[e] = (g == my_rank) ? next_local++ : -1;
    }
    *num_dest = (stage == HMO_RECV_INTRA_NODE) ? ranks_per_node : next_local;
    return HMO_OK;
}

/*
 * hmo_level_dest_map -- the destination table of one hop of the d-dimensional exchange (Section
 * III-A/B: Inter-level-i, or the final Intra-level, seen from `my_rank`).  The G ranks are cut into
 * parent_groups (= U[i-1]) and into child_groups (= U[i], or G for the Intra-level hop) contiguous
 * equal groups, parent | child | G.  Experts whose rank lies in my parent group map to the index
 * of their child group inside that parent, 0 .. child/parent - 1 -- these are the U[i]/U[i-1]
 * peers of Eq.(4) (G/U[d-1] peers in Eq.(5)); experts in other parent groups map to -1 (their
 * copies were routed elsewhere by an earlier hop); invalid placement entries to -2.
 * parent = 1, child = nodes is the sender's node-level cut; parent = nodes, child = G is the
 * intra-node hop of HD2.
 */
int hmo_level_dest_map(const int32_t *expert_to_rank, int32_t E, int32_t G, int32_t my_rank, int32_t parent_groups,
                       int32_t child_groups, int32_t *dest_map, int32_t *num_dest)
{
    if (!expert_to_rank || !dest_map || !num_dest || E <= 0 || G <= 0 || G > 64) return HMO_ERR_ARG;
    if (my_rank < 0 || my_rank >= G || parent_groups < 1 || child_groups < parent_groups || child_groups > G) return HMO_ERR_ARG;
    if (child_groups % parent_groups != 0 || G % child_groups != 0) return HMO_ERR_ARG;
    const int32_t ranks_per_parent = G / parent_groups, ranks_per_child = G / child_groups;
    const int32_t children_per_parent = child_groups / parent_groups;
    for (int32_t e = 0; e < E; ++e) {
        const int32_t g = expert_to_rank[e];
        if (g < 0 || g >= G) dest_map[e] = -2;
        else if (g / ranks_per_parent != my_rank / ranks_per_parent) dest_map[e] = -1;
        else dest_map[e] = (g / ranks_per_child) % children_per_parent;
    }
    *num_dest = children_per_parent;
    return HMO_OK;
}

/*
 * hmo_plan_mapped -- the plan of hmo_plan for an arbitrary expert -> destination table:
 * dest_map[e] in [0,num_dest) is a destination, -1 means "no copy at this hop" (the slot is
 * skipped without error: slot_row = -1, slot_keep = 0), anything else or an id outside [0,E) is
 * invalid (skipped, *status = HMO_BAD_ID).  dedup != 0 keeps one row per (row, destination) as in
 * Eq.(7), the lowest k owning it; dedup == 0 gives every valid slot its own row.  Everything else
 * (counts, offsets, stable order, row weights) is as in hmo_plan.  dest_mask[i] (optional) gets
 * bit d set iff row i has a valid slot for destination d.
 */
int hmo_plan_mapped(const int32_t *ids, const float *weights, const int32_t *dest_map, int32_t rows, int32_t K,
                    int32_t E, int32_t num_dest, int32_t dedup, int32_t *dest_count, int32_t *dest_offset,
                    int32_t *row_token, int32_t *slot_row, uint8_t *slot_keep, float *row_weight,
                    uint64_t *dest_mask, int32_t *status)
{
    if (!ids || !weights || !dest_map || !dest_count || !dest_offset || !row_token || !slot_row || !slot_keep ||
        !row_weight || !status)
        return HMO_ERR_ARG;
    if (rows < 0 || K <= 0 || E <= 0 || num_dest <= 0 || num_dest > 64) return HMO_ERR_ARG;
    *status = HMO_OK;
    for (int32_t d = 0; d < num_dest; ++d) dest_count[d] = 0;
    /* destination of every slot, ownership flags, counts */
    for (int32_t i = 0; i < rows; ++i) {
        uint64_t mask = 0;
        for (int32_t k = 0; k < K; ++k) {
            const size_t s = (size_t)i * K + k;
            const int32_t id = ids[s];
            int32_t d = -1;
            if (id == -1) d = -1;                  /* drop marker: skipped silently */
            else if (id < 0 || id >= E) *status = HMO_BAD_ID;
            else if (dest_map[id] >= 0 && dest_map[id] < num_dest) d = dest_map[id];
            else if (dest_map[id] != -1) *status = HMO_BAD_ID;
            slot_row[s] = d;                       /* holds the destination until rows are numbered */
            int keep = d >= 0;
            if (keep && dedup)
                for (int32_t k1 = 0; k1 < k; ++k1)
                    if (slot_row[(size_t)i * K + k1] == d) keep = 0;
            slot_keep[s] = (uint8_t)keep;
            if (keep) dest_count[d] += 1;
            if (d >= 0) mask |= (uint64_t)1 << d;
        }
        if (dest_mask) dest_mask[i] = mask;
    }
    dest_offset[0] = 0;
    for (int32_t d = 0; d < num_dest; ++d) dest_offset[d + 1] = dest_offset[d] + dest_count[d];
    /* number the rows: ascending flat slot index inside each destination */
    int32_t cursor[64], row_of[64];
    for (int32_t d = 0; d < num_dest; ++d) cursor[d] = dest_offset[d];
    for (int32_t i = 0; i < rows; ++i) {
        for (int32_t d = 0; d < num_dest; ++d) row_of[d] = -1;
        for (int32_t k = 0; k < K; ++k) {
            const size_t s = (size_t)i * K + k;
            const int32_t d = slot_row[s];
            if (d < 0) continue;                   /* stays -1 */
            if (slot_keep[s]) {
                const int32_t row = cursor[d]++;
                row_token[row] = i;
                row_weight[row] = weights[s];
                row_of[d] = row;
                slot_row[s] = row;
            } else {
                slot_row[s] = row_of[d];
                row_weight[row_of[d]] = row_weight[row_of[d]] + weights[s];   /* ascending k, binary32 */
            }
        }
    }
    return HMO_OK;
}

/*
 * hmo_combine_mix -- the merge a receiving rank performs before it sends results back one hop:
 * the row it returns for a received token is the weight-normalised mixture of what came back
 * for that token's slots,
 *     out[i][j] = bf16( (sum_k w[i,k] * Y[slot_row[i,k]][j]) / (sum_k w[i,k]) ),
 * both sums over the slots with slot_row >= 0, in binary64, rounded once.  With these mixtures
 * as the packed-layout Y of the previous hop, hmo_combine at the source reproduces
 * sum_k w_k f_k(x) exactly (up to the bf16 roundings of the rows in flight).  A row without a
 * valid slot gives zeros.
 */
int hmo_combine_mix(const uint16_t *y, int64_t y_rows, const float *weights, const int32_t *slot_row,
                    int64_t rows, int32_t K, int64_t H, uint16_t *out)
{
    if (!y || !weights || !slot_row || !out || rows < 0 || K <= 0 || H <= 0) return HMO_ERR_ARG;
    for (int64_t i = 0; i < rows; ++i) {
        double wsum = 0.0;
        for (int32_t k = 0; k < K; ++k)
            if (slot_row[i * K + k] >= 0) wsum += (double)weights[i * K + k];
        for (int64_t j = 0; j < H; ++j) {
            double acc = 0.0;
            for (int32_t k = 0; k < K; ++k) {
                const int64_t row = slot_row[i * K + k];
                if (row < 0) continue;
                if (row >= y_rows) return HMO_ERR_ARG;
                acc += (double)weights[i * K + k] * bf16_to_f64(y[row * H + j]);
            }
            out[i * H + j] = f64_to_bf16_rne(wsum != 0.0 ? acc / wsum : 0.0);
        }
    }
    return HMO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Choosing the dimension of the hierarchical exchange (Section III-B/C, Eq.(1)-(6), Alg.1).
 * ------------------------------------------------------------------------------------------------ */

/*
 * hmo_group_counts -- the duplicate-free counts of Eq.(7) for several group sizes at once:
 * counts[l*64 + j] = number of tokens with a valid slot whose rank lies in group j when the G
 * ranks are cut into groups[l] contiguous equal groups (groups[l] must divide G).  groups = {G}
 * gives p of Eq.(2); groups = {U[i]} gives p^(i,U[i]) on this rank's own tokens.
 */
int hmo_group_counts(const int32_t *topk_ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                     int32_t G, int32_t depth, const int32_t *groups, int32_t *counts, int32_t *status)
{
    if (!topk_ids || !expert_to_rank || !groups || !counts || !status) return HMO_ERR_ARG;
    if (T < 0 || K <= 0 || E <= 0 || G <= 0 || G > 64 || depth < 1 || depth > 4) return HMO_ERR_ARG;
    for (int32_t l = 0; l < depth; ++l)
        if (groups[l] < 1 || groups[l] > G || G % groups[l] != 0) return HMO_ERR_ARG;
    *status = HMO_OK;
    for (int32_t i = 0; i < depth * 64; ++i) counts[i] = 0;
    for (int32_t t = 0; t < T; ++t)
        for (int32_t l = 0; l < depth; ++l) {
            int in_group[64] = {0};
            const int32_t ranks_per_group = G / groups[l];
            for (int32_t k = 0; k < K; ++k) {
                const int rank = slot_rank(expert_to_rank, E, G, topk_ids[(size_t)t * K + k]);
                if (rank < 0) { if (rank == -1) *status = HMO_BAD_ID; continue; }
                in_group[rank / ranks_per_group] = 1;
            }
            for (int32_t j = 0; j < groups[l]; ++j) counts[l * 64 + j] += in_group[j];
        }
    return HMO_OK;
}

static double max_count(const int32_t *p, int32_t n)
{
    int32_t m = 0;
    for (int32_t j = 0; j < n; ++j)
        if (p[j] > m) m = p[j];
    return (double)m;
}

/*
 * hmo_alltoall_times -- estimated time of the d-dimensional deduplicated exchange for d = 1..D and
 * the dimension to use.
 *   U[0..D-1]      group counts of the Inter-level AlltoAlls, U[0] = 1 (Section III-B)
 *   p_inter[i*64+j] duplicate-free tokens per U[i]-group at the input of Inter-level-i, 1 <= i < D
 *   p_intra[l*64+j] duplicate-free tokens per GPU at the input of Intra-level-l, 0 <= l < D
 *                  (l = 0: the one-dimensional exchange, p of Eq.(2))
 *   alpha/beta_inter[i], alpha/beta_intra[l]: the linear model of Eq.(1) per kind of AlltoAll;
 *                  index 0 of the intra arrays is the standard AlltoAll (the convention of Eq.(8))
 *   n_inter(i) = U[i]/U[i-1] * max(p_inter[i]) * M * v                              Eq.(4)
 *   n_intra(l) = G/U[l]      * max(p_intra[l]) * M * v                              Eq.(2),(5)
 *   t_d = sum_{i=1}^{d-1} (alpha_inter[i] + n_inter(i) beta_inter[i])
 *         + alpha_intra[d-1] + n_intra(d-1) beta_intra[d-1]                         Eq.(1),(3)
 *   d* = 1 if t_1 < min_{d>1} t_d, else the (lowest) d > 1 with the smallest t_d    Eq.(6)
 * times[d-1] receives t_d; *best receives d*.
 */
int hmo_alltoall_times(int32_t D, const int32_t *U, int32_t G, double M, double v, const int32_t *p_inter,
                       const int32_t *p_intra, const double *alpha_inter, const double *beta_inter,
                       const double *alpha_intra, const double *beta_intra, double *times, int32_t *best)
{
    if (!U || !p_inter || !p_intra || !alpha_inter || !beta_inter || !alpha_intra || !beta_intra || !times || !best)
        return HMO_ERR_ARG;
    if (D < 1 || D > 4 || G < 1 || G > 64 || U[0] != 1) return HMO_ERR_ARG;
    for (int32_t i = 1; i < D; ++i)
        if (U[i] < U[i - 1] || U[i] > G || U[i] % U[i - 1] != 0 || G % U[i] != 0) return HMO_ERR_ARG;
    for (int32_t d = 1; d <= D; ++d) {
        double t = 0.0;
        for (int32_t i = 1; i <= d - 1; ++i) {
            const double n = (double)(U[i] / U[i - 1]) * max_count(p_inter + i * 64, U[i]) * M * v;
            t = t + (alpha_inter[i] + n * beta_inter[i]);
        }
        const double n = (double)(G / U[d - 1]) * max_count(p_intra + (d - 1) * 64, G) * M * v;
        t = t + (alpha_intra[d - 1] + n * beta_intra[d - 1]);
        times[d - 1] = t;
    }
    int32_t arg = 1;
    if (D > 1) {
        arg = 2;
        for (int32_t d = 3; d <= D; ++d)
            if (times[d - 1] < times[arg - 1]) arg = d;
        if (times[0] < times[arg - 1]) arg = 1;
    }
    *best = arg;
    return HMO_OK;
}

/* ------------------------------------------------------------------------------------------------
 * Hierarchical expert swap, HierD-ES (Section IV, Eq.(8)-(11)).
 * ------------------------------------------------------------------------------------------------ */

/* Duplicate-free tokens per group for a placement, ranks cut into ng contiguous groups; slots with
 * an invalid id or placement entry are ignored.  (Eq.(7) by sets.) */
static void count_groups(const int32_t *ids, const int32_t *placement, int32_t T, int32_t K, int32_t E, int32_t G,
                         int32_t ng, int32_t *out)
{
    const int32_t per = G / ng;
    for (int32_t j = 0; j < ng; ++j) out[j] = 0;
    for (int32_t t = 0; t < T; ++t) {
        int in_group[64] = {0};
        for (int32_t k = 0; k < K; ++k) {
            const int rank = slot_rank(placement, E, G, ids[(size_t)t * K + k]);
            if (rank >= 0) in_group[rank / per] = 1;
        }
        for (int32_t j = 0; j < ng; ++j) out[j] += in_group[j];
    }
}

/*
 * hmo_swap_counts_naive -- the definition of Z (Section IV-A): Z[r][c][j] = duplicate-free number
 * of tokens assigned to group j after the positions of experts r and c are exchanged, i.e. the
 * counts of Eq.(7) under the placement with entries r and c swapped.  O(E^2 T K).
 * A pair in which either expert has no valid placement keeps the unswapped counts, and *status
 * is set to HMO_BAD_ID (as for any invalid slot).
 */
int hmo_swap_counts_naive(const int32_t *ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                          int32_t G, int32_t ng, int32_t *Z, int32_t *status)
{
    if (!ids || !expert_to_rank || !Z || !status) return HMO_ERR_ARG;
    if (T < 0 || K <= 0 || E <= 0 || G <= 0 || G > 64 || ng < 1 || ng > G || G % ng != 0) return HMO_ERR_ARG;
    *status = HMO_OK;
    for (size_t s = 0; s < (size_t)T * K; ++s)
        if (slot_rank(expert_to_rank, E, G, ids[s]) == -1) *status = HMO_BAD_ID;
    int32_t *placement = (int32_t *)malloc(sizeof(int32_t) * (size_t)E);
    if (!placement) return HMO_ERR_ARG;
    for (int32_t r = 0; r < E; ++r)
        for (int32_t c = 0; c < E; ++c) {
            for (int32_t e = 0; e < E; ++e) placement[e] = expert_to_rank[e];
            const int valid_r = expert_to_rank[r] >= 0 && expert_to_rank[r] < G;
            const int valid_c = expert_to_rank[c] >= 0 && expert_to_rank[c] < G;
            if (valid_r && valid_c) {
                placement[r] = expert_to_rank[c];
                placement[c] = expert_to_rank[r];
            } else {
                *status = HMO_BAD_ID;
            }
            count_groups(ids, placement, T, K, E, G, ng, Z + ((size_t)r * E + c) * ng);
        }
    free(placement);
    return HMO_OK;
}

/*
 * hmo_swap_counts_incremental -- the paper's O(T K E) procedure (Section IV-A, the four cases of
 * Fig.8): start every Z[r][c][:] from the counts without a swap; then for every token and every
 * pair (A selected, B not selected) in different groups:
 *   the group of B gains the token unless the token already selects an expert there (cases 1,2 / 3,4);
 *   the group of A loses the token if A is its only selected expert there (cases 2,4 / 1,3).
 * Pairs both selected or both unselected change nothing.  The update goes to Z[A][B] and Z[B][A].
 */
int hmo_swap_counts_incremental(const int32_t *ids, const int32_t *expert_to_rank, int32_t T, int32_t K, int32_t E,
                                int32_t G, int32_t ng, int32_t *Z, int32_t *status)
{
    if (!ids || !expert_to_rank || !Z || !status) return HMO_ERR_ARG;
    if (T < 0 || K <= 0 || E <= 0 || G <= 0 || G > 64 || ng < 1 || ng > G || G % ng != 0) return HMO_ERR_ARG;
    *status = HMO_OK;
    const int32_t per = G / ng;
    int32_t base[64];
    count_groups(ids, expert_to_rank, T, K, E, G, ng, base);
    for (int32_t e = 0; e < E; ++e)
        if (expert_to_rank[e] < 0 || expert_to_rank[e] >= G) *status = HMO_BAD_ID;
    for (size_t rc = 0; rc < (size_t)E * E; ++rc)
        for (int32_t j = 0; j < ng; ++j) Z[rc * ng + j] = base[j];
    uint8_t *selected = (uint8_t *)malloc((size_t)E);
    if (!selected) return HMO_ERR_ARG;
    for (int32_t t = 0; t < T; ++t) {
        int in_group[64] = {0};                       /* selected experts of the token per group */
        for (int32_t e = 0; e < E; ++e) selected[e] = 0;
        for (int32_t k = 0; k < K; ++k) {
            const int32_t id = ids[(size_t)t * K + k];
            const int rank = slot_rank(expert_to_rank, E, G, id);
            if (rank < 0) { if (rank == -1) *status = HMO_BAD_ID; continue; }
            if (!selected[id]) { selected[id] = 1; in_group[rank / per] += 1; }
        }
        for (int32_t a = 0; a < E; ++a) {
            if (!selected[a]) continue;
            const int32_t ga = expert_to_rank[a] / per;
            for (int32_t b = 0; b < E; ++b) {
                if (selected[b]) continue;
                if (expert_to_rank[b] < 0 || expert_to_rank[b] >= G) continue;   /* pair keeps the unswapped counts */
                const int32_t gb = expert_to_rank[b] / per;
                if (ga == gb) continue;
                const int gain = in_group[gb] == 0;   /* B's group had none of the token's experts   */
                const int loss = in_group[ga] == 1;   /* A was the token's only expert in its group  */
                int32_t *zab = Z + ((size_t)a * E + b) * ng, *zba = Z + ((size_t)b * E + a) * ng;
                zab[gb] += gain; zba[gb] += gain;
                zab[ga] -= loss; zba[ga] -= loss;
            }
        }
    }
    free(selected);
    return HMO_OK;
}

/* Eq.(11): max(x) * (sum_i (x_i/max(x))^gamma)^(1/gamma); the plain maximum for gamma <= 0. */
static double smooth_max(const int32_t *x, int32_t n, double gamma)
{
    const double m = max_count(x, n);
    if (gamma <= 0.0 || m == 0.0) return m;
    double sum = 0.0;
    for (int32_t i = 0; i < n; ++i) sum += pow((double)x[i] / m, gamma);
    return m * pow(sum, 1.0 / gamma);
}

/*
 * hmo_swap_select -- Eq.(8)-(10) for one dimension d: the estimated time of the d-dimensional
 * exchange after swapping experts r and c, for every pair, and the pair that minimises it.
 *   z_inter[i] (1 <= i < d): Z of the U[i]-group cut, [E][E][U[i]];  z_intra: Z of the G-group cut.
 *   scale_inter[i], scale_intra: multipliers on the counts (the fan-in of the level; 1 for own counts)
 *   N_inter(i)[r,c] = U[i]/U[i-1] * scale_inter[i] * smax(z_inter[i][r,c,:]) * M * v            Eq.(9)
 *   N_intra[r,c]    = G/U[d-1]    * scale_intra    * smax(z_intra[r,c,:])    * M * v            Eq.(9)
 *   Q[r,c] = sum_{i<d} (N_inter(i) beta_inter[i] + alpha_inter[i]) + N_intra beta_intra + alpha_intra   Eq.(8)
 *   (r*,c*) = argmin Q, the first pair in row-major order among equals                          Eq.(10)
 * smax is the smooth maximum of Eq.(11) with parameter gamma (plain max if gamma <= 0).
 */
int hmo_swap_select(int32_t d, const int32_t *U, int32_t G, int32_t E, double M, double v,
                    const int32_t *const *z_inter, const int32_t *z_intra, const double *scale_inter,
                    double scale_intra, const double *alpha_inter, const double *beta_inter, double alpha_intra,
                    double beta_intra, double gamma, double *Q, int32_t *best_pair, double *best_time)
{
    if (!U || !z_intra || !Q || !best_pair || !best_time) return HMO_ERR_ARG;
    if (d < 1 || d > 4 || E < 1 || G < 1 || G > 64 || U[0] != 1) return HMO_ERR_ARG;
    if (d > 1 && (!z_inter || !scale_inter || !alpha_inter || !beta_inter)) return HMO_ERR_ARG;
    for (int32_t i = 1; i < d; ++i)
        if (!z_inter[i] || U[i] < U[i - 1] || U[i] % U[i - 1] != 0 || G % U[i] != 0) return HMO_ERR_ARG;
    double best = 0.0;
    int32_t br = -1, bc = -1;
    for (int32_t r = 0; r < E; ++r)
        for (int32_t c = 0; c < E; ++c) {
            const size_t rc = (size_t)r * E + c;
            double q = 0.0;
            for (int32_t i = 1; i < d; ++i) {
                const double n = (double)(U[i] / U[i - 1]) * scale_inter[i] * smooth_max(z_inter[i] + rc * U[i], U[i], gamma) * M * v;
                q = q + (n * beta_inter[i] + alpha_inter[i]);
            }
            const double n = (double)(G / U[d - 1]) * scale_intra * smooth_max(z_intra + rc * G, G, gamma) * M * v;
            q = q + (n * beta_intra + alpha_intra);
            Q[rc] = q;
            if (br < 0 || q < best) { best = q; br = r; bc = c; }
        }
    best_pair[0] = br;
    best_pair[1] = bc;
    *best_time = best;
    return HMO_OK;
}

/*
 * hmo_swap_apply -- carry out the chosen swap (Section IV: the positions of the two selected
 * experts are exchanged, once per planner step): the placement entries of experts pair[0] and
 * pair[1] trade places.  A pair on the diagonal (the unswapped placement won Eq.(10)) or with an
 * index outside [0,E) changes nothing.
 */
int hmo_swap_apply(int32_t *expert_to_rank, int32_t E, const int32_t *pair)
{
    if (!expert_to_rank || !pair || E < 1) return HMO_ERR_ARG;
    const int32_t r = pair[0], c = pair[1];
    if (r < 0 || r >= E || c < 0 || c >= E || r == c) return HMO_OK;
    const int32_t g = expert_to_rank[r];
    expert_to_rank[r] = expert_to_rank[c];
    expert_to_rank[c] = g;
    return HMO_OK;
}

/* Exposed so tests can pin the rounding routine by itself. */
uint16_t hmo_f64_to_bf16(double v) { return f64_to_bf16_rne(v); }
