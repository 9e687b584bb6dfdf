/*
 * squeezed_attention.h -- C ABI of the MI355X (gfx950) implementation of the online path of
 * Squeezed Attention (arxiv 2411.09688): centroid scoring, threshold selection with key-range
 * compaction, sparse flash attention for decode and prefill, and the two-level centroid lookup.
 *
 * Conventions shared by every entry point
 *   - Every tensor pointer is a DEVICE pointer owned by the caller, contiguous in the stated
 *     layout, 16-byte aligned, and never retained after the call returns.
 *   - fp16 tensors are IEEE binary16 passed as `const void*`; "f32"/"i32"/"u32" are 4-byte types.
 *   - `stream` is a hipStream_t passed as void* (NULL = the default stream).  Calls only enqueue
 *     work on it and never synchronise; outputs are valid once the stream reaches that point.
 *   - The library allocates nothing.  Scratch is a caller-provided device workspace `ws` of at
 *     least sq_workspace_bytes(shape, which) bytes, 256-byte aligned; its contents are private to
 *     one call and may be reused afterwards.  Two calls that share a workspace must be ordered on
 *     the same stream.
 *   - Return value: SQ_OK or a negative sq_status; sq_last_error() gives a thread-local message.
 *     Invalid arguments are rejected on the host before anything is enqueued.
 *   - Empty selections, zero-size clusters and U == 0 are legal inputs and never fault.
 *
 * Data layout of the fixed context (Section 3.1: keys are clustered offline; here they are stored
 * sorted by cluster id, so a cluster is a contiguous key range):
 *   K_fixed, V_fixed  f16 [H, L, d]      keys/values of the fixed context, shared by all B sequences
 *   centroids         f16 [H, C, d]      mean key of each cluster
 *   sizes             i32 [H, C]         N_i, number of keys in cluster i (0 allowed)
 *   offsets           i32 [H, C+1]       exclusive prefix sum of sizes; cluster i = keys
 *                                        [offsets[i], offsets[i] + sizes[i])
 *   thresh            f32 [H]            threshold T per head (a global T is a broadcast)
 * Queries q are f16 [B, H, Lq, d]; user / generated keys K_user, V_user are f16 [B, H, U, d].
 */
#ifndef SQUEEZED_ATTENTION_H
#define SQUEEZED_ATTENTION_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum sq_status {
    SQ_OK = 0,
    SQ_ERR_INVALID_ARG = -1, /* null pointer, misalignment, non-positive dimension, bad enum */
    SQ_ERR_UNSUPPORTED = -2, /* d != 128, Lq != 1 where decode is required, device is not gfx950 */
    SQ_ERR_WORKSPACE = -3,   /* ws == NULL or ws_bytes too small */
    SQ_ERR_HIP = -4          /* a launch or runtime call failed; see sq_last_error() */
} sq_status;

typedef enum sq_call {
    SQ_CALL_CENTROID_SCORE = 0,
    SQ_CALL_SELECT = 1,
    SQ_CALL_ATTN_DECODE = 2,
    SQ_CALL_ATTN_PREFILL = 3,
    SQ_CALL_HIER_SELECT = 4,
    SQ_CALL_DECODE_STEP = 5,
    SQ_CALL_HIER_DECODE_STEP = 6,
    SQ_CALL_SELECT_MEAN = 7,
    SQ_CALL_ATTN_PREFILL_SHARED = 8,
    SQ_CALL_PREFILL_STEP = 9,
    SQ_CALL_PREFILL_MEAN_STEP = 10,
    SQ_CALL_GQA_DECODE_STEP = 11,
    SQ_CALL_MULTILEVEL_SELECT = 12,
    SQ_CALL_MULTILEVEL_DECODE_STEP = 13,
    SQ_CALL_KMEANS_STEP = 14,
    SQ_CALL_CALIBRATE = 15,
    SQ_CALL_HIER_PREFILL_MEAN_STEP = 16,
    SQ_CALL_GQA_MEAN_DECODE_STEP = 17,
    SQ_CALL_HIER_PREFILL_STEP = 18
} sq_call;

/*
 * Problem shape.  B sequences, H heads, head dim d (must be 128), L fixed-context keys per head,
 * C clusters per head (the fine level C2 for the two-level calls), Lq queries per sequence
 * (1 in decode), U user keys per sequence.  sm_scale multiplies every logit, both q.C_i in Eq. 1
 * and q.k_j in attention (Eq. 1 is an estimate of the attention softmax, so it takes the same
 * scale; sm_scale = 1 gives the equation as printed).  causal_user != 0: query t sees user keys
 * 0..t only (prefill; the user input follows the fixed context, which stays fully visible).
 */
typedef struct sq_shape_t {
    int32_t B, H, d, L, C, Lq, U;
    float sm_scale;
    int32_t causal_user;
} sq_shape_t;

/* Bytes of workspace the given call needs for this shape (0 if none).  Host only. */
size_t sq_workspace_bytes(const sq_shape_t *shape, int which_call);

/* Message of the last error raised on the calling thread ("" if none).  Host only. */
const char *sq_last_error(void);

/* Library version, major*10000 + minor*100 + patch. */
int sq_version(void);

/*
 * Cluster scores of Eq. 1 (Section 3.2) in the max-subtracted form of Appendix D
 * ("Generation Stage"): for every query row r = (b, h, t)
 *     logits[r, i] = sm_scale * sum_u q[r, u] * centroids[h, i, u]          (fp32 accumulation)
 *     row_max[r]   = max over clusters with sizes > 0 of logits[r, i]       (-inf if none)
 *     denom[r]     = sum_i sizes[h, i] * exp(logits[r, i] - row_max[r])     (D of Appendix D)
 * so that S_i = exp(logits[r,i] - row_max[r]) / denom[r].
 * Out: logits f32 [B,H,Lq,C], row_max f32 [B,H,Lq], denom f32 [B,H,Lq].  No workspace needed
 * (ws may be NULL).
 */
int sq_centroid_score(const sq_shape_t *shape, const void *q, const void *centroids, const int32_t *sizes,
                      float *logits, float *row_max, float *denom,
                      void *ws, size_t ws_bytes, void *stream);

/*
 * Threshold rule of Sections 3.2 / 4.1 ("load cluster i iff S_i > T", strict), evaluated without a
 * division as exp(logits - row_max) > T * denom (Appendix D), followed by compaction of the kept
 * clusters into key ranges (the key-index tensor of Section 4.2, as ranges because clusters are
 * contiguous).  Clusters with sizes == 0 are never kept.
 * Out: keep_mask u32 [B,H,Lq,ceil(C/32)]  bit (i % 32) of word (i / 32) = cluster i kept;
 *      ranges    i32 [B,H,Lq,C,2]         (first key, key count) per kept cluster, ascending; entries
 *                                         past n_ranges are left untouched.  May be NULL (mask only).
 *      n_ranges  i32 [B,H,Lq]             number of kept clusters
 *      n_keys    i32 [B,H,Lq]             total keys in kept clusters
 * No workspace needed.
 */
int sq_select(const sq_shape_t *shape, const float *logits, const float *row_max, const float *denom,
              const float *thresh, const int32_t *sizes, const int32_t *offsets,
              uint32_t *keep_mask, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys,
              void *ws, size_t ws_bytes, void *stream);

/*
 * Decode-time sparse attention (Section 4.2, Lq must be 1): exact softmax attention of each query
 * over the fixed-context keys listed in its ranges together with all U user keys of its sequence,
 * one softmax over the union.  Work is split along the key dimension into equal-sized chunks of
 * keys (the split-KV scheme of Section 4.2, so heads that keep more keys get more workgroups), each
 * chunk producing a partial (max, sum, output), merged in a second phase.
 * In:  ranges i32 [B,H,1,range_cap,2] (first key, count), ascending, disjoint, within [0, L);
 *      n_ranges, n_keys i32 [B,H,1] with n_keys = sum of counts; range_cap = shape->C.
 *      The key counts are taken from the ranges themselves: n_keys must be a valid pointer (it keeps the
 *      argument list of sq_select's outputs) but its values are not read.
 *      Input outside this contract never faults and is not reported: of a row, only the first range_cap ranges
 *      and the first L listed keys are used, entries with count <= 0 are skipped, and a key row outside
 *      [0, L) is read as the nearest row inside.
 * Out: out f16 [B,H,1,d]; lse f32 [B,H,1] = log sum exp of the scaled logits, or NULL.
 *      A query with no visible key gets out = 0 and lse = -inf.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_ATTN_DECODE).
 */
int sq_sparse_attn_decode(const sq_shape_t *shape, const void *q, const void *K_fixed, const void *V_fixed,
                          const int32_t *ranges, const int32_t *n_ranges, const int32_t *n_keys,
                          const void *K_user, const void *V_user,
                          void *out, float *lse, void *ws, size_t ws_bytes, void *stream);

/*
 * Prefill-time sparse attention (Section 4.2) with PER-QUERY selection: query t of sequence b
 * attends to the keys of the clusters set in its own keep_mask row, plus user keys 0..t
 * (causal_user != 0) or all U user keys (causal_user == 0).
 * In:  keep_mask u32 [B,H,Lq,ceil(C/32)], offsets i32 [H,C+1].
 * Out: out f16 [B,H,Lq,d]; lse f32 [B,H,Lq] or NULL.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_ATTN_PREFILL).
 * Cost: the keys are walked in blocks of 64 by groups of 64 consecutive query tokens.  A block in which no token of
 * the group kept a cluster is not read at all, provided at least an eighth of all (group, block) pairs are of that
 * kind (counted on the device from keep_mask, no host synchronisation) and L <= 262144; otherwise every group walks
 * every block and only the matrix products of such a block are skipped.  The result does not depend on which.
 */
int sq_sparse_attn_prefill(const sq_shape_t *shape, const void *q, const void *K_fixed, const void *V_fixed,
                           const int32_t *offsets, const uint32_t *keep_mask,
                           const void *K_user, const void *V_user,
                           void *out, float *lse, void *ws, size_t ws_bytes, void *stream);

/*
 * Prefill selection as the paper does it (Appendix D, "Prefill Stage"): the cluster scores of Eq. 1,
 * S_i(t) = exp(x_i(t) - m(t)) / D(t), are averaged over the Lq query tokens of a (sequence, head) and
 * cluster i is kept iff N_i > 0 and the average is > thresh[h] (strict): ONE kept set for all query
 * tokens of that sequence and head.  fp32 throughout (per-token scores, a fixed-order sum, one division).
 * In:  logits, row_max, denom as written by sq_centroid_score.
 * Out: keep_mask u32 [B,H,ceil(C/32)]; ranges i32 [B,H,C,2] (may be NULL) = (first key, count) of the
 *      kept clusters in ascending order; n_ranges, n_keys i32 [B,H].
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_SELECT_MEAN).
 */
int sq_select_mean(const sq_shape_t *shape, const float *logits, const float *row_max, const float *denom,
                   const float *thresh, const int32_t *sizes, const int32_t *offsets,
                   uint32_t *keep_mask, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys,
                   void *ws, size_t ws_bytes, void *stream);

/*
 * Prefill-time sparse attention (Section 4.2) with ONE kept set per (sequence, head), as produced by
 * sq_select_mean: every query token t of sequence b attends to the keys of ranges[b,h,0..n_ranges) plus
 * user keys 0..t (causal_user != 0) or all U user keys.  The ranges are expanded into a list of key rows
 * (the key-index tensor of Section 4.2) that the attention kernel gathers; there are no per-query masks.
 * In:  ranges i32 [B,H,C,2], n_ranges i32 [B,H] (entries with count 0 are skipped; at most L keys per
 *      row are used), n_keys i32 [B,H] (informational; the kernels recount).
 * Out: out f16 [B,H,Lq,d]; lse f32 [B,H,Lq] or NULL.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_ATTN_PREFILL_SHARED).
 */
int sq_sparse_attn_prefill_shared(const sq_shape_t *shape, const void *q, const void *K_fixed, const void *V_fixed,
                                  const int32_t *ranges, const int32_t *n_ranges, const int32_t *n_keys,
                                  const void *K_user, const void *V_user,
                                  void *out, float *lse, void *ws, size_t ws_bytes, void *stream);

/*
 * Two-level centroid lookup (Section 3.3, Eq. 2 and Eq. 3; Lq must be 1).  shape->C is the number
 * of fine (level-2) clusters C2; C1 is the number of coarse clusters.
 *   level 1: scores of Eq. 2 on (centroids1, sizes1) against thresh1 -> keep_mask1;
 *   expansion: the candidates are fine clusters child_offsets[j] .. child_offsets[j+1]-1 of every
 *            kept coarse cluster j (fine clusters are stored grouped by parent);
 *   level 2: scores of Eq. 3 on the candidates only -- the max and the normaliser run over the
 *            candidates, not over all fine clusters -- against thresh2 -> keep_mask2, ranges.
 * In:  centroids1 f16 [H,C1,d], sizes1 i32 [H,C1] (keys under each coarse cluster),
 *      child_offsets i32 [H,C1+1] (non-decreasing, child_offsets[C1] <= C2), thresh1 f32 [H],
 *      centroids2 f16 [H,C2,d], sizes2 i32 [H,C2], offsets2 i32 [H,C2+1], thresh2 f32 [H].
 * Out: keep_mask1 u32 [B,H,ceil(C1/32)], keep_mask2 u32 [B,H,ceil(C2/32)],
 *      ranges i32 [B,H,1,C2,2] (may be NULL), n_ranges, n_keys i32 [B,H,1] as in sq_select.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_HIER_SELECT) (depends on C1 only through C2 >= C1).
 */
int sq_hier_select(const sq_shape_t *shape, int32_t C1, const void *q,
                   const void *centroids1, const int32_t *sizes1, const int32_t *child_offsets,
                   const float *thresh1,
                   const void *centroids2, const int32_t *sizes2, const int32_t *offsets2,
                   const float *thresh2,
                   uint32_t *keep_mask1, uint32_t *keep_mask2,
                   int32_t *ranges, int32_t *n_ranges, int32_t *n_keys,
                   void *ws, size_t ws_bytes, void *stream);

/*
 * One whole decode step (Lq must be 1): sq_centroid_score + sq_select + sq_sparse_attn_decode
 * enqueued back to back with the intermediate results kept in the workspace -- the end-to-end
 * quantity the paper times (lookup + argument set-up + sparse attention, Appendix "Kernel
 * Benchmarking").  The selection is bit-identical to the three separate calls; the attention output
 * agrees up to rounding (the keys are split over workgroups differently).
 * With B >= 2 the sequences share K_fixed/V_fixed (the shared-prefix setting of Section 1) and each
 * sequence still selects on its own.  From B = 8 on, the step streams the union of the selections of every
 * group of 16 sequences, so a key kept by several sequences is read once; the probabilities are then rounded
 * to fp16 before they multiply V (matrix-core product, fp32 accumulation), as in sq_sparse_attn_prefill.
 * Below that the selections overlap too little to pay for the union and every sequence is handled by itself.
 * Out: out f16 [B,H,1,d]; optional (NULL to skip): lse f32 [B,H,1], keep_mask u32 [B,H,1,ceil(C/32)],
 *      n_keys i32 [B,H,1].
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_DECODE_STEP).
 */
int sq_decode_step(const sq_shape_t *shape, const void *q,
                   const void *centroids, const int32_t *sizes, const int32_t *offsets, const float *thresh,
                   const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                   void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                   void *ws, size_t ws_bytes, void *stream);

/*
 * sq_decode_step for callers that cannot allocate device memory or hand over a workspace: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results and error behaviour as
 * sq_decode_step, without the workspace: the step's intermediate state (logits, key-index lists, partial
 * results) lives in a device array of SQ_NOALLOC_SCRATCH_BYTES that is part of the library's code object -- one copy
 * per GPU the library runs on, held until the process ends.  The call allocates and frees nothing.  A shape whose
 * sq_workspace_bytes(shape, SQ_CALL_DECODE_STEP) exceeds SQ_NOALLOC_SCRATCH_BYTES is rejected with SQ_ERR_WORKSPACE
 * (the limit covers one sequence of 32 heads over a 32K-key context with 1024 clusters and 512 user keys).
 * All calls on one GPU share that GPU's array: calls that overlap in time on one GPU (different streams or threads)
 * race; calls enqueued one after the other on one stream do not.
 */
#define SQ_NOALLOC_SCRATCH_BYTES (16u << 20)
int sq_decode_step_noalloc(const sq_shape_t *shape, const void *q,
                           const void *centroids, const int32_t *sizes, const int32_t *offsets, const float *thresh,
                           const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                           void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys, void *stream);

/*
 * One whole decode step with GROUPED-QUERY attention (Lq must be 1): G query heads of a sequence share one K/V
 * head -- its fixed-context keys, centroids, threshold and the sequence's user keys -- and every query head
 * selects its clusters independently (the setting of the appendix "Additional Longbench Evaluation": keys and
 * values shared amongst a subset of the heads, each head selecting on its own).  shape->H is the number of K/V
 * heads; query head hq = h * G + g uses K/V head h.  The B * G (sequence, query head) pairs of a K/V head are
 * handled like B * G sequences over a shared context: from B * G = 8 on, the union of the selections of every group
 * of 16 of them is streamed once, so a key kept by several query heads leaves HBM once; below that every pair is a
 * row of the per-sequence kernels, which read the K/V head once per query head (same kernels, arithmetic and
 * rounding as sq_decode_step; G = 1 is that call).  1 <= G <= 16; a group size that does not divide 16 (3 or 6 query
 * heads per K/V head) takes the per-sequence kernels at any batch size.
 * In:  q f16 [B, H*G, 1, d]; centroids, sizes, offsets, thresh, K_fixed, V_fixed per K/V head as everywhere;
 *      K_user, V_user f16 [B, H, U, d].
 * Out: out f16 [B, H*G, 1, d]; optional (NULL to skip): lse f32 [B, H*G, 1], keep_mask u32 [B, H*G, 1, ceil(C/32)],
 *      n_keys i32 [B, H*G, 1].
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_GQA_DECODE_STEP) (sized for G = 16).
 */
int sq_gqa_decode_step(const sq_shape_t *shape, int32_t G, const void *q,
                       const void *centroids, const int32_t *sizes, const int32_t *offsets, const float *thresh,
                       const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                       void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                       void *ws, size_t ws_bytes, void *stream);

/*
 * Grouped-query decode with ONE kept set per (sequence, K/V head): the aggregation across the heads of a group that
 * the paper's appendix ("Additional Longbench Evaluation") leaves as future work, read as the average: the Eq. 1
 * scores of the G query heads that share a K/V head are averaged (Appendix D's rule with the heads in the place of
 * the query tokens) and cluster i is kept iff the average exceeds thresh (up to the fp32 rounding of sum_i N_i * mean_i,
 * which is 1 in exact arithmetic); every head of the group attends to those keys plus the sequence's user keys, and
 * each kept key is read once per group.  Arguments, layouts and G as sq_gqa_decode_step; keep_mask u32
 * [B,H*G,1,ceil(C/32)] and n_keys i32 [B,H*G,1] (optional) repeat the group's set for each of its heads.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_GQA_MEAN_DECODE_STEP).
 */
int sq_gqa_mean_decode_step(const sq_shape_t *shape, int32_t G, const void *q, const void *centroids,
                            const int32_t *sizes, const int32_t *offsets, const float *thresh,
                            const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                            void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                            void *ws, size_t ws_bytes, void *stream);

/*
 * One whole prefill step with PER-QUERY selection: the lookup of sq_centroid_score + sq_select for every
 * query token, then sq_sparse_attn_prefill.  The lookup makes two passes over the centroids (normaliser,
 * then scores; Section 4.1) and writes no [queries x clusters] intermediate.  Its normaliser is summed in
 * a different order than sq_centroid_score's, so a cluster whose score is within rounding of the threshold
 * may be decided differently from the separate calls; everything else is identical.
 * Out: out f16 [B,H,Lq,d]; optional (NULL to skip): lse f32 [B,H,Lq], keep_mask u32 [B,H,Lq,ceil(C/32)],
 *      n_keys i32 [B,H,Lq].
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_PREFILL_STEP).
 */
int sq_prefill_step(const sq_shape_t *shape, const void *q,
                    const void *centroids, const int32_t *sizes, const int32_t *offsets, const float *thresh,
                    const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                    void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                    void *ws, size_t ws_bytes, void *stream);

/*
 * One whole prefill step with the selection on AVERAGED scores (Appendix D, "Prefill Stage"): the same
 * two-pass lookup, the scores of Eq. 1 averaged over the Lq query tokens, one kept set per (sequence, head)
 * as in sq_select_mean, then sq_sparse_attn_prefill_shared on it.  The same remark on rounding applies.
 * Out: out f16 [B,H,Lq,d]; optional (NULL to skip): lse f32 [B,H,Lq], keep_mask u32 [B,H,ceil(C/32)],
 *      n_keys i32 [B,H].
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_PREFILL_MEAN_STEP).
 */
int sq_prefill_mean_step(const sq_shape_t *shape, const void *q,
                         const void *centroids, const int32_t *sizes, const int32_t *offsets, const float *thresh,
                         const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                         void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * One whole decode step with the two-level lookup (Lq must be 1): sq_hier_select followed by
 * sq_sparse_attn_decode on its ranges, intermediates kept in the workspace.  Arguments as in those two
 * calls; keep_mask2 and n_keys are optional outputs (NULL to skip).
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_HIER_DECODE_STEP).
 */
int sq_hier_decode_step(const sq_shape_t *shape, int32_t C1, const void *q,
                        const void *centroids1, const int32_t *sizes1, const int32_t *child_offsets,
                        const float *thresh1,
                        const void *centroids2, const int32_t *sizes2, const int32_t *offsets2,
                        const float *thresh2,
                        const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                        void *out, float *lse, uint32_t *keep_mask2, int32_t *n_keys,
                        void *ws, size_t ws_bytes, void *stream);

/*
 * Centroid lookup through a hierarchy of n_levels levels (1 .. SQ_MAX_LEVELS), coarsest first: Section 3.3's Eq. 2
 * and Eq. 3 applied level after level (the section notes that the two-level scheme extends to more levels).
 * Level 0 scores all of its clusters against its threshold; at every further level the candidates are the
 * children of the clusters kept one level up, and the maximum and the normaliser of the scores run over those
 * candidates only.  n_levels = 2 is sq_hier_select, n_levels = 1 the one-level selection.
 * One level: centroids f16 [H, C, d]; sizes i32 [H, C] (keys under each cluster of this level); child_offsets
 * i32 [H, C+1] -- cluster j's children at the next level are child_offsets[j] .. child_offsets[j+1]-1 (clusters of
 * a level are stored grouped by parent), and at the LAST level child_offsets are the key offsets of the clusters
 * (cluster j = keys [child_offsets[j], child_offsets[j] + sizes[j])); thresh f32 [H].  All device pointers; the
 * `levels` array itself is host memory read during the call.  C must not exceed shape->C, and the last level's C
 * must equal shape->C.
 * Out: keep_masks (host array of n_levels device pointers, or NULL; entries may be NULL): level k's mask
 *      u32 [B,H,ceil(C_k/32)]; ranges i32 [B,H,1,C,2] (may be NULL), n_ranges, n_keys i32 [B,H,1] of the last level.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_MULTILEVEL_SELECT).  Lq must be 1.
 */
#define SQ_MAX_LEVELS 4
typedef struct sq_level_t {
    int32_t C;
    const void *centroids;
    const int32_t *sizes;
    const int32_t *child_offsets;
    const float *thresh;
} sq_level_t;

int sq_multilevel_select(const sq_shape_t *shape, int32_t n_levels, const sq_level_t *levels, const void *q,
                         uint32_t *const *keep_masks, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys,
                         void *ws, size_t ws_bytes, void *stream);

/*
 * One whole decode step with the lookup of sq_multilevel_select followed by sq_sparse_attn_decode on its ranges,
 * intermediates kept in the workspace.  keep_mask (last level) and n_keys are optional outputs (NULL to skip).
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_MULTILEVEL_DECODE_STEP).
 */
int sq_multilevel_decode_step(const sq_shape_t *shape, int32_t n_levels, const sq_level_t *levels, const void *q,
                              const void *K_fixed, const void *V_fixed, const void *K_user, const void *V_user,
                              void *out, float *lse, uint32_t *keep_mask, int32_t *n_keys,
                              void *ws, size_t ws_bytes, void *stream);

/*
 * Prefill through the two-level lookup (Section 3.3; the paper builds the hierarchy for generation only), with the
 * paper's prefill rule (Appendix D, "Prefill Stage": scores averaged over the Lq query tokens, ONE kept set per
 * (sequence, head)) at both levels: the coarse scores of Eq. 2 averaged over the tokens select coarse clusters by
 * thresh1; the fine scores of Eq. 3 -- per token, normaliser over the children of the kept coarse clusters only --
 * are averaged over the tokens and compared with thresh2; attention as in sq_sparse_attn_prefill_shared on the kept
 * fine clusters' keys.  Arguments as sq_hier_decode_step, with q f16 [B,H,Lq,d], out f16 [B,H,Lq,d],
 * lse f32 [B,H,Lq] (or NULL), keep_mask2 u32 [B,H,ceil(C/32)] and n_keys i32 [B,H] (optional outputs).
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_HIER_PREFILL_MEAN_STEP).
 */
int sq_hier_prefill_mean_step(const sq_shape_t *shape, int32_t C1, const void *q,
                              const void *centroids1, const int32_t *sizes1, const int32_t *child_offsets,
                              const float *thresh1, const void *centroids2, const int32_t *sizes2,
                              const int32_t *offsets2, const float *thresh2, const void *K_fixed, const void *V_fixed,
                              const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask2,
                              int32_t *n_keys, void *ws, size_t ws_bytes, void *stream);

/*
 * The same with PER-QUERY selection (every query token selects for itself, as sq_prefill_step): token t keeps coarse
 * clusters by Eq. 2 and thresh1, and fine clusters among the children of ITS kept coarse clusters by Eq. 3
 * (normaliser over those children only) and thresh2; attention as in sq_sparse_attn_prefill with the per-token fine
 * masks.  The fine centroids are scored densely for every token (a token's non-candidates are treated as clusters
 * without keys), so this form saves no centroid comparisons over sq_prefill_step: it applies the hierarchical rule.
 * keep_mask2 u32 [B,H,Lq,ceil(C/32)] and n_keys i32 [B,H,Lq] are optional outputs.  C1 <= 1024.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_HIER_PREFILL_STEP).
 */
int sq_hier_prefill_step(const sq_shape_t *shape, int32_t C1, const void *q,
                         const void *centroids1, const int32_t *sizes1, const int32_t *child_offsets,
                         const float *thresh1, const void *centroids2, const int32_t *sizes2,
                         const int32_t *offsets2, const float *thresh2, const void *K_fixed, const void *V_fixed,
                         const void *K_user, const void *V_user, void *out, float *lse, uint32_t *keep_mask2,
                         int32_t *n_keys, void *ws, size_t ws_bytes, void *stream);

/*
 * Offline clustering of the fixed-context keys (Section 3.1: K-means on normalised key vectors; the centroid of a
 * cluster is the mean of its vectors).  The paper fixes neither initialisation nor iteration count, so the unit
 * here is one Lloyd iteration; the caller chooses the initial centres (e.g. normalised keys drawn at random) and
 * how often to iterate.  Every (sequence, head) pair of the shape is clustered on its own; shape->Lq, U and
 * sm_scale are not used (give Lq = 1, U = 0, sm_scale = 1).
 *
 * sq_kmeans_normalize: X[b,h,j,:] = K[b,h,j,:] / |K[b,h,j,:]| (fp32 arithmetic, rounded to f16; a zero row stays
 *   zero).  K, X f16 [B,H,L,d]; X may alias K.  No workspace.
 */
int sq_kmeans_normalize(const sq_shape_t *shape, const void *K, void *X, void *stream);

/*
 * One Lloyd iteration on the rows of X (f16 [B,H,L,d]) with the centres centers_in (f16 [B,H,C,d]):
 *   assign  i32 [B,H,L]    nearest centre of each row in squared Euclidean distance, evaluated as
 *                          argmax_c (x.c - |c|^2/2) with fp32 accumulation; equal scores go to the lowest index
 *   sizes   i32 [B,H,C]    members per centre;  offsets i32 [B,H,C+1] their exclusive prefix sum (last = L)
 *   perm    i32 [B,H,L]    row indices grouped by centre, ascending inside a centre (a stable sort by centre id):
 *                          centre c's members are perm[offsets[c] .. offsets[c] + sizes[c])
 *   centers_out f16 [B,H,C,d]  mean of each centre's members (fp32 sum, rounded to f16); a centre without members
 *                          keeps its value.  May alias centers_in.
 * C <= L required.  Workspace: sq_workspace_bytes(shape, SQ_CALL_KMEANS_STEP).
 */
int sq_kmeans_step(const sq_shape_t *shape, const void *X, const void *centers_in, void *centers_out,
                   int32_t *assign, int32_t *sizes, int32_t *offsets, int32_t *perm,
                   void *ws, size_t ws_bytes, void *stream);

/*
 * From a grouping (perm, sizes, offsets as written by sq_kmeans_step) to the inputs of the online calls above:
 * K_sorted[b,h,i,:] = K[b,h,perm[i],:], likewise V_sorted, so that each cluster's keys are contiguous, and
 * centroids f16 [B,H,C,d] = mean of the RAW keys of each cluster (Section 3.1; zeros for an empty cluster).
 * K, V, K_sorted, V_sorted f16 [B,H,L,d]; the outputs must not alias the inputs.  V and V_sorted may be NULL (keys
 * only); K_sorted may be NULL too (centroids only), and then perm may be NULL: cluster c is rows
 * offsets[c] .. offsets[c] + sizes[c] of K as they stand.  No workspace.
 */
int sq_cluster_layout(const sq_shape_t *shape, const void *K, const void *V, const int32_t *perm,
                      const int32_t *sizes, const int32_t *offsets, void *K_sorted, void *V_sorted,
                      void *centroids, void *stream);

/*
 * Nesting for the hierarchical lookup (Section 3.3: the coarse level is a clustering of the fine centroids).  After
 * the keys were clustered into shape->C fine clusters (assign_fine i32 [B,H,L], from sq_kmeans_step) and the fine
 * centroids into C1 coarse clusters (a second sq_kmeans_step run on the centroids, with L = C and C = C1: its perm
 * is perm_coarse i32 [B,H,C], its offsets are child_offsets i32 [B,H,C1+1]), this call renumbers the fine clusters
 * in perm_coarse order, so that the children of a coarse cluster are the consecutive fine clusters
 * child_offsets[j] .. child_offsets[j+1]-1, and groups the keys again:
 *   assign_new i32 [B,H,L]   new fine cluster id of each key
 *   sizes i32 [B,H,C], offsets i32 [B,H,C+1], perm i32 [B,H,L]   the keys grouped by new id (as sq_kmeans_step)
 *   sizes_coarse i32 [B,H,C1]   keys under each coarse cluster
 * Then sq_cluster_layout on (perm, sizes, offsets) gives K/V and the fine centroids in the new order, and
 * sq_cluster_layout with L = C, C = C1 on those centroids (perm NULL, sizes = the coarse run's sizes, offsets =
 * child_offsets) gives the coarse centroids as the unweighted mean of their children.
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_KMEANS_STEP).
 */
int sq_cluster_nest(const sq_shape_t *shape, int32_t C1, const int32_t *assign_fine, const int32_t *perm_coarse,
                    const int32_t *child_offsets, int32_t *assign_new, int32_t *sizes, int32_t *offsets,
                    int32_t *perm, int32_t *sizes_coarse, void *ws, size_t ws_bytes, void *stream);

/*
 * Threshold calibration (Appendix C: the threshold is set so that a target share of the keys is retrieved on
 * calibration queries; the paper states the goal, the procedure is this library's).  The B * Lq rows of each head are
 * its calibration queries: their cluster scores S_i = exp(logits - row_max) / denom (Eq. 1, fp32, as written by
 * sq_centroid_score) are pooled, each weighing sizes[i] keys, and walked from the highest score down until
 * target_keys keys are covered (clamped to what the head's queries can retrieve at all); thresh[h] is the geometric
 * mean of the last score needed and the highest score strictly below it (half the last score if there is none, or
 * if it is 0), so that the strict rule S > thresh keeps exactly the walked scores, ties included.
 * In:  logits f32 [B,H,Lq,C], row_max, denom f32 [B,H,Lq], sizes i32 [H,C]; target_keys = pooled key budget per head
 *      (e.g. keep_fraction * B * Lq * L).  B * Lq * L must stay below 2^31.
 * Out: thresh f32 [H].
 * Workspace: sq_workspace_bytes(shape, SQ_CALL_CALIBRATE).
 */
int sq_calibrate_threshold(const sq_shape_t *shape, const float *logits, const float *row_max, const float *denom,
                           const int32_t *sizes, int64_t target_keys, float *thresh,
                           void *ws, size_t ws_bytes, void *stream);

/* ------------------------------------------------------------------------------------------------------------------
 * MEASUREMENT HOOKS -- sq_profile_begin / sq_profile_end / sq_probe_stream_read.  Not part of the method and not
 * part of the path's boundary: nothing above calls them and no result depends on them.  They exist so that a
 * benchmark can time the dominant kernel and the device's streaming-read ceiling from inside its own process.
 * They keep process-wide state and are not thread-safe.
 * ---------------------------------------------------------------------------------------------------------------- */

/*
 * Measurement hook for benchmarks (for callers that want a kernel's duration
 * without an external profiler).  Between sq_profile_begin(n) and sq_profile_end(), every launch of
 * the dominant kernel of a step -- the split-KV partial-attention kernel, which reads the selected K/V rows,
 * i.e. nearly all bytes of a decode step (Section 4.2, phase 1); the attention kernel of a prefill step --
 * carries a pair of HIP events attached to its dispatch on the stream it is launched on (start and end of the
 * kernel itself), up to n launches.  sq_profile_end() waits for those events, writes the
 * average / minimum / maximum elapsed time per launch in microseconds (any pointer may be NULL),
 * returns the number of launches measured (or a negative sq_status), and releases the events.
 * Host only; process-wide state, not thread-safe; creates HIP events (no device memory).  Not to be used while
 * the stream is being captured into a graph.
 */
int sq_profile_begin(int max_launches);
int sq_profile_end(float *avg_us, float *min_us, float *max_us);

/*
 * Measurement probe: a plain streaming read of `bytes` bytes of device memory at `buf` (16-byte aligned)
 * by `workgroups` workgroups of 256 threads, enqueued on `stream`; `sink` is >= 1 KiB of device memory
 * that may receive a word.  Timed by the caller, it gives the read bandwidth an HBM-bound kernel can
 * approach on the device at hand, to put beside the published peak.
 */
int sq_probe_stream_read(const void *buf, size_t bytes, void *sink, int workgroups, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* SQUEEZED_ATTENTION_H */
