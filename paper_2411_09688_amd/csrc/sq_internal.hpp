// Host-side launcher declarations shared between the kernel files and the C-ABI file.
#pragma once
#include <hip/hip_ext.h>
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sq_common.hpp"

namespace sq {

struct Shape {
    int B, H, L, C, Lq, U;
    float sm_scale;
    int causal_user;
};

// Internal plan of the split-KV decode kernel, held in the workspace.
//   rec       per row, one record per kept range: (first key, count, selected keys before it, 0)
//   hdr       per row: (number of records, number of selected keys)
//   row_items per row: (first work item, number of work items); items of a row are consecutive
//   total     two ints: work items of the whole call, rows that have placed their items
//   row_rank  per row (may be null): how many rows had placed their items before this one
//   item      per work item (= one chunk of up to KPC keys of one row) ITEM_STRIDE int2 slots:
//             slot 0 = (row, keys in the chunk), slot 1 = (records in the chunk, position of the chunk's first key
//             in its row's selection) or, for a chunk of user keys, (-1, first user key), slots 2.. = the chunk's own copy of the range records it touches, as
//             (position of the record's first key relative to the chunk, fixed-context row of that key
//             minus that position): key slot t of the chunk lies in the last record whose position is
//             <= t and reads row t + delta.  This is the key-index tensor of Section 4.2 in run-length
//             form, stored chunk by chunk so an attention workgroup gets it with one coalesced load.
constexpr int ITEM_STRIDE = KPC + 2;     // int2 slots per item: a chunk of KPC keys touches <= KPC records
struct DecodePlan {
    int4 *rec;        // [rows, rec_cap]
    int2 *hdr;        // [rows]
    int2 *row_items;  // [rows]
    int *total;       // [2], 8-byte aligned (both words are advanced by one 64-bit atomic)
    int *row_rank;    // [rows] or null
    int2 *item;       // [item_cap, ITEM_STRIDE]
    int rec_cap;
    int item_cap;     // rows * (user chunks + ceil(L / KPC))
    int L;
};

inline int chunk_cap_for(int L) { return (L + KPC - 1) / KPC; }
inline int user_chunks_for(int U) { return (U + KPC - 1) / KPC; }

// Row-wise selection stages a row's logits and cluster sizes in LDS.
constexpr int SELECT_MAX_C = 16384;
constexpr int LDS_BYTES_MAX = 160 * 1024 - 8192;   // gfx950: 160 KB per workgroup, minus the static arrays
// Scheduling keeps two ints per chunk of a row in LDS (same budget as the staged logits).
constexpr int MAX_L = SELECT_MAX_C * KPC;

// zero_counter (may be null) points at the two counters of a decode step's work list; the kernel zeroes them.
hipError_t launch_score(const void *q, const void *centroids, float *logits, int *zero_counter, int B, int H, int Lq,
                        int C, float sm_scale, hipStream_t s);
hipError_t launch_row_stats(const float *logits, const int32_t *sizes, float *row_max, float *denom, int rows,
                            int H, int Lq, int C, hipStream_t s);
// Averaged-score prefill selection: partial sums of the per-token scores over blocks of MEAN_ROWS query tokens,
// part_sum [B*H, mean_parts_for(Lq), C].
constexpr int MEAN_ROWS = 64;
inline int mean_parts_for(int Lq) { return (Lq + MEAN_ROWS - 1) / MEAN_ROWS; }
hipError_t launch_mean_score(const float *logits, const float *row_max, const float *denom, float *part_sum, int BH,
                             int Lq, int C, hipStream_t s);
// Fused prefill lookup (scores, statistics and the per-token decision in one kernel, nothing materialised): one
// wave handles LOOKUP_ROWS query tokens.  mean == false writes keep_mask [B*H*Lq, ceil(C/32)] and the per-token
// counts; mean == true writes part_sum [B*H, lookup_parts_for(Lq), C] for the selection on averaged scores.
constexpr int LOOKUP_ROWS = 16;
__host__ __device__ inline int lookup_parts_for(int Lq) { return (Lq + LOOKUP_ROWS - 1) / LOOKUP_ROWS; }
hipError_t launch_prefill_lookup(const void *q, const void *centroids, const int32_t *sizes, const float *thresh,
                                 uint32_t *keep_mask, int32_t *n_ranges, int32_t *n_keys, float *part_sum, bool mean,
                                 int B, int H, int Lq, int C, float sm_scale, hipStream_t s,
                                 const int32_t *cand_id = nullptr, const int2 *cand_hdr = nullptr,
                                 const int32_t *parent = nullptr, const uint32_t *mask1 = nullptr, int C1 = 0);
// (parent [H, C] / mask1 [B*H*Lq, ceil(C1/32)] given, per-query mode: a cluster counts for a token only if the token's
// level-1 mask holds its parent: level 2 of a hierarchical lookup with per-token candidates; C1 <= 1024.)
hipError_t launch_child_parent(const int32_t *child_offsets, int32_t *parent, int H, int C1, int C2, hipStream_t s);
// (cand_id [B*H, C] / cand_hdr [B*H] given, with mean: only the hdr.y candidates listed for a (sequence, head) are
// scored, statistics over them alone, part_sum in candidate order: level 2 of a hierarchical lookup.)
// Kept ranges (records of a plan) -> flat index lists idx [rows, L]: the key rows of the attention, or the candidate
// clusters of the next level.
hipError_t launch_expand_ranges(DecodePlan plan, int32_t *idx, int rows, int L, hipStream_t s);
// Options of the row-wise selection for the two-level lookup (all zero for the one-level path).
struct SelectOpts {
    const int32_t *cand_id;          // level 2: `logits` is [rows, C] in candidate order, cand_id [rows, C] the
    const int2 *cand_hdr;            //   candidates' cluster ids (ascending), cand_hdr[row].y their number
    int len_from_offsets;            // level 1: emitted range length = offsets[i+1] - offsets[i] (child clusters)
    int mean_parts;                  // averaged-score selection: `logits` holds this many partial score sums per
    float mean_div;                  //   row, [rows, mean_parts, C]; their sum / mean_div is compared with T
    int union_rows;                  // shared-context decode: rows are union rows (sequence group, head)
    int B;                           // shared-context decode: number of query rows that share a head's K/V (B * G)
    int G;                           // shared-context decode: query rows per (sequence, head), see shared_row
    int replay;                      // set by launch_select: multi-step rows write their work items from the staged row
    int masks_ready;                 // union rows: set by launch_select when the per-sequence masks are already in keep_mask
    const int4 *cand_rec;            // level 2, optional: the candidates' records and the statistics of the work items
    const float2 *cand_stats;        //   that listed them (see launch_gather_score), cand_items[row] = (first item,
    const int2 *cand_items;          //   items) of the row: the row is then staged from these streams alone
};

// Dense attention over the rows' user keys as a rider on the selection launch (see sq_user_attn.hpp): q [rows, d],
// user keys [rows / G, U, d]; row r leaves nuq = ceil(U / KPC) partial results, one per chunk of user keys, at slots
// slot_base + r * nuq + (0 .. nuq - 1) of `partials`.  q == nullptr: none.
struct UserAttn {
    const _Float16 *q, *Ku, *Vu;
    float *partials;
    int rows, U, G, slot_base, nuq;
    float sm_scale;
};

// Batched decode over a shared fixed context: sequences are handled in groups of SG; a "union row" is one
// (group, head) pair and its work items cover the clusters kept by ANY sequence of the group, each key
// carrying the set of sequences that kept it, so a key leaves HBM once per group instead of once per sequence.
// Items of a union row use the layout above with these differences: slot 0.x is the union row; slot 1.x of a
// user chunk is -1 - (real sequence within the group: its G virtual sequences own the chunk); a record's x packs (position clamped to >= 0) | (set of
// sequences << 16).
// With grouped-query attention, G query heads of a sequence share one K/V head (and the sequence's user keys) and
// select independently: the B * G (sequence, query head) pairs that share a K/V head are handled exactly like
// B * G sequences over a shared context.  "Virtual sequence" vs = b * G + g; its query, keep mask, counts and
// output sit at row ((b * H + h) * G + g) of the [B, H, G] tensors (H = K/V heads).  G = 1 is the plain batch.
// G must divide SG so that the G virtual sequences of one real sequence never straddle two groups.
constexpr int SG = 16;
inline int seq_groups_for(int BV) { return (BV + SG - 1) / SG; }
__host__ __device__ inline size_t shared_row(int vs, int h, int H, int G)
{
    return ((size_t)(vs / G) * H + h) * G + vs % G;
}
// Workgroups of the shared-context partial kernel: three per compute unit.
constexpr int SHARED_ATTN_GRID = 256 * 3;

// stats_in == true: use row_max/denom; false: the kernel derives them from logits itself.
hipError_t launch_select(const float *logits, const float *row_max, const float *denom, bool stats_in,
                         const float *thresh, const int32_t *sizes, const int32_t *offsets, uint32_t *keep_mask,
                         int32_t *ranges, int32_t *n_ranges, int32_t *n_keys, DecodePlan plan, bool schedule, int U,
                         SelectOpts opt, int rows, int H, int Lq, int C, hipStream_t s,
                         const UserAttn *user = nullptr);   // rider: only with schedule, computed statistics, plain rows
// Level-2 scoring of the two-level lookup: logits of the candidate fine centroids listed by the work
// items of `cand` (chunks of candidate clusters), written in candidate order: logits2[row, j], cand_id[row, j],
// cand_rec[row, j] = (logit bits, id | bit 31 if N == 0, offsets[id], range length: N, or offsets[id + 1] - offsets[id]
// with len_from_offsets),
// and per item cand_stats[item] = (max, sum N exp(x - max)) over the item's candidates with N > 0.
hipError_t launch_gather_score(const void *q, const void *centroids2, DecodePlan cand, const int32_t *sizes2,
                               const int32_t *offsets2, int len_from_offsets, float *logits2, int32_t *cand_id,
                               int4 *cand_rec, float2 *cand_stats, int *zero_counter, int H, int C2, float sm_scale,
                               hipStream_t s, uint32_t *zero_mask = nullptr, size_t zero_words = 0);
// (zero_mask: zero_words words cleared by the launch, for the selection that follows to set bits in.)
// Rows [BH, G, C] of logits -> ln of the group's averaged Eq. 1 scores, written to all G rows (in place).
hipError_t launch_group_mean_logits(float *logits, const int32_t *sizes, int BH, int H, int G, int C, hipStream_t s);
// Caller-style ranges [rows, range_cap, 2] -> records + header per row.
hipError_t launch_ranges_to_rec(const int32_t *ranges, const int32_t *n_ranges, DecodePlan plan, int rows,
                                int range_cap, hipStream_t s);
// Records + headers of all rows -> work items.
hipError_t launch_schedule(DecodePlan plan, int rows, int U, hipStream_t s);
// user_slot_base >= 0: the rows' user keys are already in `partials` (nuq results per row from that slot on, see
// UserAttn) and the plan holds no user chunks.
hipError_t launch_decode_attn(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                              DecodePlan plan, float *partials, void *out, float *lse, const Shape &sh,
                              hipStream_t s, int user_slot_base = -1, int nuq = 0);

// Shared-context decode: per-sequence selection (keep_masks, n_ranges, n_keys: [B*H] rows) and the work items of
// every union row in one launch (needs the two counters at plan.total zeroed), and the partial + merge kernels.  partials: (SHARED_ATTN_GRID + union
// rows) * SG slots of PART_STRIDE floats.
hipError_t launch_union_schedule(const float *logits, const float *thresh, const int32_t *sizes,
                                 const int32_t *offsets, uint32_t *keep_masks, int32_t *n_ranges, int32_t *n_keys,
                                 DecodePlan plan, int U, int B, int G, int H, int C, hipStream_t s);
hipError_t launch_decode_attn_shared(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                                     DecodePlan plan, float *partials, void *out, float *lse, const Shape &sh,
                                     hipStream_t s);

// The masked prefill's block table blk_info: an int per (head, 64-key block), then, 8-byte aligned, the 64-bit count of
// (workgroup, block) pairs in which no query of the workgroup kept a cluster.
__host__ __device__ inline size_t prefill_skip_count_at(int H, int L) { return ((size_t)H * ((L + 63) / 64) + 1) & ~(size_t)1; }
inline size_t prefill_blk_info_ints(int H, int L) { return prefill_skip_count_at(H, L) + 2; }

// Prefill attention with per-query keep masks; key_cid [H, L] and blk_info [prefill_blk_info_ints(H, L)] are workspace
// (the key -> cluster map and the block table).
hipError_t launch_prefill_attn(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                               const uint32_t *keep_mask, const int32_t *offsets, int32_t *key_cid, int32_t *blk_info,
                               void *out, float *lse, const Shape &sh, hipStream_t s);

// Prefill attention with ONE kept set per (sequence, head): plan.rec / plan.hdr hold the kept ranges' records
// (from launch_ranges_to_rec); key_idx [B*H, L] is workspace for the list of kept key rows.
hipError_t launch_prefill_attn_shared(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                                      DecodePlan plan, int32_t *key_idx, void *out, float *lse, const Shape &sh,
                                      hipStream_t s);

// Offline clustering (sq_kmeans.hip).  hn: [heads * C] floats; hist: [heads * parts * C] ints with
// parts = ceil(L / kmeans_part_len(L)).
int kmeans_part_len(int L);
hipError_t launch_normalize_rows(const void *K, void *X, size_t rows, hipStream_t s);
hipError_t launch_kmeans_step(const void *X, const void *centers_in, void *centers_out, int32_t *assign,
                              int32_t *sizes, int32_t *offsets, int32_t *perm, float *hn, int32_t *hist, int heads,
                              int L, int C, hipStream_t s);
hipError_t launch_cluster_nest(const int32_t *assign_fine, const int32_t *perm_coarse, const int32_t *child_offsets,
                               int32_t *assign_new, int32_t *sizes, int32_t *offsets, int32_t *perm,
                               int32_t *sizes_coarse, int32_t *inv, int32_t *hist, int heads, int L, int C2, int C1,
                               hipStream_t s);
hipError_t launch_cluster_layout(const void *K, const void *V, const int32_t *perm, const int32_t *sizes,
                                 const int32_t *offsets, void *K_sorted, void *V_sorted, void *centroids, int heads,
                                 int L, int C, hipStream_t s);

// Threshold calibration (sq_calibrate.hip).  S: [H, B * Lq, C] floats of workspace.
hipError_t launch_calibrate(const float *logits, const float *row_max, const float *denom, const int32_t *sizes,
                            float *S, float *thresh, int target, int B, int H, int Lq, int C, hipStream_t s);

// Decode step through a key-index list (sq_decode_keyidx.hip): the selection writes, per query row, the rows of the
// kept keys in ascending order (key_idx [rows, L]) and the number of them (row_keys [rows]); the partial kernel cuts
// the rows' lists, laid end to end, into equal shares of keys.  For rows of at most KI_MAX_C clusters and calls of at
// most KI_MAX_ROWS query rows.
constexpr int KI_MAX_C = 4096;
constexpr int KI_SLICE = 128;          // clusters per selection workgroup
constexpr int KI_MAX_ROWS = 1024;
constexpr int KI_MIN_SHARE = 128;      // keys per workgroup of the partial kernel, at least
constexpr int KI_ATTN_GRID = 256;      // workgroups of the partial kernel that stream selected keys: one per compute unit
struct KeyIndexPlan {
    int32_t *key_idx;                  // [rows, L]
    int32_t *row_keys;                 // [rows]
    int L;
};
// Partial results: KI_ATTN_GRID + rows slots for the selected keys, then rows * nuq for the user keys.
inline size_t keyidx_partial_slots(int rows, int nuq) { return (size_t)KI_ATTN_GRID + rows + (size_t)rows * nuq; }
hipError_t launch_select_index(const float *logits, const float *thresh, const int32_t *sizes, const int32_t *offsets,
                               uint32_t *keep_mask, int32_t *n_ranges, int32_t *n_keys, KeyIndexPlan plan, int rows,
                               int H, int G, int C, hipStream_t s);
// Last level of a hierarchical lookup, selected in slices of 256 candidates per workgroup (two launches: count, then
// write).  rec / hdr / stats / row_items: the candidates' records, per-row candidate counts (hdr[row].y), per-item
// statistics and per-row (first item, items), as launch_gather_score leaves them; slice_cnt [rows, cand_slices_for(C)]
// is scratch.  keep_mask (optional) must have been zeroed (launch_gather_score does it).  C <= SELECT_MAX_C, at most
// 1024 rows.  (The lookup without attention, which returns ranges, keeps the one-workgroup-per-row selection: over all
// queries of a workload its single launch is faster than these two.)
struct CandSelect {
    const int4 *rec;
    const int2 *hdr;
    const float2 *stats;
    const int2 *row_items;
    int2 *slice_cnt;
    float2 *row_stat;                  // [rows] scratch: the row's (maximum, T * D), from the counting to the writing launch
};
inline int cand_slices_for(int C) { return (C + 255) / 256; }
hipError_t launch_cand_select(CandSelect cs, const float *thresh, uint32_t *keep_mask, int32_t *n_ranges, int32_t *n_keys,
                              KeyIndexPlan plan, int rows, int H, int C, hipStream_t s);
// Partial kernel over the selected keys + merge.  user (may be null): the rows' dense attention over their user keys
// runs in extra workgroups of the partial kernel, one per piece of USER_PIECE keys: row r leaves user->nuq =
// user_pieces_for(U) partial results at slots user->slot_base + r * nuq + (0 .. nuq - 1) of `partials`.
constexpr int USER_PIECE = 64;
inline int user_pieces_for(int U) { return (U + USER_PIECE - 1) / USER_PIECE; }
hipError_t launch_decode_attn_index(const void *q, const void *Kf, const void *Vf, KeyIndexPlan plan, float *partials,
                                    void *out, float *lse, int rows, int H, int G, float sm_scale, const UserAttn *user,
                                    hipStream_t s);

// Records the calling thread's error message (what sq_last_error returns) and hands back `code`.
int set_error(int code, const char *fmt, ...) __attribute__((format(printf, 2, 3)));

// Measurement hook (sq_profile.hip): when enabled, hands out the next pair of events; the caller attaches them to
// the dominant kernel's dispatch (hipExtLaunchKernelGGL), so they carry the start and end time of that kernel
// itself rather than of marker packets around it.
bool profile_pair(hipEvent_t *start, hipEvent_t *stop);

}  // namespace sq
