// Host-side launcher declarations shared between the kernel files and the C-ABI file.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "sq_common.hpp"

namespace sq {

struct Shape {
    int B, H, L, C, Lq, U;
    float sm_scale;
    int causal_user;
};

// Internal per-row plan of the split-KV decode kernel: one record per kept range with the number of
// selected keys in front of it, and for every chunk of KPC selected keys the first record it touches.
struct DecodePlan {
    int4 *rec;          // [rows, rec_cap]  (first key, count, keys before, 0)
    int *chunk_first;   // [rows, chunk_cap]
    int2 *hdr;          // [rows] (number of records, number of selected keys)
    int rec_cap;
    int chunk_cap;
};

inline int chunk_cap_for(int L) { return (L + KPC - 1) / KPC; }
inline int user_chunks_for(int U) { return (U + KPC - 1) / KPC; }

hipError_t launch_score(const void *q, const void *centroids, float *logits, int B, int H, int Lq, int C,
                        float sm_scale, hipStream_t s);
hipError_t launch_row_stats(const float *logits, const int32_t *sizes, float *row_max, float *denom,
                            int rows, int H, int Lq, int C, hipStream_t s);
// stats_in == true: use row_max/denom; false: the kernel derives them from logits itself.
hipError_t launch_select(const float *logits, const float *row_max, const float *denom, bool stats_in,
                         const float *thresh, const int32_t *sizes, const int32_t *offsets,
                         uint32_t *keep_mask, int32_t *ranges, int32_t *n_ranges, int32_t *n_keys,
                         DecodePlan plan, int rows, int H, int Lq, int C, hipStream_t s);
hipError_t launch_plan_from_ranges(const int32_t *ranges, const int32_t *n_ranges, DecodePlan plan, int rows,
                                   int range_cap, hipStream_t s);
hipError_t launch_decode_attn(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                              DecodePlan plan, const int32_t *n_ranges, const int32_t *n_keys, float *partials,
                              void *out, float *lse, const Shape &sh, hipStream_t s);

}  // namespace sq
