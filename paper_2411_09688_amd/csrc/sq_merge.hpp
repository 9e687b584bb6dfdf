// Phase 2 of the split-KV decode (Section 4.2): merge of the partial (max, sum, output) results of one row.
#pragma once
#include "sq_common.hpp"

namespace sq {

// Merge of n partials of one row by a 1024-thread workgroup:
//   out = sum_c e^{m_c - M} o_c / sum_c e^{m_c - M} l_c,   lse = M + log(sum_c e^{m_c - M} l_c).
// 32 groups of 32 threads; group g folds partials g, g+32, ... with a running maximum (a thread owns
// four output dimensions, 16-byte loads, four partials in flight), then the groups are folded in LDS.
// slot_ptr(c) -> the c-th partial of the row (PART_STRIDE floats: m, l, pad, pad, o[128]).
// GUARD: a partial whose m is -inf is empty and its o[] was never written.
constexpr int MERGE_THREADS = 1024;
constexpr int MERGE_GROUPS = MERGE_THREADS / 32;
template <bool GUARD, class SlotPtr>
__device__ __forceinline__ void merge_row(SlotPtr slot_ptr, int n, _Float16 *__restrict__ out_row, float *lse_row,
                                          float *s_red /*[MERGE_GROUPS * 130]*/, int tid)
{
    const int quad = tid & 31, grp = tid >> 5;
    float M = SQ_NEG_INF, lsum = 0.0f;
    f4 acc = {0.f, 0.f, 0.f, 0.f};
    const f4 zero4 = {0.f, 0.f, 0.f, 0.f};
    // weight of a partial with maximum mx under the running maximum Mn (Mn >= mx)
    auto wgt = [](float mx, float Mn) { return mx == SQ_NEG_INF ? 0.0f : __expf(mx - Mn); };
    int c = grp;
    for (; c + 3 * MERGE_GROUPS < n; c += 4 * MERGE_GROUPS) {
        const float *p0 = slot_ptr(c), *p1 = slot_ptr(c + MERGE_GROUPS), *p2 = slot_ptr(c + 2 * MERGE_GROUPS),
                    *p3 = slot_ptr(c + 3 * MERGE_GROUPS);
        const float2 a0 = *reinterpret_cast<const float2 *>(p0), a1 = *reinterpret_cast<const float2 *>(p1),
                     a2 = *reinterpret_cast<const float2 *>(p2), a3 = *reinterpret_cast<const float2 *>(p3);
        f4 o0 = *reinterpret_cast<const f4 *>(p0 + 4 + quad * 4), o1 = *reinterpret_cast<const f4 *>(p1 + 4 + quad * 4),
           o2 = *reinterpret_cast<const f4 *>(p2 + 4 + quad * 4), o3 = *reinterpret_cast<const f4 *>(p3 + 4 + quad * 4);
        if (GUARD) {
            o0 = a0.x == SQ_NEG_INF ? zero4 : o0;
            o1 = a1.x == SQ_NEG_INF ? zero4 : o1;
            o2 = a2.x == SQ_NEG_INF ? zero4 : o2;
            o3 = a3.x == SQ_NEG_INF ? zero4 : o3;
        }
        const float Mn = fmaxf(fmaxf(M, fmaxf(a0.x, a1.x)), fmaxf(a2.x, a3.x));
        const float sc = wgt(M, Mn);                     // M = -inf before the first partial: scale 0
        const float w0 = wgt(a0.x, Mn), w1 = wgt(a1.x, Mn), w2 = wgt(a2.x, Mn), w3 = wgt(a3.x, Mn);
        acc = acc * sc + o0 * w0 + o1 * w1 + o2 * w2 + o3 * w3;
        lsum = lsum * sc + a0.y * w0 + a1.y * w1 + a2.y * w2 + a3.y * w3;
        M = Mn;
    }
    for (; c + MERGE_GROUPS < n; c += 2 * MERGE_GROUPS) {       // two partials in flight (rows of 33 .. 128 partials)
        const float *p0 = slot_ptr(c), *p1 = slot_ptr(c + MERGE_GROUPS);
        const float2 a0 = *reinterpret_cast<const float2 *>(p0), a1 = *reinterpret_cast<const float2 *>(p1);
        f4 o0 = *reinterpret_cast<const f4 *>(p0 + 4 + quad * 4), o1 = *reinterpret_cast<const f4 *>(p1 + 4 + quad * 4);
        if (GUARD) {
            o0 = a0.x == SQ_NEG_INF ? zero4 : o0;
            o1 = a1.x == SQ_NEG_INF ? zero4 : o1;
        }
        const float Mn = fmaxf(M, fmaxf(a0.x, a1.x));
        const float sc = wgt(M, Mn), w0 = wgt(a0.x, Mn), w1 = wgt(a1.x, Mn);
        acc = acc * sc + o0 * w0 + o1 * w1;
        lsum = lsum * sc + a0.y * w0 + a1.y * w1;
        M = Mn;
    }
    for (; c < n; c += MERGE_GROUPS) {
        const float *p = slot_ptr(c);
        const float2 a = *reinterpret_cast<const float2 *>(p);
        f4 o = *reinterpret_cast<const f4 *>(p + 4 + quad * 4);
        if (GUARD) o = a.x == SQ_NEG_INF ? zero4 : o;
        const float Mn = fmaxf(M, a.x);
        const float sc = wgt(M, Mn), w = wgt(a.x, Mn);
        acc = acc * sc + o * w;
        lsum = lsum * sc + a.y * w;
        M = Mn;
    }
    // Fold the groups: s_red[g] = (M_g, l_g, o_g[128]).  A group that saw no partial has M_g = -inf.
    float *mine = s_red + grp * 130;
    if (quad == 0) {
        mine[0] = M;
        mine[1] = lsum;
    }
#pragma unroll
    for (int e = 0; e < 4; ++e) mine[2 + quad * 4 + e] = acc[e];
    __syncthreads();
    if (tid < D) {
        float Mt = SQ_NEG_INF;
#pragma unroll
        for (int g = 0; g < MERGE_GROUPS; ++g) Mt = fmaxf(Mt, s_red[g * 130]);
        float a = 0.0f, l = 0.0f;
#pragma unroll
        for (int g = 0; g < MERGE_GROUPS; ++g) {
            const float mg = s_red[g * 130];
            const float w = mg == SQ_NEG_INF ? 0.0f : __expf(mg - Mt);
            a += w * s_red[g * 130 + 2 + tid];
            l += w * s_red[g * 130 + 1];
        }
        const bool empty = n == 0 || !(l > 0.0f);
        out_row[tid] = (_Float16)(empty ? 0.0f : a / l);
        if (lse_row && tid == 0) *lse_row = empty ? SQ_NEG_INF : Mt + logf(l);
    }
}

}  // namespace sq
