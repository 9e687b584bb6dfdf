// Dense attention of one query row over its user/generated keys (Section 3.2: they are attended to densely, whatever
// the lookup keeps), as partial results for the split-KV merge.  The user keys do not depend on the selection, so a
// decode step computes this part in extra workgroups of a launch that leaves the memory system idle, and the partial
// kernel's other workgroups stream only the selected fixed-context keys.  Two forms:
//
// user_chunk_partial (steps on the work-list kernels): extra workgroups of the SELECTION launch -- a launch that occupies
// one compute unit per row and leaves the rest of the chip idle.  One 1024-thread workgroup per (row, chunk of KPC user
// keys) -- a compute unit pulls ~27 GB/s at most, so the chunks of a row must not share one -- with the arithmetic of
// the partial kernel: a wave owns 8 key slots of the chunk, 16 lanes per key row, every K/V load in flight before the
// arithmetic.  The 16 waves' results are folded in LDS into ONE partial result at slot slot_base + row * nuq + chunk
// (nuq = chunks per row).
//
// user_piece_partial (steps through the key-index list): extra workgroups of the PARTIAL kernel's launch, 256 threads per
// piece of USER_PIECE keys (see there).
#pragma once
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

__device__ __forceinline__ void user_chunk_partial(const UserAttn &ua, int unit, float *s_part /*[16][PART_STRIDE]*/)
{
    constexpr int KW = KPC / 16, NI = KW / 4;               // key slots per wave; loads per lane (4 rows per wave load)
    const int row = unit / ua.nuq, c = unit - row * ua.nuq;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, p = lane & 15;
    const size_t bkv = (size_t)row / ua.G;                  // (sequence, K/V head): G query rows share its user keys
    const int first = c * KPC, nvalid = min(KPC, ua.U - first);
    const _Float16 *Kb = ua.Ku + (bkv * (size_t)ua.U + first) * D, *Vb = ua.Vu + (bkv * (size_t)ua.U + first) * D;
    const h8 qv = *reinterpret_cast<const h8 *>(ua.q + (size_t)row * D + p * 8);
    h8 kreg[NI], vreg[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int kl = wave * KW + i * 4 + g;
        const size_t off = (size_t)min(kl, nvalid - 1) * D + p * 8;   // slots past the end re-read a valid row
        kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Kb + off));
        vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Vb + off));
    }
    float s[NI], m_w = SQ_NEG_INF;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int kl = wave * KW + i * 4 + g;
        const float d = row16_sum(dot8(qv, kreg[i], 0.0f)) * ua.sm_scale;
        s[i] = kl < nvalid ? d : SQ_NEG_INF;
        m_w = fmaxf(m_w, s[i]);
    }
    m_w = cross16_max(m_w);                                 // maximum over the wave's slots (-inf: none valid)
    float l_run = 0.0f, o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.0f;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const float pr = s[i] == SQ_NEG_INF ? 0.0f : __expf(s[i] - m_w);
        l_run += pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += pr * (float)vreg[i][e];
    }
    // The four lane groups of a wave, then the 16 waves.
    const float l_w = cross16_sum(l_run);
    float ow[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ow[e] = cross16_sum(o[e]);
    float *mine = s_part + (size_t)wave * PART_STRIDE;
    if (g == 0) {
        if (p == 0) {
            mine[0] = m_w;
            mine[1] = l_w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) mine[4 + p * 8 + e] = ow[e];
    }
    __syncthreads();
    if (tid < D) {
        float M = SQ_NEG_INF;
#pragma unroll
        for (int w = 0; w < 16; ++w) M = fmaxf(M, s_part[w * PART_STRIDE]);
        float lsum = 0.0f, acc = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; ++w) {
            const float mw = s_part[w * PART_STRIDE];
            const float sc = mw == SQ_NEG_INF ? 0.0f : __expf(mw - M);
            lsum += sc * s_part[w * PART_STRIDE + 1];
            acc += sc * s_part[w * PART_STRIDE + 4 + tid];
        }
        float *dst = ua.partials + ((size_t)ua.slot_base + unit) * PART_STRIDE;
        if (tid == 0) {
            dst[0] = M;
            dst[1] = lsum;
        }
        dst[4 + tid] = acc;
    }
}

// Dense attention of one query row over one piece of USER_PIECE of its user keys (Section 3.2: the user input is
// attended to densely, whatever the lookup keeps), as a partial (max, sum, output) for the split-KV merge.  The user keys
// depend on nothing the lookup computes: the decode step through the key-index list reads them in extra workgroups of
// its partial kernel, whose other workgroups spend their first microseconds on two dependent round trips (key counts,
// then index entries) and leave the memory system idle.  256 threads: a wave owns 16 of the piece's 64 keys (16 lanes per key row, four wave-wide loads of
// four whole rows), the four waves' results are folded in LDS.
__device__ __forceinline__ void user_piece_partial(const UserAttn &ua, int piece, float (*s_part)[PART_STRIDE])
{
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, g = lane >> 4, p = lane & 15;
    const int row = piece / ua.nuq, c = piece - row * ua.nuq;
    const size_t bkv = (size_t)row / ua.G;                  // (sequence, K/V head): G query rows share its user keys
    const int first = c * USER_PIECE, nvalid = min(USER_PIECE, ua.U - first);
    const _Float16 *Kb = ua.Ku + (bkv * (size_t)ua.U + first) * D, *Vb = ua.Vu + (bkv * (size_t)ua.U + first) * D;
    h8 kreg[4], vreg[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const size_t off = (size_t)min(wave * 16 + i * 4 + g, nvalid - 1) * D + p * 8;   // slots past the end re-read a valid row
        kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Kb + off));
        vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Vb + off));
    }
    const h8 qv = *reinterpret_cast<const h8 *>(ua.q + (size_t)row * D + p * 8);
    float s[4], m_w = SQ_NEG_INF;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float d = row16_sum(dot8(qv, kreg[i], 0.0f)) * ua.sm_scale;
        s[i] = wave * 16 + i * 4 + g < nvalid ? d : SQ_NEG_INF;
        m_w = fmaxf(m_w, s[i]);
    }
    m_w = cross16_max(m_w);                                 // maximum over the wave's slots (-inf: none valid)
    float l_run = 0.0f, o[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = 0.0f;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        const float pr = s[i] == SQ_NEG_INF ? 0.0f : __expf(s[i] - m_w);
        l_run += pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += pr * (float)vreg[i][e];
    }
    const float l_w = cross16_sum(l_run);
    float ow[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) ow[e] = cross16_sum(o[e]);
    if (g == 0) {
        if (p == 0) {
            s_part[wave][0] = m_w;
            s_part[wave][1] = l_w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) s_part[wave][4 + p * 8 + e] = ow[e];
    }
    __syncthreads();
    if (tid < D) {
        const float M = fmaxf(fmaxf(s_part[0][0], s_part[1][0]), fmaxf(s_part[2][0], s_part[3][0]));
        float lsum = 0.0f, acc = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = s_part[w][0];
            const float sc = mw == SQ_NEG_INF ? 0.0f : __expf(mw - M);
            lsum += sc * s_part[w][1];
            acc += sc * s_part[w][4 + tid];
        }
        float *dst = ua.partials + ((size_t)ua.slot_base + piece) * PART_STRIDE;
        if (tid == 0) {
            dst[0] = M;
            dst[1] = lsum;
        }
        dst[4 + tid] = acc;
    }
}

}  // namespace sq
