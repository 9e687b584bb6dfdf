// Decode-time sparse attention (Section 4.2): exact attention of one query per (sequence, head) over
// the selected fixed-context key ranges plus the dense user keys, split along the key dimension into
// chunks of KPC keys (the split-KV scheme: a head that keeps more keys gets more workgroups), each
// chunk producing a partial (max, sum, output) that a second phase merges.
//
// The kernel is bound by HBM: every selected K and V row (256 B each) is read exactly once.  A
// workgroup owns one chunk; 16 lanes share a row (16 B per lane, so a wave-wide load covers four
// whole rows), and every lane issues all of its K and V loads before any arithmetic, so a
// workgroup keeps its whole 128 KiB chunk in flight.  Scores are reduced over the 16 lanes of a row
// with DPP rotations; the softmax runs per wave and the four wave results are combined in LDS.
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

constexpr int KW = KPC / 4;     // keys per wave
constexpr int NI = KW / 4;      // loads per lane (4 rows per wave-wide load)

__global__ __launch_bounds__(256) void decode_partial_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ Kf, const _Float16 *__restrict__ Vf,
    const _Float16 *__restrict__ Ku, const _Float16 *__restrict__ Vu, DecodePlan plan,
    float *__restrict__ partials, int H, int L, int U, int n_user_chunks, float sm_scale)
{
    __shared__ int4 s_rec[KPC];
    __shared__ int s_rows[KPC];
    __shared__ float s_part[4][PART_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, p = lane & 15;
    const int c = blockIdx.x;
    const size_t bh = blockIdx.y;
    const int h = (int)(bh % H);
    const int chunks_per_row = n_user_chunks + plan.chunk_cap;

    const h8 qv = *reinterpret_cast<const h8 *>(q + bh * D + p * 8);

    const _Float16 *Kbase, *Vbase;
    int nvalid;
    const bool user = c < n_user_chunks;
    if (user) {
        const int k0 = c * KPC;
        nvalid = min(KPC, U - k0);
        Kbase = Ku + (bh * U + k0) * D;
        Vbase = Vu + (bh * U + k0) * D;
    } else {
        const int cf = c - n_user_chunks;
        const int2 hdr = plan.hdr[bh];                 // (records, selected keys)
        const int key0 = cf * KPC;
        if (key0 >= hdr.y) return;                     // chunk past the selection: whole workgroup leaves
        nvalid = min(KPC, hdr.y - key0);
        const int first = plan.chunk_first[bh * plan.chunk_cap + cf];
        // A chunk of KPC keys touches at most KPC records (each holds at least one of its keys).
        {
            const int idx = first + tid;
            int4 r = make_int4(0, 0, 0x7fffffff, 0);
            if (idx < hdr.x) r = plan.rec[bh * plan.rec_cap + idx];
            s_rec[tid] = r;
        }
        __syncthreads();
        {
            // Last staged record whose key prefix is <= this thread's key (records ascend in .z).
            const int kk = key0 + min(tid, nvalid - 1);
            int lo = 0;
#pragma unroll
            for (int step = KPC / 2; step > 0; step >>= 1)
                if (s_rec[lo + step].z <= kk) lo += step;
            const int4 r = s_rec[lo];
            int rowi = r.x + (kk - r.z);
            rowi = max(0, min(rowi, L - 1));           // malformed ranges cannot leave the tensor
            s_rows[tid] = rowi;
        }
        __syncthreads();
        Kbase = Kf + (size_t)h * L * D;
        Vbase = Vf + (size_t)h * L * D;
    }

    // Issue every K and V load of this lane.
    h8 kreg[NI], vreg[NI];
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int kl = wave * KW + i * 4 + g;
        const int rowi = user ? min(kl, nvalid - 1) : s_rows[kl];
        const size_t o = (size_t)rowi * D + p * 8;
        kreg[i] = *reinterpret_cast<const h8 *>(Kbase + o);
        vreg[i] = *reinterpret_cast<const h8 *>(Vbase + o);
    }

    // Scores of this lane-group's keys and the wave-local softmax.
    float s[NI];
    float m_w = SQ_NEG_INF;
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const int kl = wave * KW + i * 4 + g;
        float d = row16_sum(dot8(qv, kreg[i], 0.0f)) * sm_scale;
        s[i] = kl < nvalid ? d : SQ_NEG_INF;
        m_w = fmaxf(m_w, s[i]);
    }
    m_w = cross16_max(m_w);
    float l_w = 0.0f;
    float o[8] = {0, 0, 0, 0, 0, 0, 0, 0};
#pragma unroll
    for (int i = 0; i < NI; ++i) {
        const float pr = s[i] == SQ_NEG_INF ? 0.0f : __expf(s[i] - m_w);
        l_w += pr;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] += pr * (float)vreg[i][e];
    }
    l_w = cross16_sum(l_w);
#pragma unroll
    for (int e = 0; e < 8; ++e) o[e] = cross16_sum(o[e]);
    if (g == 0) {
        if (p == 0) {
            s_part[wave][0] = m_w;
            s_part[wave][1] = l_w;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) s_part[wave][4 + p * 8 + e] = o[e];
    }
    __syncthreads();

    // Combine the four waves; threads 0..127 own one output dimension each.
    if (tid < D) {
        float M = fmaxf(fmaxf(s_part[0][0], s_part[1][0]), fmaxf(s_part[2][0], s_part[3][0]));
        float lsum = 0.0f, acc = 0.0f;
#pragma unroll
        for (int w = 0; w < 4; ++w) {
            const float mw = s_part[w][0];
            const float sc = mw == SQ_NEG_INF ? 0.0f : __expf(mw - M);
            lsum += sc * s_part[w][1];
            acc += sc * s_part[w][4 + tid];
        }
        float *dst = partials + (bh * chunks_per_row + c) * PART_STRIDE;
        if (tid == 0) {
            dst[0] = M;
            dst[1] = lsum;
        }
        dst[4 + tid] = acc;
    }
}

// Phase 2: merge the partials of one (sequence, head):  out = sum_c e^{m_c - M} o_c / sum_c e^{m_c - M} l_c.
__global__ __launch_bounds__(128) void decode_merge_kernel(const float *__restrict__ partials, DecodePlan plan,
                                                           _Float16 *__restrict__ out, float *__restrict__ lse,
                                                           int U, int n_user_chunks)
{
    const size_t bh = blockIdx.x;
    const int tid = threadIdx.x;
    const int chunks_per_row = n_user_chunks + plan.chunk_cap;
    const int n_fixed = (plan.hdr[bh].y + KPC - 1) / KPC;
    const float *base = partials + bh * chunks_per_row * PART_STRIDE;
    // Valid chunks: user chunks 0..n_user_chunks-1, fixed chunks n_user_chunks..n_user_chunks+n_fixed-1.
    const int n = n_user_chunks + n_fixed;
    float M = SQ_NEG_INF;
    for (int c = 0; c < n; ++c) M = fmaxf(M, base[c * PART_STRIDE]);
    float lsum = 0.0f, acc = 0.0f;
    for (int c = 0; c < n; ++c) {
        const float *pc = base + c * PART_STRIDE;
        const float sc = __expf(pc[0] - M);
        lsum += sc * pc[1];
        acc += sc * pc[4 + tid];
    }
    const bool empty = n == 0 || lsum == 0.0f;
    out[bh * D + tid] = (_Float16)(empty ? 0.0f : acc / lsum);
    if (lse && tid == 0) lse[bh] = empty ? SQ_NEG_INF : M + logf(lsum);
}

hipError_t launch_decode_attn(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                              DecodePlan plan, const int32_t *, const int32_t *, float *partials, void *out,
                              float *lse, const Shape &sh, hipStream_t s)
{
    const int nuc = user_chunks_for(sh.U);
    const int rows = sh.B * sh.H;
    dim3 grid(nuc + plan.chunk_cap, rows);
    hipLaunchKernelGGL(decode_partial_kernel, grid, dim3(256), 0, s, (const _Float16 *)q, (const _Float16 *)Kf,
                       (const _Float16 *)Vf, (const _Float16 *)Ku, (const _Float16 *)Vu, plan, partials, sh.H, sh.L,
                       sh.U, nuc, sh.sm_scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_merge_kernel, dim3(rows), dim3(128), 0, s, partials, plan, (_Float16 *)out, lse, sh.U,
                       nuc);
    return hipGetLastError();
}

}  // namespace sq
