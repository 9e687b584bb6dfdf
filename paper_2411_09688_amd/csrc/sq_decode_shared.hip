// Decode-time sparse attention for a batch of sequences over ONE shared fixed context (Section 4.2 applied
// to the shared-prefix setting of Section 1): each sequence selects its own clusters, but a cluster kept by
// several sequences is read from HBM once.  Sequences are handled in groups of SG = 16; the work items of a
// (group, head) "union row" are chunks of KPC keys drawn from the clusters kept by ANY sequence of the group,
// every key carrying the set of sequences that kept it.  The user keys of a sequence are chunks owned by that
// one sequence.
//
// With 16 sequences per group the scores of a chunk form a 16-column matrix, which is the shape of a CDNA4
// matrix-core tile, so the arithmetic runs on MFMA and the kernel stays bound by the K/V stream:
//   * a workgroup takes a run of consecutive work items; each of its four waves owns 32 of an item's 128 key
//     slots and works alone between segment ends (no workgroup barrier inside a union row);
//   * scores are S^T = K Q^T on 16x16x32 fp16 tiles (A = 16 keys, B = the 16 queries of the group, kept in
//     registers per head).  K rows are loaded whole (16 lanes per 256-byte row, non-temporal: a row is needed once)
//     and reach the A-operand layout through the wave's LDS tile (row-major store, 16-byte reads);
//   * in the accumulator layout a lane owns ONE sequence (column) and a few keys, so the per-(key, sequence)
//     ownership bit, the running maximum, the running sum and the output rescaling are per-lane scalars;
//   * V rows are loaded whole (16 lanes per 256-byte row, a wave-wide load = 4 rows), stored row-major in a
//     wave-private LDS tile and read back as V^T tiles with the transposing LDS read; O^T += V^T P^T runs on MFMA
//     with P^T taken from the score accumulators in place;
//   * a lane's output accumulators hold its sequence's 128 dimensions spread over the four lane groups: 32
//     registers of state for all 16 sequences.
//
// Partial results and merge follow the single-sequence kernel: per (workgroup, union row) segment the four
// waves' results are combined in LDS and written as SG partial results (one per sequence of the group; those of
// sequences that owned no key in the segment are marked empty), and a second kernel merges the partials of every
// (sequence, head) row.  Rows are placed in the item list in the order they arrive and a row's rank in that
// order is recorded with it; segment (workgroup w, row) writes slot w + rank(row), which is unique because both
// w and the rank never decrease along the item list and one of them increases from one segment to the next.
#include <stdlib.h>

#include "sq_common.hpp"
#include "sq_internal.hpp"
#include "sq_merge.hpp"

namespace sq {

// The work list of `total` items is cut into one run of consecutive items per workgroup, kq = total / G items each
// and one more for the first total % G workgroups: every workgroup is busy, and since compute units take workgroups
// round robin and stream at the same rate each, every compute unit gets the same number of chunks to within three.
struct RunSplit {
    int kq, rem;
    __device__ __forceinline__ int start(int w) const { return w * kq + min(w, rem); }
    __device__ __forceinline__ int owner(int x) const      // the workgroup whose run holds item x
    {
        const int head = rem * (kq + 1);                   // items held by the longer runs
        return x < head ? x / (kq + 1) : rem + (x - head) / max(kq, 1);
    }
};
__device__ __forceinline__ RunSplit run_split(int total, int grid)
{
    RunSplit rs;
    rs.kq = total / grid;
    rs.rem = total - rs.kq * grid;
    return rs;
}


static_assert(KPC == 128 && SG == 16, "the shared-context kernel is written for 128-key chunks and 16 sequences");
constexpr int SV_STRIDE = D + 16; // halves per V row in LDS (288 B: the transposing reads hit 32 distinct banks)
constexpr int SK_STRIDE = D + 8;  // halves per K row in the same tile (272 B: conflict-free 16-byte reads)

struct WaveLds {                 // private to one wave, except while a segment's results are combined
    int pos[KPC], delta[KPC];    // run-length records of the current item
    uint32_t rset[KPC];          // set of sequences per record
    int rows[32];                // K/V row of the wave's key slots (-1 past the end)
    uint32_t kset[32];           // set of sequences per key slot (0 past the end)
    float ml[2 * SG];            // segment end: (m, l) of every sequence
    _Float16 Vt[32 * SV_STRIDE]; // K rows, then V rows of the current 32-key step; segment end: o[SG][D] as fp32
};
static_assert(sizeof(_Float16) * 32 * SV_STRIDE >= sizeof(float) * SG * D, "the V tile doubles as the output staging");

// LDS traffic inside a wave needs no hardware barrier (a wave's LDS operations complete in order), only a point
// the compiler does not move LDS accesses across.
__device__ __forceinline__ void wave_lds_sync()
{
    __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
    __builtin_amdgcn_wave_barrier();
    __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
}

__global__ __launch_bounds__(256, 3) void decode_attn_shared_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ Kf, const _Float16 *__restrict__ Vf,
    const _Float16 *__restrict__ Ku, const _Float16 *__restrict__ Vu, DecodePlan plan,
    float *__restrict__ partials, int BV, int G, int H, int L, int U, float sm_scale)
{
    __shared__ __align__(16) WaveLds s_w[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    WaveLds &S = s_w[wave];
    const int col = lane & 15, kg = lane >> 4;             // sequence of this lane; lane group
    const int j0 = wave * 32;                              // this wave's 32 key slots of every item

    const int total = min(plan.total[0], plan.item_cap);
    const RunSplit rs = run_split(total, (int)gridDim.x);
    int item = rs.start((int)blockIdx.x);
    const int item_end = rs.start((int)blockIdx.x + 1);
    if (item >= item_end) return;                          // whole workgroup

    const float c2 = sm_scale * 1.44269504088896341f;      // exp(sm_scale * s) = exp2(c2 * s)
    float m_run = SQ_NEG_INF, l_run = 0.0f;                // of sequence `col`; raw logit units; l is this lane's share
    f4 o[8];
#pragma unroll
    for (int dt = 0; dt < 8; ++dt) o[dt] = f4{0.f, 0.f, 0.f, 0.f};
    h8 bq[4] = {};                                         // Q^T operand: sequence col, dims s*32 + kg*8 .. +8
    int cur_row = -1;

    // End of a (workgroup, union row) segment: the four waves' running results are combined in LDS and written
    // as SG partials at slots (blockIdx.x + rank(row)) * SG + sequence.  Contains workgroup barriers.
    auto flush = [&](int row) {
        const float lt = cross16_sum(l_run);
        float *so = reinterpret_cast<float *>(S.Vt);       // [SG][D]
        wave_lds_sync();                                   // the last step's readers of V^T are done
        if (kg == 0) {
            S.ml[col * 2] = m_run;
            S.ml[col * 2 + 1] = lt;
        }
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) *reinterpret_cast<f4 *>(so + col * D + dt * 16 + kg * 4) = o[dt];
        __syncthreads();
        const int slot0 = ((int)blockIdx.x + plan.row_rank[row]) * SG;
        // thread t: dimension t % 128 of sequences t / 128, t / 128 + 2, ...
        const int dim = tid & (D - 1);
        for (int sq_ = tid >> 7; sq_ < SG; sq_ += 2) {
            float mw[4];
#pragma unroll
            for (int w = 0; w < 4; ++w) mw[w] = s_w[w].ml[sq_ * 2];
            const float M = fmaxf(fmaxf(mw[0], mw[1]), fmaxf(mw[2], mw[3]));
            float lsum = 0.0f, acc = 0.0f;
#pragma unroll
            for (int w = 0; w < 4; ++w) {
                const float sc = mw[w] == SQ_NEG_INF ? 0.0f : __builtin_amdgcn_exp2f((mw[w] - M) * c2);
                lsum += sc * s_w[w].ml[sq_ * 2 + 1];
                acc += sc * reinterpret_cast<const float *>(s_w[w].Vt)[sq_ * D + dim];
            }
            float *dst = partials + (size_t)(slot0 + sq_) * PART_STRIDE;
            const bool empty = M == SQ_NEG_INF;            // the sequence owned no key of this segment
            if (dim == 0) {
                dst[0] = empty ? SQ_NEG_INF : M * sm_scale;
                dst[1] = lsum;
            }
            if (!empty) dst[4 + dim] = acc;
        }
        __syncthreads();
    };

    // Header and this lane's two records of the next item travel in registers behind the K/V stream.
    int2 h0n, h1n, rcn[2];
    auto prefetch = [&](int i) {
        const int2 *it = plan.item + (size_t)i * ITEM_STRIDE;
        h0n = it[0];
        h1n = it[1];
        rcn[0] = it[2 + lane];
        rcn[1] = it[2 + 64 + lane];                        // inside the item's ITEM_STRIDE slots whatever its record count
    };
    prefetch(item);

    for (; item < item_end; ++item) {
        const int2 h0 = h0n, h1 = h1n;                     // (union row, keys) (records | -1 - sequence, first user key)
        const int2 rc[2] = {rcn[0], rcn[1]};
        const int row = h0.x, h = row % H, grp = row / H;
        if (row != cur_row) {                              // workgroup-uniform
            if (cur_row >= 0) {
                flush(cur_row);
                m_run = SQ_NEG_INF;
                l_run = 0.0f;
#pragma unroll
                for (int dt = 0; dt < 8; ++dt) o[dt] = f4{0.f, 0.f, 0.f, 0.f};
            }
            cur_row = row;
            const int vs = grp * SG + col;                 // virtual sequence of this lane's column
            if (vs < BV) {
                const h8 *qp = reinterpret_cast<const h8 *>(q + shared_row(vs, h, H, G) * D);
#pragma unroll
                for (int s = 0; s < 4; ++s) bq[s] = qp[s * 4 + kg];
            } else {
#pragma unroll
                for (int s = 0; s < 4; ++s) bq[s] = h8{0, 0, 0, 0, 0, 0, 0, 0};
            }
        }
        const int nvalid = h0.y;
        if (j0 >= nvalid) {                                // wave-uniform: a short chunk has no keys for this wave
            if (item + 1 < item_end) prefetch(item + 1);
            continue;
        }
        const bool user = h1.x < 0;
        const char *Kbase, *Vbase;                         // byte pointers; a row is 256 B
        const int t_my = j0 + (lane & 31);                 // key slot this lane resolves (both halves of the wave agree)
        wave_lds_sync();                                   // the previous item's readers are done
        if (user) {
            const int jb = -1 - h1.x;                      // real sequence within the group; its G columns own the chunk
            const size_t bh = (size_t)(grp * SG / G + jb) * H + h;
            Kbase = reinterpret_cast<const char *>(Ku + (bh * U + h1.y) * D);
            Vbase = reinterpret_cast<const char *>(Vu + (bh * U + h1.y) * D);
            if (lane < 32) {
                S.rows[lane] = t_my < nvalid ? t_my : -1;
                S.kset[lane] = t_my < nvalid ? (((1u << G) - 1u) << (jb * G)) : 0u;
            }
        } else {
            Kbase = reinterpret_cast<const char *>(Kf + (size_t)h * L * D);
            Vbase = reinterpret_cast<const char *>(Vf + (size_t)h * L * D);
            const int nrec = min(h1.x, KPC);
#pragma unroll
            for (int u = 0; u < 2; ++u) {
                const int t = lane + 64 * u;
                S.pos[t] = rc[u].x & 0xffff;
                S.rset[t] = (uint32_t)rc[u].x >> 16;
                S.delta[t] = rc[u].y;
            }
            wave_lds_sync();
            int lo = 0;
#pragma unroll
            for (int step = KPC / 2; step > 0; step >>= 1)
                if (lo + step < nrec && S.pos[lo + step] <= t_my) lo += step;
            const int r = t_my + S.delta[lo];
            const uint32_t ks = S.rset[lo];
            if (lane < 32) {
                S.rows[lane] = t_my < nvalid ? max(0, min(r, L - 1)) : -1;   // malformed input stays in the tensor
                S.kset[lane] = t_my < nvalid ? ks : 0u;
            }
        }
        wave_lds_sync();
        const int r_last = S.rows[min(nvalid - j0, 32) - 1];

        // ---- loads: K and V rows whole: lane group kg takes keys kg*8 + i, 16 bytes per lane --------------------------
        h8 kr[8], vr[8];
        {
            const int4 rv0 = *reinterpret_cast<const int4 *>(&S.rows[kg * 8]), rv1 = *reinterpret_cast<const int4 *>(&S.rows[kg * 8 + 4]);
            const int rv[8] = {rv0.x, rv0.y, rv0.z, rv0.w, rv1.x, rv1.y, rv1.z, rv1.w};
#pragma unroll
            for (int i = 0; i < 8; ++i)                    // slots past the end re-read a valid row
                kr[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Kbase + (size_t)(rv[i] < 0 ? r_last : rv[i]) * 256 + col * 16));
#pragma unroll
            for (int i = 0; i < 8; ++i)
                vr[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Vbase + (size_t)(rv[i] < 0 ? r_last : rv[i]) * 256 + col * 16));
        }
        if (item + 1 < item_end) prefetch(item + 1);
        // ownership bits of this lane's (key, sequence) pairs: element e = t*4 + v <-> key t*16 + kg*4 + v
        uint32_t msk[8];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            const uint4 ks = *reinterpret_cast<const uint4 *>(&S.kset[t * 16 + kg * 4]);
            msk[t * 4 + 0] = (uint32_t)__builtin_amdgcn_sbfe((int)ks.x, col, 1);
            msk[t * 4 + 1] = (uint32_t)__builtin_amdgcn_sbfe((int)ks.y, col, 1);
            msk[t * 4 + 2] = (uint32_t)__builtin_amdgcn_sbfe((int)ks.z, col, 1);
            msk[t * 4 + 3] = (uint32_t)__builtin_amdgcn_sbfe((int)ks.w, col, 1);
        }

        // ---- S^T = K Q^T ---------------------------------------------------------------------------------------------
        // K rows -> the wave's LDS tile (row-major) -> A-operand layout (tile t: key t*16 + col, dims s*32 + kg*8 .. +8)
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<h8 *>(S.Vt + (kg * 8 + i) * SK_STRIDE + col * 8) = kr[i];
        wave_lds_sync();
        h8 ka[2][4];
#pragma unroll
        for (int t = 0; t < 2; ++t)
#pragma unroll
            for (int s = 0; s < 4; ++s)
                ka[t][s] = *reinterpret_cast<const h8 *>(S.Vt + (t * 16 + col) * SK_STRIDE + s * 32 + kg * 8);
        wave_lds_sync();                                   // the tile is free for V
        f4 sacc[2];
#pragma unroll
        for (int t = 0; t < 2; ++t) {
            sacc[t] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s)
                sacc[t] = __builtin_amdgcn_mfma_f32_16x16x32_f16(ka[t][s], bq[s], sacc[t], 0, 0, 0);
        }

        // ---- V -> wave-private LDS, row-major ----------------------------------------------------------------------
#pragma unroll
        for (int i = 0; i < 8; ++i) *reinterpret_cast<h8 *>(S.Vt + (kg * 8 + i) * SV_STRIDE + col * 8) = vr[i];

        // ---- online softmax of column `col` -----------------------------------------------------------------------
        float sv[8];
        float mx = SQ_NEG_INF;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const float sraw = sacc[e >> 2][e & 3];        // (a copy: the bit cast below must not see a vector element)
            const uint32_t bits = __builtin_bit_cast(uint32_t, sraw);
            sv[e] = __builtin_bit_cast(float, (msk[e] & bits) | (~msk[e] & 0xff800000u));   // not owned: -inf
            mx = fmaxf(mx, sv[e]);
        }
        mx = cross16_max(mx);                              // the 4 lane groups hold the other keys of the column
        const float m_new = fmaxf(m_run, mx);
        const float mneg = m_new == SQ_NEG_INF ? 0.0f : -m_new * c2;   // nothing seen yet: exp2(-inf) = 0
        // (exactly 1 while the maximum stands still: m * c2 + fl(-m * c2) is the rounding error of the product, not 0)
        const float alpha = m_new == m_run ? 1.0f : __builtin_amdgcn_exp2f(fmaf(m_run, c2, mneg));
        float psum = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            sv[e] = __builtin_amdgcn_exp2f(fmaf(sv[e], c2, mneg));
            psum += sv[e];
        }
        m_run = m_new;
        l_run = l_run * alpha + psum;
        if (__ballot(alpha != 1.0f) != 0ull) {
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) o[dt] *= alpha;
        }
        h8 bp;                                             // P^T operand: sequence col, keys at positions kg*8 .. +8
#pragma unroll
        for (int e = 0; e < 8; ++e) bp[e] = (_Float16)sv[e];

        // ---- O^T += V^T P^T -----------------------------------------------------------------------------------------
        wave_lds_sync();                                   // V is written
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            // keys t*16 + kg*4 + (0..3) for t = 0, 1: the order P^T sits in the score accumulators
            const _Float16 *vp = S.Vt + (kg * 4 + (col >> 2)) * SV_STRIDE + dt * 16 + (col & 3) * 4;
            const h4 a0 = lds_read_tr16(vp), a1 = lds_read_tr16(vp + 16 * SV_STRIDE);
            const h8 a = {a0[0], a0[1], a0[2], a0[3], a1[0], a1[1], a1[2], a1[3]};
            o[dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bp, o[dt], 0, 0, 0);
        }
    }
    flush(cur_row);
}

// Phase 2: one workgroup per (sequence, head) row merges the partials its union row's segments wrote for
// that sequence.
__global__ __launch_bounds__(MERGE_THREADS) void decode_merge_shared_kernel(const float *__restrict__ partials,
                                                                            DecodePlan plan, _Float16 *__restrict__ out,
                                                                            float *__restrict__ lse, int H, int G,
                                                                            int attn_grid)
{
    __shared__ float s_red[MERGE_GROUPS * 130];
    const size_t bh = blockIdx.x;                    // output row (b, h, g) of the [B, H, G] tensors
    const int g = (int)(bh % G), h = (int)((bh / G) % H), vs = (int)(bh / ((size_t)G * H)) * G + g;
    const int urow = (vs / SG) * H + h, sq_ = vs % SG;
    const int2 it = plan.row_items[urow];            // (first item, items) of the union row
    const int rank = plan.row_rank[urow];
    const int total = min(plan.total[0], plan.item_cap);
    const RunSplit rs = run_split(total, attn_grid);
    const int w_lo = rs.owner(it.x);                 // the attention workgroups that hold the row's items
    const int n = it.y == 0 ? 0 : rs.owner(it.x + it.y - 1) - w_lo + 1;
    auto slot_ptr = [&](int c) { return partials + ((size_t)(w_lo + c + rank) * SG + sq_) * PART_STRIDE; };
    merge_row<true>(slot_ptr, n, out + bh * D, lse ? lse + bh : nullptr, s_red, threadIdx.x);
}

hipError_t launch_decode_attn_shared(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                                     DecodePlan plan, float *partials, void *out, float *lse, const Shape &sh,
                                     hipStream_t s)
{
    const int G = sh.Lq;                             // query rows per (sequence, head): 1, or the GQA group size
    const int rows = sh.B * sh.H * G;
    hipEvent_t ev0, ev1;
    if (profile_pair(&ev0, &ev1))
        hipExtLaunchKernelGGL(decode_attn_shared_kernel, dim3(SHARED_ATTN_GRID), dim3(256), 0, s, ev0, ev1, 0,
                              (const _Float16 *)q, (const _Float16 *)Kf, (const _Float16 *)Vf, (const _Float16 *)Ku,
                              (const _Float16 *)Vu, plan, partials, sh.B * G, G, sh.H, sh.L, sh.U, sh.sm_scale);
    else
        hipLaunchKernelGGL(decode_attn_shared_kernel, dim3(SHARED_ATTN_GRID), dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)Kf, (const _Float16 *)Vf, (const _Float16 *)Ku, (const _Float16 *)Vu, plan,
                           partials, sh.B * G, G, sh.H, sh.L, sh.U, sh.sm_scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_merge_shared_kernel, dim3(rows), dim3(MERGE_THREADS), 0, s, partials, plan,
                       (_Float16 *)out, lse, sh.H, G, SHARED_ATTN_GRID);
    return hipGetLastError();
}

}  // namespace sq
