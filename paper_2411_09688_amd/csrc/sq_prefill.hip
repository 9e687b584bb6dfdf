// Prefill-time sparse attention (Section 4.2) with per-query selection: every query token attends to the
// keys of the clusters set in its own keep mask, plus the (causal) user keys, one softmax over the union.
//
// Layout of the computation (FlashAttention-2 style: grid over heads x query blocks, loop over key blocks,
// online softmax), written for CDNA4 matrix cores:
//   * a workgroup = 4 waves x 16*QT queries; all waves walk the same 64-key blocks, whose K tile and
//     transposed V tile are staged in LDS once per workgroup;
//   * scores are computed TRANSPOSED, S^T = K Q^T, with 16x16x32 fp16 MFMA tiles (A = 16 keys, B = 16
//     queries).  In the accumulator layout a lane then owns ONE query column for the whole kernel (and four
//     keys per tile), so the running maximum, the running sum and the rescaling of the output are per-lane
//     scalars, and P^T is repacked into the B operand of the next product in registers, with no
//     cross-lane traffic;
//   * O^T = V^T P^T uses A = V^T tiles read from an LDS copy of V that was transposed on the way in, with
//     the keys of each 32-key group permuted so that the eight keys a lane needs are 16 contiguous bytes;
//   * the per-query keep masks are applied per (query, key): a small pre-kernel expands the cluster offsets
//     into a key -> cluster map, each key block brings the (at most three) mask words that can cover its
//     clusters for every query of the workgroup, and a wave skips the products of a block none of its
//     queries kept.
// The user block is causal when causal_user is set (query t sees user keys 0..t); the fixed context is
// always fully visible.
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

constexpr int PF_BN = 64;                 // keys per block
constexpr int PF_KS_STRIDE = D + 8;       // halves per K row in LDS (272 B: conflict-free 16-B reads)
constexpr int PF_VT_STRIDE = PF_BN + 8;   // halves per V^T row in LDS (144 B)

// key -> cluster id map of every head (clusters are contiguous key ranges).
__global__ __launch_bounds__(256) void key_cluster_kernel(const int32_t *__restrict__ offsets, int32_t *__restrict__ cid,
                                                          int C, int L)
{
    const int h = blockIdx.y;
    const int32_t *off = offsets + (size_t)h * (C + 1);
    for (int c = blockIdx.x * 4 + (threadIdx.x >> 6); c < C; c += gridDim.x * 4) {
        const int a = max(0, off[c]), b = min(L, off[c + 1]);
        for (int j = a + (threadIdx.x & 63); j < b; j += 64) cid[(size_t)h * L + j] = c;
    }
}

__device__ __forceinline__ int s_cid_first(const int32_t *key_cid, int h, int L, int j0, int C)
{
    return min(key_cid[(size_t)h * L + j0], C - 1);
}

// Position of key kappa (0..63) of a block inside a V^T row: within each 32-key group, key (t*16 + g*4 + j)
// goes to g*8 + t*4 + j, so that the B operand's keys (two accumulator tiles x 4 keys) are contiguous.
__device__ __forceinline__ int vt_pos(int kappa)
{
    const int ks = kappa >> 5, k2 = kappa & 31, t = k2 >> 4, g = (k2 & 15) >> 2, j = k2 & 3;
    return ks * 32 + g * 8 + t * 4 + j;
}

template <int QT>
__global__ __launch_bounds__(256) void prefill_attn_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ Kf, const _Float16 *__restrict__ Vf,
    const _Float16 *__restrict__ Ku, const _Float16 *__restrict__ Vu, const uint32_t *__restrict__ keep_mask,
    const int32_t *__restrict__ key_cid, _Float16 *__restrict__ out, float *__restrict__ lse, int H, int L, int C,
    int Lq, int U, int causal_user, float sm_scale)
{
    constexpr int BM = 64 * QT;           // queries per workgroup
    __shared__ __align__(16) _Float16 s_K[PF_BN * PF_KS_STRIDE];
    __shared__ __align__(16) _Float16 s_Vt[D * PF_VT_STRIDE];
    __shared__ __align__(16) int s_cid[PF_BN];
    __shared__ __align__(16) uint32_t s_mw[BM * 4];       // up to 3 mask words per query for the current block
    __shared__ int s_w0, s_wide;

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const int h = blockIdx.y, b = blockIdx.z;
    const int q0 = blockIdx.x * BM;                       // first query of the workgroup
    const int W = (C + 31) >> 5;
    const size_t row0 = ((size_t)b * H + h) * Lq;         // query-row index of query 0 of this (b, h)

    // Queries of this lane: n[qt] = q0 + wave*16*QT + qt*16 + col; B operand of S^T = K Q^T.
    h8 bq[QT][4];
    int nq[QT];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        nq[qt] = q0 + wave * 16 * QT + qt * 16 + col;
        const int nc = min(nq[qt], Lq - 1);
        const h8 *qp = reinterpret_cast<const h8 *>(q + (row0 + nc) * D);
#pragma unroll
        for (int s = 0; s < 4; ++s) bq[qt][s] = qp[s * 4 + kg];
    }

    float m_run[QT], l_run[QT];
    f4 o[QT][8];
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        m_run[qt] = SQ_NEG_INF;
        l_run[qt] = 0.0f;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) o[qt][dt] = f4{0.f, 0.f, 0.f, 0.f};
    }

    const _Float16 *Kfh = Kf + (size_t)h * L * D, *Vfh = Vf + (size_t)h * L * D;
    const _Float16 *Kuh = Ku + ((size_t)b * H + h) * (size_t)U * D, *Vuh = Vu + ((size_t)b * H + h) * (size_t)U * D;
    const int nblk_fixed = (L + PF_BN - 1) / PF_BN;
    // Causal user block: queries of this workgroup see user keys 0 .. min(U, q0 + BM) - 1 at most.
    const int u_vis = causal_user ? min(U, q0 + BM) : U;
    const int nblk_user = (u_vis + PF_BN - 1) / PF_BN;

    for (int blk = 0; blk < nblk_fixed + nblk_user; ++blk) {
        const bool user = blk >= nblk_fixed;
        const int j0 = (user ? blk - nblk_fixed : blk) * PF_BN;       // first key of the block
        const int nkeys = user ? U : L;
        const _Float16 *Kb = user ? Kuh : Kfh, *Vb = user ? Vuh : Vfh;

        // ---- stage the block: K rows, V transposed, cluster ids, mask words --------------------------------
        __syncthreads();                                   // previous block's LDS reads are done
        if (!user) {
            if (tid < PF_BN) {
                const int j = j0 + tid;
                const int c = j < L ? key_cid[(size_t)h * L + j] : 0x7fffffff;
                s_cid[tid] = c;
                if (tid == 0) s_w0 = min(c, C - 1) >> 5;
                // Last real key of the block: if its cluster lies more than two mask words past the first
                // key's (empty clusters in between), the staged words do not cover the block.
                if (j == min(j0 + PF_BN, L) - 1) s_wide = (c >> 5) - (s_cid_first(key_cid, h, L, j0, C) >> 5) > 2;
            }
        }
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int key = i * 16 + (tid >> 4), chunk = tid & 15;
            const int j = min(j0 + key, nkeys - 1);
            const h8 kv = *reinterpret_cast<const h8 *>(Kb + (size_t)j * D + chunk * 8);
            const h8 vv = *reinterpret_cast<const h8 *>(Vb + (size_t)j * D + chunk * 8);
            *reinterpret_cast<h8 *>(s_K + key * PF_KS_STRIDE + chunk * 8) = kv;
            const int pos = vt_pos(key);
#pragma unroll
            for (int e = 0; e < 8; ++e) s_Vt[(chunk * 8 + e) * PF_VT_STRIDE + pos] = vv[e];
        }
        __syncthreads();
        if (!user) {
            // Mask words w0 .. w0+2 of every query of the workgroup (64 consecutive clusters span <= 3 words).
            const int w0 = s_w0;
            for (int t = tid; t < BM * 3; t += 256) {
                const int ql = t / 3, wi = t - ql * 3;
                const int n = min(q0 + ql, Lq - 1);
                const int w = w0 + wi;
                s_mw[ql * 4 + wi] = w < W ? keep_mask[(row0 + n) * W + w] : 0u;
            }
            __syncthreads();
        }

        // ---- visibility of this lane's (query, key) pairs --------------------------------------------------
        // vis[qt] bit (kt*4 + v): key kt*16 + kg*4 + v of the block is visible to query nq[qt].
        uint32_t vis[QT];
        bool any = false;
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            uint32_t bits = 0;
            if (!user) {
                const int w0 = s_w0;
                const bool wide = s_wide != 0;                     // workgroup-uniform, rare
                const uint4 mw = *reinterpret_cast<const uint4 *>(s_mw + (wave * 16 * QT + qt * 16 + col) * 4);
                const uint32_t *mrow = keep_mask + (row0 + min(nq[qt], Lq - 1)) * W;
#pragma unroll
                for (int kt = 0; kt < 4; ++kt) {
                    const int4 c4 = *reinterpret_cast<const int4 *>(s_cid + kt * 16 + kg * 4);
                    const int cc[4] = {c4.x, c4.y, c4.z, c4.w};
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int wi = (cc[v] >> 5) - w0;          // 0..2 for real keys, huge for padding
                        uint32_t word = wi == 0 ? mw.x : (wi == 1 ? mw.y : (wi == 2 ? mw.z : 0u));
                        if (wide && cc[v] < C) word = mrow[cc[v] >> 5];   // block spans > 3 mask words
                        bits |= ((word >> (cc[v] & 31)) & 1u) << (kt * 4 + v);
                    }
                }
            } else {
#pragma unroll
                for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const int j = j0 + kt * 16 + kg * 4 + v;
                        const bool ok = j < U && (!causal_user || j <= nq[qt]);
                        bits |= (ok ? 1u : 0u) << (kt * 4 + v);
                    }
            }
            if (nq[qt] >= Lq) bits = 0;
            vis[qt] = bits;
            any |= bits != 0;
        }
        if (__ballot(any) == 0ull) continue;                // none of this wave's queries sees the block

        // ---- S^T = K Q^T -----------------------------------------------------------------------------------
        f4 st[QT][4];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt)
#pragma unroll
            for (int kt = 0; kt < 4; ++kt) st[qt][kt] = f4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int kt = 0; kt < 4; ++kt) {
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const h8 a = *reinterpret_cast<const h8 *>(s_K + (kt * 16 + col) * PF_KS_STRIDE + s * 32 + kg * 8);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    st[qt][kt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq[qt][s], st[qt][kt], 0, 0, 0);
            }
        }

        // ---- online softmax per query column; P^T packed as the B operand of the next product ---------------
        h8 bp[QT][2];
#pragma unroll
        for (int qt = 0; qt < QT; ++qt) {
            float mx = SQ_NEG_INF;
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const bool ok = (vis[qt] >> (kt * 4 + v)) & 1u;
                    const float sv = ok ? st[qt][kt][v] * sm_scale : SQ_NEG_INF;
                    st[qt][kt][v] = sv;
                    mx = fmaxf(mx, sv);
                }
            mx = cross16_max(mx);                           // the 4 lane groups hold the other keys of the column
            const float m_new = fmaxf(m_run[qt], mx);
            const float alpha = m_new == SQ_NEG_INF ? 1.0f : __expf(m_run[qt] - m_new);
            float psum = 0.0f;
            float pv[16];
#pragma unroll
            for (int kt = 0; kt < 4; ++kt)
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const float sv = st[qt][kt][v];
                    const float p = sv == SQ_NEG_INF ? 0.0f : __expf(sv - m_new);
                    pv[kt * 4 + v] = p;
                    psum += p;
                }
            m_run[qt] = m_new;
            l_run[qt] = l_run[qt] * alpha + psum;           // per-lane partial; groups are summed at the end
#pragma unroll
            for (int dt = 0; dt < 8; ++dt) o[qt][dt] *= alpha;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                h8 bv;
#pragma unroll
                for (int j = 0; j < 4; ++j) {
                    bv[j] = (_Float16)pv[(2 * ks) * 4 + j];
                    bv[4 + j] = (_Float16)pv[(2 * ks + 1) * 4 + j];
                }
                bp[qt][ks] = bv;
            }
        }

        // ---- O^T += V^T P^T --------------------------------------------------------------------------------
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const h8 a = *reinterpret_cast<const h8 *>(s_Vt + (dt * 16 + col) * PF_VT_STRIDE + ks * 32 + kg * 8);
#pragma unroll
                for (int qt = 0; qt < QT; ++qt)
                    o[qt][dt] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bp[qt][ks], o[qt][dt], 0, 0, 0);
            }
        }
    }

    // ---- normalise and store: lane holds query column nq[qt], dims dt*16 + kg*4 + v ---------------------------
#pragma unroll
    for (int qt = 0; qt < QT; ++qt) {
        const float lt = cross16_sum(l_run[qt]);
        if (nq[qt] >= Lq) continue;
        const bool empty = !(lt > 0.0f);
        const float inv = empty ? 0.0f : 1.0f / lt;
        _Float16 *orow = out + (row0 + nq[qt]) * D;
#pragma unroll
        for (int dt = 0; dt < 8; ++dt) {
            h4 hv;
#pragma unroll
            for (int v = 0; v < 4; ++v) hv[v] = (_Float16)(o[qt][dt][v] * inv);
            *reinterpret_cast<h4 *>(orow + dt * 16 + kg * 4) = hv;
        }
        if (lse && kg == 0) lse[row0 + nq[qt]] = empty ? SQ_NEG_INF : m_run[qt] + logf(lt);
    }
}

hipError_t launch_prefill_attn(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                               const uint32_t *keep_mask, const int32_t *offsets, int32_t *key_cid, void *out,
                               float *lse, const Shape &sh, hipStream_t s)
{
    hipLaunchKernelGGL(key_cluster_kernel, dim3(64, sh.H), dim3(256), 0, s, offsets, key_cid, sh.C, sh.L);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    constexpr int QT = 1;
    dim3 grid((sh.Lq + 64 * QT - 1) / (64 * QT), sh.H, sh.B);
    const bool prof = profile_mark(s, true);
    hipLaunchKernelGGL(prefill_attn_kernel<QT>, grid, dim3(256), 0, s, (const _Float16 *)q, (const _Float16 *)Kf,
                       (const _Float16 *)Vf, (const _Float16 *)Ku, (const _Float16 *)Vu, keep_mask, key_cid,
                       (_Float16 *)out, lse, sh.H, sh.L, sh.C, sh.Lq, sh.U, sh.causal_user, sh.sm_scale);
    if (prof) profile_mark(s, false);
    return hipGetLastError();
}

}  // namespace sq
