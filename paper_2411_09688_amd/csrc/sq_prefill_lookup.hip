// Centroid lookup for prefill (Section 4.1): grid over (sequence, head) x query blocks; a workgroup makes two
// passes over the head's centroids.  Pass 1 accumulates, per query token, the maximum and the size-weighted
// normaliser of Eq. 1; pass 2 recomputes the same logits and turns them into scores, so no [queries x clusters]
// intermediate is ever written to memory (the centroids are read twice instead, from L2).
//
// Scores run on the matrix cores as S^T = C Q^T (16x16x32 fp16 tiles: A = 16 centroids, B = a wave's 16 query
// tokens, kept in registers), so a lane owns ONE query token (column) and four centroids per tile: maximum,
// normaliser and threshold test are per-lane scalars, combined over the four lane groups once per pass.  The
// four waves of a workgroup (64 tokens) share the centroid stream: groups of 64 centroids travel global memory ->
// registers (issued two groups ahead) -> one of two LDS stages -> A operands, one barrier per group.
//
//   MEAN == false  per-query selection: keep cluster i for token t iff N_i > 0 and exp(x_i - m) > T * D; the
//                  keep bits of two tiles are gathered into one mask word per token.
//   MEAN == true   selection on averaged scores (Appendix D, "Prefill Stage"), first half: the scores
//                  S_i(t) = exp(x_i - m) / D of a wave's 16 tokens are summed per cluster and written as one
//                  part of part_sum [B*H, ceil(Lq/16), C]; the row-wise selection kernel adds the parts.
//   CANDS == true  (with MEAN) second level of a hierarchical lookup (Section 3.3, Eq. 3): the clusters scored are the
//                  n candidates cand_id[bh, 0..n) of the (sequence, head) -- the children of the coarse clusters kept
//                  one level up -- so maximum and normaliser run over the candidates only; part_sum is written in
//                  candidate order.
//   PARENTS == true (per-query selection) second level of a hierarchical lookup with per-token candidates: fine
//                  cluster i counts for token t only if t kept its parent coarse cluster (bit parent[i] of the
//                  token's level-1 mask); the others are treated like clusters without keys, so maximum,
//                  normaliser and threshold test of Eq. 3 run over the token's candidates only.
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

constexpr int LK_TU = 4;                     // centroid tiles per group
constexpr int LK_G = LK_TU * 16;             // centroids per group
constexpr int LK_STRIDE = D + 8;             // halves per centroid row in LDS (272 B: conflict-free 16-B reads)

struct LkStage {
    _Float16 Ct[LK_G * LK_STRIDE];
    float Wt[LK_G];                          // cluster sizes as floats (exact: a head has fewer than 2^24 keys)
    float bias[LK_G];                        // 0 for a cluster with keys, -inf for one without (or past the end): the
                                             // score products start from it, so such a cluster's logit is -inf and
                                             // it drops out of maximum, normaliser and scores without a test
    int P[LK_G];                             // parent coarse cluster (PARENTS only)
};

constexpr int LK_MAX_W1 = 32;                // level-1 mask words per token held in LDS: at most 1024 coarse clusters

template <bool MEAN, bool CANDS = false, bool PARENTS = false>
__global__ __launch_bounds__(256) void prefill_lookup_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ cent, const int32_t *__restrict__ sizes,
    const float *__restrict__ thresh, uint32_t *__restrict__ keep_mask, int32_t *__restrict__ n_ranges,
    int32_t *__restrict__ n_keys, float *__restrict__ part_sum, const int32_t *__restrict__ cand_id,
    const int2 *__restrict__ cand_hdr, const uint32_t *__restrict__ mask1, int W1, int H, int Lq, int C_all,
    float sm_scale)
{
    __shared__ __align__(16) LkStage stage[2];
    __shared__ uint32_t s_m1[PARENTS ? 64 * LK_MAX_W1 : 1];   // level-1 masks of the workgroup's 64 tokens
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const int bh = blockIdx.y, h = bh % H;
    // C: the clusters this workgroup scores (all of the head's, or its candidates); C_all: row length of the arrays.
    const int C = CANDS ? min(cand_hdr[bh].y, C_all) : C_all;
    if (CANDS && C <= 0) return;                            // no candidate: nothing to score (workgroup-uniform)
    const int32_t *cid = CANDS ? cand_id + (size_t)bh * C_all : nullptr;
    const int32_t *par = PARENTS ? cand_id + (size_t)h * C_all : nullptr;     // (PARENTS: cand_id is parent [H, C])
    if (PARENTS) {
        for (int idx = threadIdx.x; idx < 64 * W1; idx += 256) {
            const int t = idx / W1, w = idx - t * W1;
            const int token = min((int)blockIdx.x * 64 + t, Lq - 1);
            s_m1[t * W1 + w] = mask1[((size_t)bh * Lq + token) * W1 + w];
        }
    }
    const int q0 = (blockIdx.x * 4 + wave) * LOOKUP_ROWS;   // first token of this wave (may lie past the end)
    const int nq = q0 + col;
    const bool valid = nq < Lq;
    const size_t row = (size_t)bh * Lq + min(nq, Lq - 1);
    const int W = (C + 31) >> 5;
    const int nt = (C + 15) >> 4, ng = (C + LK_G - 1) / LK_G;

    h8 bq[4];
    {
        const h8 *qp = reinterpret_cast<const h8 *>(q + row * D);
#pragma unroll
        for (int s = 0; s < 4; ++s) bq[s] = qp[s * 4 + kg];
    }
    const char *ch = reinterpret_cast<const char *>(cent + (size_t)h * C_all * D);
    const int32_t *Nh = sizes + (size_t)h * C_all;

    // This thread's share of a group: rows i*16 + tid/16 (i = 0..3), 16-byte chunk tid%16; size of cluster tid.
    h8 pk[4];
    int pn = 0, pp = 0;
    auto fetch = [&](int g) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            int c_row = min(g * LK_G + i * 16 + (tid >> 4), C - 1);          // rows past the end repeat the last one
            if (CANDS) c_row = min(max(cid[c_row], 0), C_all - 1);
            pk[i] = *reinterpret_cast<const h8 *>(ch + (size_t)c_row * 256 + (tid & 15) * 16);
        }
        if (tid < LK_G) {                                                    // 0 past the last cluster
            const int c = g * LK_G + tid;
            pn = c < C ? Nh[CANDS ? min(max(cid[c], 0), C_all - 1) : c] : 0;
            if (PARENTS) pp = c < C ? min(max(par[c], 0), W1 * 32 - 1) : 0;
        }
    };
    auto commit = [&](LkStage &st) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<h8 *>(st.Ct + (i * 16 + (tid >> 4)) * LK_STRIDE + (tid & 15) * 8) = pk[i];
        if (tid < LK_G) {
            st.Wt[tid] = (float)pn;
            st.bias[tid] = pn > 0 ? 0.0f : SQ_NEG_INF;
            if (PARENTS) st.P[tid] = pp;
        }
    };
    const float c2 = sm_scale * 1.44269504088896341f;
    // Logits of the staged group in units of log 2 (the exponentials below are base-2: one instruction each):
    // x[u][v] = sm_scale * log2(e) * q . C_c, c = g*64 + u*16 + kg*4 + v, and the cluster sizes.
    auto scores = [&](const LkStage &st, float (&x)[LK_TU][4], float (&nv)[LK_TU][4]) {
#pragma unroll
        for (int u = 0; u < LK_TU; ++u) {
            f4 acc = *reinterpret_cast<const f4 *>(st.bias + u * 16 + kg * 4);
#pragma unroll
            for (int s = 0; s < 4; ++s) {
                const h8 a = *reinterpret_cast<const h8 *>(st.Ct + (u * 16 + col) * LK_STRIDE + s * 32 + kg * 8);
                acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bq[s], acc, 0, 0, 0);
            }
            const f4 n4 = *reinterpret_cast<const f4 *>(st.Wt + u * 16 + kg * 4);
            nv[u][0] = n4.x;
            nv[u][1] = n4.y;
            nv[u][2] = n4.z;
            nv[u][3] = n4.w;
            if (PARENTS) {                                  // not a candidate of this lane's token: as if it had no keys
                const int4 p4 = *reinterpret_cast<const int4 *>(st.P + u * 16 + kg * 4);
                const uint32_t *mrow = s_m1 + (wave * 16 + col) * W1;
                const int pv[4] = {p4.x, p4.y, p4.z, p4.w};
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (!((mrow[pv[v] >> 5] >> (pv[v] & 31)) & 1u)) {
                        nv[u][v] = 0.0f;
                        acc[v] = SQ_NEG_INF;
                    }
            }
#pragma unroll
            for (int v = 0; v < 4; ++v) x[u][v] = acc[v] * c2;   // (-inf stays -inf: sm_scale > 0)
        }
    };

    float m = SQ_NEG_INF, Dsum = 0.0f, thr = 0.0f, inv_D = 0.0f, m_ref = 0.0f;
    uint32_t word = 0u;
    int cnt = 0;
    float keys = 0.0f;                                       // (exact in fp32, like the sizes)
    const int part = q0 / LOOKUP_ROWS, n_part = lookup_parts_for(Lq);

    // One loop over both passes: iteration it handles group it % ng; the stream of groups never drains in between.
    fetch(0);
    commit(stage[0]);
    if (2 * ng > 1) fetch(1 % ng);
    __syncthreads();
    for (int it = 0; it < 2 * ng; ++it) {
        const int g = it % ng;
        if (it + 1 < 2 * ng) {
            commit(stage[(it + 1) & 1]);                    // group it+1 (in registers since the last iteration)
            if (it + 2 < 2 * ng) fetch((it + 2) % ng);
        }
        float x[LK_TU][4];
        float nv[LK_TU][4];
        scores(stage[it & 1], x, nv);
        if (it < ng) {
            // ---- pass 1: m = max over clusters with keys, D = sum N_i exp(x_i - m), per token ---------------------
            // (a cluster without keys has x = -inf: it does not move the maximum and adds 0 * exp(-inf) = +0)
            float mt = m;
#pragma unroll
            for (int u = 0; u < LK_TU; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v) mt = fmaxf(mt, x[u][v]);
            if (mt != SQ_NEG_INF) {
                Dsum *= __builtin_amdgcn_exp2f(m - mt);      // m = -inf: Dsum is 0 and stays 0
#pragma unroll
                for (int u = 0; u < LK_TU; ++u)
#pragma unroll
                    for (int v = 0; v < 4; ++v) Dsum += nv[u][v] * __builtin_amdgcn_exp2f(x[u][v] - mt);
                m = mt;
            }
            if (it == ng - 1) {                              // the four lane groups hold the other clusters of the token
#pragma unroll
                for (int off = 16; off <= 32; off <<= 1) {
                    const float mo = __shfl_xor(m, off), Do = __shfl_xor(Dsum, off);
                    const float M = fmaxf(m, mo);
                    const float wa = m == SQ_NEG_INF ? 0.0f : __builtin_amdgcn_exp2f(m - M);
                    const float wb = mo == SQ_NEG_INF ? 0.0f : __builtin_amdgcn_exp2f(mo - M);
                    Dsum = Dsum * wa + Do * wb;
                    m = M;
                }
                thr = thresh[h] * Dsum;
                inv_D = valid && Dsum > 0.0f ? 1.0f / Dsum : 0.0f;   // scores of pass 2: e * (1 / D), one division per token
                m_ref = m == SQ_NEG_INF ? 0.0f : m;          // (no cluster with keys at all: exp(-inf - 0) = 0, not NaN)
            }
        } else {
            // ---- pass 2: the same logits again, now as scores ---------------------------------------------------------
#pragma unroll
            for (int u = 0; u < LK_TU; ++u) {
                const int t = g * LK_TU + u;
                if (t >= nt) break;                          // workgroup-uniform
                float e[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) e[v] = __builtin_amdgcn_exp2f(x[u][v] - m_ref);   // 0 for a cluster without keys
                if (!MEAN) {
#pragma unroll
                    for (int v = 0; v < 4; ++v) {
                        const bool keep = nv[u][v] > 0.0f && e[v] > thr;
                        word |= (uint32_t)keep << ((t & 1) * 16 + kg * 4 + v);
                        cnt += keep;
                        keys += keep ? nv[u][v] : 0.0f;
                    }
                    if ((t & 1) || t == nt - 1) {            // a mask word is complete
                        word = cross16_or(word);
                        if (kg == 0 && valid) keep_mask[row * W + (t >> 1)] = word;
                        word = 0u;
                    }
                } else {
                    float sums[4];
#pragma unroll
                    for (int v = 0; v < 4; ++v)             // over the wave's tokens
                        sums[v] = row16_sum(e[v] * inv_D);
                    if (col == 0 && part < n_part) {
                        float *dst = part_sum + ((size_t)bh * n_part + part) * C_all + t * 16 + kg * 4;
#pragma unroll
                        for (int v = 0; v < 4; ++v)
                            if (t * 16 + kg * 4 + v < C) dst[v] = sums[v];
                    }
                }
            }
        }
        __syncthreads();                                     // stage it & 1 may be overwritten; stage (it+1) & 1 is complete
    }
    if (!MEAN) {
        cnt = cross16_sum_i(cnt);
        const int keys_i = cross16_sum_i((int)keys);
        if (kg == 0 && valid) {
            n_ranges[row] = cnt;
            n_keys[row] = keys_i;
        }
    }
}

hipError_t launch_prefill_lookup(const void *q, const void *centroids, const int32_t *sizes, const float *thresh,
                                 uint32_t *keep_mask, int32_t *n_ranges, int32_t *n_keys, float *part_sum, bool mean,
                                 int B, int H, int Lq, int C, float sm_scale, hipStream_t s, const int32_t *cand_id,
                                 const int2 *cand_hdr, const int32_t *parent, const uint32_t *mask1, int C1)
{
    const dim3 grid((Lq + 4 * LOOKUP_ROWS - 1) / (4 * LOOKUP_ROWS), B * H);
    const uint32_t *no_mask = nullptr;
    if (parent) {
        if (mean || cand_id || !mask1 || C1 <= 0 || (C1 + 31) / 32 > LK_MAX_W1) return hipErrorInvalidValue;
        hipLaunchKernelGGL((prefill_lookup_kernel<false, false, true>), grid, dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)centroids, sizes, thresh, keep_mask, n_ranges, n_keys, part_sum, parent,
                           (const int2 *)nullptr, mask1, (C1 + 31) / 32, H, Lq, C, sm_scale);
    } else if (cand_id) {
        if (!mean || !cand_hdr) return hipErrorInvalidValue;
        hipLaunchKernelGGL((prefill_lookup_kernel<true, true>), grid, dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)centroids, sizes, thresh, keep_mask, n_ranges, n_keys, part_sum, cand_id,
                           cand_hdr, no_mask, 0, H, Lq, C, sm_scale);
    } else if (mean)
        hipLaunchKernelGGL((prefill_lookup_kernel<true, false>), grid, dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)centroids, sizes, thresh, keep_mask, n_ranges, n_keys, part_sum,
                           (const int32_t *)nullptr, (const int2 *)nullptr, no_mask, 0, H, Lq, C, sm_scale);
    else
        hipLaunchKernelGGL((prefill_lookup_kernel<false, false>), grid, dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)centroids, sizes, thresh, keep_mask, n_ranges, n_keys, part_sum,
                           (const int32_t *)nullptr, (const int2 *)nullptr, no_mask, 0, H, Lq, C, sm_scale);
    return hipGetLastError();
}

// parent[h, c] = the coarse cluster whose child range child_offsets[j] .. child_offsets[j+1]-1 holds fine cluster c
// (binary search; C1 - 1 for ids past the last range).
__global__ __launch_bounds__(256) void child_parent_kernel(const int32_t *__restrict__ child_offsets,
                                                           int32_t *__restrict__ parent, int C1, int C2)
{
    const int h = blockIdx.y, c = blockIdx.x * 256 + threadIdx.x;
    if (c >= C2) return;
    const int32_t *co = child_offsets + (size_t)h * (C1 + 1);
    int lo = 0, hi = C1;                                     // invariant: co[lo] <= c (co[0] = 0), answer in [lo, hi)
    while (hi - lo > 1) {
        const int mid = (lo + hi) >> 1;
        if (co[mid] <= c) lo = mid;
        else hi = mid;
    }
    parent[(size_t)h * C2 + c] = lo;
}

hipError_t launch_child_parent(const int32_t *child_offsets, int32_t *parent, int H, int C1, int C2, hipStream_t s)
{
    hipLaunchKernelGGL(child_parent_kernel, dim3((C2 + 255) / 256, H), dim3(256), 0, s, child_offsets, parent, C1, C2);
    return hipGetLastError();
}

}  // namespace sq
