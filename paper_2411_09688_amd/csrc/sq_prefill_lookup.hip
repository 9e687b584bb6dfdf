// Centroid lookup for prefill (Section 4.1): grid over (sequence, head) x query blocks; a workgroup makes two
// passes over the head's centroids.  Pass 1 accumulates, per query token, the maximum and the size-weighted
// normaliser of Eq. 1; pass 2 recomputes the same logits and turns them into scores, so no [queries x clusters]
// intermediate is ever written to memory (the centroids are read twice instead, from L2).
//
// Scores run on the matrix cores as S^T = C Q^T (16x16x32 fp16 tiles: A = 16 centroids, loaded from global
// memory directly in the operand layout, B = the wave's 16 query tokens, kept in registers), so a lane owns ONE
// query token (column) and four centroids per tile: maximum, normaliser and threshold test are per-lane scalars,
// combined over the four lane groups once per pass.  Waves never synchronise.
//
//   MEAN == false  per-query selection: keep cluster i for token t iff N_i > 0 and exp(x_i - m) > T * D; the
//                  keep bits of two tiles are gathered into one mask word per token.
//   MEAN == true   selection on averaged scores (Appendix D, "Prefill Stage"), first half: the scores
//                  S_i(t) = exp(x_i - m) / D of a wave's 16 tokens are summed per cluster and written as one
//                  part of part_sum [B*H, ceil(Lq/16), C]; the row-wise selection kernel adds the parts.
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

constexpr int LK_TU = 4;         // centroid tiles in flight per step

template <bool MEAN>
__global__ __launch_bounds__(256) void prefill_lookup_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ cent, const int32_t *__restrict__ sizes,
    const float *__restrict__ thresh, uint32_t *__restrict__ keep_mask, int32_t *__restrict__ n_ranges,
    int32_t *__restrict__ n_keys, float *__restrict__ part_sum, int H, int Lq, int C, float sm_scale)
{
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const int bh = blockIdx.y, h = bh % H;
    const int q0 = (blockIdx.x * 4 + wave) * LOOKUP_ROWS;   // first token of this wave
    if (q0 >= Lq) return;                                   // this wave only: the kernel has no barrier
    const int nq = q0 + col;
    const bool valid = nq < Lq;
    const size_t row = (size_t)bh * Lq + min(nq, Lq - 1);
    const int W = (C + 31) >> 5;
    const int nt = (C + 15) >> 4;

    h8 bq[4];
    {
        const h8 *qp = reinterpret_cast<const h8 *>(q + row * D);
#pragma unroll
        for (int s = 0; s < 4; ++s) bq[s] = qp[s * 4 + kg];
    }
    const char *ch = reinterpret_cast<const char *>(cent + (size_t)h * C * D);
    const int32_t *Nh = sizes + (size_t)h * C;

    // Logits of LK_TU tiles starting at tile t0: x[u][v] = sm_scale * q . C_c, c = (t0+u)*16 + kg*4 + v, with
    // the cluster sizes nv[u][v] (0 past the last cluster).
    auto tiles = [&](int t0, float (&x)[LK_TU][4], int (&nv)[LK_TU][4]) {
        h8 a[LK_TU][4];
#pragma unroll
        for (int u = 0; u < LK_TU; ++u) {
            const int c_row = min((t0 + u) * 16 + col, C - 1);              // rows past the end repeat the last one
            const char *p = ch + (size_t)c_row * 256 + kg * 16;
#pragma unroll
            for (int s = 0; s < 4; ++s) a[u][s] = *reinterpret_cast<const h8 *>(p + s * 64);
#pragma unroll
            for (int v = 0; v < 4; ++v) {
                const int c = (t0 + u) * 16 + kg * 4 + v;
                nv[u][v] = c < C ? Nh[c] : 0;
            }
        }
#pragma unroll
        for (int u = 0; u < LK_TU; ++u) {
            f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[u][s], bq[s], acc, 0, 0, 0);
#pragma unroll
            for (int v = 0; v < 4; ++v) x[u][v] = acc[v] * sm_scale;
        }
    };

    // ---- pass 1: m = max over clusters with keys, D = sum N_i exp(x_i - m), per token ---------------------------
    float m = SQ_NEG_INF, Dsum = 0.0f;
    for (int t0 = 0; t0 < nt; t0 += LK_TU) {
        float x[LK_TU][4];
        int nv[LK_TU][4];
        tiles(t0, x, nv);
        float mt = m;
#pragma unroll
        for (int u = 0; u < LK_TU; ++u)
#pragma unroll
            for (int v = 0; v < 4; ++v)
                if (nv[u][v] > 0) mt = fmaxf(mt, x[u][v]);
        if (mt != SQ_NEG_INF) {
            Dsum *= __expf(m - mt);                          // m = -inf: Dsum is 0 and stays 0
#pragma unroll
            for (int u = 0; u < LK_TU; ++u)
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (nv[u][v] > 0) Dsum += (float)nv[u][v] * __expf(x[u][v] - mt);
            m = mt;
        }
    }
#pragma unroll
    for (int off = 16; off <= 32; off <<= 1) {              // the four lane groups hold the other clusters of the token
        const float mo = __shfl_xor(m, off), Do = __shfl_xor(Dsum, off);
        const float M = fmaxf(m, mo);
        const float wa = m == SQ_NEG_INF ? 0.0f : __expf(m - M), wb = mo == SQ_NEG_INF ? 0.0f : __expf(mo - M);
        Dsum = Dsum * wa + Do * wb;
        m = M;
    }
    const float thr = thresh[h] * Dsum;

    // ---- pass 2: the same logits again, now as scores ---------------------------------------------------------------
    uint32_t word = 0u;
    int cnt = 0, keys = 0;
    const int part = q0 / LOOKUP_ROWS, n_part = lookup_parts_for(Lq);
    for (int t0 = 0; t0 < nt; t0 += LK_TU) {
        float x[LK_TU][4];
        int nv[LK_TU][4];
        tiles(t0, x, nv);
#pragma unroll
        for (int u = 0; u < LK_TU; ++u) {
            const int t = t0 + u;
            if (t >= nt) break;                              // wave-uniform
            float e[4];
#pragma unroll
            for (int v = 0; v < 4; ++v) e[v] = nv[u][v] > 0 ? __expf(x[u][v] - m) : 0.0f;
            if (!MEAN) {
#pragma unroll
                for (int v = 0; v < 4; ++v) {
                    const bool keep = nv[u][v] > 0 && e[v] > thr;
                    word |= (uint32_t)keep << ((t & 1) * 16 + kg * 4 + v);
                    cnt += keep;
                    keys += keep ? nv[u][v] : 0;
                }
                if ((t & 1) || t == nt - 1) {                // a mask word is complete
                    word |= __shfl_xor(word, 16);
                    word |= __shfl_xor(word, 32);
                    if (kg == 0 && valid) keep_mask[row * W + (t >> 1)] = word;
                    word = 0u;
                }
            } else {
                float sums[4];
#pragma unroll
                for (int v = 0; v < 4; ++v) sums[v] = row16_sum(valid && Dsum > 0.0f ? e[v] / Dsum : 0.0f);   // over the wave's tokens
                if (col == 0) {
                    float *dst = part_sum + ((size_t)bh * n_part + part) * C + t * 16 + kg * 4;
#pragma unroll
                    for (int v = 0; v < 4; ++v)
                        if (t * 16 + kg * 4 + v < C) dst[v] = sums[v];
                }
            }
        }
    }
    if (!MEAN) {
        cnt += __shfl_xor(cnt, 16);
        cnt += __shfl_xor(cnt, 32);
        keys += __shfl_xor(keys, 16);
        keys += __shfl_xor(keys, 32);
        if (kg == 0 && valid) {
            n_ranges[row] = cnt;
            n_keys[row] = keys;
        }
    }
}

hipError_t launch_prefill_lookup(const void *q, const void *centroids, const int32_t *sizes, const float *thresh,
                                 uint32_t *keep_mask, int32_t *n_ranges, int32_t *n_keys, float *part_sum, bool mean,
                                 int B, int H, int Lq, int C, float sm_scale, hipStream_t s)
{
    const dim3 grid((Lq + 4 * LOOKUP_ROWS - 1) / (4 * LOOKUP_ROWS), B * H);
    if (mean)
        hipLaunchKernelGGL(prefill_lookup_kernel<true>, grid, dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)centroids, sizes, thresh, keep_mask, n_ranges, n_keys, part_sum, H, Lq, C,
                           sm_scale);
    else
        hipLaunchKernelGGL(prefill_lookup_kernel<false>, grid, dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)centroids, sizes, thresh, keep_mask, n_ranges, n_keys, part_sum, H, Lq, C,
                           sm_scale);
    return hipGetLastError();
}

}  // namespace sq
