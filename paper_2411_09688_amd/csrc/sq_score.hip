// Centroid scoring: logits[r, i] = sm_scale * q_r . C_i  (argument of exp in Eq. 1, Section 3.2) and
// the row statistics (m, D) of the max-subtracted form (Appendix D, "Generation Stage").
//
// The score is a small matrix product per head -- centroids [C x 128] times queries [128 x Nq] -- so it
// runs on the matrix cores: one 16x16x32 fp16 MFMA tile covers 16 centroid rows x 16 queries, with the
// centroid rows streamed straight from HBM into the A operand (each lane loads 16 contiguous bytes of
// a row, no LDS).  In decode only some of the 16 query columns are live; the kernel is bound by
// the centroid bytes either way.
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

constexpr int SCORE_TILES_PER_WAVE = 2;                              // 16-row tiles per wave
constexpr int SCORE_ROWS_PER_WG = 4 * 16 * SCORE_TILES_PER_WAVE;     // 4 waves

__global__ __launch_bounds__(256) void score_kernel(const _Float16 *__restrict__ q,
                                                    const _Float16 *__restrict__ cent,
                                                    float *__restrict__ logits, int *__restrict__ zero_counter,
                                                    int B, int H, int Lq, int C, float sm_scale)
{
    if (zero_counter && blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0 && threadIdx.x == 0)
        zero_counter[0] = zero_counter[1] = 0;              // (items, rows placed) of the step's work list
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const int h = blockIdx.y;
    const int NQ = B * Lq;
    const int n = blockIdx.z * 16 + col;          // query column of this lane (per head)
    const bool n_ok = n < NQ;
    size_t qrow = 0;
    h8 bq[4];
    if (n_ok) {
        int b = n / Lq, t = n - b * Lq;
        qrow = ((size_t)b * H + h) * Lq + t;
        const h8 *qp = reinterpret_cast<const h8 *>(q + qrow * D);
#pragma unroll
        for (int s = 0; s < 4; ++s) bq[s] = qp[s * 4 + kg];
    } else {
#pragma unroll
        for (int s = 0; s < 4; ++s) bq[s] = h8{0, 0, 0, 0, 0, 0, 0, 0};
    }
    const int i_base = (blockIdx.x * 4 + wave) * 16 * SCORE_TILES_PER_WAVE;
    h8 a[SCORE_TILES_PER_WAVE][4];
#pragma unroll
    for (int tile = 0; tile < SCORE_TILES_PER_WAVE; ++tile) {
        int row = i_base + tile * 16 + col;
        row = row < C ? row : C - 1;              // clamp: rows past C are computed and discarded
        const h8 *cp = reinterpret_cast<const h8 *>(cent + ((size_t)h * C + row) * D);
#pragma unroll
        for (int s = 0; s < 4; ++s) a[tile][s] = cp[s * 4 + kg];
    }
#pragma unroll
    for (int tile = 0; tile < SCORE_TILES_PER_WAVE; ++tile) {
        const int i0 = i_base + tile * 16 + kg * 4;   // first of this lane's 4 centroid rows
        f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[tile][s], bq[s], acc, 0, 0, 0);
        if (n_ok && i0 < C) {
            float *dst = logits + qrow * (size_t)C + i0;
            if (i0 + 3 < C && (C & 3) == 0) {
                *reinterpret_cast<f4 *>(dst) = acc * sm_scale;
            } else {
#pragma unroll
                for (int v = 0; v < 4; ++v)
                    if (i0 + v < C) dst[v] = acc[v] * sm_scale;
            }
        }
    }
}

__global__ __launch_bounds__(256) void row_stats_kernel(const float *__restrict__ logits,
                                                        const int32_t *__restrict__ sizes,
                                                        float *__restrict__ row_max, float *__restrict__ denom,
                                                        int rows, int H, int Lq, int C)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const int h = (row / Lq) % H;
    float m, Dsum;
    wave_row_stats(logits + (size_t)row * C, sizes + (size_t)h * C, C, lane, m, Dsum);
    if (lane == 0) {
        row_max[row] = m;
        denom[row] = Dsum;
    }
}

// The same statistics with a 1024-thread workgroup per row, for launches of few rows (decode): thread v adds clusters
// v, v+1024, ... ascending, a butterfly inside each wave, the 16 wave sums in ascending order -- the library's one
// summation order computed side by side instead of group after group: bit-identical to wave_row_stats.
__global__ __launch_bounds__(1024) void row_stats_block_kernel(const float *__restrict__ logits,
                                                               const int32_t *__restrict__ sizes,
                                                               float *__restrict__ row_max, float *__restrict__ denom,
                                                               int H, int Lq, int C)
{
    __shared__ float s_red[16];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x, h = (row / Lq) % H;
    const float *x = logits + (size_t)row * C;
    const int32_t *N = sizes + (size_t)h * C;
    float m = SQ_NEG_INF;
    for (int i = tid; i < C; i += 1024)
        if (N[i] > 0) m = fmaxf(m, x[i]);
    m = wave_max(m);
    if (lane == 0) s_red[wave] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < 16; ++w) m = fmaxf(m, s_red[w]);
    __syncthreads();                                         // s_red is reused
    float local = 0.0f;
    for (int i = tid; i < C; i += 1024) {
        const int Ni = N[i];
        if (Ni > 0) local = __fmaf_rn((float)Ni, expf(x[i] - m), local);
    }
    local = wave_sum(local);
    if (lane == 0) s_red[wave] = local;
    __syncthreads();
    if (tid == 0) {
        float Dsum = 0.0f;
#pragma unroll
        for (int w = 0; w < 16; ++w) Dsum += s_red[w];
        row_max[row] = m;
        denom[row] = Dsum;
    }
}

// Prefill selection on averaged scores (Appendix D, "Prefill Stage"), first half: the per-token scores
// S_i(t) = exp(x_i(t) - m(t)) / D(t) of Eq. 1 summed over a block of MEAN_ROWS query tokens of one
// (sequence, head), t ascending, one thread per cluster (coalesced along i).  The selection kernel adds the
// blocks' sums in ascending order and divides by Lq.
__global__ __launch_bounds__(256) void mean_score_kernel(const float *__restrict__ logits,
                                                         const float *__restrict__ row_max,
                                                         const float *__restrict__ denom, float *__restrict__ part_sum,
                                                         int Lq, int C, int n_part)
{
    __shared__ float s_m[MEAN_ROWS], s_D[MEAN_ROWS];
    const int bh = blockIdx.y, part = blockIdx.x;
    const int t0 = part * MEAN_ROWS, nt = min(MEAN_ROWS, Lq - t0);
    const size_t row0 = (size_t)bh * Lq + t0;
    if ((int)threadIdx.x < nt) {
        s_m[threadIdx.x] = row_max[row0 + threadIdx.x];
        const float Dt = denom[row0 + threadIdx.x];
        s_D[threadIdx.x] = Dt > 0.0f ? 1.0f / Dt : 0.0f;     // scores are e * (1 / D): one division per token
    }
    __syncthreads();
    for (int i = threadIdx.x; i < C; i += 256) {
        const float *x = logits + row0 * C + i;
        float acc = 0.0f;
        int t = 0;
        for (; t + 8 <= nt; t += 8) {                      // eight loads in flight
            float xv[8];
#pragma unroll
            for (int u = 0; u < 8; ++u) xv[u] = x[(size_t)(t + u) * C];
#pragma unroll
            for (int u = 0; u < 8; ++u) acc += expf(xv[u] - s_m[t + u]) * s_D[t + u];
        }
        for (; t < nt; ++t) acc += expf(x[(size_t)t * C] - s_m[t]) * s_D[t];
        part_sum[((size_t)bh * n_part + part) * C + i] = acc;
    }
}

// Grouped-query attention with one kept set per K/V head: the scores S_i = exp(x_i - m) / D (Eq. 1) of the G query
// heads of a (sequence, K/V head) are averaged, g ascending, and every head's logit row is replaced by
// ln(mean score) (-inf where the mean is 0).  A selection run on such a row finds max = ln(max mean),
// D = sum N_i mean_i / max mean, and therefore keeps cluster i iff mean_i > T * sum_j N_j mean_j, the sum being 1 up
// to fp32 rounding: the per-row threshold rule applied to the group's averaged scores, identically for the G rows.
__global__ __launch_bounds__(1024) void group_mean_logits_kernel(float *__restrict__ logits,
                                                                 const int32_t *__restrict__ sizes, int H, int G, int C)
{
    __shared__ float s_red[SG][16], s_m[SG], s_D[SG];
    const int bh = blockIdx.x, h = bh % H;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row0 = (size_t)bh * G;                       // first of the G rows of this (sequence, K/V head)
    const int32_t *N = sizes + (size_t)h * C;
    // (m, D) of Eq. 1 for the G query heads side by side: row g is handled by the 16 / G waves w with w % G == g
    // (G divides 16), each covering every (16 / G)-th block of 64 clusters.
    const int g = wave % G, j = wave / G, nw = 16 / G;
    const float *x = logits + (row0 + g) * C;
    // This wave's entries i = j*64 + lane + k*64*nw stay in registers between the two passes when there are at most
    // GM_REG of them per lane (rows of up to 1024 * 16 / G clusters).
    constexpr int GM_REG = 16;
    const bool in_regs = C <= 64 * nw * GM_REG;              // workgroup-uniform
    float xr[GM_REG];
    int nr[GM_REG];
    float m = SQ_NEG_INF;
    if (in_regs) {
#pragma unroll
        for (int k = 0; k < GM_REG; ++k) {
            const int i = j * 64 + lane + k * 64 * nw;
            nr[k] = i < C ? N[i] : 0;
            xr[k] = i < C ? x[i] : 0.0f;
        }
#pragma unroll
        for (int k = 0; k < GM_REG; ++k)
            if (nr[k] > 0) m = fmaxf(m, xr[k]);
    } else {
        for (int i = j * 64 + lane; i < C; i += 64 * nw)
            if (N[i] > 0) m = fmaxf(m, x[i]);
    }
    m = wave_max(m);
    if (lane == 0) s_red[g][j] = m;
    __syncthreads();
    for (int k = 0; k < nw; ++k) m = fmaxf(m, s_red[g][k]);
    __syncthreads();                                          // s_red is reused
    float d = 0.0f;
    if (in_regs) {
#pragma unroll
        for (int k = 0; k < GM_REG; ++k)                     // (k ascending: the same order as the loop below)
            if (nr[k] > 0) d += (float)nr[k] * expf(xr[k] - m);
    } else {
        for (int i = j * 64 + lane; i < C; i += 64 * nw)
            if (N[i] > 0) d += (float)N[i] * expf(x[i] - m);
    }
    d = wave_sum(d);
    if (lane == 0) s_red[g][j] = d;
    __syncthreads();
    if (tid < G) {
        float Dsum = 0.0f;
        for (int k = 0; k < nw; ++k) Dsum += s_red[tid][k];
        s_D[tid] = Dsum > 0.0f ? 1.0f / Dsum : 0.0f;         // the scores below are e * (1 / D): one division per row
    }
    if (j == 0 && lane == 0) s_m[g] = m;
    __syncthreads();
    for (int i = tid; i < C; i += 1024) {
        float sum = 0.0f;
        if (N[i] > 0)
            for (int gg = 0; gg < G; ++gg) sum += expf(logits[(row0 + gg) * C + i] - s_m[gg]) * s_D[gg];
        const float mean = sum / (float)G;
        const float xl = mean > 0.0f ? logf(mean) : SQ_NEG_INF;
        for (int gg = 0; gg < G; ++gg) logits[(row0 + gg) * C + i] = xl;
    }
}

hipError_t launch_group_mean_logits(float *logits, const int32_t *sizes, int BH, int H, int G, int C, hipStream_t s)
{
    hipLaunchKernelGGL(group_mean_logits_kernel, dim3(BH), dim3(1024), 0, s, logits, sizes, H, G, C);
    return hipGetLastError();
}

// Level-2 scoring of the two-level lookup (Section 3.3, Eq. 3 numerator): the fine centroids to score are
// the children of the kept coarse clusters, listed by work items of KPC candidate clusters each (built
// by the level-1 selection: a balanced number of centroids per workgroup, Appendix D).  A persistent
// grid walks the items; each wave scores 16-cluster MFMA tiles of its share, gathering the centroid rows
// by cluster id.  Per candidate j of the row (candidate order) it writes the logit, the cluster id and the 16-byte
// record (logit, id | no-keys flag, first key | first child, range length) the selection needs, so that the selection
// -- one workgroup per row -- reads ONE coalesced stream instead of gathering by id; per item it writes the statistics of Eq. 3's
// denominator over the item's candidates, (m, sum N exp(x - m)) over those with N > 0, which the selection
// merges in item order.
__global__ __launch_bounds__(256) void gather_score_kernel(const _Float16 *__restrict__ q,
                                                           const _Float16 *__restrict__ cent2, DecodePlan cand,
                                                           const int32_t *__restrict__ sizes2,
                                                           const int32_t *__restrict__ offsets2, int len_from_offsets,
                                                           float *__restrict__ logits2,
                                                           int32_t *__restrict__ cand_id, int4 *__restrict__ cand_rec,
                                                           float2 *__restrict__ cand_stats,
                                                           int *__restrict__ zero_counter, int H, int C2,
                                                           float sm_scale, uint32_t *__restrict__ zero_mask,
                                                           size_t zero_words)
{
    __shared__ int s_pos[KPC], s_delta[KPC], s_rows[KPC];
    __shared__ __align__(16) float s_x[KPC];
    __shared__ float s_red[4];
    if (zero_counter && blockIdx.x == 0 && threadIdx.x == 0) zero_counter[0] = zero_counter[1] = 0;
    for (size_t w = (size_t)blockIdx.x * 256 + threadIdx.x; w < zero_words; w += (size_t)gridDim.x * 256) zero_mask[w] = 0u;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    constexpr int TILES = KPC / 64;                 // 16-cluster tiles per wave
    static_assert(KPC == 128, "two waves hold an item's candidates");
    const int total = min(*cand.total, cand.item_cap);
    for (int item = blockIdx.x; item < total; item += gridDim.x) {
        const int2 *it = cand.item + (size_t)item * ITEM_STRIDE;
        const int2 h0 = it[0], h1 = it[1];          // (row, clusters in chunk) (records, chunk's first candidate in its row)
        const int2 rc = it[2 + (tid < KPC ? tid : 0)];
        const size_t bh = (size_t)h0.x;
        const int h = (int)(bh % H);
        const int j0 = h1.y;                        // this chunk's first candidate within its row
        chunk_rows_from_records<KPC>(rc.x, rc.y, min(h1.x, KPC), h0.y, C2, s_pos, s_delta, s_rows, tid);
        __syncthreads();
        h8 bq[4];
        {
            const h8 *qp = reinterpret_cast<const h8 *>(q + bh * D);
#pragma unroll
            for (int s = 0; s < 4; ++s) bq[s] = col == 0 ? qp[s * 4 + kg] : h8{0, 0, 0, 0, 0, 0, 0, 0};
        }
        const int r_last = s_rows[h0.y - 1];
        h8 a[TILES][4];
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            int r = s_rows[wave * (KPC / 4) + t * 16 + col];
            r = r < 0 ? r_last : r;
            const h8 *cp = reinterpret_cast<const h8 *>(cent2 + ((size_t)h * C2 + r) * D);
#pragma unroll
            for (int s = 0; s < 4; ++s) a[t][s] = cp[s * 4 + kg];
        }
        // the candidate's record, one candidate per thread of the first two waves (loads run under the products)
        const int my_r = tid < KPC ? s_rows[tid] : -1;
        int my_N = 0, my_start = 0, my_next = 0;
        if (my_r >= 0) {
            my_N = sizes2[(size_t)h * C2 + my_r];
            my_start = offsets2[(size_t)h * (C2 + 1) + my_r];
            if (len_from_offsets) my_next = offsets2[(size_t)h * (C2 + 1) + my_r + 1];
        }
#pragma unroll
        for (int t = 0; t < TILES; ++t) {
            f4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int s = 0; s < 4; ++s) acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(a[t][s], bq[s], acc, 0, 0, 0);
            if (col == 0) *reinterpret_cast<f4 *>(&s_x[wave * (KPC / 4) + t * 16 + kg * 4]) = acc * sm_scale;
        }
        __syncthreads();
        if (wave < 2) {                             // wave-uniform
            const float xj = s_x[tid];
            const bool ok = my_r >= 0 && j0 + tid < C2;
            if (ok) {
                const size_t j = bh * (size_t)C2 + j0 + tid;
                logits2[j] = xj;
                cand_id[j] = my_r;
                // (logit, id with bit 31 set for a cluster without keys, first key | first child, range length)
                cand_rec[j] = make_int4(__float_as_int(xj), my_N > 0 ? my_r : (int)(0x80000000u | (uint32_t)my_r), my_start,
                                        len_from_offsets ? my_next - my_start : my_N);
            }
            const bool live = ok && my_N > 0;
            const float mw = wave_max(live ? xj : SQ_NEG_INF);
            if (lane == 0) s_red[wave] = mw;
        }
        __syncthreads();
        if (wave < 2) {
            const float m = fmaxf(s_red[0], s_red[1]);
            const bool live = my_r >= 0 && j0 + tid < C2 && my_N > 0;
            const float sw = wave_sum(live ? __fmul_rn((float)my_N, expf(s_x[tid] - m)) : 0.0f);
            if (lane == 0) s_red[2 + wave] = sw;
        }
        __syncthreads();                            // (LDS is reused by the next item)
        if (tid == 0) cand_stats[item] = make_float2(fmaxf(s_red[0], s_red[1]), s_red[2] + s_red[3]);
    }
}

hipError_t launch_gather_score(const void *q, const void *centroids2, DecodePlan cand, const int32_t *sizes2,
                               const int32_t *offsets2, int len_from_offsets, float *logits2, int32_t *cand_id,
                               int4 *cand_rec, float2 *cand_stats, int *zero_counter, int H, int C2, float sm_scale,
                               hipStream_t s, uint32_t *zero_mask, size_t zero_words)
{
    const int grid = cand.item_cap < 2048 ? cand.item_cap : 2048;
    hipLaunchKernelGGL(gather_score_kernel, dim3(grid), dim3(256), 0, s, (const _Float16 *)q,
                       (const _Float16 *)centroids2, cand, sizes2, offsets2, len_from_offsets, logits2, cand_id,
                       cand_rec, cand_stats, zero_counter, H, C2, sm_scale, zero_mask, zero_mask ? zero_words : 0);
    return hipGetLastError();
}

hipError_t launch_score(const void *q, const void *centroids, float *logits, int *zero_counter, int B, int H, int Lq,
                        int C, float sm_scale, hipStream_t s)
{
    dim3 grid((C + SCORE_ROWS_PER_WG - 1) / SCORE_ROWS_PER_WG, H, (B * Lq + 15) / 16);
    hipLaunchKernelGGL(score_kernel, grid, dim3(256), 0, s, (const _Float16 *)q, (const _Float16 *)centroids, logits,
                       zero_counter, B, H, Lq, C, sm_scale);
    return hipGetLastError();
}

hipError_t launch_mean_score(const float *logits, const float *row_max, const float *denom, float *part_sum, int BH,
                             int Lq, int C, hipStream_t s)
{
    const int n_part = mean_parts_for(Lq);
    hipLaunchKernelGGL(mean_score_kernel, dim3(n_part, BH), dim3(256), 0, s, logits, row_max, denom, part_sum, Lq, C,
                       n_part);
    return hipGetLastError();
}

hipError_t launch_row_stats(const float *logits, const int32_t *sizes, float *row_max, float *denom, int rows,
                            int H, int Lq, int C, hipStream_t s)
{
    if (rows <= 2048)                                        // few rows: a whole workgroup per row
        hipLaunchKernelGGL(row_stats_block_kernel, dim3(rows), dim3(1024), 0, s, logits, sizes, row_max, denom, H, Lq, C);
    else
        hipLaunchKernelGGL(row_stats_kernel, dim3((rows + 3) / 4), dim3(256), 0, s, logits, sizes, row_max, denom, rows,
                           H, Lq, C);
    return hipGetLastError();
}

}  // namespace sq
