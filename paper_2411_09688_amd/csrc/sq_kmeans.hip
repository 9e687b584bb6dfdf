// Offline clustering of the fixed-context keys (Section 3.1): K-means on NORMALISED key vectors, the centroid of
// a cluster being the mean of its vectors.  One call makes one Lloyd iteration:
//
//   half norms  hn_c = |c|^2 / 2 of the current centres                         (one wave per centre)
//   assignment  a(x) = argmin_c |x - c|^2 = argmax_c (x . c - hn_c)              (matrix cores, below)
//   grouping    stable counting sort of the key indices by centre id: per-part histograms, a scan over parts
//               and centres, and a scatter in key order -- sizes, offsets and the member list of every cluster
//   update      centre = mean of its members' vectors (a cluster without members keeps its centre)
//
// and a last call turns an assignment into what the online path reads: keys and values reordered so that each
// cluster is contiguous, and the centroid of every cluster as the mean of its RAW keys.
//
// The assignment is the only dense contraction: S^T = C X^T on 16x16x32 fp16 MFMA tiles, A = 16 centres read
// from LDS, B = 16 key vectors held in registers.  A wave holds four B sets (64 keys), so every A operand read
// feeds four MFMAs; the four waves of a workgroup (256 keys) share the centre stream, which travels global
// memory -> registers (two groups ahead) -> one of two LDS stages, one barrier per group of 64 centres.  A lane
// owns one key per B set and four centres per tile, so the running (best score, best centre) is a per-lane
// scalar pair; the four lane groups are combined once at the end.  Ties go to the lowest centre index: a lane
// visits its centres in ascending order and replaces only on a strictly larger score, and the final combination
// prefers the lower index on equal scores.
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

constexpr int KM_G = 64;                     // centres per staged group
constexpr int KM_STRIDE = D + 8;             // halves per centre row in LDS (272 B: conflict-free 16-B reads)
constexpr int KM_RW = 4;                     // B sets (16 keys each) per wave
constexpr int KM_ROWS_PER_WG = 4 * 16 * KM_RW;

struct KmStage {
    _Float16 Ct[KM_G * KM_STRIDE];
    float nhn[KM_G];                         // minus the half norm: the accumulator's starting value
};

// x / |x| per row (fp32 arithmetic), one wave per row; a zero row stays zero.
__global__ __launch_bounds__(256) void normalize_rows_kernel(const _Float16 *__restrict__ K, _Float16 *__restrict__ X,
                                                             size_t rows)
{
    const int lane = threadIdx.x & 63;
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const h2 v = reinterpret_cast<const h2 *>(K + row * D)[lane];
    const float a = (float)v[0], b = (float)v[1];
    const float ss = wave_sum(a * a + b * b);
    const float inv = ss > 0.0f ? 1.0f / sqrtf(ss) : 0.0f;
    h2 o;
    o[0] = (_Float16)(a * inv);
    o[1] = (_Float16)(b * inv);
    reinterpret_cast<h2 *>(X + row * D)[lane] = o;
}

__global__ __launch_bounds__(256) void half_norm_kernel(const _Float16 *__restrict__ cent, float *__restrict__ hn,
                                                        int rows)
{
    const int lane = threadIdx.x & 63;
    const int row = blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= rows) return;
    const h2 v = reinterpret_cast<const h2 *>(cent + (size_t)row * D)[lane];
    const float a = (float)v[0], b = (float)v[1];
    const float ss = wave_sum(a * a + b * b);
    if (lane == 0) hn[row] = 0.5f * ss;
}

__global__ __launch_bounds__(256) void kmeans_assign_kernel(const _Float16 *__restrict__ X,
                                                            const _Float16 *__restrict__ cent,
                                                            const float *__restrict__ hn,
                                                            int32_t *__restrict__ assign, int L, int C)
{
    __shared__ __align__(16) KmStage stage[2];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    const int h = blockIdx.y;
    const int r0 = (blockIdx.x * 4 + wave) * 16 * KM_RW;      // first key of this wave (may lie past the end)
    const int ng = (C + KM_G - 1) / KM_G;

    h8 bx[KM_RW][4];
#pragma unroll
    for (int r = 0; r < KM_RW; ++r) {
        const int row = min(r0 + r * 16 + col, L - 1);        // keys past the end repeat the last one
        const h8 *xp = reinterpret_cast<const h8 *>(X + ((size_t)h * L + row) * D);
#pragma unroll
        for (int s = 0; s < 4; ++s) bx[r][s] = xp[s * 4 + kg];
    }
    const char *ch = reinterpret_cast<const char *>(cent + (size_t)h * C * D);
    const float *hh = hn + (size_t)h * C;

    // This thread's share of a group: rows i*16 + tid/16 (i = 0..3), 16-byte chunk tid%16; half norm of centre tid.
    h8 pk[4];
    float pn = 0.0f;
    auto fetch = [&](int g) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int c_row = min(g * KM_G + i * 16 + (tid >> 4), C - 1);
            pk[i] = *reinterpret_cast<const h8 *>(ch + (size_t)c_row * 256 + (tid & 15) * 16);
        }
        if (tid < KM_G) pn = g * KM_G + tid < C ? -hh[g * KM_G + tid] : SQ_NEG_INF;   // past the end: never best
    };
    auto commit = [&](KmStage &st) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
            *reinterpret_cast<h8 *>(st.Ct + (i * 16 + (tid >> 4)) * KM_STRIDE + (tid & 15) * 8) = pk[i];
        if (tid < KM_G) st.nhn[tid] = pn;
    };

    float best[KM_RW];
    int bi[KM_RW];
#pragma unroll
    for (int r = 0; r < KM_RW; ++r) {
        best[r] = SQ_NEG_INF;
        bi[r] = 0;
    }
    // Scores of tile u of a staged group: acc[r][v] = x_r . c - hn_c for c = u*16 + kg*4 + v (the accumulator starts
    // at -hn_c).
    auto tile = [&](const KmStage &st, int u, f4 (&acc)[KM_RW]) {
        const f4 nh = *reinterpret_cast<const f4 *>(st.nhn + u * 16 + kg * 4);
#pragma unroll
        for (int s = 0; s < 4; ++s) {
            const h8 a = *reinterpret_cast<const h8 *>(st.Ct + (u * 16 + col) * KM_STRIDE + s * 32 + kg * 8);
#pragma unroll
            for (int r = 0; r < KM_RW; ++r)
                acc[r] = __builtin_amdgcn_mfma_f32_16x16x32_f16(a, bx[r][s], s == 0 ? nh : acc[r], 0, 0, 0);
        }
    };
    auto take = [&](const f4 (&acc)[KM_RW], int c0) {
#pragma unroll
        for (int v = 0; v < 4; ++v)
#pragma unroll
            for (int r = 0; r < KM_RW; ++r)
                if (acc[r][v] > best[r]) {
                    best[r] = acc[r][v];
                    bi[r] = c0 + v;
                }
    };
    // The running best is updated one tile behind the matrix cores: the compares of a tile come after the MFMAs of
    // the next one in program order, which lets the compiler interleave the two kinds of work.
    f4 cur[KM_RW];
#pragma unroll
    for (int r = 0; r < KM_RW; ++r) cur[r] = f4{SQ_NEG_INF, SQ_NEG_INF, SQ_NEG_INF, SQ_NEG_INF};
    int cur_c0 = 0;
    fetch(0);
    commit(stage[0]);
    if (ng > 1) fetch(1);
    __syncthreads();
    for (int g = 0; g < ng; ++g) {
        if (g + 1 < ng) {
            commit(stage[(g + 1) & 1]);
            if (g + 2 < ng) fetch(g + 2);
        }
        const KmStage &st = stage[g & 1];
#pragma unroll
        for (int u = 0; u < KM_G / 16; ++u) {
            f4 nxt[KM_RW];
            tile(st, u, nxt);
            take(cur, cur_c0);
#pragma unroll
            for (int r = 0; r < KM_RW; ++r) cur[r] = nxt[r];
            cur_c0 = g * KM_G + u * 16 + kg * 4;
        }
        __syncthreads();                                      // stage g & 1 may be overwritten; the other is complete
    }
    take(cur, cur_c0);
#pragma unroll
    for (int r = 0; r < KM_RW; ++r) {
#pragma unroll
        for (int off = 16; off <= 32; off <<= 1) {
            const float so = __shfl_xor(best[r], off);
            const int io = __shfl_xor(bi[r], off);
            if (so > best[r] || (so == best[r] && io < bi[r])) {
                best[r] = so;
                bi[r] = io;
            }
        }
        const int row = r0 + r * 16 + col;
        if (kg == 0 && row < L) assign[(size_t)h * L + row] = bi[r];
    }
}

// Grouping, step 1: histogram of centre ids over one part of a head's keys.
__global__ __launch_bounds__(256) void kmeans_hist_kernel(const int32_t *__restrict__ assign, int32_t *__restrict__ hist,
                                                          int L, int C, int PL, int P)
{
    extern __shared__ int s_cnt[];
    const int p = blockIdx.x, h = blockIdx.y;
    for (int c = threadIdx.x; c < C; c += 256) s_cnt[c] = 0;
    __syncthreads();
    const int k_end = min(L, (p + 1) * PL);
    for (int k = p * PL + threadIdx.x; k < k_end; k += 256)      // (an id out of range counts for the nearest valid one)
        atomicAdd(&s_cnt[min(max(assign[(size_t)h * L + k], 0), C - 1)], 1);
    __syncthreads();
    int32_t *dst = hist + ((size_t)h * P + p) * C;
    for (int c = threadIdx.x; c < C; c += 256) dst[c] = s_cnt[c];
}

// Grouping, step 2 (one workgroup of 1024 threads per head): per centre, the part counts become exclusive prefixes
// over the parts and their total the cluster size; the sizes are scanned over the centres into offsets.
__global__ __launch_bounds__(1024) void kmeans_scan_kernel(int32_t *__restrict__ hist, int32_t *__restrict__ sizes,
                                                           int32_t *__restrict__ offsets, int L, int C, int P)
{
    __shared__ int s_wave[16];
    __shared__ int s_carry;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x;
    if (tid == 0) s_carry = 0;
    __syncthreads();
    for (int base = 0; base < C; base += 1024) {
        const int c = base + tid;
        int total = 0;
        if (c < C) {
            int32_t *col = hist + (size_t)h * P * C + c;
            int p = 0;
            for (; p + 8 <= P; p += 8) {                        // eight loads in flight
                int t8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) t8[u] = col[(size_t)(p + u) * C];
#pragma unroll
                for (int u = 0; u < 8; ++u) {
                    col[(size_t)(p + u) * C] = total;
                    total += t8[u];
                }
            }
            for (; p < P; ++p) {
                const int t = col[(size_t)p * C];
                col[(size_t)p * C] = total;
                total += t;
            }
            sizes[(size_t)h * C + c] = total;
        }
        const int inc = wave_inclusive_scan(total, lane);
        if (lane == 63) s_wave[wave] = inc;
        __syncthreads();
        int before = s_carry;
        for (int w = 0; w < wave; ++w) before += s_wave[w];
        if (c < C) offsets[(size_t)h * (C + 1) + c] = before + inc - total;
        __syncthreads();
        if (tid == 1023) s_carry = before + inc;
        __syncthreads();
    }
    if (tid == 0) offsets[(size_t)h * (C + 1) + C] = L;
}

// Grouping, step 3: one WAVE per part walks the part's keys in index order, 64 at a time.  The lanes that hold the
// same centre id are found in registers (a ballot per bit of the id); a lane's slot is the cluster's cursor plus the number of matching lanes below it, so members appear in
// ascending key order inside every cluster (a stable sort).  The cursors live in LDS and are touched by this one
// wave only, in program order (all lanes of a group read the cursor, then its last lane advances it): no atomics.
__global__ __launch_bounds__(64) void kmeans_scatter_kernel(const int32_t *__restrict__ assign,
                                                            const int32_t *__restrict__ hist,
                                                            const int32_t *__restrict__ offsets,
                                                            int32_t *__restrict__ perm, int L, int C, int PL, int P)
{
    extern __shared__ int s_cur[];
    const int p = blockIdx.x, h = blockIdx.y, lane = threadIdx.x;
    const int32_t *hp = hist + ((size_t)h * P + p) * C;
    const int32_t *op = offsets + (size_t)h * (C + 1);
    for (int c = lane; c < C; c += 64) s_cur[c] = op[c] + hp[c];
    __syncthreads();
    const int k_end = min(L, (p + 1) * PL);
    const int nbits = 32 - __clz(max(C - 1, 1));           // bits of a centre id
    for (int k0 = p * PL; k0 < k_end; k0 += 64) {
        const int k = k0 + lane;
        const bool valid = k < k_end;
        const int c = valid ? min(max(assign[(size_t)h * L + k], 0), C - 1) : -1;   // clamped like the counts
        // Lanes with the same centre id, found bit by bit: a lane keeps the lanes that agree with it on every bit of
        // the id (one ballot per bit, no data-dependent loop).
        uint64_t m = __ballot(valid);
        for (int b = 0; b < nbits; ++b) {                  // uniform trip count
            const bool bit = (c >> b) & 1;
            const uint64_t bal = __ballot(valid && bit);
            m &= bit ? bal : ~bal;
        }
        const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(m >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)m, 0u));
        const int cnt = __popcll(m);
        if (valid) {
            const int cur = s_cur[c];
            if (rank == cnt - 1) s_cur[c] = cur + cnt;
            perm[(size_t)h * L + cur + rank] = k;
        }
    }
}

// Mean of the rows of `src` listed for one cluster (members perm[off .. off + n) of head h), fp32 accumulation in
// a fixed order: 16 member slots x 16 sixteen-byte pieces of a row, then the slots are added in ascending order.
// An empty cluster copies prev (the centre it had) or, with prev == NULL, writes zeros.  perm == NULL: the members of
// a cluster are the rows off .. off + n themselves.
__global__ __launch_bounds__(256) void cluster_mean_kernel(const _Float16 *__restrict__ src,
                                                           const int32_t *perm,
                                                           const int32_t *__restrict__ sizes,
                                                           const int32_t *__restrict__ offsets,
                                                           const _Float16 *prev, _Float16 *out, int L, int C)
{
    __shared__ float s_acc[16][D + 4];
    const int c = blockIdx.x, h = blockIdx.y, tid = threadIdx.x;
    const int slot = tid >> 4, piece = tid & 15;
    const int off = min(max(offsets[(size_t)h * (C + 1) + c], 0), L);
    const int n = min(max(sizes[(size_t)h * C + c], 0), L - off);
    _Float16 *dst = out + ((size_t)h * C + c) * D;
    if (n == 0) {
        if (tid < D) dst[tid] = prev ? prev[((size_t)h * C + c) * D + tid] : (_Float16)0.0f;
        return;
    }
    const int32_t *mem = perm ? perm + (size_t)h * L + off : nullptr;
    auto member = [&](int m) { return mem ? min(max(mem[m], 0), L - 1) : off + m; };
    const _Float16 *rows = src + (size_t)h * L * D;
    float acc[8];
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[j] = 0.0f;
    int m = slot;
    for (; m + 16 < n; m += 32) {                             // two rows in flight
        const int i0 = member(m), i1 = member(m + 16);
        const h8 a = *reinterpret_cast<const h8 *>(rows + (size_t)i0 * D + piece * 8);
        const h8 b = *reinterpret_cast<const h8 *>(rows + (size_t)i1 * D + piece * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (float)a[j];
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (float)b[j];
    }
    if (m < n) {
        const h8 a = *reinterpret_cast<const h8 *>(rows + (size_t)member(m) * D + piece * 8);
#pragma unroll
        for (int j = 0; j < 8; ++j) acc[j] += (float)a[j];
    }
#pragma unroll
    for (int j = 0; j < 8; ++j) s_acc[slot][piece * 8 + j] = acc[j];
    __syncthreads();
    if (tid < D) {
        float s = 0.0f;
#pragma unroll
        for (int k = 0; k < 16; ++k) s += s_acc[k][tid];
        dst[tid] = (_Float16)(s / (float)n);
    }
}

// dst[h, i, :] = src[h, perm[h, i], :] for up to two tensors (blockIdx.z), 16 rows per workgroup.
__global__ __launch_bounds__(256) void gather_rows_kernel(const _Float16 *__restrict__ src0, _Float16 *__restrict__ dst0,
                                                          const _Float16 *__restrict__ src1, _Float16 *__restrict__ dst1,
                                                          const int32_t *__restrict__ perm, int L)
{
    const int h = blockIdx.y;
    const int i = blockIdx.x * 16 + (threadIdx.x >> 4), piece = threadIdx.x & 15;
    if (i >= L) return;
    const _Float16 *src = blockIdx.z ? src1 : src0;
    _Float16 *dst = blockIdx.z ? dst1 : dst0;
    const int k = min(max(perm[(size_t)h * L + i], 0), L - 1);
    *reinterpret_cast<h8 *>(dst + ((size_t)h * L + i) * D + piece * 8) =
        *reinterpret_cast<const h8 *>(src + ((size_t)h * L + k) * D + piece * 8);
}

int kmeans_part_len(int L)
{
    const int want = (L + 63) / 64;                           // at most 64 parts per head
    const int pl = ((want + 255) / 256) * 256;
    return pl < 512 ? 512 : pl;
}

hipError_t launch_normalize_rows(const void *K, void *X, size_t rows, hipStream_t s)
{
    hipLaunchKernelGGL(normalize_rows_kernel, dim3((unsigned)((rows + 3) / 4)), dim3(256), 0, s, (const _Float16 *)K,
                       (_Float16 *)X, rows);
    return hipGetLastError();
}

// Stable grouping of the rows by centre id: sizes, offsets and the member list of every centre.
static void launch_group(const int32_t *assign, int32_t *sizes, int32_t *offsets, int32_t *perm, int32_t *hist, int H,
                         int L, int C, hipStream_t s)
{
    const int PL = kmeans_part_len(L), P = (L + PL - 1) / PL;
    hipLaunchKernelGGL(kmeans_hist_kernel, dim3(P, H), dim3(256), (size_t)C * 4, s, assign, hist, L, C, PL, P);
    hipLaunchKernelGGL(kmeans_scan_kernel, dim3(H), dim3(1024), 0, s, hist, sizes, offsets, L, C, P);
    hipLaunchKernelGGL(kmeans_scatter_kernel, dim3(P, H), dim3(64), (size_t)C * 4, s, assign, (const int32_t *)hist,
                       (const int32_t *)offsets, perm, L, C, PL, P);
}

hipError_t launch_kmeans_step(const void *X, const void *centers_in, void *centers_out, int32_t *assign,
                              int32_t *sizes, int32_t *offsets, int32_t *perm, float *hn, int32_t *hist, int H, int L,
                              int C, hipStream_t s)
{
    hipLaunchKernelGGL(half_norm_kernel, dim3((H * C + 3) / 4), dim3(256), 0, s, (const _Float16 *)centers_in, hn, H * C);
    const dim3 grid_a((L + KM_ROWS_PER_WG - 1) / KM_ROWS_PER_WG, H);
    hipEvent_t ev0, ev1;
    if (profile_pair(&ev0, &ev1))
        hipExtLaunchKernelGGL(kmeans_assign_kernel, grid_a, dim3(256), 0, s, ev0, ev1, 0, (const _Float16 *)X,
                              (const _Float16 *)centers_in, (const float *)hn, assign, L, C);
    else
        hipLaunchKernelGGL(kmeans_assign_kernel, grid_a, dim3(256), 0, s, (const _Float16 *)X,
                           (const _Float16 *)centers_in, (const float *)hn, assign, L, C);
    launch_group(assign, sizes, offsets, perm, hist, H, L, C, s);
    hipLaunchKernelGGL(cluster_mean_kernel, dim3(C, H), dim3(256), 0, s, (const _Float16 *)X, (const int32_t *)perm,
                       (const int32_t *)sizes, (const int32_t *)offsets, (const _Float16 *)centers_in,
                       (_Float16 *)centers_out, L, C);
    return hipGetLastError();
}

// Nesting fine clusters under coarse ones (Section 3.3: the coarse level is a clustering of the fine centroids).
// perm_coarse lists the fine cluster ids grouped by coarse cluster; the fine clusters are renumbered in that order
// (inv[old id] = new id), every key's cluster id is translated, and the keys are grouped again.
__global__ __launch_bounds__(256) void invert_perm_kernel(const int32_t *__restrict__ perm, int32_t *__restrict__ inv,
                                                          int n)
{
    const int h = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    if (j >= n) return;
    const int f = perm[(size_t)h * n + j];
    if ((unsigned)f < (unsigned)n) inv[(size_t)h * n + f] = j;     // (a value out of range is ignored)
}

__global__ __launch_bounds__(256) void relabel_kernel(const int32_t *__restrict__ assign, const int32_t *__restrict__ inv,
                                                      int32_t *__restrict__ assign_new, int L, int C)
{
    const int h = blockIdx.y, k = blockIdx.x * 256 + threadIdx.x;
    if (k >= L) return;
    const int a = min(max(assign[(size_t)h * L + k], 0), C - 1);        // ids are clamped into range, so that malformed
    assign_new[(size_t)h * L + k] = min(max(inv[(size_t)h * C + a], 0), C - 1);   // input cannot index out of bounds later
}

// Keys under each coarse cluster: its children are fine clusters child_offsets[j] .. child_offsets[j+1]-1.
__global__ __launch_bounds__(256) void coarse_sizes_kernel(const int32_t *__restrict__ offsets_fine,
                                                           const int32_t *__restrict__ child_offsets,
                                                           int32_t *__restrict__ sizes_coarse, int C1, int C2)
{
    const int h = blockIdx.y, j = blockIdx.x * 256 + threadIdx.x;
    if (j >= C1) return;
    const int32_t *co = child_offsets + (size_t)h * (C1 + 1), *of = offsets_fine + (size_t)h * (C2 + 1);
    const int lo = min(max(co[j], 0), C2), hi = min(max(co[j + 1], lo), C2);
    sizes_coarse[(size_t)h * C1 + j] = of[hi] - of[lo];
}

hipError_t launch_cluster_nest(const int32_t *assign_fine, const int32_t *perm_coarse, const int32_t *child_offsets,
                               int32_t *assign_new, int32_t *sizes, int32_t *offsets, int32_t *perm,
                               int32_t *sizes_coarse, int32_t *inv, int32_t *hist, int H, int L, int C2, int C1,
                               hipStream_t s)
{
    hipLaunchKernelGGL(invert_perm_kernel, dim3((C2 + 255) / 256, H), dim3(256), 0, s, perm_coarse, inv, C2);
    hipLaunchKernelGGL(relabel_kernel, dim3((L + 255) / 256, H), dim3(256), 0, s, assign_fine, (const int32_t *)inv,
                       assign_new, L, C2);
    launch_group(assign_new, sizes, offsets, perm, hist, H, L, C2, s);
    hipLaunchKernelGGL(coarse_sizes_kernel, dim3((C1 + 255) / 256, H), dim3(256), 0, s, (const int32_t *)offsets,
                       child_offsets, sizes_coarse, C1, C2);
    return hipGetLastError();
}

hipError_t launch_cluster_layout(const void *K, const void *V, const int32_t *perm, const int32_t *sizes,
                                 const int32_t *offsets, void *K_sorted, void *V_sorted, void *centroids, int H, int L,
                                 int C, hipStream_t s)
{
    if (K_sorted)                                             // (V_sorted == NULL: keys only)
        hipLaunchKernelGGL(gather_rows_kernel, dim3((L + 15) / 16, H, V_sorted ? 2 : 1), dim3(256), 0, s,
                           (const _Float16 *)K, (_Float16 *)K_sorted, (const _Float16 *)V, (_Float16 *)V_sorted, perm, L);
    hipLaunchKernelGGL(cluster_mean_kernel, dim3(C, H), dim3(256), 0, s, (const _Float16 *)K, perm, sizes, offsets,
                       (const _Float16 *)nullptr, (_Float16 *)centroids, L, C);
    return hipGetLastError();
}

}  // namespace sq
