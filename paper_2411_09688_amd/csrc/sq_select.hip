// Threshold selection and compaction (Sections 3.2 / 4.1; Appendix D): keep cluster i iff
// exp(x_i - m) > T * D (strict), then turn the kept clusters of each query row into an ascending
// list of key ranges -- the role the key-index tensor plays in Section 4.2; ranges suffice because
// clusters are stored contiguously.
//
// One workgroup (4 waves) per query row walks the clusters 256 at a time.  Inside a wave the
// rank of a kept cluster comes from a 64-bit ballot + population count, the number of keys in front
// of it from a shuffle prefix scan; the four waves are stitched through LDS.  The ballot words are
// the keep mask.  The same pass emits the decode plan: per kept range the count of selected keys
// before it, and for each chunk of KPC selected keys the first range it touches, so the split-KV
// attention kernel can find its keys without scanning the whole list.
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

// Block-wide exclusive offsets of (count, keys) for one 256-wide step.  Returns this thread's
// exclusive rank / key prefix inside the block and the block totals.
struct ScanOut {
    int rank, key_prefix, total_cnt, total_keys;
};

__device__ __forceinline__ ScanOut block_scan_kept(bool keep, int nkeys, int lane, int wave, int *s_cnt, int *s_keys,
                                                   unsigned long long &ballot_out)
{
    const unsigned long long bal = __ballot(keep);
    ballot_out = bal;
    const int lane_rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
    const int kv = keep ? nkeys : 0;
    const int incl = wave_inclusive_scan(kv, lane);
    if (lane == 63) {
        s_cnt[wave] = __popcll(bal);
        s_keys[wave] = incl;
    }
    __syncthreads();
    ScanOut o{lane_rank, incl - kv, 0, 0};
#pragma unroll
    for (int w = 0; w < 4; ++w) {
        int c = s_cnt[w], k = s_keys[w];
        if (w < wave) {
            o.rank += c;
            o.key_prefix += k;
        }
        o.total_cnt += c;
        o.total_keys += k;
    }
    __syncthreads();
    return o;
}

// Record r of a row: (first key, count, selected keys before it); it is the first record of every
// chunk whose first key falls inside it.
__device__ __forceinline__ void emit_plan_record(const DecodePlan &plan, size_t row, int r, int start, int len, int cum)
{
    plan.rec[row * plan.rec_cap + r] = make_int4(start, len, cum, 0);
    const int c_lo = (cum + KPC - 1) / KPC, c_hi = (cum + len - 1) / KPC;
    for (int c = c_lo; c <= c_hi && c < plan.chunk_cap; ++c) plan.chunk_first[row * plan.chunk_cap + c] = r;
}

template <bool STATS_IN>
__global__ __launch_bounds__(256) void select_kernel(const float *__restrict__ logits,
                                                     const float *__restrict__ row_max,
                                                     const float *__restrict__ denom,
                                                     const float *__restrict__ thresh,
                                                     const int32_t *__restrict__ sizes,
                                                     const int32_t *__restrict__ offsets,
                                                     uint32_t *__restrict__ keep_mask, int32_t *__restrict__ ranges,
                                                     int32_t *__restrict__ n_ranges, int32_t *__restrict__ n_keys,
                                                     DecodePlan plan, int H, int Lq, int C)
{
    __shared__ int s_cnt[4], s_keys[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = blockIdx.x;
    const int h = (int)((row / Lq) % H);
    const float *x = logits + row * C;
    const int32_t *N = sizes + (size_t)h * C;
    const int32_t *off = offsets + (size_t)h * (C + 1);
    const int W = (C + 31) >> 5;

    float m, Dsum;
    if (STATS_IN) {
        m = row_max[row];
        Dsum = denom[row];
    } else {
        wave_row_stats(x, N, C, lane, m, Dsum);      // every wave derives the same (m, D)
    }
    const float thr = thresh[h] * Dsum;

    int base_r = 0, base_k = 0;
    for (int i0 = 0; i0 < C; i0 += 256) {
        const int i = i0 + tid;
        const int Ni = i < C ? N[i] : 0;
        const bool keep = Ni > 0 && expf(x[i] - m) > thr;
        unsigned long long bal;
        const ScanOut sc = block_scan_kept(keep, Ni, lane, wave, s_cnt, s_keys, bal);
        if (lane == 0 && keep_mask) {
            const int w0 = (i0 >> 5) + wave * 2;
            if (w0 < W) keep_mask[row * W + w0] = (uint32_t)bal;
            if (w0 + 1 < W) keep_mask[row * W + w0 + 1] = (uint32_t)(bal >> 32);
        }
        if (keep) {
            const int r = base_r + sc.rank, cum = base_k + sc.key_prefix, start = off[i];
            if (ranges) *reinterpret_cast<int2 *>(ranges + (row * C + r) * 2) = make_int2(start, Ni);
            if (plan.rec) emit_plan_record(plan, row, r, start, Ni, cum);
        }
        base_r += sc.total_cnt;
        base_k += sc.total_keys;
    }
    if (tid == 0) {
        n_ranges[row] = base_r;
        n_keys[row] = base_k;
        if (plan.rec) plan.hdr[row] = make_int2(base_r, base_k);
    }
}

// Plan for ranges that came from the caller (standalone attention call): prefix-sum the counts.
__global__ __launch_bounds__(256) void plan_from_ranges_kernel(const int32_t *__restrict__ ranges,
                                                               const int32_t *__restrict__ n_ranges, DecodePlan plan,
                                                               int range_cap)
{
    __shared__ int s_cnt[4], s_keys[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = blockIdx.x;
    const int nr = n_ranges[row];
    int base_r = 0, base_k = 0;
    for (int r0 = 0; r0 < nr; r0 += 256) {
        const int r = r0 + tid;
        int2 rg = make_int2(0, 0);
        if (r < nr) rg = *reinterpret_cast<const int2 *>(ranges + (row * range_cap + r) * 2);
        const bool live = r < nr && rg.y > 0;          // empty ranges are dropped from the plan
        unsigned long long bal;
        const ScanOut sc = block_scan_kept(live, rg.y, lane, wave, s_cnt, s_keys, bal);
        if (live) emit_plan_record(plan, row, base_r + sc.rank, rg.x, rg.y, base_k + sc.key_prefix);
        base_r += sc.total_cnt;
        base_k += sc.total_keys;
    }
    if (tid == 0) plan.hdr[row] = make_int2(base_r, base_k);
}

hipError_t launch_select(const float *logits, const float *row_max, const float *denom, bool stats_in,
                         const float *thresh, const int32_t *sizes, const int32_t *offsets, uint32_t *keep_mask,
                         int32_t *ranges, int32_t *n_ranges, int32_t *n_keys, DecodePlan plan, int rows, int H, int Lq,
                         int C, hipStream_t s)
{
    if (stats_in)
        hipLaunchKernelGGL(select_kernel<true>, dim3(rows), dim3(256), 0, s, logits, row_max, denom, thresh, sizes,
                           offsets, keep_mask, ranges, n_ranges, n_keys, plan, H, Lq, C);
    else
        hipLaunchKernelGGL(select_kernel<false>, dim3(rows), dim3(256), 0, s, logits, row_max, denom, thresh, sizes,
                           offsets, keep_mask, ranges, n_ranges, n_keys, plan, H, Lq, C);
    return hipGetLastError();
}

hipError_t launch_plan_from_ranges(const int32_t *ranges, const int32_t *n_ranges, DecodePlan plan, int rows,
                                   int range_cap, hipStream_t s)
{
    hipLaunchKernelGGL(plan_from_ranges_kernel, dim3(rows), dim3(256), 0, s, ranges, n_ranges, plan, range_cap);
    return hipGetLastError();
}

}  // namespace sq
