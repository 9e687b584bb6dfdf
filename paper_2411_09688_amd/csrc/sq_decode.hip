// Decode-time sparse attention (Section 4.2): exact attention of one query per (sequence, head) over
// the selected fixed-context keys plus the dense user keys, split along the key dimension into
// chunks of KPC keys (the split-KV scheme: a head that keeps more keys gets more workgroups).  A
// workgroup folds the consecutive chunks it owns into one partial (max, sum, output) per row; a second
// kernel merges the partials of every row (phase 2 of Section 4.2).
//
// The kernel is bound by HBM: every selected K and V row (256 B each) is read exactly once.  A
// workgroup owns one chunk; its 256 threads fetch the chunk's range records with one coalesced load
// and turn them into one row index per key in LDS, then 16 lanes share a row (16 B per lane, a wave-wide load covers four whole rows) and every lane
// issues all of its K and V loads before any arithmetic, so a workgroup keeps its whole chunk in
// flight.  Scores are reduced over the 16 lanes of a row with DPP rotations; the softmax runs per
// wave and the four wave results are combined in LDS.

#include "sq_common.hpp"
#include "sq_internal.hpp"
#include "sq_merge.hpp"

namespace sq {

constexpr int KW = KPC / 4;     // keys per wave
constexpr int NI = KW / 4;      // loads per lane (4 rows per wave-wide load)
constexpr int REG_RECORDS = 16; // chunks of at most this many records find their rows in registers (else through LDS)

// How the work list of `total` items is split over the G workgroups of the partial kernel (the merge kernel derives
// the same numbers).  Compute units take workgroups round robin and each streams at the same rate, so what counts is
// equal bytes per compute unit.
//   total <= G        workgroup w takes item w;
//   total <  2 G      workgroup w takes item w and, for w < total - G, also item G + w: with four workgroups per
//                     compute unit that is 4 or 5 chunks each (runs of two consecutive items over total / 2
//                     workgroups would give 4 or 6); the first item is item w itself, fetched before the count is known;
//   otherwise         runs of kq = ceil(total / G) consecutive items (8 or 9 chunks per workgroup hardly differ, and
//                     consecutive chunks of a row fold into one partial result).
struct WorkSplit {
    int kq, rem, R;                      // items per run, items past the runs, first index past the runs
};
__device__ __forceinline__ WorkSplit work_split(int total, int grid)
{
    WorkSplit ws;
    if (total < 2 * grid) {
        ws.kq = 1;
        ws.R = min(total, grid);
        ws.rem = total - ws.R;
    } else {
        ws.kq = (total + grid - 1) / grid;
        ws.R = total;
        ws.rem = 0;
    }
    return ws;
}
// Index (past the runs) of the extra item of workgroup w, or -1.
__device__ __forceinline__ int extra_of(const WorkSplit &ws, int w) { return w < ws.rem ? w : -1; }

// Phase 1: one work item = one chunk of up to KPC keys of one (sequence, head) row.  The grid is a fixed number of
// workgroups and the work list is split over them as described at work_split: no workgroup is launched for chunks
// that do not exist.  (Handing items out through a device-wide counter was measured too: a thousand increments of one
// address serialise, and the step got 4 us slower.  Several runs per workgroup buy no better balance and cost more
// partial results to merge.)
// Consecutive items of one row inside a run are folded into one running (max, sum, output) per lane, so a
// partial result is written once per (run, row) segment, at the index of the segment's first item; an extra item
// is a segment of its own.
__global__ __launch_bounds__(256) void decode_attn_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ Kf, const _Float16 *__restrict__ Vf,
    const _Float16 *__restrict__ Ku, const _Float16 *__restrict__ Vu, DecodePlan plan,
    float *__restrict__ partials, int H, int G, int L, int U, float sm_scale)
{
    __shared__ int s_pos[KPC], s_delta[KPC];
    __shared__ int s_rows[KPC];
    __shared__ float s_part[4][PART_STRIDE];

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, p = lane & 15;

    // The work list is read with as few dependent round trips as possible: the item this workgroup starts with
    // when the list is shorter than twice the grid is fetched together with the item count; only a longer list
    // costs a second fetch.  (The grid never exceeds item_cap, so the speculative read stays inside the item array; slots
    // past the count hold stale data that is not used.)
    const int2 *it = plan.item + (size_t)blockIdx.x * ITEM_STRIDE;
    int2 h0_next = it[0], h1_next = it[1], rec_next = it[2 + lane];   // every wave holds records 0..63 in its lanes
    const int total = min(*plan.total, plan.item_cap);
    const WorkSplit ws = work_split(total, (int)gridDim.x);
    const int run0 = (int)blockIdx.x * ws.kq;               // this workgroup's run [run0, run0 + run_len)
    const int run_len = run0 < ws.R ? min(ws.kq, ws.R - run0) : 0;
    const int extra = extra_of(ws, (int)blockIdx.x);
    const int n_my = run_len + (extra >= 0 ? 1 : 0);
    if (n_my == 0) return;                                 // whole workgroup
    auto item_at = [&](int j) { return j < run_len ? run0 + j : ws.R + extra; };
    if (item_at(0) != (int)blockIdx.x) {                   // (only lists of 2 G items or more)
        it = plan.item + (size_t)item_at(0) * ITEM_STRIDE;
        h0_next = it[0];
        h1_next = it[1];
        rec_next = it[2 + lane];
    }

    // Running state of the current (run, row) segment.  m is wave-uniform; l and o are this lane's
    // share (its 16-lane group's keys), summed over the four groups only when the segment is flushed.
    float m_run, l_run;
    float o[8];

    auto flush = [&](int slot) {
        const float l_w = cross16_sum(l_run);
        float ow[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) ow[e] = cross16_sum(o[e]);
        if (g == 0) {
            if (p == 0) {
                s_part[wave][0] = m_run;
                s_part[wave][1] = l_w;
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) s_part[wave][4 + p * 8 + e] = ow[e];
        }
        __syncthreads();
        // Combine the four waves; threads 0..127 own one output dimension each.
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
            float *dst = partials + (size_t)slot * PART_STRIDE;
            if (tid == 0) {
                dst[0] = M;
                dst[1] = lsum;
            }
            dst[4 + tid] = acc;
        }
        __syncthreads();
    };

    {
        m_run = SQ_NEG_INF;
        l_run = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.0f;
        int seg_first = item_at(0);
        int cur_row = h0_next.x;
        for (int j = 0; j < n_my; ++j) {
            const int item = item_at(j);
            const int2 h0 = h0_next, h1 = h1_next, rc = rec_next;   // (row, keys) (records | -1, first user key)
            if (h0.x != cur_row || (j == run_len && j > 0)) {   // workgroup-uniform: the previous segment ends
                flush(seg_first);
                m_run = SQ_NEG_INF;
                l_run = 0.0f;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] = 0.0f;
                seg_first = item;
                cur_row = h0.x;
            }
            const size_t bh = (size_t)h0.x;
            const int nvalid = h0.y;
            const bool user = h1.x < 0;
            const int nrec = min(h1.x, KPC);
            // Row bh = (sequence, K/V head, query head of the group): G query heads share the K/V head and the
            // sequence's user keys (G = 1 without grouped-query attention).
            const size_t bkv = bh / G;                     // (sequence, K/V head)
            const int h = (int)(bkv % H);
            const _Float16 *Kbase, *Vbase;
            const h8 qv = *reinterpret_cast<const h8 *>(q + bh * D + p * 8);
            // Rows of this lane's NI key slots (slot = wave * KW + i * 4 + g) and of the chunk's last valid slot.
            // A slot lies in the last record whose position is <= the slot and reads row slot + delta.  With few
            // records (the usual case: a chunk of 128 keys spans a handful of clusters) the records are broadcast
            // from the wave's lanes and the rows found in registers: no LDS, no barrier on the way to the K/V loads.
            int rows[NI], r_last;
            if (user) {
                Kbase = Ku + (bkv * U + h1.y) * D;
                Vbase = Vu + (bkv * U + h1.y) * D;
#pragma unroll
                for (int i = 0; i < NI; ++i) rows[i] = wave * KW + i * 4 + g;
                r_last = nvalid - 1;
            } else {
                Kbase = Kf + (size_t)h * L * D;
                Vbase = Vf + (size_t)h * L * D;
                if (nrec <= REG_RECORDS) {                  // workgroup-uniform
                    int dl[NI], d_last;
                    const int d0 = __builtin_amdgcn_readlane(rc.y, 0);
#pragma unroll
                    for (int i = 0; i < NI; ++i) dl[i] = d0;
                    d_last = d0;
                    for (int r = 1; r < nrec; ++r) {
                        const int pr = __builtin_amdgcn_readlane(rc.x, r), dr = __builtin_amdgcn_readlane(rc.y, r);
#pragma unroll
                        for (int i = 0; i < NI; ++i)
                            if (pr <= wave * KW + i * 4 + g) dl[i] = dr;
                        if (pr <= nvalid - 1) d_last = dr;
                    }
#pragma unroll
                    for (int i = 0; i < NI; ++i) rows[i] = max(0, min(wave * KW + i * 4 + g + dl[i], L - 1));
                    r_last = max(0, min(nvalid - 1 + d_last, L - 1));
                } else {
                    const int2 rcl = plan.item[(size_t)item * ITEM_STRIDE + 2 + (tid < KPC ? tid : 0)];
                    __syncthreads();                        // (the previous item's readers of s_rows are done)
                    chunk_rows_from_records<KPC>(rcl.x, rcl.y, nrec, nvalid, L, s_pos, s_delta, s_rows, tid);
                    __syncthreads();
#pragma unroll
                    for (int i = 0; i < NI; ++i) rows[i] = s_rows[wave * KW + i * 4 + g];
                    r_last = s_rows[nvalid - 1];
                }
            }

            // Issue every K and V load of this lane.
            h8 kreg[NI], vreg[NI];
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int kl = wave * KW + i * 4 + g;
                const int r = kl < nvalid ? rows[i] : r_last;     // slots past the chunk re-read a valid row
                const size_t off = (size_t)r * D + p * 8;
                // (streamed once: non-temporal loads keep the rows from displacing the centroids, records and
                // partial results that the step's other kernels find in the cache)
                kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Kbase + off));
                vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Vbase + off));
            }
            // Metadata of this workgroup's next item,
            // fetched behind the K/V stream.
            if (j + 1 < n_my) {
                const int2 *nx = plan.item + (size_t)item_at(j + 1) * ITEM_STRIDE;
                h0_next = nx[0];
                h1_next = nx[1];
                rec_next = nx[2 + lane];
            }

            // Scores of this lane-group's keys, folded into the running softmax.
            float s[NI];
            float m_it = SQ_NEG_INF;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const int kl = wave * KW + i * 4 + g;
                const float d = row16_sum(dot8(qv, kreg[i], 0.0f)) * sm_scale;
                s[i] = kl < nvalid ? d : SQ_NEG_INF;
                m_it = fmaxf(m_it, s[i]);
            }
            m_it = cross16_max(m_it);
            const float m_new = fmaxf(m_run, m_it);
            const float alpha = m_new == SQ_NEG_INF ? 1.0f : __expf(m_run - m_new);   // exp(-inf) = 0 on the first item
            l_run *= alpha;
#pragma unroll
            for (int e = 0; e < 8; ++e) o[e] *= alpha;
#pragma unroll
            for (int i = 0; i < NI; ++i) {
                const float pr = s[i] == SQ_NEG_INF ? 0.0f : __expf(s[i] - m_new);
                l_run += pr;
#pragma unroll
                for (int e = 0; e < 8; ++e) o[e] += pr * (float)vreg[i][e];
            }
            m_run = m_new;
        }
        flush(seg_first);
    }
}

// Phase 2 (Section 4.2): one workgroup per (sequence, head) merges the row's partials.  A separate
// launch, so the kernel boundary makes the partials visible: a device-wide fence inside the partial
// kernel would write back a whole L2 per workgroup and costs far more than this launch.
__global__ __launch_bounds__(MERGE_THREADS) void decode_merge_kernel(const float *__restrict__ partials,
                                                                     DecodePlan plan, _Float16 *__restrict__ out,
                                                                     float *__restrict__ lse, int attn_grid,
                                                                     int user_slot_base, int nuq)
{
    __shared__ float s_red[MERGE_GROUPS * 130];
    const size_t bh = blockIdx.x;
    const int2 it = plan.row_items[bh];              // (first item, items) of this row
    const int total = min(*plan.total, plan.item_cap);
    const WorkSplit ws = work_split(total, attn_grid);
    // The row's items are [first, first + items).  Inside the runs its partials sit at `first` and at every multiple
    // of kq inside (first, end of the row or of the runs); past the runs every item has a partial of its own.
    const int first = it.x, last = it.x + it.y, kq = ws.kq, fk = first / kq;
    const int e1 = min(last, ws.R);
    const int n_run = (it.y > 0 && first < ws.R) ? 1 + (e1 - 1) / kq - fk : 0;
    const int t0 = max(first, ws.R);
    const int n_sel = n_run + max(0, last - t0);
    // After them, the row's user-key partials when the selection launch computed those (user_slot_base >= 0).
    const int n = n_sel + (user_slot_base >= 0 ? nuq : 0);
    auto slot_ptr = [&](int c) {
        const int idx = c >= n_sel ? user_slot_base + (int)bh * nuq + (c - n_sel)
                                   : (c >= n_run ? t0 + (c - n_run) : (c == 0 ? first : (fk + c) * kq));
        return partials + (size_t)idx * PART_STRIDE;
    };
    merge_row<false>(slot_ptr, n, out + bh * D, lse ? lse + bh : nullptr, s_red, threadIdx.x);
}

// Workgroups of the persistent partial kernel: four per compute unit.
constexpr int ATTN_GRID = 256 * 4;

hipError_t launch_decode_attn(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                              DecodePlan plan, float *partials, void *out, float *lse, const Shape &sh,
                              hipStream_t s, int user_slot_base, int nuq)
{
    const int G = sh.Lq;                             // query heads per K/V head (1, or the group size)
    const int rows = sh.B * sh.H * G;
    const int grid = plan.item_cap < ATTN_GRID ? plan.item_cap : ATTN_GRID;
    hipEvent_t ev0, ev1;
    if (profile_pair(&ev0, &ev1))
        hipExtLaunchKernelGGL(decode_attn_kernel, dim3(grid), dim3(256), 0, s, ev0, ev1, 0, (const _Float16 *)q,
                              (const _Float16 *)Kf, (const _Float16 *)Vf, (const _Float16 *)Ku, (const _Float16 *)Vu, plan,
                              partials, sh.H, G, sh.L, sh.U, sh.sm_scale);
    else
        hipLaunchKernelGGL(decode_attn_kernel, dim3(grid), dim3(256), 0, s, (const _Float16 *)q, (const _Float16 *)Kf,
                           (const _Float16 *)Vf, (const _Float16 *)Ku, (const _Float16 *)Vu, plan, partials, sh.H, G,
                           sh.L, sh.U, sh.sm_scale);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_merge_kernel, dim3(rows), dim3(MERGE_THREADS), 0, s, partials, plan, (_Float16 *)out, lse,
                       grid, user_slot_base, nuq);
    return hipGetLastError();
}

}  // namespace sq
