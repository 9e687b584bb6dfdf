// Decode step through a key-index list (Sections 3.2, 4.1, 4.2; Appendix D "Generation Stage").
//
// The sparse attention kernel of Section 4.2 is driven by a list of the indices of the keys to load; this file
// builds that list and lets every launch of the step run across the whole chip:
//
//   select_index_kernel      one workgroup per (query row, slice of 128 clusters).  Every workgroup of a row
//                            recomputes the row's statistics (m, D) of Eq. 1 and all of its keep decisions -- a row is
//                            a few KB of logits, so the redundancy is cheaper than one workgroup per row walking a
//                            long dependent chain on one compute unit -- and therefore knows, without talking to the
//                            other slices, how many clusters and keys are kept in front of its own slice.  It writes
//                            the slice's mask words and, for every kept cluster of the slice, the rows of its keys
//                            into the row's key-index list key_idx[row, position].
//   decode_attn_index_kernel the selected keys of all rows, laid end to end, are cut into EQUAL shares of keys, one
//                            per workgroup (the split-KV scheme of Section 4.2 with the balance taken to the key: every
//                            compute unit streams the same number of bytes whatever the heads keep).  A workgroup
//                            derives its share from the per-row key counts alone, walks it in batches of up to 64
//                            keys (one batch computed while the next one's K/V rows stream in and the index entries of
//                            the one after are fetched), and leaves one partial (max, sum, output) per row it touches.
//                            What a workgroup has to read -- key counts, then index entries, then K/V rows -- is two
//                            dependent round trips before the first selected byte moves; the dense attention over the
//                            user keys (Section 3.2), whose addresses depend on nothing, is dealt over the same
//                            workgroups in equal runs and streams during exactly that time.
//   decode_merge_index_kernel  phase 2 of Section 4.2: the partial results of a row, found from the same key counts.
//
// No counters, no atomics, nothing to clear between steps: every buffer is written before it is read.
#include <algorithm>

#include "sq_common.hpp"
#include "sq_internal.hpp"
#include "sq_merge.hpp"
#include "sq_user_attn.hpp"

namespace sq {

constexpr int KI_THREADS = 1024;                 // selection workgroup: thread v owns clusters v, v + 1024, ...
constexpr int KI_STEPS = KI_MAX_C / KI_THREADS;  // clusters per thread, at most
constexpr int KI_WAVES = KI_THREADS / 64;
static_assert(KI_SLICE == 128, "a slice is the clusters of two waves of one step");

// LDS of one selection workgroup.
struct SelectLds {
    float red[KI_WAVES];
    int cnt[KI_STEPS * KI_WAVES + 1], keys[KI_STEPS * KI_WAVES + 1];
    int4 rec[KI_SLICE];                          // kept clusters of the slice: (first key, keys, keys before, -)
};

// Selection of ONE query row by a 1024-thread workgroup that is responsible for slice `sl` (clusters sl * 128 .. + 127)
// of the row: the statistics (m, D) of Eq. 1 and the keep decision of EVERY cluster of the row (thread v holds the
// logits xv[k] and sizes nv[k] of clusters v + 1024 k), then the outputs of the slice alone: its mask words, the rows of
// its kept keys at their positions in the row's key-index list, and (slice 0) the row's counts.  start_s: first key of
// this thread's cluster in the slice's step (waves of the slice only).  STEPS: clusters per thread the caller holds.
// Key-index entries of the kept clusters rec[0..n) = (first key, keys, position in the row's list) of a slice: eight
// lanes per cluster, so 8 x (waves of the workgroup) clusters are written per round.  (A wave per cluster took eight
// rounds for a 128-cluster slice of a row that keeps everything, and the launch waited 1.6 us for that row's workgroups;
// measured on the whole step at 32 heads x 32K keys: a wave per cluster 28.10 us, 16 lanes 27.82, 8 lanes 27.70, the
// group width chosen by the number of clusters 27.81.)  The eight lanes write the first 64 keys of their cluster; the
// rest of a longer cluster is written by the whole wave.  Called by every thread of the workgroup.
constexpr int KI_WRITE_SH = 3;                                       // log2 of the lanes per cluster
__device__ __forceinline__ void write_key_index(const int4 *rec, int n, int32_t *__restrict__ idx_row, int L, int threads)
{
    constexpr int LPC = 1 << KI_WRITE_SH, PER_WAVE = 64 / LPC;
    const int lane = threadIdx.x & 63;
    for (int c0 = (threadIdx.x >> 6) * PER_WAVE; c0 < n; c0 += (threads >> 6) * PER_WAVE) {   // (wave-uniform bounds)
        const int c = c0 + (lane >> KI_WRITE_SH);
        const int4 rc = c < n ? rec[c] : make_int4(0, 0, 0, 0);
        const int head = min(rc.y, 64);
        for (int j = lane & (LPC - 1); j < head && rc.z + j < L; j += LPC)
            idx_row[rc.z + j] = max(0, min(rc.x + j, L - 1));        // malformed offsets stay in the tensor
        unsigned long long big = __ballot(rc.y > 64);
        while (big) {                                                // wave-uniform; rare
            const int src = __builtin_ctzll(big);                    // a lane of the long cluster's group
            big &= ~(((1ull << LPC) - 1ull) << (src & ~(LPC - 1)));
            const int bx = __shfl(rc.x, src), by = __shfl(rc.y, src), bz = __shfl(rc.z, src);
            for (int j = 64 + lane; j < by && bz + j < L; j += 64) idx_row[bz + j] = max(0, min(bx + j, L - 1));
        }
    }
}

template <int STEPS>
__device__ __forceinline__ void select_row_slice(float (&xv)[STEPS], const int (&nv)[STEPS], int start_s, float T, int C,
                                                 int row, int sl, uint32_t *__restrict__ keep_mask,
                                                 int32_t *__restrict__ n_ranges, int32_t *__restrict__ n_keys,
                                                 const KeyIndexPlan &plan, SelectLds &S)
{
    static_assert(STEPS <= KI_STEPS, "");
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int W = (C + 31) >> 5;
    // The slice's clusters are those of waves wv_s, wv_s + 1 in step k_s.
    const int k_s = (sl * KI_SLICE) / KI_THREADS, wv_s = ((sl * KI_SLICE) % KI_THREADS) >> 6;
    const bool mine = wave == wv_s || wave == wv_s + 1;      // wave-uniform

    // m = max over clusters with keys; e_i = exp(x_i - m); D in the library's one summation order (see wave_row_stats:
    // thread v adds clusters v, v + 1024, ... with fused multiply-adds, a butterfly inside each wave, the 16 wave sums
    // in ascending order) -- bit-identical to sq_centroid_score's denominator.
    float m = SQ_NEG_INF;
#pragma unroll
    for (int k = 0; k < STEPS; ++k)
        if (nv[k] > 0) m = fmaxf(m, xv[k]);
    m = wave_max(m);
    if (lane == 0) S.red[wave] = m;
    __syncthreads();
#pragma unroll
    for (int w = 0; w < KI_WAVES; ++w) m = fmaxf(m, S.red[w]);
    __syncthreads();                                         // S.red is reused
    float local = 0.0f;
#pragma unroll
    for (int k = 0; k < STEPS; ++k) {
        xv[k] = nv[k] > 0 ? expf(xv[k] - m) : 0.0f;          // e_i, kept for the comparison (Appendix D)
        if (nv[k] > 0) local = __fmaf_rn((float)nv[k], xv[k], local);
    }
    local = wave_sum(local);
    if (lane == 0) S.red[wave] = local;
    __syncthreads();
    float Dsum = 0.0f;
#pragma unroll
    for (int w = 0; w < KI_WAVES; ++w) Dsum += S.red[w];
    const float thr = T * Dsum;

    // Keep decisions of the whole row; kept clusters and keys per (step, wave), then their exclusive prefix.
    const int n_steps = (C + KI_THREADS - 1) / KI_THREADS;
    bool keep_s = false;                                     // this thread's cluster of the slice's step
    int nv_s = 0;
    unsigned long long bal_s = 0ull;
#pragma unroll
    for (int k = 0; k < STEPS; ++k) {
        if (k >= n_steps) break;                             // workgroup-uniform
        const bool keep = nv[k] > 0 && xv[k] > thr;
        const unsigned long long bal = __ballot(keep);
        const int wkeys = wave_sum_i(keep ? nv[k] : 0);
        if (lane == 0) {
            S.cnt[k * KI_WAVES + wave] = __popcll(bal);
            S.keys[k * KI_WAVES + wave] = wkeys;
        }
        if (k == k_s) {
            keep_s = keep;
            nv_s = nv[k];
            bal_s = bal;
        }
    }
    __syncthreads();
    static_assert(KI_STEPS * KI_WAVES == 64, "the (step, wave) table is scanned by one wave");
    if (wave == 0) {                                         // 64 entries: one per lane
        const int n_ent = n_steps * KI_WAVES;
        const int c = lane < n_ent ? S.cnt[lane] : 0, kk = lane < n_ent ? S.keys[lane] : 0;
        const int ci = wave_inclusive_scan(c, lane), ki = wave_inclusive_scan(kk, lane);
        S.cnt[lane] = ci - c;
        S.keys[lane] = ki - kk;
        if (lane == 63) {
            S.cnt[KI_STEPS * KI_WAVES] = ci;
            S.keys[KI_STEPS * KI_WAVES] = ki;
        }
    }
    __syncthreads();
    const int tot_r = S.cnt[KI_STEPS * KI_WAVES], tot_k = S.keys[KI_STEPS * KI_WAVES];
    if (sl == 0 && tid == 0) {
        n_ranges[row] = tot_r;
        n_keys[row] = tot_k;
        plan.row_keys[row] = min(tot_k, plan.L);             // (sizes that exceed the context stay inside the list)
    }
    // The slice's two waves: mask words, and the kept clusters' records into LDS (slice order).
    const int ent0 = k_s * KI_WAVES + wv_s;
    const int slice_r0 = S.cnt[ent0];
    if (mine) {
        const int ent = k_s * KI_WAVES + wave;
        const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal_s >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal_s, 0));
        const int kv = keep_s ? nv_s : 0;
        const int incl = wave_inclusive_scan(kv, lane);
        if (keep_s) S.rec[S.cnt[ent] + rank - slice_r0] = make_int4(start_s, kv, S.keys[ent] + incl - kv, 0);
        if (keep_mask && lane == 0) {
            const int w0 = (k_s * KI_THREADS + wave * 64) >> 5;
            if (w0 < W) keep_mask[(size_t)row * W + w0] = (uint32_t)bal_s;
            if (w0 + 1 < W) keep_mask[(size_t)row * W + w0 + 1] = (uint32_t)(bal_s >> 32);
        }
    }
    __syncthreads();
    // kept clusters of the slice: prefix of the entry after its second wave (the same step: wv_s is even) minus its own
    const int e_next = ent0 + 2;
    const int n_slice = (e_next < KI_STEPS * KI_WAVES ? S.cnt[e_next] : tot_r) - slice_r0;
    write_key_index(S.rec, n_slice, plan.key_idx + (size_t)row * plan.L, plan.L, KI_THREADS);
    __syncthreads();                                         // (the caller may select another row with the same LDS)
}

// Selection from logits in memory: one workgroup per (query row, slice).
__global__ __launch_bounds__(KI_THREADS) void select_index_kernel(
    const float *__restrict__ logits, const float *__restrict__ thresh, const int32_t *__restrict__ sizes,
    const int32_t *__restrict__ offsets, uint32_t *__restrict__ keep_mask, int32_t *__restrict__ n_ranges,
    int32_t *__restrict__ n_keys, KeyIndexPlan plan, int H, int G, int C, int nsl)
{
    __shared__ SelectLds S;
    const int unit = blockIdx.x;
    const int tid = threadIdx.x, wave = tid >> 6;
    const int row = unit / nsl, sl = unit - row * nsl;
    const int h = (row / G) % H;
    const float *x = logits + (size_t)row * C;
    const int32_t *N = sizes + (size_t)h * C;
    const int32_t *off = offsets + (size_t)h * (C + 1);
    float xv[KI_STEPS];
    int nv[KI_STEPS];
#pragma unroll
    for (int k = 0; k < KI_STEPS; ++k) {
        const int i = k * KI_THREADS + tid;
        nv[k] = i < C ? N[i] : 0;
        xv[k] = i < C ? x[i] : 0.0f;
    }
    const int k_s = (sl * KI_SLICE) / KI_THREADS, wv_s = ((sl * KI_SLICE) % KI_THREADS) >> 6;
    const int i_s = k_s * KI_THREADS + tid;                  // this thread's cluster in the slice's step
    const bool mine = wave == wv_s || wave == wv_s + 1;
    const int start_s = (mine && i_s < C) ? off[i_s] : 0;    // fetched with the logits: no second round trip
    select_row_slice<KI_STEPS>(xv, nv, start_s, thresh[h], C, row, sl, keep_mask, n_ranges, n_keys, plan, S);
}

// How the partial kernel's workgroups divide the selected keys (the merge kernel derives the same numbers): the kept
// keys of all rows are laid end to end, every row that has keys followed by KI_ROW_PAD positions that stand for no key,
// and this sequence is cut into equal shares, workgroup w taking positions [w * share, (w + 1) * share).  The padding
// prices what a row boundary inside a share costs its workgroup (a drained pipeline and one more partial result), so
// that a share over several short rows holds fewer keys (measured at 32 heads x 32K keys, keep 1/8, whole step: no
// padding 30.95 us, 48 positions 29.5, 128 to 384 positions 28.9; one workgroup per compute unit 28.2 against 28.9 with
// two and 31 with four).  The grid is a multiple of the compute units: every compute unit holds the same number of shares.
constexpr int KI_ROW_PAD = 128;
constexpr int SB_ROUNDS = 8;                 // rounds of 16 keys whose rows a lane holds at a time
constexpr int SB_KEYS = SB_ROUNDS * 16;      // = one "super-batch": two batches of K/V loads
constexpr int NB = SB_ROUNDS / 2;            // rounds per batch
__device__ __forceinline__ int padded(int n) { return n > 0 ? n + KI_ROW_PAD : 0; }
__device__ __forceinline__ int share_of(int P_total, int grid) { return max(KI_MIN_SHARE, (P_total + grid - 1) / grid); }

// One query row's running (max, sum, output) over the keys a workgroup has seen, per lane: m is wave-uniform, l and o
// are the share of the lane's 16-lane group, summed over the four groups only when the state is written out.
struct RowState {
    float m, l, o[8];
    __device__ __forceinline__ void reset()
    {
        m = SQ_NEG_INF;
        l = 0.0f;
#pragma unroll
        for (int e = 0; e < 8; ++e) o[e] = 0.0f;
    }
};

// One super-batch: up to SB_KEYS consecutive keys of one row's index list (all workgroup-uniform).
struct SuperBatch {
    int r;             // query row
    int pos0, n;       // first position in the row's list, keys
};

__global__ __launch_bounds__(256) void decode_attn_index_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ Kf, const _Float16 *__restrict__ Vf,
    KeyIndexPlan plan, float *__restrict__ partials, int rows, int H, int G, float sm_scale, int grid, UserAttn ua)
{
    __shared__ int s_pref[KI_MAX_ROWS + 1];      // prefix of the rows' padded key counts
    __shared__ int s_w[4];
    __shared__ int s_r0;
    __shared__ float s_part[4][PART_STRIDE];
    // The workgroups past the first `grid` attend to the rows' user keys, one piece each: they stream at once, while
    // the others make their two dependent round trips (key counts, then index entries).
    if ((int)blockIdx.x >= grid) {                           // workgroup-uniform
        user_piece_partial(ua, (int)blockIdx.x - grid, s_part);
        return;
    }
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int g = lane >> 4, p = lane & 15;
    const int L = plan.L;
    const int wg = (int)blockIdx.x;
    const int my_slot = wave * 4 + g;                        // this lane group's key slot within a round of 16

    // ---- the rows' key counts -> padded prefix -> this workgroup's share [lo, hi) and the row that holds position lo ----
    int lo, hi, cur_r;
    if (rows <= 64) {                                        // workgroup-uniform: one count per lane, scanned per wave
        const int v = lane < rows ? padded(plan.row_keys[min(lane, rows - 1)]) : 0;
        const int incl = wave_inclusive_scan(v, lane);
        const int P = __builtin_amdgcn_readlane(incl, 63);
        const int share = share_of(P, grid);
        lo = min(P, wg * share);
        hi = min(P, lo + share);
        const unsigned long long above = __ballot(incl > lo);   // the first row whose inclusive prefix exceeds lo
        cur_r = above ? __ffsll((long long)above) - 1 : 0;
        if (wave == 0) s_pref[lane + 1] = incl;
        if (tid == 0) s_pref[0] = 0;
        __syncthreads();
    } else {
        constexpr int PER = KI_MAX_ROWS / 256;               // consecutive rows per thread
        int rk[PER], sum = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            const int v = plan.row_keys[min(tid * PER + u, rows - 1)];
            rk[u] = tid * PER + u < rows ? padded(v) : 0;
            sum += rk[u];
        }
        const int incl = wave_inclusive_scan(sum, lane);
        if (lane == 63) s_w[wave] = incl;
        __syncthreads();
        int base = incl - sum;
#pragma unroll
        for (int w = 0; w < 4; ++w)
            if (w < wave) base += s_w[w];
        if (tid == 0) s_pref[0] = 0;
#pragma unroll
        for (int u = 0; u < PER; ++u) {
            base += rk[u];
            if (tid * PER + u < rows) s_pref[tid * PER + u + 1] = base;
        }
        __syncthreads();
        const int P = __builtin_amdgcn_readfirstlane(s_pref[rows]);
        const int share = share_of(P, grid);
        lo = min(P, wg * share);
        hi = min(P, lo + share);
        if (lo < hi)
            for (int r = tid; r < rows; r += 256)
                if (s_pref[r] <= lo && lo < s_pref[r + 1]) s_r0 = r;   // exactly one row holds position lo
        __syncthreads();
        cur_r = lo < hi ? __builtin_amdgcn_readfirstlane(s_r0) : 0;
    }
    // Cursor over the share: the next super-batch of real keys, skipping padding and rows without keys.
    int cur_pos = lo;
    // (returns the super-batch by value, in scalars: r < 0 means none left)
    auto next_sb = [&]() -> SuperBatch {
        SuperBatch b{-1, 0, 0};
        while (cur_pos < hi) {
            const int p0 = __builtin_amdgcn_readfirstlane(s_pref[cur_r]), p1 = __builtin_amdgcn_readfirstlane(s_pref[cur_r + 1]);
            const int n_r = p1 - p0 - KI_ROW_PAD;            // keys of the row (negative: a row without keys)
            const int a = cur_pos - p0, e = min(min(hi, p1) - p0, n_r);   // row-local positions [a, e) are real keys
            if (a < e) {
                b.r = cur_r;
                b.pos0 = a;
                b.n = min(SB_KEYS, e - a);
                cur_pos += b.n;
                break;
            }
            cur_pos = max(cur_pos, min(hi, p1));             // past this row's padding (or an empty row)
            if (cur_pos >= p1) ++cur_r;
        }
        return b;
    };
    // Everything below that loads is written WITHOUT branches around the loads: the hardware returns loads in issue
    // order and the compiler can only let later loads stay in flight across a wait when it knows they were issued,
    // so slots and whole super-batches that do not exist re-read a valid row instead of being skipped (those repeats
    // are served by the caches; only their arithmetic result is masked).
    //
    // Rows of this lane's slots in the super-batch's rounds and the lane's piece of the row's query.
    auto fetch_rows = [&](const SuperBatch &b, int (&kr)[SB_ROUNDS], h8 &qv) {
        const int32_t *idx = plan.key_idx + (size_t)b.r * L + b.pos0;
#pragma unroll
        for (int i = 0; i < SB_ROUNDS; ++i) kr[i] = idx[min(i * 16 + my_slot, b.n - 1)];
        qv = *reinterpret_cast<const h8 *>(q + (size_t)b.r * D + p * 8);
    };
    auto set_base = [&](const SuperBatch &b, const _Float16 *&Kb, const _Float16 *&Vb) {
        const size_t h = ((size_t)b.r / G) % H;              // K/V head: G query rows of a sequence share it
        Kb = Kf + h * L * D;
        Vb = Vf + h * L * D;
    };
    // K/V rows of rounds [r0, r0 + NB) of a super-batch: every lane issues its loads, nothing waits.
    auto fetch_kv = [&](const _Float16 *Kb, const _Float16 *Vb, const int (&kr)[SB_ROUNDS], int r0, h8 (&kreg)[NB],
                        h8 (&vreg)[NB]) {
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const size_t o16 = (size_t)kr[r0 + i] * D + p * 8;
            // (streamed once: non-temporal loads keep the rows from displacing what the step's other kernels find in
            // the cache)
            kreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Kb + o16));
            vreg[i] = __builtin_nontemporal_load(reinterpret_cast<const h8 *>(Vb + o16));
        }
    };
    RowState st;
    st.reset();
    // Scores of rounds [r0, r0 + NB) folded into the running softmax of the row (n: keys of the super-batch).
    auto compute = [&](const h8 &qv, int r0, int n, const h8 (&kreg)[NB], const h8 (&vreg)[NB]) {
        float s[NB];
        float m_it = SQ_NEG_INF;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const float d = row16_sum(dot8(qv, kreg[i], 0.0f)) * sm_scale;
            s[i] = (r0 + i) * 16 + my_slot < n ? d : SQ_NEG_INF;
            m_it = fmaxf(m_it, s[i]);
        }
        m_it = cross16_max(m_it);
        const float m_new = fmaxf(st.m, m_it);
        const float alpha = m_new == SQ_NEG_INF ? 1.0f : __expf(st.m - m_new);   // exp(-inf) = 0 on the first keys
        st.l *= alpha;
#pragma unroll
        for (int e = 0; e < 8; ++e) st.o[e] *= alpha;
#pragma unroll
        for (int i = 0; i < NB; ++i) {
            const float pr = s[i] == SQ_NEG_INF ? 0.0f : __expf(s[i] - m_new);
            st.l += pr;
#pragma unroll
            for (int e = 0; e < 8; ++e) st.o[e] += pr * (float)vreg[i][e];
        }
        st.m = m_new;
    };

    SuperBatch cur, nxt;
    int kr[SB_ROUNDS], kr_n[SB_ROUNDS];
    h8 qv, qv_n;
    h8 kA[NB], vA[NB], kB[NB], vB[NB];
    const _Float16 *Kb, *Vb, *Kb_n, *Vb_n;
    cur = next_sb();
    if (cur.r < 0) return;                                   // whole workgroup: nothing in its share
    fetch_rows(cur, kr, qv);
    set_base(cur, Kb, Vb);
    fetch_kv(Kb, Vb, kr, 0, kA, vA);
    // Invariant at the top: the first batch of `cur` is in flight in (kA, vA).
    while (true) {
        // the next super-batch: its description, then its index entries and query -- issued BEFORE this one's second
        // batch, so that waiting for them later does not wait for that batch
        nxt = next_sb();
        const bool have_n = nxt.r >= 0;
        if (!have_n) {                                       // none left: loads that are never used re-read ONE key row
            nxt = cur;
            nxt.n = 1;
        }
        fetch_rows(nxt, kr_n, qv_n);
        set_base(nxt, Kb_n, Vb_n);
        fetch_kv(Kb, Vb, kr, NB, kB, vB);
        compute(qv, 0, cur.n, kA, vA);
        fetch_kv(Kb_n, Vb_n, kr_n, 0, kA, vA);               // the next super-batch's first batch leaves now
        compute(qv, NB, cur.n, kB, vB);
        if (!have_n || nxt.r != cur.r) {                     // the row's part of the share is complete: one partial result
            const float l_w = cross16_sum(st.l);
            float ow[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) ow[e] = cross16_sum(st.o[e]);
            if (g == 0) {
                if (p == 0) {
                    s_part[wave][0] = st.m;
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
                float *dst = partials + (size_t)(wg + cur.r) * PART_STRIDE;
                if (tid == 0) {
                    dst[0] = M;
                    dst[1] = lsum;
                }
                dst[4 + tid] = acc;
            }
            __syncthreads();
            st.reset();
        }
        if (!have_n) break;
        cur = nxt;
        qv = qv_n;
        Kb = Kb_n;
        Vb = Vb_n;
#pragma unroll
        for (int i = 0; i < SB_ROUNDS; ++i) kr[i] = kr_n[i];
    }
}

// Phase 2 (Section 4.2): one workgroup per row.  The row's keys are positions pref .. pref + n - 1 of the padded
// end-to-end sequence, so its partial results come from workgroups pref / share .. (pref + n - 1) / share of the
// partial kernel, at slots workgroup + row (both never decrease along the sequence and one of them grows from one
// segment to the next: the slots are unique, grid + rows of them at most); after them the row's user-key partials,
// nuq of them from slot user_slot_base + row * nuq on.
__global__ __launch_bounds__(MERGE_THREADS) void decode_merge_index_kernel(const float *__restrict__ partials,
                                                                           KeyIndexPlan plan,
                                                                           _Float16 *__restrict__ out,
                                                                           float *__restrict__ lse, int rows,
                                                                           int attn_grid, int user_slot_base, int nuq)
{
    __shared__ float s_red[MERGE_GROUPS * 130];
    __shared__ int s_sum[2][MERGE_THREADS / 64];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x;
    static_assert(KI_MAX_ROWS <= MERGE_THREADS, "one row count per thread");
    const int v = tid < rows ? padded(plan.row_keys[min(tid, rows - 1)]) : 0;
    const int n_row = plan.row_keys[row];
    int pref, P;
    if (rows <= 64) {                                        // every wave holds all counts: no LDS, no barrier
        const int incl = wave_inclusive_scan(lane < rows ? padded(plan.row_keys[min(lane, rows - 1)]) : 0, lane);
        P = __builtin_amdgcn_readlane(incl, 63);
        pref = row > 0 ? __builtin_amdgcn_readlane(incl, row - 1) : 0;
    } else {
        const int before = wave_sum_i(tid < row ? v : 0), all = wave_sum_i(v);
        if (lane == 0) {
            s_sum[0][wave] = before;
            s_sum[1][wave] = all;
        }
        __syncthreads();
        pref = 0;
        P = 0;
#pragma unroll
        for (int w = 0; w < MERGE_THREADS / 64; ++w) {
            pref += s_sum[0][w];
            P += s_sum[1][w];
        }
    }
    const int share = share_of(P, attn_grid);
    const int w_first = pref / share;
    const int n_sel = n_row > 0 ? (pref + n_row - 1) / share - w_first + 1 : 0;
    const int n = n_sel + nuq;
    auto slot_ptr = [&](int c) {
        const int idx = c < n_sel ? w_first + c + row : user_slot_base + row * nuq + (c - n_sel);
        return partials + (size_t)idx * PART_STRIDE;
    };
    merge_row<false>(slot_ptr, n, out + (size_t)row * D, lse ? lse + row : nullptr, s_red, tid);
}

// Last level of a hierarchical lookup (Section 3.3, Eq. 3) into the same outputs.  The row's entries are its candidate
// clusters in candidate order, each with a 16-byte record (logit, id | bit 31 if it has no keys, first key, keys), and the
// statistics (max, sum N exp(x - max)) of every work item that scored them (see launch_gather_score).  A row can list
// up to C candidates, so one workgroup takes a slice of CAND_SLICE of them: a quarter of its threads hold a candidate
// each, all of them write the key-index entries (eight lanes per kept cluster, see write_key_index: a slice that
// keeps everything is written in two rounds); the row's maximum and
// normaliser are merged from the items' pairs by every workgroup (item v by thread v; wave sums ascending):
// bit-identical whichever slice asks.  Two launches: the first counts the kept clusters and keys of every slice and
// sets the mask bits (by cluster id, into a mask the scoring launch zeroed); the second, knowing the counts of the
// slices in front of its own, writes the key rows into the row's key-index list and (slice 0) the row's counts.
constexpr int CAND_THREADS = 1024;                               // = items of a row, at most
constexpr int CAND_SLICE = 256;
constexpr int CAND_WAVES = CAND_SLICE / 64;                      // waves that hold candidates
constexpr int CAND_ITEM_WAVES = CAND_THREADS / 64;
static_assert(CAND_SLICE == 256, "cand_slices_for counts slices of 256 candidates");

template <bool EMIT>
struct CandLds {
    float red[CAND_ITEM_WAVES];
    int cnt[CAND_WAVES + 1], keys[CAND_WAVES + 1], base[2];
    int wsum[CAND_ITEM_WAVES], unit[3];
    int4 rec[EMIT ? CAND_SLICE : 1];
};

// Slice `sl` of row `row` (n candidates), by the whole workgroup.  Leaves the LDS free for the next slice.
template <bool EMIT>
__device__ __forceinline__ void cand_select_slice(const CandSelect &cs, const float *__restrict__ thresh,
                                                  uint32_t *__restrict__ keep_mask,
                                                  int32_t *__restrict__ n_ranges, int32_t *__restrict__ n_keys,
                                                  const KeyIndexPlan &plan, int H, int C, int nsl, int row, int sl, int n,
                                                  CandLds<EMIT> &S)
{
    float (&s_red)[CAND_ITEM_WAVES] = S.red;
    int (&s_cnt)[CAND_WAVES + 1] = S.cnt, (&s_keys)[CAND_WAVES + 1] = S.keys, (&s_base)[2] = S.base;
    int4 (&s_rec)[EMIT ? CAND_SLICE : 1] = S.rec;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int j = sl * CAND_SLICE + tid;
    const int4 rv = tid < CAND_SLICE && j < n ? cs.rec[(size_t)row * C + j] : make_int4(0, (int)0x80000000u, 0, 0);
    const int n_sl = (n + CAND_SLICE - 1) / CAND_SLICE;         // slices with candidates: at most 64
    int2 sc = make_int2(0, 0);
    float m, thr;                                               // the row's maximum and T * D
    if constexpr (EMIT) {
        // (the counting launch left them: the same bits, without the round trip to the items' pairs and three barriers)
        if (tid < n_sl) sc = cs.slice_cnt[(size_t)row * nsl + tid];
        const float2 rs = cs.row_stat[row];
        m = rs.x;
        thr = rs.y;
    } else {
        const int2 ri = n > 0 ? cs.row_items[row] : make_int2(0, 0);   // (first item, items): at most CAND_THREADS items
        const float2 ms = tid < ri.y ? cs.stats[ri.x + tid] : make_float2(SQ_NEG_INF, 0.0f);
        const float T = thresh[row % H];
        const float mw = wave_max(ms.x);
        if (lane == 0) s_red[wave] = mw;
        __syncthreads();
        m = s_red[0];
#pragma unroll
        for (int w = 1; w < CAND_ITEM_WAVES; ++w) m = fmaxf(m, s_red[w]);
        __syncthreads();                                        // s_red is reused
        const float part = ms.y > 0.0f ? __fmul_rn(ms.y, expf(ms.x - m)) : 0.0f;
        const float pw = wave_sum(part);
        if (lane == 0) s_red[wave] = pw;
        __syncthreads();
        float Dsum = 0.0f;                                      // the 16 wave sums in ascending order, by every thread
#pragma unroll
        for (int w = 0; w < CAND_ITEM_WAVES; ++w) Dsum += s_red[w];
        thr = T * Dsum;
        if (sl == 0 && tid == 0) cs.row_stat[row] = make_float2(m, thr);   // for the writing launch
    }
    const bool keep = tid < CAND_SLICE && j < n && rv.y >= 0 && expf(__int_as_float(rv.x) - m) > thr;

    const unsigned long long bal = __ballot(keep);
    const int kv = keep ? rv.w : 0;
    const int incl = wave_inclusive_scan(kv, lane);
    if (lane == 63 && wave < CAND_WAVES) {
        s_cnt[wave] = __popcll(bal);
        s_keys[wave] = incl;
    }
    if (!EMIT && keep_mask && wave < CAND_WAVES)
        wave_mask_or(keep_mask + (size_t)row * ((C + 31) >> 5), rv.y & 0x7fffffff, keep, lane);
    __syncthreads();
    if (!EMIT) {
        if (tid == 0) {
            int r = 0, k = 0;
#pragma unroll
            for (int w = 0; w < CAND_WAVES; ++w) {
                r += s_cnt[w];
                k += s_keys[w];
            }
            cs.slice_cnt[(size_t)row * nsl + sl] = make_int2(r, k);
        }
        __syncthreads();                                        // (the LDS is free for the next slice)
        return;
    }
    if (wave == 0) {
        // exclusive prefix of the per-wave counts; records and keys of the slices in front; the row's totals
        const int c = lane < CAND_WAVES ? s_cnt[lane] : 0, kk = lane < CAND_WAVES ? s_keys[lane] : 0;
        const int ci = wave_inclusive_scan(c, lane), ki = wave_inclusive_scan(kk, lane);
        const int before_r = wave_sum_i(lane < sl ? sc.x : 0), before_k = wave_sum_i(lane < sl ? sc.y : 0);
        const int tot_r = wave_sum_i(sc.x), tot_k = wave_sum_i(sc.y);
        if (lane < CAND_WAVES) {
            s_cnt[lane] = ci - c;
            s_keys[lane] = ki - kk;
        }
        if (lane == 63) {
            s_cnt[CAND_WAVES] = ci;
            s_base[0] = before_r;
            s_base[1] = before_k;
            if (sl == 0) {
                n_ranges[row] = tot_r;
                n_keys[row] = tot_k;
                plan.row_keys[row] = min(tot_k, plan.L);
            }
        }
    }
    __syncthreads();
    if (keep) {
        const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0));
        const int r = s_cnt[wave] + rank;
        s_rec[r] = make_int4(rv.z, kv, s_base[1] + s_keys[wave] + incl - kv, 0);
    }
    __syncthreads();
    write_key_index(s_rec, s_cnt[CAND_WAVES], plan.key_idx + (size_t)row * plan.L, plan.L, CAND_THREADS);
    __syncthreads();                                            // (the LDS is free for the next slice)
}

// Workgroups -> slices (rows <= CAND_THREADS): a fixed grid; every workgroup reads all rows' candidate counts and takes
// the non-empty slices u = workgroup, workgroup + grid, ... of the rows laid end to end (a row without candidates counts
// as one slice: its counts are still written), so no workgroup is launched only to find that its slice is empty.
template <bool EMIT>
__global__ __launch_bounds__(CAND_THREADS) void cand_select_kernel(CandSelect cs, const float *__restrict__ thresh,
                                                                   uint32_t *__restrict__ keep_mask,
                                                                   int32_t *__restrict__ n_ranges,
                                                                   int32_t *__restrict__ n_keys, KeyIndexPlan plan,
                                                                   int rows, int H, int C, int nsl)
{
    __shared__ CandLds<EMIT> S;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int n_t = tid < rows ? min(cs.hdr[tid].y, C) : 0;
    const int cnt = tid < rows ? max(1, (n_t + CAND_SLICE - 1) / CAND_SLICE) : 0;
    const int incl = wave_inclusive_scan(cnt, lane);
    if (lane == 63) S.wsum[wave] = incl;
    __syncthreads();
    int start = incl - cnt, total = 0;
#pragma unroll
    for (int w = 0; w < CAND_ITEM_WAVES; ++w) {
        const int ws = S.wsum[w];
        if (w < wave) start += ws;
        total += ws;
    }
    for (int u = blockIdx.x; u < total; u += gridDim.x) {       // workgroup-uniform
        if (u >= start && u < start + cnt) {
            S.unit[0] = tid;
            S.unit[1] = u - start;
            S.unit[2] = n_t;
        }
        __syncthreads();
        const int row = S.unit[0], sl = S.unit[1], n = S.unit[2];
        cand_select_slice<EMIT>(cs, thresh, keep_mask, n_ranges, n_keys, plan, H, C, nsl, row, sl, n, S);
    }
}

hipError_t launch_cand_select(CandSelect cs, const float *thresh, uint32_t *keep_mask, int32_t *n_ranges, int32_t *n_keys,
                              KeyIndexPlan plan, int rows, int H, int C, hipStream_t s)
{
    const int nsl = cand_slices_for(C);
    if (nsl > 64 || chunk_cap_for(C) > CAND_ITEM_WAVES * 64 || rows > CAND_THREADS || !plan.key_idx || !plan.row_keys)
        return hipErrorInvalidValue;
    const int grid = (int)std::min<long long>((long long)rows * nsl, 2 * 256);   // two workgroups per compute unit
    hipLaunchKernelGGL(cand_select_kernel<false>, dim3(grid), dim3(CAND_THREADS), 0, s, cs, thresh, keep_mask, n_ranges,
                       n_keys, plan, rows, H, C, nsl);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(cand_select_kernel<true>, dim3(grid), dim3(CAND_THREADS), 0, s, cs, thresh, keep_mask, n_ranges,
                       n_keys, plan, rows, H, C, nsl);
    return hipGetLastError();
}


hipError_t launch_select_index(const float *logits, const float *thresh, const int32_t *sizes, const int32_t *offsets,
                               uint32_t *keep_mask, int32_t *n_ranges, int32_t *n_keys, KeyIndexPlan plan, int rows,
                               int H, int G, int C, hipStream_t s)
{
    if (C > KI_MAX_C || rows > KI_MAX_ROWS) return hipErrorInvalidValue;
    const int nsl = (C + KI_SLICE - 1) / KI_SLICE;
    hipLaunchKernelGGL(select_index_kernel, dim3(rows * nsl), dim3(KI_THREADS), 0, s, logits, thresh, sizes, offsets,
                       keep_mask, n_ranges, n_keys, plan, H, G, C, nsl);
    return hipGetLastError();
}

hipError_t launch_decode_attn_index(const void *q, const void *Kf, const void *Vf, KeyIndexPlan plan, float *partials,
                                    void *out, float *lse, int rows, int H, int G, float sm_scale, const UserAttn *user,
                                    hipStream_t s)
{
    if (rows > KI_MAX_ROWS) return hipErrorInvalidValue;
    UserAttn ua{};
    if (user && user->q) {
        if (user->nuq != user_pieces_for(user->U) || user->rows != rows || user->partials != partials) return hipErrorInvalidValue;
        ua = *user;
    }
    const int grid = KI_ATTN_GRID, launched = grid + (ua.q ? rows * ua.nuq : 0);
    hipEvent_t ev0, ev1;
    if (profile_pair(&ev0, &ev1))
        hipExtLaunchKernelGGL(decode_attn_index_kernel, dim3(launched), dim3(256), 0, s, ev0, ev1, 0, (const _Float16 *)q,
                              (const _Float16 *)Kf, (const _Float16 *)Vf, plan, partials, rows, H, G, sm_scale, grid, ua);
    else
        hipLaunchKernelGGL(decode_attn_index_kernel, dim3(launched), dim3(256), 0, s, (const _Float16 *)q,
                           (const _Float16 *)Kf, (const _Float16 *)Vf, plan, partials, rows, H, G, sm_scale, grid, ua);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(decode_merge_index_kernel, dim3(rows), dim3(MERGE_THREADS), 0, s, partials, plan, (_Float16 *)out,
                       lse, rows, grid, ua.q ? ua.slot_base : 0, ua.q ? ua.nuq : 0);
    return hipGetLastError();
}

}  // namespace sq
