// Threshold selection and compaction (Sections 3.2 / 4.1; Appendix D): keep cluster i iff
// exp(x_i - m) > T * D (strict), then turn the kept clusters of each query row into an ascending
// list of key ranges -- the role the key-index tensor plays in Section 4.2; ranges suffice because
// clusters are stored contiguously.
//
// select_kernel: one workgroup of 16 waves per query row.  The row's logits are staged in LDS and
// replaced there by e_i = exp(x_i - m), so the comparison with T * D re-reads stored exponentials
// instead of recomputing anything (the stored-exponential scheme of Appendix D).  Inside a wave the
// rank of a kept cluster comes from a 64-bit ballot + population count and the number of keys in
// front of it from a prefix scan in the vector ALU (data-parallel-primitive row shifts); the waves
// are stitched through LDS.  The ballot words are the keep mask.
//
// ranges_to_rec_kernel turns a caller's range list into the same records the selection emits, and
// schedule_kernel turns the records of all rows into the work items of the split-KV attention
// kernel: chunks of KPC selected keys (Section 4.2: a fixed number of keys per workgroup, so rows
// that keep more keys get more workgroups), each carrying its own copy of the records it touches.
#include "sq_common.hpp"
#include "sq_internal.hpp"
#include "sq_user_attn.hpp"

namespace sq {

constexpr int SEL_THREADS = 1024;
constexpr int SEL_WAVES = SEL_THREADS / 64;

struct ScanOut {
    int rank, key_prefix, total_cnt, total_keys;
};

// Block-wide exclusive rank / key prefix of the kept items of one block-wide step (NW waves).
template <int NW>
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
    for (int w = 0; w < NW; ++w) {
        const int c = s_cnt[w], k = s_keys[w];
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

// Work items of one row, written by the calling workgroup (nthreads threads).  The row owns
// n_user_chunks + ceil(n_sel / KPC) consecutive items starting at *s_base_ptr (read after the first
// barrier, so the caller may still be fetching it); each record copies itself into every chunk it
// touches.  s_first: LDS scratch, two ints per fixed-context chunk of the row.
// REG: the caller's threads each hold at most one record (have_rec, my_r, my_rec) in registers, as they
// do after a single selection step; otherwise the records are read back from plan.rec.
// SHARED: the row is a union row of a sequence group; its n_user_chunks = sequences * chunks_per_seq user
// chunks name their sequence, and every record carries the set of sequences (rec.w) that kept its cluster.
template <bool REG, bool SHARED = false>
__device__ __forceinline__ void emit_row_items(const DecodePlan &plan, int row, const int *s_base_ptr, int n_rec,
                                               int n_sel, int U, int n_user_chunks, int *s_first, int tid,
                                               int nthreads, bool have_rec, int my_r, int4 my_rec,
                                               int chunks_per_seq = 1)
{
    const int n_fixed = (n_sel + KPC - 1) / KPC;
    int *s_firstz = s_first + n_fixed;                      // selected keys before the chunk's first record
    const int4 *rec_row = plan.rec + (size_t)row * plan.rec_cap;
    // Pass 1: the record that holds a chunk's first key is the chunk's first record.
    auto first_of = [&](int r, const int4 rc) {
        const int c_lo = (rc.z + KPC - 1) / KPC, c_hi = min((rc.z + rc.y - 1) / KPC, n_fixed - 1);
        for (int c = c_lo; c <= c_hi; ++c) {
            s_first[c] = r;
            s_firstz[c] = rc.z;
        }
    };
    constexpr int RB = 8;                                   // records fetched together (all loads in flight)
    if (REG) {
        if (have_rec) first_of(my_r, my_rec);
    } else {
        for (int r0 = tid; r0 < n_rec; r0 += nthreads * RB) {
            int4 rc[RB];
#pragma unroll
            for (int u = 0; u < RB; ++u) rc[u] = r0 + u * nthreads < n_rec ? rec_row[r0 + u * nthreads] : make_int4(0, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < RB; ++u)
                if (r0 + u * nthreads < n_rec) first_of(r0 + u * nthreads, rc[u]);
        }
    }
    __syncthreads();
    const int base = *s_base_ptr;
    if (tid == 0) plan.row_items[row] = make_int2(base, n_user_chunks + n_fixed);
    for (int c = tid; c < n_user_chunks; c += nthreads) {
        int2 *it = plan.item + (size_t)(base + c) * ITEM_STRIDE;
        const int seq = SHARED ? c / chunks_per_seq : 0, cu = SHARED ? c % chunks_per_seq : c;
        it[0] = make_int2(row, min(KPC, U - cu * KPC));
        it[1] = make_int2(-1 - seq, cu * KPC);
    }
    // Pass 2: every record writes its (position, delta) into the chunks it touches.
    auto place = [&](int r, const int4 rc) {
        const int c_lo = rc.z / KPC, c_hi = min((rc.z + rc.y - 1) / KPC, n_fixed - 1);
        for (int c = c_lo; c <= c_hi; ++c) {
            int2 *it = plan.item + (size_t)(base + n_user_chunks + c) * ITEM_STRIDE;
            const int pos = rc.z - c * KPC;                 // negative for a record that began in an earlier chunk
            it[2 + r - s_first[c]] = make_int2(SHARED ? (int)((uint32_t)max(pos, 0) | ((uint32_t)rc.w << 16)) : pos, rc.x - pos);
        }
    };
    if (REG) {
        if (have_rec) place(my_r, my_rec);
    } else {
        for (int r0 = tid; r0 < n_rec; r0 += nthreads * RB) {
            int4 rc[RB];
#pragma unroll
            for (int u = 0; u < RB; ++u) rc[u] = r0 + u * nthreads < n_rec ? rec_row[r0 + u * nthreads] : make_int4(0, 0, 0, 0);
#pragma unroll
            for (int u = 0; u < RB; ++u)
                if (r0 + u * nthreads < n_rec) place(r0 + u * nthreads, rc[u]);
        }
    }
    // Chunk headers.  The last record touching chunk c is the first record of chunk c+1 if that record
    // began before the boundary, else the one before it.
    for (int c = tid; c < n_fixed; c += nthreads) {
        int2 *it = plan.item + (size_t)(base + n_user_chunks + c) * ITEM_STRIDE;
        int last;
        if (c + 1 < n_fixed) {
            const int f = s_first[c + 1];
            last = s_firstz[c + 1] == (c + 1) * KPC ? f - 1 : f;
        } else {
            last = n_rec - 1;
        }
        it[0] = make_int2(row, min(KPC, n_sel - c * KPC));
        it[1] = make_int2(last - s_first[c] + 1, c * KPC);   // (records, first position of the chunk in its row)
    }
}

// Selection of one query row by ONE wave, mask and counts only: keep cluster i iff N_i > 0 and
// exp(x_i - m) > T * D.  The row statistics (m, D) are given (STATS_IN) or derived here in the library's one
// summation order (see wave_row_stats), so the decision is bit-identical to the row-wise selection kernel.
// A row of up to 1024 clusters is held in registers after a single round of loads.
template <bool STATS_IN>
__device__ __forceinline__ void wave_select_mask(const float *__restrict__ x, const int32_t *__restrict__ N, int C, float T,
                                                 float m_in, float D_in, uint32_t *__restrict__ mask_row,
                                                 int32_t *n_ranges_out, int32_t *n_keys_out, int lane,
                                                 uint32_t *lds_row = nullptr)   // optional second copy of the mask words
{
    const int W = (C + 31) >> 5;
    int cnt = 0, keys = 0;
    if (C <= 1024) {
        float xv[16];
        int nv[16];
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            const int i = g * 64 + lane;
            nv[g] = i < C ? N[i] : 0;
            xv[g] = i < C ? x[i] : 0.0f;
        }
        float m = m_in, Dsum = D_in;
        if (!STATS_IN) {
            m = SQ_NEG_INF;
#pragma unroll
            for (int g = 0; g < 16; ++g)
                if (nv[g] > 0) m = fmaxf(m, xv[g]);
            m = wave_max(m);
        }
#pragma unroll
        for (int g = 0; g < 16; ++g) xv[g] = nv[g] > 0 ? expf(xv[g] - m) : 0.0f;   // e_i, stored (Appendix D)
        if (!STATS_IN) {
            Dsum = 0.0f;
#pragma unroll
            for (int g = 0; g < 16; ++g)                       // rounded products: nothing may be fused into the sums
                Dsum += wave_sum(nv[g] > 0 ? __fmul_rn((float)nv[g], xv[g]) : 0.0f);
        }
        const float thr = T * Dsum;
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            if (g * 64 >= C) break;
            const bool keep = nv[g] > 0 && xv[g] > thr;
            const unsigned long long bal = __ballot(keep);
            if (lane == 0) {
                const int w0 = g * 2;
                mask_row[w0] = (uint32_t)bal;
                if (w0 + 1 < W) mask_row[w0 + 1] = (uint32_t)(bal >> 32);
                if (lds_row) {
                    lds_row[w0] = (uint32_t)bal;
                    if (w0 + 1 < W) lds_row[w0 + 1] = (uint32_t)(bal >> 32);
                }
            }
            cnt += __popcll(bal);
            keys += keep ? nv[g] : 0;
        }
    } else {
        float m = m_in, Dsum = D_in;
        if (!STATS_IN) wave_row_stats(x, N, C, lane, m, Dsum);
        const float thr = T * Dsum;
        for (int i0 = 0; i0 < C; i0 += 64 * 4) {                 // four loads in flight
            float xv[4];
            int nv[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * 64 + lane;
                nv[u] = i < C ? N[i] : 0;
                xv[u] = i < C ? x[i] : 0.0f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int i = i0 + u * 64;                       // first cluster of this 64-wide step
                if (i >= C) break;
                const bool keep = nv[u] > 0 && expf(xv[u] - m) > thr;
                const unsigned long long bal = __ballot(keep);
                if (lane == 0) {
                    const int w0 = i >> 5;
                    mask_row[w0] = (uint32_t)bal;
                    if (w0 + 1 < W) mask_row[w0 + 1] = (uint32_t)(bal >> 32);
                    if (lds_row) {
                        lds_row[w0] = (uint32_t)bal;
                        if (w0 + 1 < W) lds_row[w0 + 1] = (uint32_t)(bal >> 32);
                    }
                }
                cnt += __popcll(bal);
                keys += keep ? nv[u] : 0;
            }
        }
    }
    keys = wave_sum_i(keys);
    if (lane == 0) {
        *n_ranges_out = cnt;
        *n_keys_out = keys;
    }
}

// UNION: the row is a union row (sequence group, head) of a batched decode over a shared context.  First every
// sequence of the group is selected by one wave of the workgroup (logits [B*H, C]; keep_mask, n_ranges, n_keys
// are the per-sequence outputs), then cluster i is kept for the union row iff any sequence of the group kept
// it, and the set of those sequences travels with the record.  Always with SCHEDULE.
// CAND: level 2 of the two-level lookup (Section 3.3, Eq. 3).  The row's entries are its candidates j = 0..n-1 (the
// children of the kept coarse clusters, ascending), logits[row, j] is the logit of fine cluster opt.cand_id[row, j],
// and the maximum, the normaliser and the compaction run over those n entries only; mask bits are set by cluster id.
template <bool STATS_IN, bool SCHEDULE, bool UNION = false, bool CAND = false>
__global__ __launch_bounds__(SEL_THREADS) void select_kernel(
    const float *__restrict__ logits, const float *__restrict__ row_max, const float *__restrict__ denom,
    const float *__restrict__ thresh, const int32_t *__restrict__ sizes, const int32_t *__restrict__ offsets,
    uint32_t *__restrict__ keep_mask, int32_t *__restrict__ ranges, int32_t *__restrict__ n_ranges,
    int32_t *__restrict__ n_keys, DecodePlan plan, SelectOpts opt, int H, int Lq, int C, int U, int n_user_chunks,
    UserAttn ua)
{
    extern __shared__ __align__(16) unsigned char smem[];
    // Rider (plain scheduling rows only): the workgroups past the first ua.rows compute the rows' attention over their
    // user keys, one chunk each, which does not depend on the selection, while the first ua.rows select.
    if (SCHEDULE && !STATS_IN && !UNION && !CAND) {
        if (ua.q && (int)blockIdx.x >= ua.rows) {            // workgroup-uniform
            user_chunk_partial(ua, (int)blockIdx.x - ua.rows, reinterpret_cast<float *>(smem));
            return;
        }
    }
    __shared__ float s_wred[SEL_WAVES];
    __shared__ int s_base;
    __shared__ float s_thr;
    float *s_e = reinterpret_cast<float *>(smem);          // [C] logits, then e_i
    int32_t *s_N = reinterpret_cast<int32_t *>(s_e + C);   // [C]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = blockIdx.x;
    const int h = (int)((row / Lq) % H);
    const float *x = logits + row * C;
    const int32_t *N = sizes + (size_t)h * C;
    const int32_t *off = offsets + (size_t)h * (C + 1);
    const int W = (C + 31) >> 5;
    const float T = UNION ? 0.0f : thresh[h];
    (void)T;
    // Entries of the row: all C clusters, or (CAND) the row's candidates; entry i is cluster id_of(i).
    const int32_t *cid = CAND ? opt.cand_id + row * C : nullptr;
    const int n = CAND ? min(opt.cand_hdr[row].y, C) : C;
    auto id_of = [&](int i) { return CAND ? cid[i] : i; };
    __shared__ uint32_t s_mask[CAND ? SELECT_MAX_C / 32 : 1];
    uint32_t *s_set = reinterpret_cast<uint32_t *>(s_e);   // UNION: set of sequences per cluster instead of e_i
    const int n_seq = UNION ? min(SG, opt.B - (int)(row / H) * SG) : 1;   // (virtual) sequences of this group
    const int n_real = UNION ? (n_seq + opt.G - 1) / opt.G : 1;            // real sequences: owners of user keys
    // Candidate rows staged from records keep their entries in registers: entry st*SEL_THREADS + tid of this thread is
    // (first key | -1 if dropped, range length).  Indexed with constants only (the step loops below are unrolled).
    int kz[CAND ? 16 : 1], kl[CAND ? 16 : 1];
    int sr[CAND ? 16 : 1], sk[CAND ? 16 : 1];              // their record index (-1: none) and key prefix, from the first walk

    if (UNION) {
        static_assert(SG == SEL_WAVES, "one wave per sequence of the group");
        const int vs0 = (int)(row / H) * SG;                         // first virtual sequence of the group
        if (wave < n_seq) {
            const size_t bh = shared_row(vs0 + wave, h, H, opt.G);
            // the mask words also go to LDS ([SG][W] words at the start of the staging area: W * 32 <= C + 31)
            if (opt.masks_ready) {                                   // selected by a launch of its own (see launch_select)
                for (int w = lane; w < W; w += 64) s_set[wave * W + w] = keep_mask[bh * W + w];
            } else {
                wave_select_mask<false>(logits + bh * C, N, C, thresh[h], 0.0f, 0.0f, keep_mask + bh * W, n_ranges + bh,
                                        n_keys + bh, lane, s_set + wave * W);
            }
        }
        __syncthreads();                                             // the group's masks are in LDS
        uint32_t setv[16];                                           // C <= 16 * SEL_THREADS
#pragma unroll
        for (int k = 0; k < 16; ++k) setv[k] = 0u;
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (k * SEL_THREADS >= C) break;                         // (one jump past the steps the row does not have)
            const int i = k * SEL_THREADS + tid;
            uint32_t set = 0u;
            if (i < C) {
#pragma unroll
                for (int sq_ = 0; sq_ < SG; ++sq_) {
                    const uint32_t word = sq_ < n_seq ? s_set[sq_ * W + (i >> 5)] : 0u;
                    set |= ((word >> (i & 31)) & 1u) << sq_;
                }
            }
            setv[k] = set;
        }
        __syncthreads();                                             // the mask words are consumed: the area is reused
#pragma unroll
        for (int k = 0; k < 16; ++k) {
            if (k * SEL_THREADS >= C) break;
            const int i = k * SEL_THREADS + tid;
            if (i < C) {
                s_set[i] = setv[k];
                s_N[i] = N[i];
            }
        }
    } else if (CAND && !STATS_IN && opt.cand_rec) {
        // Candidates with their records and per-item statistics at hand (see launch_gather_score): the row's maximum
        // and normaliser are merged from its items' pairs (items in ascending order), every entry is decided as its
        // logit and record arrive, and the row is staged directly as (first key | -1, range length).
        for (int w = tid; w < W; w += SEL_THREADS) s_mask[w] = 0u;
        int4 rv[16];                                        // all loads of the (up to 16) steps in flight together:
        const int4 *crec = opt.cand_rec + row * C;          // (logit, id | bit 31 if no keys, first key, range length)
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int i = st * SEL_THREADS + tid;
            rv[st] = i < n ? crec[i] : make_int4(0, (int)0x80000000u, 0, 0);
        }
        const int2 ri = opt.cand_items[row];                // (first item, items): at most chunk_cap_for(C) <= SEL_THREADS
        const float2 ms = tid < ri.y ? opt.cand_stats[ri.x + tid] : make_float2(SQ_NEG_INF, 0.0f);
        float mw = wave_max(ms.x);
        if (lane == 0) s_wred[wave] = mw;
        __syncthreads();
        float m = s_wred[0];
#pragma unroll
        for (int w = 1; w < SEL_WAVES; ++w) m = fmaxf(m, s_wred[w]);
        __syncthreads();                                    // every wave has read the maxima: s_wred is reused
        const float part = ms.y > 0.0f ? __fmul_rn(ms.y, expf(ms.x - m)) : 0.0f;
        const float pw = wave_sum(part);
        if (lane == 0) s_wred[wave] = pw;
        __syncthreads();
        float Dsum = 0.0f;                                  // every thread adds the wave sums in the same order
#pragma unroll
        for (int w = 0; w < SEL_WAVES; ++w) Dsum += s_wred[w];
        const float thr_c = T * Dsum;
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int i = st * SEL_THREADS + tid;
            const bool k = i < n && rv[st].y >= 0 && expf(__int_as_float(rv[st].x) - m) > thr_c;
            kz[CAND ? st : 0] = k ? rv[st].z : -1;
            kl[CAND ? st : 0] = k ? rv[st].w : 0;
            if (st * SEL_THREADS < n) wave_mask_or(s_mask, rv[st].y & 0x7fffffff, k, lane);   // mask bit by cluster id
        }
    } else if (CAND) {
        for (int w = tid; w < W; w += SEL_THREADS) s_mask[w] = 0u;
        int idv[16], nv[16];                                // all loads of the (up to 16) steps in flight together
        float xv[16];
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int i = st * SEL_THREADS + tid;
            idv[st] = i < n ? cid[i] : 0;
            if (STATS_IN && opt.mean_parts) {               // averaged scores of the candidates (parts in ascending order)
                const float *ps = logits + row * (size_t)opt.mean_parts * C;
                float sum = 0.0f;
                if (i < n)
                    for (int p = 0; p < opt.mean_parts; ++p) sum += ps[(size_t)p * C + i];
                xv[st] = sum / opt.mean_div;
            } else {
                xv[st] = i < n ? x[i] : 0.0f;
            }
        }
#pragma unroll
        for (int st = 0; st < 16; ++st) nv[st] = st * SEL_THREADS + tid < n ? N[idv[st]] : 0;
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int i = st * SEL_THREADS + tid;
            if (i < n) {
                s_e[i] = xv[st];
                s_N[i] = nv[st];
            }
        }
    } else if (opt.mean_parts) {
        // Averaged-score selection (Appendix D, prefill): the staged value is the mean score itself.
        const float *ps = logits + row * (size_t)opt.mean_parts * C;
        for (int i = tid; i < C; i += SEL_THREADS) {
            float sum = 0.0f;                               // parts added in ascending order
            int p = 0;
            for (; p + 8 <= opt.mean_parts; p += 8) {       // eight loads in flight
                float v8[8];
#pragma unroll
                for (int u = 0; u < 8; ++u) v8[u] = ps[(size_t)(p + u) * C + i];
#pragma unroll
                for (int u = 0; u < 8; ++u) sum += v8[u];
            }
            for (; p < opt.mean_parts; ++p) sum += ps[(size_t)p * C + i];
            s_e[i] = sum / opt.mean_div;
            s_N[i] = N[i];
        }
    } else {
#pragma unroll 4
        for (int i = tid; i < C; i += SEL_THREADS) {
            s_e[i] = x[i];
            s_N[i] = N[i];
        }
    }
    const bool cand_fast = CAND && !STATS_IN && opt.cand_rec != nullptr;   // workgroup-uniform
    float m, thr = 0.0f;
    if (cand_fast) {
        __syncthreads();                                    // the row is staged
    } else if (UNION) {
        if (tid == 0) s_thr = 0.0f;
    } else if (STATS_IN && opt.mean_parts) {
        if (tid == 0) s_thr = T;                            // keep iff mean score > T
        __syncthreads();
        for (int i = tid; i < n; i += SEL_THREADS) s_e[i] = s_N[i] > 0 ? s_e[i] : 0.0f;
    } else if (STATS_IN) {
        m = row_max[row];
        if (tid == 0) s_thr = T * denom[row];
        __syncthreads();
        for (int i = tid; i < n; i += SEL_THREADS) s_e[i] = s_N[i] > 0 ? expf(s_e[i] - m) : 0.0f;
    } else {
        __syncthreads();
        m = SQ_NEG_INF;
        for (int i = tid; i < n; i += SEL_THREADS)
            if (s_N[i] > 0) m = fmaxf(m, s_e[i]);
        m = wave_max(m);
        if (lane == 0) s_wred[wave] = m;
        __syncthreads();
        m = s_wred[0];
#pragma unroll
        for (int w = 1; w < SEL_WAVES; ++w) m = fmaxf(m, s_wred[w]);
        for (int i = tid; i < n; i += SEL_THREADS) s_e[i] = s_N[i] > 0 ? expf(s_e[i] - m) : 0.0f;
        __syncthreads();                                     // every wave has read the maxima: s_wred is reused below
        // D in the library's one summation order (see wave_row_stats): thread v adds clusters v, v+1024, ...
        // ascending, butterfly inside each wave, then the 16 wave sums in ascending order.
        float local = 0.0f;
        for (int i = tid; i < n; i += SEL_THREADS) {
            const int Ni = s_N[i];
            if (Ni > 0) local = __fmaf_rn((float)Ni, s_e[i], local);
        }
        local = wave_sum(local);
        if (lane == 0) s_wred[wave] = local;
        __syncthreads();
        float Dsum = 0.0f;                                   // every thread adds the 16 wave sums, in the same order
#pragma unroll
        for (int w = 0; w < SEL_WAVES; ++w) Dsum += s_wred[w];
        thr = T * Dsum;
    }
    if (UNION || STATS_IN) {
        __syncthreads();
        thr = s_thr;
    }

    // Compaction in two passes over the (up to 16) block-wide steps, with one barrier between them.
    // Pass 1: every wave counts the ranges it will emit and their keys, step by step, into a small LDS
    // table, and writes the mask words.  The table's exclusive prefix in (step, wave) order gives every
    // wave of every step its first record index and key prefix.  Pass 2 repeats the cheap ballot and
    // lane scan and emits.
    __shared__ int s_tcnt[16 * SEL_WAVES + 1], s_tkeys[16 * SEL_WAVES + 1];
    const int n_steps = (n + SEL_THREADS - 1) / SEL_THREADS;
    const int id_first = tid < n ? id_of(tid) : 0;
    const int start_first = (tid < n) ? off[id_first] : 0;  // offsets of the first step, fetched early
    const int next_first = (opt.len_from_offsets && tid < n) ? off[id_first + 1] : 0;
    // Rows of more than one step: every global load of the compaction is issued here, for all (up to 16) steps at
    // once, so that no step below waits on memory.  The staged value of entry i becomes the first key of its range
    // (-1 if the cluster is dropped) and s_N[i] the range's length; a thread re-reads only entries it wrote itself.
    const bool staged_ranges = (!UNION && n_steps > 1) || cand_fast;
    if (staged_ranges && !cand_fast) {
        int idv[16], sv[16], lv[16];
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int i = st * SEL_THREADS + tid;
            const bool k = i < n && s_N[i] > 0 && s_e[i] > thr;
            idv[st] = k ? id_of(i) : -1;
        }
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            sv[st] = idv[st] >= 0 ? off[idv[st]] : -1;
            lv[st] = (opt.len_from_offsets && idv[st] >= 0) ? off[idv[st] + 1] : 0;
        }
#pragma unroll
        for (int st = 0; st < 16; ++st) {
            const int i = st * SEL_THREADS + tid;
            if (i < n) {
                s_e[i] = __int_as_float(sv[st]);
                if (opt.len_from_offsets) s_N[i] = idv[st] >= 0 ? lv[st] - sv[st] : 0;
            }
            if (CAND) wave_mask_or(s_mask, idv[st], i < n && idv[st] >= 0, lane);   // mask bit by cluster id
        }
    }
    // Entry i of step st: kept?, first key and length of its range.
    auto entry = [&](int st, int i, bool &keep, int &start, int &len) {
        if (CAND && cand_fast) {
            start = kz[CAND ? st : 0];
            keep = start >= 0;
            len = kl[CAND ? st : 0];
        } else if (staged_ranges) {
            start = i < n ? __float_as_int(s_e[i]) : -1;
            keep = start >= 0;
            len = keep ? s_N[i] : 0;
        } else {
            const int Ni = i < n ? s_N[i] : 0;
            keep = Ni > 0 && (UNION ? s_set[i] != 0u : s_e[i] > thr);
            start = st == 0 ? start_first : (keep ? off[i] : 0);    // later steps: union rows only
            len = opt.len_from_offsets ? (keep ? next_first - start_first : 0) : Ni;
        }
    };
    // The block-wide steps of the row.  Candidate rows: unrolled, so that `st` is a constant in the body (register
    // entries) and the steps, which do not depend on each other, overlap.
    auto for_steps = [&](auto &&body) {
        if constexpr (CAND) {
#pragma unroll
            for (int st = 0; st < 16; ++st)
                if (st < n_steps) body(st);              // workgroup-uniform
        } else {
            for (int st = 0; st < n_steps; ++st) body(st);
        }
    };
    for_steps([&](int st) {
        const int i = st * SEL_THREADS + tid;
        bool keep;
        int start, len;
        entry(st, i, keep, start, len);
        const bool emit = keep && len > 0;              // a kept coarse cluster without children emits nothing
        const unsigned long long bal = __ballot(keep), bal_emit = __ballot(emit);
        const int wkeys = wave_sum_i(emit ? len : 0);
        if (lane == 0) {
            s_tcnt[st * SEL_WAVES + wave] = __popcll(bal_emit);
            s_tkeys[st * SEL_WAVES + wave] = wkeys;
            if (keep_mask && !UNION && !CAND) {          // (a union row has no mask of its own)
                const int w0 = (i >> 5);
                if (w0 < W) keep_mask[row * W + w0] = (uint32_t)bal;
                if (w0 + 1 < W) keep_mask[row * W + w0 + 1] = (uint32_t)(bal >> 32);
            }
        }
        if (CAND && !staged_ranges) wave_mask_or(s_mask, id_first, keep, lane);
    });
    __syncthreads();
    if (CAND && keep_mask)
        for (int w = tid; w < W; w += SEL_THREADS) keep_mask[row * W + w] = s_mask[w];
    // Work items of the row are placed at a base taken from a device-wide counter (zeroed by the scoring kernel
    // that ran before): rows land in arrival order, which moves chunks between workgroups but changes no result.
    // The add is issued as soon as the row's totals are known, so its round trip runs under the second pass.
    auto take_items = [&](int total_keys) {
        const int n_items = n_user_chunks * n_real + (min(total_keys, plan.L) + KPC - 1) / KPC;
        // One 64-bit add advances (items, rows placed) together, so rows are ranked in item order.
        const unsigned long long old = atomicAdd(reinterpret_cast<unsigned long long *>(plan.total),
                                                 (1ull << 32) | (unsigned long long)(unsigned)n_items);
        s_base = (int)(old & 0xffffffffull);
        if (plan.row_rank) plan.row_rank[row] = (int)(old >> 32);
    };
    int base_r, base_k;                                      // totals of the row
    int pre_r = 0, pre_k = 0;                                // single step: records / keys of the waves before this one
    if (n_steps == 1) {
        // One step: every thread adds the 16 per-wave counts itself (no second barrier).
        base_r = 0;
        base_k = 0;
#pragma unroll
        for (int w = 0; w < SEL_WAVES; ++w) {
            const int c = s_tcnt[w], k = s_tkeys[w];
            if (w < wave) {
                pre_r += c;
                pre_k += k;
            }
            base_r += c;
            base_k += k;
        }
        if (SCHEDULE && tid == 0) take_items(base_k);
    } else {
        if (wave == 0) {                                     // exclusive prefix of the n_steps*16 (<= 256) entries
            const int n_ent = n_steps * SEL_WAVES;
            int c4[4], k4[4], cs = 0, ks = 0;
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = lane * 4 + u;
                c4[u] = e < n_ent ? s_tcnt[e] : 0;
                k4[u] = e < n_ent ? s_tkeys[e] : 0;
                cs += c4[u];
                ks += k4[u];
            }
            int cpre = wave_inclusive_scan(cs, lane) - cs, kpre = wave_inclusive_scan(ks, lane) - ks;
            const int ctot = __shfl(cpre + cs, 63), ktot = __shfl(kpre + ks, 63);
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                const int e = lane * 4 + u;
                if (e < n_ent) {
                    s_tcnt[e] = cpre;
                    s_tkeys[e] = kpre;
                }
                cpre += c4[u];
                kpre += k4[u];
            }
            if (lane == 0) {
                s_tcnt[16 * SEL_WAVES] = ctot;
                s_tkeys[16 * SEL_WAVES] = ktot;
                if (SCHEDULE) take_items(ktot);
            }
        }
        __syncthreads();
        base_r = s_tcnt[16 * SEL_WAVES];
        base_k = s_tkeys[16 * SEL_WAVES];
    }
    bool have_rec = false;                                   // this thread's record of the (only) step
    int my_r = 0;
    int4 my_rec = make_int4(0, 0, 0, 0);
    // Walks the row's records in order: fn(r, (first key, keys, keys before, set)) for every kept entry with keys,
    // r and the key prefix from the (step, wave) table plus a ballot and a lane scan.  Can be run more than once:
    // the staged row stays in LDS.
    auto for_each_record = [&](auto &&fn) {
        for_steps([&](int st) {
            const int i = st * SEL_THREADS + tid;
            bool keep;
            int start, len;
            entry(st, i, keep, start, len);
            const bool emit = keep && len > 0;
            const unsigned long long bal_emit = __ballot(emit);
            if (bal_emit == 0ull) return;                // wave-uniform
            const int rank = __builtin_amdgcn_mbcnt_hi((uint32_t)(bal_emit >> 32),
                                                       __builtin_amdgcn_mbcnt_lo((uint32_t)bal_emit, 0));
            const int kv = emit ? len : 0;
            const int incl = wave_inclusive_scan(kv, lane);
            if (emit) {
                const int r = (n_steps == 1 ? pre_r : s_tcnt[st * SEL_WAVES + wave]) + rank;
                const int kbefore = (n_steps == 1 ? pre_k : s_tkeys[st * SEL_WAVES + wave]) + incl - kv;
                fn(r, make_int4(start, len, kbefore, UNION ? (int)s_set[i] : 0), st);
            }
        });
    };
    // Rows of more than one step that schedule (opt.replay: the table below fits behind the staged row): the work
    // items are written from two walks over the records instead of reading them back from memory.  Walk 1 (together
    // with the outputs) notes, per chunk of KPC kept keys, the record that holds the chunk's first key (bit 31: the
    // record begins exactly there); walk 2 copies every record into the chunks it touches.
    const bool replay = SCHEDULE && CAND && n_steps > 1 && opt.replay;     // workgroup-uniform; candidate rows only
    int *s_tab = reinterpret_cast<int *>(smem + (size_t)C * 8);
    const int n_sel = SCHEDULE ? min(base_k, plan.L) : 0;
    const int n_fixed = (n_sel + KPC - 1) / KPC;
    constexpr uint32_t EXACT = 0x80000000u;
    if (CAND) {
#pragma unroll
        for (int st = 0; st < (CAND ? 16 : 1); ++st) sr[st] = -1;
    }
    for_each_record([&](int r, const int4 rc, int st) {
        if (ranges) *reinterpret_cast<int2 *>(ranges + (row * C + r) * 2) = make_int2(rc.x, rc.y);
        my_rec = rc;
        my_r = r;
        have_rec = true;
        if (CAND) {                                          // (st is a constant here: the step loop is unrolled)
            sr[CAND ? st : 0] = r;
            sk[CAND ? st : 0] = rc.z;
        }
        if (plan.rec && !replay) plan.rec[row * plan.rec_cap + r] = rc;
        if (replay) {
            const int c_lo = (rc.z + KPC - 1) / KPC, c_hi = min((rc.z + rc.y - 1) / KPC, n_fixed - 1);
            for (int c = c_lo; c <= c_hi; ++c) s_tab[c] = (int)((uint32_t)r | (rc.z == c * KPC ? EXACT : 0u));
        }
    });
    if (tid == 0) {
        if (!UNION) {                                        // a union row has no outputs of its own
            n_ranges[row] = base_r;
            n_keys[row] = base_k;
        }
        if (plan.rec) plan.hdr[row] = make_int2(base_r, base_k);
    }
    if (SCHEDULE && replay) {
        const int n_uc = n_user_chunks * n_real;            // every real sequence of a union row has its own user keys
        __syncthreads();                                    // the chunk table is complete
        const int base = s_base;
        if (tid == 0) plan.row_items[row] = make_int2(base, n_uc + n_fixed);
        for (int c = tid; c < n_uc; c += SEL_THREADS) {
            int2 *it = plan.item + (size_t)(base + c) * ITEM_STRIDE;
            const int seq = UNION ? c / n_user_chunks : 0, cu = UNION ? c % n_user_chunks : c;
            it[0] = make_int2((int)row, min(KPC, U - cu * KPC));
            it[1] = make_int2(-1 - seq, cu * KPC);
        }
        // Second walk.  Rows staged from records kept every entry's record index and key prefix in registers.
        auto for_each_again = [&](auto &&fn) {
            if (CAND && cand_fast) {
                for_steps([&](int st) {
                    if (sr[CAND ? st : 0] >= 0)
                        fn(sr[CAND ? st : 0], make_int4(kz[CAND ? st : 0], kl[CAND ? st : 0], sk[CAND ? st : 0], 0), st);
                });
            } else {
                for_each_record(fn);
            }
        };
        for_each_again([&](int r, const int4 rc, int) {
            const int c_lo = rc.z / KPC, c_hi = min((rc.z + rc.y - 1) / KPC, n_fixed - 1);
            for (int c = c_lo; c <= c_hi; ++c) {
                int2 *it = plan.item + (size_t)(base + n_uc + c) * ITEM_STRIDE;
                const int pos = rc.z - c * KPC;              // negative for a record that began in an earlier chunk
                const int first = (int)((uint32_t)s_tab[c] & ~EXACT);
                it[2 + r - first] = make_int2(UNION ? (int)((uint32_t)max(pos, 0) | ((uint32_t)rc.w << 16)) : pos, rc.x - pos);
            }
        });
        // Chunk headers.  The last record touching chunk c is the first record of chunk c+1 if that record began
        // before the boundary, else the one before it.
        for (int c = tid; c < n_fixed; c += SEL_THREADS) {
            int2 *it = plan.item + (size_t)(base + n_uc + c) * ITEM_STRIDE;
            const int first = (int)((uint32_t)s_tab[c] & ~EXACT);
            int last;
            if (c + 1 < n_fixed) {
                const uint32_t t = (uint32_t)s_tab[c + 1];
                last = (int)(t & ~EXACT) - ((t & EXACT) ? 1 : 0);
            } else {
                last = base_r - 1;
            }
            it[0] = make_int2((int)row, min(KPC, n_sel - c * KPC));
            it[1] = make_int2(last - first + 1, c * KPC);   // (records, first position of the chunk in its row)
        }
    } else if (SCHEDULE) {
        // This row's work items (their base was taken above).  The records written above are read back after
        // the barrier.
        const int n_uc = n_user_chunks * n_real;            // every real sequence of a union row has its own user keys
        __syncthreads();                                    // every thread is done with the staged row (s_first aliases it)
        int *s_first = reinterpret_cast<int *>(smem);       // the staged logits are no longer needed
        if (C <= SEL_THREADS) {
            emit_row_items<true, UNION>(plan, (int)row, &s_base, base_r, n_sel, U, n_uc, s_first, tid, SEL_THREADS,
                                        have_rec, my_r, my_rec, n_user_chunks);
        } else {
            emit_row_items<false, UNION>(plan, (int)row, &s_base, base_r, n_sel, U, n_uc, s_first, tid, SEL_THREADS,
                                         false, 0, my_rec, n_user_chunks);
        }
    }
}

// Mask-only selection, one wave per query row and no LDS: the form prefill uses, where tens of thousands
// of rows each need only their keep mask and counts (no ranges).
template <bool STATS_IN>
__global__ __launch_bounds__(256) void select_mask_kernel(const float *__restrict__ logits,
                                                          const float *__restrict__ row_max,
                                                          const float *__restrict__ denom,
                                                          const float *__restrict__ thresh,
                                                          const int32_t *__restrict__ sizes,
                                                          uint32_t *__restrict__ keep_mask,
                                                          int32_t *__restrict__ n_ranges, int32_t *__restrict__ n_keys,
                                                          int rows, int H, int Lq, int C)
{
    const int lane = threadIdx.x & 63;
    const size_t row = (size_t)blockIdx.x * 4 + (threadIdx.x >> 6);
    if (row >= (size_t)rows) return;
    const int h = (int)((row / Lq) % H);
    const int W = (C + 31) >> 5;
    wave_select_mask<STATS_IN>(logits + row * C, sizes + (size_t)h * C, C, thresh[h], STATS_IN ? row_max[row] : 0.0f,
                               STATS_IN ? denom[row] : 0.0f, keep_mask + row * W, n_ranges + row, n_keys + row, lane);
}

// Caller-provided ranges -> records (start, count, keys before) + header.  Empty ranges are dropped.
__global__ __launch_bounds__(256) void ranges_to_rec_kernel(const int32_t *__restrict__ ranges,
                                                            const int32_t *__restrict__ n_ranges, DecodePlan plan,
                                                            int range_cap)
{
    __shared__ int s_cnt[4], s_keys[4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const size_t row = blockIdx.x;
    const int nr = min(n_ranges[row], range_cap);
    int4 *rec_row = plan.rec + row * plan.rec_cap;
    int base_r = 0, base_k = 0;
    for (int r0 = 0; r0 < nr; r0 += 256) {
        const int r = r0 + tid;
        int2 rg = make_int2(0, 0);
        if (r < nr) rg = *reinterpret_cast<const int2 *>(ranges + (row * range_cap + r) * 2);
        const bool live = r < nr && rg.y > 0;
        unsigned long long bal;
        const ScanOut sc = block_scan_kept<4>(live, rg.y, lane, wave, s_cnt, s_keys, bal);
        if (live && base_r + sc.rank < plan.rec_cap)
            rec_row[base_r + sc.rank] = make_int4(rg.x, rg.y, base_k + sc.key_prefix, 0);
        base_r += sc.total_cnt;
        base_k += sc.total_keys;
    }
    if (tid == 0) plan.hdr[row] = make_int2(min(base_r, plan.rec_cap), base_k);
}

// Work items from the records of all rows, in row order: every workgroup derives its row's first item
// from the headers of all rows (a few hundred integers), so the rows need no second pass.
__global__ __launch_bounds__(256) void schedule_kernel(DecodePlan plan, int rows, int U, int n_user_chunks)
{
    extern __shared__ __align__(16) unsigned char smem[];
    int *s_first = reinterpret_cast<int *>(smem);
    __shared__ int s_wsum[2][4];
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int row = blockIdx.x;
    const int L = plan.L;
    int before = 0, total = 0;
    for (int r = tid; r < rows; r += 256) {
        const int cnt = n_user_chunks + (min(plan.hdr[r].y, L) + KPC - 1) / KPC;
        total += cnt;
        if (r < row) before += cnt;
    }
    before = wave_sum_i(before);
    total = wave_sum_i(total);
    if (lane == 0) {
        s_wsum[0][wave] = before;
        s_wsum[1][wave] = total;
    }
    __syncthreads();
    __shared__ int s_base;
    total = s_wsum[1][0] + s_wsum[1][1] + s_wsum[1][2] + s_wsum[1][3];
    const int2 hdr = plan.hdr[row];
    if (tid == 0) {
        s_base = s_wsum[0][0] + s_wsum[0][1] + s_wsum[0][2] + s_wsum[0][3];
        if (row == 0) *plan.total = total;
    }
    emit_row_items<false>(plan, row, &s_base, min(hdr.x, plan.rec_cap), min(hdr.y, L), U, n_user_chunks, s_first, tid,
                          256, false, 0, make_int4(0, 0, 0, 0));
}

// schedule == true also emits the row's work items (needs *plan.total == 0 on entry).
hipError_t launch_select(const float *logits, const float *row_max, const float *denom, bool stats_in,
                         const float *thresh, const int32_t *sizes, const int32_t *offsets, uint32_t *keep_mask,
                         int32_t *ranges, int32_t *n_ranges, int32_t *n_keys, DecodePlan plan, bool schedule, int U,
                         SelectOpts opt, int rows, int H, int Lq, int C, hipStream_t s, const UserAttn *user)
{
    if (user && user->q && (!schedule || stats_in || opt.union_rows || opt.cand_id)) return hipErrorInvalidValue;
    if (!ranges && !plan.rec && !schedule && !opt.cand_id && !opt.len_from_offsets && !opt.mean_parts && keep_mask) {
        // mask and counts only (prefill): one wave per row
        if (stats_in)
            hipLaunchKernelGGL(select_mask_kernel<true>, dim3((rows + 3) / 4), dim3(256), 0, s, logits, row_max, denom,
                               thresh, sizes, keep_mask, n_ranges, n_keys, rows, H, Lq, C);
        else
            hipLaunchKernelGGL(select_mask_kernel<false>, dim3((rows + 3) / 4), dim3(256), 0, s, logits, row_max, denom,
                               thresh, sizes, keep_mask, n_ranges, n_keys, rows, H, Lq, C);
        return hipGetLastError();
    }
    // LDS: logits + sizes of the row; reused for two ints per chunk when scheduling.
    size_t smem = (size_t)C * 8;
    if (schedule && (size_t)chunk_cap_for(plan.L) * 8 > smem) smem = (size_t)chunk_cap_for(plan.L) * 8;
    // Rows of more than one step build their work items from the staged row when the per-chunk table fits behind it.
    opt.replay = 0;
    if (schedule && C > SEL_THREADS && (size_t)C * 8 + (size_t)chunk_cap_for(plan.L) * 4 <= (size_t)LDS_BYTES_MAX) {
        opt.replay = 1;
        if ((size_t)C * 8 + (size_t)chunk_cap_for(plan.L) * 4 > smem) smem = (size_t)C * 8 + (size_t)chunk_cap_for(plan.L) * 4;
    }
    if (opt.union_rows && (size_t)SG * ((C + 31) / 32) * 4 > smem) smem = (size_t)SG * ((C + 31) / 32) * 4;   // the group's masks
    if (smem > (size_t)LDS_BYTES_MAX) return hipErrorInvalidValue;
    static bool attr_set = false;   // one GPU per process in this build
    if (!attr_set) {
        const int lim = LDS_BYTES_MAX;
        const void *fns[8] = {reinterpret_cast<const void *>(select_kernel<true, false, false, true>),
                              reinterpret_cast<const void *>(select_kernel<true, false>),
                              reinterpret_cast<const void *>(select_kernel<false, false>),
                              reinterpret_cast<const void *>(select_kernel<false, true>),
                              reinterpret_cast<const void *>(select_kernel<true, true>),
                              reinterpret_cast<const void *>(select_kernel<false, true, true>),
                              reinterpret_cast<const void *>(select_kernel<false, false, false, true>),
                              reinterpret_cast<const void *>(select_kernel<false, true, false, true>)};
        for (const void *f : fns) {
            hipError_t e = hipFuncSetAttribute(f, hipFuncAttributeMaxDynamicSharedMemorySize, lim);
            if (e != hipSuccess) return e;
        }
        attr_set = true;
    }
    const int nuc = user_chunks_for(U);
    if (opt.union_rows) {
        if (!schedule || !keep_mask || !logits) return hipErrorInvalidValue;
        // Groups of many sequences: the per-sequence selections (one wave each) would share one compute unit per
        // union row and queue for its vector ALUs, so they get a launch of their own, four rows per workgroup
        // across the chip (the same function, the same bits); the union kernel then reads the mask words.
        opt.masks_ready = 0;
        if (opt.B >= 8) {
            const int seq_rows = opt.B * H;
            hipLaunchKernelGGL(select_mask_kernel<false>, dim3((seq_rows + 3) / 4), dim3(256), 0, s, logits, row_max, denom,
                               thresh, sizes, keep_mask, n_ranges, n_keys, seq_rows, H, opt.G, C);
            opt.masks_ready = 1;
        }
        hipLaunchKernelGGL((select_kernel<false, true, true>), dim3(rows), dim3(SEL_THREADS), smem, s, logits, row_max,
                           denom, thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys, plan, opt, H, Lq, C, U,
                           nuc, UserAttn{});
        return hipGetLastError();
    }
    if (opt.cand_id) {
        if ((stats_in && (!opt.mean_parts || schedule)) || !opt.cand_hdr) return hipErrorInvalidValue;
        if (stats_in)                                       // averaged scores over the candidates (prefill rule)
            hipLaunchKernelGGL((select_kernel<true, false, false, true>), dim3(rows), dim3(SEL_THREADS), smem, s, logits,
                               row_max, denom, thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys, plan, opt, H,
                               Lq, C, U, nuc, UserAttn{});
        else if (schedule)
            hipLaunchKernelGGL((select_kernel<false, true, false, true>), dim3(rows), dim3(SEL_THREADS), smem, s, logits,
                               row_max, denom, thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys, plan, opt, H,
                               Lq, C, U, nuc, UserAttn{});
        else
            hipLaunchKernelGGL((select_kernel<false, false, false, true>), dim3(rows), dim3(SEL_THREADS), smem, s, logits,
                               row_max, denom, thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys, plan, opt, H,
                               Lq, C, U, nuc, UserAttn{});
        return hipGetLastError();
    }
#define SQ_LAUNCH_SELECT(SI, SCH, GRID, UA)                                                                     \
    hipLaunchKernelGGL((select_kernel<SI, SCH>), dim3(GRID), dim3(SEL_THREADS), smem, s, logits, row_max, denom, \
                       thresh, sizes, offsets, keep_mask, ranges, n_ranges, n_keys, plan, opt, H, Lq, C, U, nuc, UA)
    if (stats_in && schedule) SQ_LAUNCH_SELECT(true, true, rows, UserAttn{});
    else if (stats_in) SQ_LAUNCH_SELECT(true, false, rows, UserAttn{});
    else if (schedule && user && user->q) {
        // The rows' user-key attention rides along: one more workgroup per (row, user chunk), and no user chunks in the work list
        // (the caller passes U = 0 for it).  Their partial results are staged in the dynamic LDS area.
        if (U != 0 || user->nuq != user_chunks_for(user->U) || user->rows != rows) return hipErrorInvalidValue;
        if (smem < (size_t)16 * PART_STRIDE * sizeof(float)) smem = (size_t)16 * PART_STRIDE * sizeof(float);
        SQ_LAUNCH_SELECT(false, true, rows + rows * user->nuq, *user);
    } else if (schedule) SQ_LAUNCH_SELECT(false, true, rows, UserAttn{});
    else SQ_LAUNCH_SELECT(false, false, rows, UserAttn{});
#undef SQ_LAUNCH_SELECT
    return hipGetLastError();
}

hipError_t launch_union_schedule(const float *logits, const float *thresh, const int32_t *sizes,
                                 const int32_t *offsets, uint32_t *keep_masks, int32_t *n_ranges, int32_t *n_keys,
                                 DecodePlan plan, int U, int B, int G, int H, int C, hipStream_t s)
{
    SelectOpts opt{};
    opt.union_rows = 1;
    opt.B = B * G;
    opt.G = G;
    return launch_select(logits, nullptr, nullptr, false, thresh, sizes, offsets, keep_masks, nullptr, n_ranges,
                         n_keys, plan, true, U, opt, seq_groups_for(B * G) * H, H, 1, C, s);
}

hipError_t launch_ranges_to_rec(const int32_t *ranges, const int32_t *n_ranges, DecodePlan plan, int rows,
                                int range_cap, hipStream_t s)
{
    hipLaunchKernelGGL(ranges_to_rec_kernel, dim3(rows), dim3(256), 0, s, ranges, n_ranges, plan, range_cap);
    return hipGetLastError();
}

hipError_t launch_schedule(DecodePlan plan, int rows, int U, hipStream_t s)
{
    const size_t smem = (size_t)chunk_cap_for(plan.L) * 8 + 16;
    static bool attr_set = false;   // one GPU per process in this build
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(schedule_kernel),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, SELECT_MAX_C * 8 + 16);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    hipLaunchKernelGGL(schedule_kernel, dim3(rows), dim3(256), smem, s, plan, rows, U, user_chunks_for(U));
    return hipGetLastError();
}

}  // namespace sq
