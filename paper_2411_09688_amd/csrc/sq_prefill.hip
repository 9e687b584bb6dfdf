// Prefill-time sparse attention (Section 4.2) with per-query selection: every query token attends to the
// keys of the clusters set in its own keep mask, plus the (causal) user keys, one softmax over the union.
//
// Layout of the computation (FlashAttention-2 style: grid over heads x query blocks, loop over key blocks,
// online softmax), written for CDNA4 matrix cores:
//   * a workgroup = 4 waves x 16 queries, two workgroups per compute unit (shared-set form: 8 waves, one
//     workgroup); all waves walk the same 64-key blocks, whose K and V tiles are staged row-major in LDS once per
//     workgroup (two LDS buffers; the next block's rows go from global memory straight into the other buffer with the
//     load-to-LDS instruction, issued a piece at a time behind the steps of the current block's score products);
//   * scores are computed TRANSPOSED, S^T = K Q^T, with 16x16x32 fp16 MFMA tiles (A = 16 keys, B = 16
//     queries).  In the accumulator layout a lane then owns ONE query column for the whole kernel (and four
//     keys per tile), so the running maximum, the running sum and the rescaling of the output are per-lane
//     scalars, and P^T is repacked into the B operand of the next product in registers, with no
//     cross-lane traffic;
//   * O^T = V^T P^T uses A = V^T tiles read from the row-major V tile with the transposing LDS read
//     (ds_read_b64_tr_b16), so V needs no transposition on its way into LDS;
//   * the per-query keep masks are applied per (query, key): a small pre-kernel expands the cluster offsets
//     into a key -> cluster map, each key block brings, for every query of the workgroup, the window of mask
//     bits that covers its clusters, the bit of a (query, key) pair is spread over a word with one signed
//     bit-field extract and blended into the score with one bit-select, and a wave skips the products of a
//     block none of its queries kept.  The mask arithmetic is issued behind the S^T products, in the same
//     straight-line block, so the vector ALU works while the matrix cores do;
//   * the masked form exists twice: a kernel that walks every key block, and one that first lists, per workgroup, the
//     blocks in which at least one of its queries kept a cluster and walks only those.  A counting launch decides which
//     of the two does the work (see PF_LIST_MIN_SHARE).
// The user block is causal when causal_user is set (query t sees user keys 0..t); the fixed context is
// always fully visible.
//
// SHARED variant (selection on averaged scores, Appendix D "Prefill Stage"): all query tokens of a (sequence,
// head) attend to ONE kept set.  The kept ranges are expanded into a list of key rows (the key-index tensor of
// Section 4.2); the kernel walks that list 64 keys at a time, gathering K and V rows by index (the indices of
// the block after next travel in registers ahead of the rows), with no per-query masks: only the tail of the
// last block and the causal user keys are masked, so every executed tile is useful work.
#include <type_traits>

#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

constexpr int PF_BN = 64;                 // keys per block
// K and V tiles in LDS: unpadded rows of 256 B, filled straight from global memory by the load-to-LDS instruction
// (global_load_lds_dwordx4: the 64 lanes of a wave write 64 x 16 contiguous bytes = four whole rows), and swizzled
// instead of padded so that the operand reads stay free of bank conflicts: the 16-byte chunk c of row r sits at slot
// c ^ swz(r).  The swizzle is applied on the global side (lane = slot: it fetches chunk slot ^ swz(r)).
//   K (16-byte reads, 16 rows at one chunk index per group of lanes): swz = r % 16 -- the 16 rows land in 16 slots.
//   V (transposing 8-byte reads, 16 rows x 32 bytes per instruction): swz = 2 * (r % 8) -- a pair of chunks stays
//   adjacent and the 8 rows of half a wave land in 8 different pairs.
__device__ __forceinline__ int pf_k_swz(int row) { return row & 15; }
__device__ __forceinline__ int pf_v_swz(int row) { return (row & 7) << 1; }

// key -> cluster id map of every head (clusters are contiguous key ranges).  Keys that no cluster covers (before
// offsets[0] or from offsets[C] on) get the "no cluster" id 0x7fffffff, which no query keeps.
__global__ __launch_bounds__(256) void key_cluster_kernel(const int32_t *__restrict__ offsets, int32_t *__restrict__ cid,
                                                          int C, int L)
{
    const int h = blockIdx.y;
    const int32_t *off = offsets + (size_t)h * (C + 1);
    if (blockIdx.x == 0) {
        const int head = max(0, min(L, off[0])), tail = max(0, min(L, off[C]));
        for (int j = threadIdx.x; j < head; j += 256) cid[(size_t)h * L + j] = 0x7fffffff;
        for (int j = tail + threadIdx.x; j < L; j += 256) cid[(size_t)h * L + j] = 0x7fffffff;
    }
    for (int c = blockIdx.x * 4 + (threadIdx.x >> 6); c < C; c += gridDim.x * 4) {
        const int a = max(0, off[c]), b = min(L, off[c + 1]);
        for (int j = a + (threadIdx.x & 63); j < b; j += 64) cid[(size_t)h * L + j] = c;
    }
}

// Per 64-key block of the fixed context: the cluster of its first key, how many cluster ids it spans, and
// whether that span fits the 31-bit window of mask bits staged per query (it always does unless the block
// crosses a long run of empty clusters).  blk_info[h, blk] = first | span << 16 | wide << 31.
__global__ __launch_bounds__(256) void block_info_kernel(const int32_t *__restrict__ cid, int32_t *__restrict__ blk_info,
                                                         int C, int L, int nblk)
{
    const int h = blockIdx.y;
    const int blk = blockIdx.x * 256 + threadIdx.x;
    if (h == 0 && blk == 0)                              // the count of skippable (workgroup, block) pairs, behind the table
        *reinterpret_cast<unsigned long long *>(blk_info + prefill_skip_count_at((int)gridDim.y, L)) = 0ull;
    if (blk >= nblk) return;
    const int first = max(0, min(cid[(size_t)h * L + blk * PF_BN], C - 1));
    const int last = max(first, min(cid[(size_t)h * L + min(L, (blk + 1) * PF_BN) - 1], C - 1));
    const int span = last - first;
    blk_info[(size_t)h * nblk + blk] = first | (min(span, 30) << 16) | (span >= 31 ? (int)0x80000000 : 0);
}

// Kept ranges of every (sequence, head) row -> list of key rows: record (first key, count, keys before) writes
// key_idx[row, before + j] = first + j, clamped into the tensor.  One wave per record at a time, the records of a row
// dealt over the gridDim.y workgroups of the row.
constexpr int EXPAND_SLICES = 16;         // workgroups per row
__global__ __launch_bounds__(256) void expand_ranges_kernel(DecodePlan plan, int32_t *__restrict__ key_idx, int L)
{
    const size_t row = blockIdx.x;
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int nrec = min(plan.hdr[row].x, plan.rec_cap);
    int32_t *dst = key_idx + row * (size_t)L;
    for (int r = (int)blockIdx.y * 4 + wave; r < nrec; r += 4 * (int)gridDim.y) {
        const int4 rc = plan.rec[row * plan.rec_cap + r];
        for (int j = lane; j < rc.y && rc.z + j < L; j += 64) dst[rc.z + j] = max(0, min(rc.x + j, L - 1));
    }
}

// Masked form, two kernels for the same work.  The plain one walks every fixed-context block (a wave still skips the
// products of a block none of its queries kept).  The listed one first builds, in LDS, the ordered list of the blocks in
// which at least one query of the workgroup kept a cluster and walks only those (Section 4.2: the work follows the kept
// set, not the context length): blocks nobody kept are neither fetched nor staged nor waited for at a barrier.  Walking
// through the list costs about 6% when nothing can be skipped (883 against 833 us at 32 heads x 1024 tokens x 32K keys,
// 1/8 kept per query), so a counting launch in front adds up the (workgroup, block) pairs that can be skipped; both
// kernels are then launched and each returns at once unless the count picks it (listed: an eighth of the pairs or more).
constexpr int PF_LIST_CAP = 4096;         // blocks (256K keys); longer contexts take the plain kernel
constexpr int PF_UMASK_WORDS = SELECT_MAX_C / 32;
constexpr size_t PF_LIST_BYTES = PF_UMASK_WORDS * 4 + PF_LIST_CAP * 2;
constexpr int PF_LIST_MIN_SHARE = 8;      // listed kernel iff skippable pairs * 8 >= all pairs

// s_um[0..W) |= keep masks of queries q0 .. q0+bm-1 (those below Lq) of query rows row0...; s_um zeroed by the caller,
// barrier after it by the caller.  A mask word of eight queries per item: eight independent loads, one LDS atomic.
__device__ __forceinline__ void pf_union_mask(uint32_t *s_um, const uint32_t *__restrict__ keep_mask, size_t row0, int q0,
                                              int bm, int Lq, int W, int tid, int threads)
{
    for (int idx = tid; idx < (bm / 8) * W; idx += threads) {
        const int g = idx / W, w = idx - g * W;
        uint32_t acc = 0u;
#pragma unroll
        for (int k = 0; k < 8; ++k)
            if (q0 + g * 8 + k < Lq) acc |= keep_mask[(row0 + q0 + g * 8 + k) * W + w];
        if (acc) atomicOr(&s_um[w], acc);
    }
}

// Does a workgroup whose queries' masks OR to s_um need the block with table entry bi?  (A block that spans more
// cluster ids than the staged window is not decided here: needed.)
__device__ __forceinline__ bool pf_block_needed(int bi, const uint32_t *s_um, int W)
{
    if (bi < 0) return true;
    const int first = bi & 0xffff, w0 = first >> 5;
    const unsigned long long two = ((unsigned long long)(w0 + 1 < W ? s_um[w0 + 1] : 0u) << 32) | s_um[w0];
    const uint32_t present = (2u << ((bi >> 16) & 31)) - 1u;   // local clusters that occur in the block
    return ((uint32_t)(two >> (first & 31)) & present) != 0u;
}

// The counting launch: one workgroup per query block of the masked kernels, *skip_count += blocks it can skip.
__global__ __launch_bounds__(256) void prefill_need_kernel(const uint32_t *__restrict__ keep_mask,
                                                           const int32_t *__restrict__ blk_info,
                                                           unsigned long long *__restrict__ skip_count, int B, int H,
                                                           int L, int C, int Lq, int bm)
{
    __shared__ uint32_t s_um[PF_UMASK_WORDS];
    __shared__ int s_cnt;
    const int tid = threadIdx.x;
    const int nqb = (Lq + bm - 1) / bm, unit = blockIdx.x;
    const int h = unit / (nqb * B), b = (unit / nqb) % B, q0 = (unit % nqb) * bm;
    const int W = (C + 31) >> 5, nblk = (L + PF_BN - 1) / PF_BN;
    const size_t row0 = ((size_t)b * H + h) * Lq;
    for (int w = tid; w < W; w += 256) s_um[w] = 0u;
    if (tid == 0) s_cnt = 0;
    __syncthreads();
    pf_union_mask(s_um, keep_mask, row0, q0, bm, Lq, W, tid, 256);
    __syncthreads();
    int skip = 0;
    for (int bb = tid; bb < nblk; bb += 256) skip += pf_block_needed(blk_info[(size_t)h * nblk + bb], s_um, W) ? 0 : 1;
    for (int o = 32; o; o >>= 1) skip += __shfl_xor(skip, o);
    if ((tid & 63) == 0 && skip) atomicAdd(&s_cnt, skip);
    __syncthreads();
    if (tid == 0 && s_cnt) atomicAdd(skip_count, (unsigned long long)s_cnt);
}

constexpr int PF_QT = 1;                  // 16-query tiles per wave
// Waves per workgroup (all walk the same staged key blocks).  Measured at the 32-head, 1024-token shape: the masked
// form is fastest with 4 (1.10 ms against 1.17 with 8: the two workgroups of a compute unit cover each other's
// barriers), the shared-set form with 8 (155 us against 171: half the global->LDS staging per product).
constexpr int pf_waves(bool shared) { return shared ? 8 : 4; }
constexpr int pf_bm(bool shared) { return 16 * PF_QT * pf_waves(shared); }   // queries per workgroup
constexpr int PF_BM_MAX = pf_bm(true);

struct PfStage {                          // one LDS buffer of a key block
    _Float16 K[PF_BN * D];
    _Float16 V[PF_BN * D];
    int cid[PF_BN];                       // cluster of each key (0x7fffffff past the end)
    int sh[PF_BN];                        // bit of the key's cluster in the staged window: cluster - first cluster of
                                          // the block (31, a bit that is never set, for keys past the end)
    uint32_t qbits[PF_BM_MAX];            // per query: mask bits of clusters first .. first+30, bit 31 clear
};

// (mask & a) | (~mask & b) on the bit patterns of floats: one v_bfi_b32.
__device__ __forceinline__ float select_bits(uint32_t mask, float a, float b)
{
    return __builtin_bit_cast(float, (mask & __builtin_bit_cast(uint32_t, a)) | (~mask & __builtin_bit_cast(uint32_t, b)));
}

// SHARED: key_cid is the key-row list [B*H, L] and blk_info the per-row (records, kept keys) headers; keep_mask is
// not used.
template <bool SHARED, bool LISTED>
__global__ __launch_bounds__(64 * pf_waves(SHARED), 8 / pf_waves(SHARED)) void prefill_attn_kernel(
    const _Float16 *__restrict__ q, const _Float16 *__restrict__ Kf, const _Float16 *__restrict__ Vf,
    const _Float16 *__restrict__ Ku, const _Float16 *__restrict__ Vu, const uint32_t *__restrict__ keep_mask,
    const int32_t *__restrict__ key_cid, const int32_t *__restrict__ blk_info, _Float16 *__restrict__ out,
    float *__restrict__ lse, int B, int H, int L, int C, int Lq, int U, int causal_user, float sm_scale)
{
    constexpr int QT = PF_QT, BM = pf_bm(SHARED);
    constexpr int PF_THREADS = 64 * pf_waves(SHARED);
    constexpr int PF_RP = PF_THREADS / 16;    // rows of a key block the workgroup moves per pass (16 lanes per row)
    constexpr int PF_NP = PF_BN / PF_RP;      // passes per block
    extern __shared__ __align__(16) unsigned char smem[];
    PfStage *stage = reinterpret_cast<PfStage *>(smem);   // [2]

    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int col = lane & 15, kg = lane >> 4;
    // Workgroup -> (head, sequence, query block).  Workgroups are dealt to the 8 XCDs round-robin by their
    // linear id; units that share a head (and so stream the same K/V) are made to land on the same XCD, so
    // one L2 fetches a head's keys once for all of its query blocks.
    const int nqb = (Lq + BM - 1) / BM;
    const int per_xcd = gridDim.x >> 3;                   // grid is a multiple of 8
    const int unit = (blockIdx.x & 7) * per_xcd + (blockIdx.x >> 3);
    if (unit >= nqb * B * H) return;
    if constexpr (!SHARED) {
        // Which of the two masked kernels does the work: the listed one iff enough (workgroup, block) pairs can be skipped.
        const int nblk_all = (L + PF_BN - 1) / PF_BN;
        const unsigned long long skip = *reinterpret_cast<const unsigned long long *>(blk_info + prefill_skip_count_at(H, L));
        const bool by_list = nblk_all <= PF_LIST_CAP && skip > 0ull &&
                             skip * PF_LIST_MIN_SHARE >= (unsigned long long)(nqb * B * H) * (unsigned long long)nblk_all;
        if (by_list != LISTED) return;
    }
    const int h = unit / (nqb * B), b = (unit / nqb) % B;
    const int q0 = (unit % nqb) * BM;                     // first query of the workgroup
    const int W = (C + 31) >> 5;
    const size_t row0 = ((size_t)b * H + h) * Lq;         // query-row index of query 0 of this (b, h)
    const float c2 = sm_scale * 1.44269504088896341f;     // exp(sm_scale * s) = exp2(c2 * s)

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

    float m_run[QT], l_run[QT];                           // running max (raw logit units) and sum per query column
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
    // keys of the fixed context this (sequence, head) walks: all of them, or the kept ones through the row list
    const int n_fixed = SHARED ? min(blk_info[2 * ((size_t)b * H + h) + 1], L) : L;
    const int32_t *idx_bh = key_cid + ((size_t)b * H + h) * (size_t)L;   // SHARED only
    const int nblk_fixed = (n_fixed + PF_BN - 1) / PF_BN;
    // Causal user block: queries of this workgroup see user keys 0 .. min(U, q0 + BM) - 1 at most.
    const int u_vis = causal_user ? min(U, q0 + BM) : U;
    const int nblk = nblk_fixed + (u_vis + PF_BN - 1) / PF_BN;
    const int32_t *binfo = blk_info + (size_t)h * ((L + PF_BN - 1) / PF_BN);
    const int32_t *cid_h = key_cid + (size_t)h * L;
    // Mask row of the query this thread stages bits for (threads 0..BM-1).
    const int my_q = q0 + tid;
    const uint32_t *my_mrow = keep_mask + (row0 + min(my_q, Lq - 1)) * W;

    // Registers that carry the next block's ids and mask words from global memory to LDS (its K and V rows go to LDS
    // directly).
    int pcid = 0, pinfo = 0;
    uint32_t pw_lo = 0u, pw_hi = 0u;
    // This thread's pieces of a 64-key block: piece i = key i*PF_RP + tid/16 (rows of 256 B), LDS slot tid%16 of that
    // row, i.e. the 16-byte chunk (tid%16) ^ swz(row) of the row in memory; row % 16 = (tid/16) % 16 for every piece.
    const uint32_t r_off = (uint32_t)(tid >> 4) * 256u;
    const uint32_t k_ch = (uint32_t)((tid & 15) ^ pf_k_swz(tid >> 4)) * 16u, v_ch = (uint32_t)((tid & 15) ^ pf_v_swz(tid >> 4)) * 16u;
    const int wave_u = __builtin_amdgcn_readfirstlane(wave);
    // SHARED: rows of this thread's pieces (keys i*16 + tid/16) of a fixed block; the indices of block b+2 are
    // loaded while block b is computed and used when block b+1's rows are fetched.
    int ik_n[PF_NP] = {}, ik_c[PF_NP] = {};
    auto fetch_idx = [&](int blk) {
        if (!SHARED || blk >= nblk_fixed) return;
        const int j0 = blk * PF_BN, last = n_fixed - 1;
#pragma unroll
        for (int i = 0; i < PF_NP; ++i) ik_n[i] = idx_bh[min(j0 + i * PF_RP + (tid >> 4), last)];
    };
    // The loads of the next block are issued in PF_NP pieces (one K and one V row chunk per thread each).  `aim` points
    // them at block `blk` and issues the block's small loads (ids, mask words); `fetch_piece` is then called from inside
    // the block body, one piece behind each step of the S^T products, so that the four waves of a workgroup do not queue
    // at the address unit all at once while the matrix cores idle.
    const char *nKb = reinterpret_cast<const char *>(Kfh), *nVb = reinterpret_cast<const char *>(Vfh);   // uniform bases
    uint32_t noff[PF_NP];                 // per-thread byte offsets of the pieces' rows, the same for K and V
#pragma unroll
    for (int i = 0; i < PF_NP; ++i) noff[i] = 0u;
    auto aim = [&](int blk) {
        const bool user = blk >= nblk_fixed;
        const int j0 = (user ? blk - nblk_fixed : blk) * PF_BN;
        const int nkeys = user ? U : L;
        if (SHARED && !user) {            // gathered rows (slots past the kept keys repeat the last kept row)
            nKb = reinterpret_cast<const char *>(Kfh);
            nVb = reinterpret_cast<const char *>(Vfh);
#pragma unroll
            for (int i = 0; i < PF_NP; ++i) noff[i] = (uint32_t)ik_c[i] * 256u;
            return;
        }
        nKb = reinterpret_cast<const char *>(user ? Kuh : Kfh) + (size_t)j0 * 256;
        nVb = reinterpret_cast<const char *>(user ? Vuh : Vfh) + (size_t)j0 * 256;
        if (j0 + PF_BN <= nkeys) {        // full block
#pragma unroll
            for (int i = 0; i < PF_NP; ++i) noff[i] = r_off + (uint32_t)i * (PF_RP * 256u);
        } else {                          // last block of a tensor: rows past the end re-read the last row
            const int last = nkeys - 1 - j0;
#pragma unroll
            for (int i = 0; i < PF_NP; ++i)
                noff[i] = (uint32_t)min(i * PF_RP + (tid >> 4), last) * 256u;
        }
        if (!user && !SHARED) {
            pinfo = binfo[blk];
            if (tid < PF_BN) pcid = j0 + tid < L ? cid_h[j0 + tid] : 0x7fffffff;
            if (tid < BM) {
                const int w0 = (pinfo & 0xffff) >> 5;
                pw_lo = my_mrow[w0];
                pw_hi = w0 + 1 < W ? my_mrow[w0 + 1] : 0u;
            }
        }
    };
    typedef __attribute__((address_space(1))) const void *gptr_t;
    typedef __attribute__((address_space(3))) void *lptr_t;
    auto fetch_piece = [&](int i, PfStage &dst) {   // i: compile-time constant at every call
        // this wave's four rows of the piece: 1 KB of the tile, lane l at byte 16 l
        _Float16 *lk = dst.K + (i * PF_RP + wave_u * 4) * D, *lv = dst.V + (i * PF_RP + wave_u * 4) * D;
        if constexpr (SHARED) {
            __builtin_amdgcn_global_load_lds((gptr_t)(nKb + (noff[i] + k_ch)), (lptr_t)lk, 16, 0, 0);
            __builtin_amdgcn_global_load_lds((gptr_t)(nVb + (noff[i] + v_ch)), (lptr_t)lv, 16, 0, 0);
        } else {
            // Written as instructions: through the builtin the compiler makes the first V read of the CURRENT buffer wait
            // for these loads into the OTHER buffer (it cannot tell the two apart).  Masked form at 32 heads x 1024 tokens x
            // 32K keys: 1042 us with the builtin, 825 us this way; the shared-set form, whose V reads come later, is faster
            // with the builtin (133 against 147 us: the asm statements pin the compiler's schedule).
            const uint32_t ak = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lptr_t)lk);
            const uint32_t av = __builtin_amdgcn_readfirstlane((uint32_t)(size_t)(lptr_t)lv);
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(ak), "v"(noff[i] + k_ch), "s"(nKb) : "m0");
            asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2" ::"s"(av), "v"(noff[i] + v_ch), "s"(nVb) : "m0");
        }
    };
    auto fetch_rest = [&](int from, PfStage &dst) {
#pragma unroll
        for (int i = 0; i < PF_NP; ++i)
            if (i >= from) fetch_piece(i, dst);
    };
    // The loads to LDS are not tracked by the compiler: before the barrier that publishes a block, every wave waits
    // for all of its outstanding memory operations itself.
    auto loads_landed = [&]() { __builtin_amdgcn_s_waitcnt(0x0f70); };   // vmcnt(0)
    auto commit = [&](int blk, PfStage &st) {   // registers -> LDS (ids, mask bits)
        const bool user = blk >= nblk_fixed;
        if (!user && !SHARED) {
            const int first = pinfo & 0xffff;
            if (tid < PF_BN) {
                st.cid[tid] = pcid;
                st.sh[tid] = (unsigned)(pcid - first) >= 31u ? 31 : pcid - first;   // (no cluster, or outside the window: bit 31 is never set)
            }
            if (tid < BM) {
                const unsigned long long two = ((unsigned long long)pw_hi << 32) | pw_lo;
                st.qbits[tid] = my_q < Lq ? ((uint32_t)(two >> (first & 31)) & 0x7fffffffu) : 0u;
            }
        }
    };

    auto take_idx = [&]() {
#pragma unroll
        for (int i = 0; i < PF_NP; ++i) ik_c[i] = ik_n[i];
    };
    // ---- listed form: the blocks this workgroup has to walk, in order ------------------------------------------------
    // s_um = OR of the keep masks of the workgroup's queries; s_list = the fixed blocks it needs.
    uint32_t *s_um = reinterpret_cast<uint32_t *>(smem + 2 * sizeof(PfStage));
    uint16_t *s_list = reinterpret_cast<uint16_t *>(s_um + PF_UMASK_WORDS);
    int n_list = nblk_fixed;
    if constexpr (LISTED) {
        __shared__ int s_wc[PF_THREADS / 64];
        for (int w = tid; w < W; w += PF_THREADS) s_um[w] = 0u;
        __syncthreads();
        pf_union_mask(s_um, keep_mask, row0, q0, BM, Lq, W, tid, PF_THREADS);
        __syncthreads();
        int base = 0;
        for (int b0 = 0; b0 < nblk_fixed; b0 += PF_THREADS) {   // in order: a ballot per wave, the waves' counts in LDS
            const int bb = b0 + tid;
            const bool need = bb < nblk_fixed && pf_block_needed(binfo[bb], s_um, W);
            const unsigned long long bal = __ballot(need);
            if (lane == 0) s_wc[wave] = __popcll(bal);
            __syncthreads();
            int before = 0, total = 0;
#pragma unroll
            for (int w = 0; w < PF_THREADS / 64; ++w) {
                if (w < wave) before += s_wc[w];
                total += s_wc[w];
            }
            if (need)
                s_list[base + before + __builtin_amdgcn_mbcnt_hi((uint32_t)(bal >> 32), __builtin_amdgcn_mbcnt_lo((uint32_t)bal, 0))] = (uint16_t)bb;
            base += total;
            __syncthreads();
        }
        n_list = __builtin_amdgcn_readfirstlane(base);
    }
    // The blocks in walking order: the (listed) fixed blocks, then the user blocks.
    const int n_seq = n_list + (nblk - nblk_fixed);
    // (the same in every lane: made scalar, or every address and branch that hangs on it would be done per lane)
    auto blk_at = [&](int i) {
        return i < n_list ? (LISTED ? __builtin_amdgcn_readfirstlane((int)s_list[i]) : i) : nblk_fixed + (i - n_list);
    };

    int info_cur = 0;
    if (n_seq > 0) {                                      // (no kept key and no user key: nothing to stage)
        fetch_idx(0);
        take_idx();
        fetch_idx(1);
        aim(blk_at(0));
        fetch_rest(0, stage[0]);
        info_cur = pinfo;
        commit(blk_at(0), stage[0]);
    }
    loads_landed();
    __syncthreads();

    // The key blocks, alternating between the two LDS buffers.  The shared-set form runs the loop unrolled over the
    // buffers, so that which buffer is read and which is filled are compile-time constants: the compiler can then tell
    // them apart (no wait for the loads to LDS in front of the V reads) and the swizzled operand addresses are
    // loop-invariant -- 133 -> 117 us at 32 heads x 1024 tokens, 1/8 of 32K keys kept.  The masked form is faster as a
    // plain loop (823 us against 896-929 us unrolled: twice the code for a body that already holds five variants of
    // the block), so the body is kept in a file of its own and included in each loop.
    if constexpr (SHARED) {
        auto one_block = [&](int blk, auto par) {
            PfStage &st = stage[par];
            PfStage &st_next = stage[par ^ 1];
#define PF_USER(b) ((b) >= nblk_fixed)
#define PF_NEXT_STAGE st_next
#define PF_HAS_NEXT (blk + 1 < nblk)
#define PF_NEXT_BLK (blk + 1)
#define PF_FETCH_IDX_AHEAD if (blk + 2 < nblk) fetch_idx(blk + 2)
#define PF_OPERANDS_AHEAD 0
#include "sq_prefill_block.inc"
#undef PF_OPERANDS_AHEAD
#undef PF_FETCH_IDX_AHEAD
#undef PF_NEXT_BLK
#undef PF_HAS_NEXT
#undef PF_NEXT_STAGE
#undef PF_USER
        };
        for (int blk = 0; blk < nblk; blk += 2) {
            one_block(blk, std::integral_constant<int, 0>{});
            if (blk + 1 < nblk) one_block(blk + 1, std::integral_constant<int, 1>{});
        }
    } else if constexpr (!LISTED) {
        for (int blk = 0; blk < nblk; ++blk) {
            PfStage &st = stage[blk & 1];
#define PF_USER(b) ((b) >= nblk_fixed)
#define PF_NEXT_STAGE stage[(blk + 1) & 1]
#define PF_HAS_NEXT (blk + 1 < nblk)
#define PF_NEXT_BLK (blk + 1)
#define PF_FETCH_IDX_AHEAD (void)0
#define PF_OPERANDS_AHEAD 3
#include "sq_prefill_block.inc"
#undef PF_OPERANDS_AHEAD
#undef PF_FETCH_IDX_AHEAD
#undef PF_NEXT_BLK
#undef PF_HAS_NEXT
#undef PF_NEXT_STAGE
#undef PF_USER
        }
    } else {
        // Two loops, fixed blocks then user blocks: each then holds only its own forms of the block, and what only the
        // other needs (base pointers, lengths) is not kept in registers through it.
        // (The list is read two blocks ahead and made scalar only after the block: the entry heads the address chain
        // of the next block's loads, and nothing in front of the block's own work waits for it.)
        int blk_cur = n_list > 0 ? blk_at(0) : 0, blk_ahead = n_seq > 1 ? blk_at(1) : 0;
        for (int it = 0; it < n_list; ++it) {
            const int blk = blk_cur, blk_nx = blk_ahead;
            int ahead_v = 0;
            if (it + 2 < n_seq) ahead_v = it + 2 < n_list ? (int)s_list[it + 2] : nblk_fixed + (it + 2 - n_list);
            PfStage &st = stage[it & 1];
#define PF_USER(b) false
#define PF_NEXT_STAGE stage[(it + 1) & 1]
#define PF_HAS_NEXT (it + 1 < n_seq)
#define PF_NEXT_BLK blk_nx
#define PF_FETCH_IDX_AHEAD (void)0
#define PF_OPERANDS_AHEAD 3
#include "sq_prefill_block.inc"
#undef PF_OPERANDS_AHEAD
#undef PF_FETCH_IDX_AHEAD
#undef PF_NEXT_BLK
#undef PF_HAS_NEXT
#undef PF_NEXT_STAGE
#undef PF_USER
            blk_cur = blk_nx;
            blk_ahead = __builtin_amdgcn_readfirstlane(ahead_v);
        }
        for (int it = n_list; it < n_seq; ++it) {
            const int blk = nblk_fixed + (it - n_list);
            PfStage &st = stage[it & 1];
#define PF_USER(b) true
#define PF_NEXT_STAGE stage[(it + 1) & 1]
#define PF_HAS_NEXT (it + 1 < n_seq)
#define PF_NEXT_BLK (blk + 1)
#define PF_FETCH_IDX_AHEAD (void)0
#define PF_OPERANDS_AHEAD 3
#include "sq_prefill_block.inc"
#undef PF_OPERANDS_AHEAD
#undef PF_FETCH_IDX_AHEAD
#undef PF_NEXT_BLK
#undef PF_HAS_NEXT
#undef PF_NEXT_STAGE
#undef PF_USER
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
        if (lse && kg == 0) lse[row0 + nq[qt]] = empty ? SQ_NEG_INF : m_run[qt] * sm_scale + logf(lt);
    }
}

namespace {

// ev0 / ev1: profiling events recorded in front of / behind the launch (either may be null).
template <bool SHARED, bool LISTED>
hipError_t launch_prefill_kernel(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                                 const uint32_t *keep_mask, const int32_t *key_cid, const int32_t *blk_info, void *out,
                                 float *lse, const Shape &sh, hipStream_t s, hipEvent_t ev0, hipEvent_t ev1)
{
    const size_t smem = 2 * sizeof(PfStage) + (LISTED ? PF_LIST_BYTES : 0);
    static bool attr_set = false;   // one GPU per process in this build
    if (!attr_set) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(prefill_attn_kernel<SHARED, LISTED>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, (int)smem);
        if (e != hipSuccess) return e;
        attr_set = true;
    }
    constexpr int PF_BM = pf_bm(SHARED), PF_THREADS = 64 * pf_waves(SHARED);
    const int units = ((sh.Lq + PF_BM - 1) / PF_BM) * sh.H * sh.B;
    dim3 grid((units + 7) / 8 * 8);
    if (ev0 || ev1)
        hipExtLaunchKernelGGL((prefill_attn_kernel<SHARED, LISTED>), grid, dim3(PF_THREADS), (uint32_t)smem, s, ev0, ev1,
                              0, (const _Float16 *)q, (const _Float16 *)Kf, (const _Float16 *)Vf, (const _Float16 *)Ku,
                              (const _Float16 *)Vu, keep_mask, key_cid, blk_info, (_Float16 *)out, lse, sh.B, sh.H, sh.L,
                              sh.C, sh.Lq, sh.U, sh.causal_user, sh.sm_scale);
    else
        hipLaunchKernelGGL((prefill_attn_kernel<SHARED, LISTED>), grid, dim3(PF_THREADS), smem, s, (const _Float16 *)q,
                           (const _Float16 *)Kf, (const _Float16 *)Vf, (const _Float16 *)Ku, (const _Float16 *)Vu,
                           keep_mask, key_cid, blk_info, (_Float16 *)out, lse, sh.B, sh.H, sh.L, sh.C, sh.Lq, sh.U,
                           sh.causal_user, sh.sm_scale);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_prefill_attn(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                               const uint32_t *keep_mask, const int32_t *offsets, int32_t *key_cid, int32_t *blk_info,
                               void *out, float *lse, const Shape &sh, hipStream_t s)
{
    const int nblk = (sh.L + PF_BN - 1) / PF_BN;
    hipLaunchKernelGGL(key_cluster_kernel, dim3(64, sh.H), dim3(256), 0, s, offsets, key_cid, sh.C, sh.L);
    hipLaunchKernelGGL(block_info_kernel, dim3((nblk + 255) / 256, sh.H), dim3(256), 0, s, key_cid, blk_info, sh.C,
                       sh.L, nblk);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    profile_pair(&ev0, &ev1);                            // (the pair brackets both attention launches)
    const bool may_list = nblk <= PF_LIST_CAP;           // else the count stays 0 and the plain kernel does the work
    if (may_list) {
        constexpr int BM = pf_bm(false);
        const int units = ((sh.Lq + BM - 1) / BM) * sh.H * sh.B;
        hipLaunchKernelGGL(prefill_need_kernel, dim3(units), dim3(256), 0, s, keep_mask, blk_info,
                           reinterpret_cast<unsigned long long *>(blk_info + prefill_skip_count_at(sh.H, sh.L)), sh.B, sh.H,
                           sh.L, sh.C, sh.Lq, BM);
        e = hipGetLastError();
        if (e != hipSuccess) return e;
    }
    e = launch_prefill_kernel<false, false>(q, Kf, Vf, Ku, Vu, keep_mask, key_cid, blk_info, out, lse, sh, s, ev0,
                                            may_list ? nullptr : ev1);
    if (e != hipSuccess || !may_list) return e;
    return launch_prefill_kernel<false, true>(q, Kf, Vf, Ku, Vu, keep_mask, key_cid, blk_info, out, lse, sh, s, nullptr,
                                              ev1);
}

hipError_t launch_expand_ranges(DecodePlan plan, int32_t *idx, int rows, int L, hipStream_t s)
{
    hipLaunchKernelGGL(expand_ranges_kernel, dim3(rows, EXPAND_SLICES), dim3(256), 0, s, plan, idx, L);
    return hipGetLastError();
}

hipError_t launch_prefill_attn_shared(const void *q, const void *Kf, const void *Vf, const void *Ku, const void *Vu,
                                      DecodePlan plan, int32_t *key_idx, void *out, float *lse, const Shape &sh,
                                      hipStream_t s)
{
    hipLaunchKernelGGL(expand_ranges_kernel, dim3(sh.B * sh.H, EXPAND_SLICES), dim3(256), 0, s, plan, key_idx, sh.L);
    hipError_t e = hipGetLastError();
    if (e != hipSuccess) return e;
    hipEvent_t ev0 = nullptr, ev1 = nullptr;
    profile_pair(&ev0, &ev1);
    return launch_prefill_kernel<true, false>(q, Kf, Vf, Ku, Vu, nullptr, key_idx,
                                              reinterpret_cast<const int32_t *>(plan.hdr), out, lse, sh, s, ev0, ev1);
}

}  // namespace sq
