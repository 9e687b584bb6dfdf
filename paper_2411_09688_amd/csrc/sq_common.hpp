// Device-side helpers and compile-time constants shared by the gfx950 kernels.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace sq {

constexpr int D = 128;            // head dimension (fp16 row = 256 B = 16 lanes x 16 B)
constexpr int KPC = 128;          // keys per split-KV chunk = one workgroup of 4 waves x KPC/4 keys
constexpr int PART_STRIDE = 132;  // floats per partial result: m, l, pad, pad, o[128]

typedef _Float16 h8 __attribute__((ext_vector_type(8)));
typedef _Float16 h4 __attribute__((ext_vector_type(4)));
typedef _Float16 h2 __attribute__((ext_vector_type(2)));
typedef float f4 __attribute__((ext_vector_type(4)));
typedef float f16v __attribute__((ext_vector_type(16)));

#define SQ_NEG_INF (-__builtin_inff())

// Data-parallel-primitive move: lane i receives `v` from the lane selected by CTRL inside its
// row of 16 lanes (0x120 + n = rotate right by n).
template <int CTRL>
__device__ __forceinline__ float dpp_f(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, false));
}

// Sum / max over each group of 16 consecutive lanes; every lane of the group gets the result.
__device__ __forceinline__ float row16_sum(float v)
{
    v += dpp_f<0x128>(v);
    v += dpp_f<0x124>(v);
    v += dpp_f<0x122>(v);
    v += dpp_f<0x121>(v);
    return v;
}

// Sum / max over the four 16-lane groups (lanes l, l^16, l^32, l^48); all lanes get the result.  Done with the CDNA4
// row-swap moves, which stay in the vector ALU (a shuffle through ds_bpermute goes to the LDS unit and back):
// v_permlane16_swap exchanges the odd rows of its first operand with the even rows of its second, so with the same
// value in both, one operand ends up holding the even row of each row pair in both rows and the other the odd row;
// v_permlane32_swap does the same with the two halves of the wave.  Each lane then combines x[l] and x[l ^ 16]
// (then x[l ^ 32]) in one order or the other: sums and maxima are commutative, so the bits equal the shuffle form's.
// (written as instructions: this compiler's builtins for the two moves hand back the first result twice.  The
// waits around them cover the vector-ALU write -> swap and swap -> vector-ALU read distances.)
__device__ __forceinline__ void swap16(float v, float &a, float &b)
{
    a = v;
    b = v;
    asm volatile("s_nop 1\n\tv_permlane16_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ void swap32(float v, float &a, float &b)
{
    a = v;
    b = v;
    asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
}
__device__ __forceinline__ float cross16_sum(float v)
{
    float a, b;
    swap16(v, a, b);
    v = a + b;
    swap32(v, a, b);
    return a + b;
}
// The same over integers: bitwise OR (mask words) and sum (counts).
__device__ __forceinline__ uint32_t cross16_or(uint32_t v)
{
    float a, b;
    swap16(__builtin_bit_cast(float, v), a, b);
    v = __builtin_bit_cast(uint32_t, a) | __builtin_bit_cast(uint32_t, b);
    swap32(__builtin_bit_cast(float, v), a, b);
    return __builtin_bit_cast(uint32_t, a) | __builtin_bit_cast(uint32_t, b);
}
__device__ __forceinline__ int cross16_sum_i(int v)
{
    float a, b;
    swap16(__builtin_bit_cast(float, v), a, b);
    v = __builtin_bit_cast(int, a) + __builtin_bit_cast(int, b);
    swap32(__builtin_bit_cast(float, v), a, b);
    return __builtin_bit_cast(int, a) + __builtin_bit_cast(int, b);
}
__device__ __forceinline__ float cross16_max(float v)
{
    float a, b;
    swap16(v, a, b);
    v = fmaxf(a, b);
    swap32(v, a, b);
    return fmaxf(a, b);
}

// Sum over the 64 lanes of a wave as an xor butterfly (partners 1, 2, 4, 8, 16, 32 lanes away, in that order);
// every lane gets the same bits.  Entirely in the vector ALU: the first two steps are quad permutes; after them
// the four lanes of a quad agree, so mirroring a half row (lane i <-> 7 - i) pairs the same values as xor 4, and
// mirroring a row (i <-> 15 - i) the same as xor 8; the last two steps add the four row sums, read with
// v_readlane, as (r0 + r1) + (r2 + r3), which is what every row's butterfly computes.  Must be called with all
// 64 lanes active.  This is the one summation order of the library for sums over a wave.
__device__ __forceinline__ float wave_sum(float v)
{
    v += dpp_f<0xb1>(v);          // quad_perm [1,0,3,2]
    v += dpp_f<0x4e>(v);          // quad_perm [2,3,0,1]
    v += dpp_f<0x141>(v);         // row_half_mirror
    v += dpp_f<0x140>(v);         // row_mirror
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return (r0 + r1) + (r2 + r3);
}
__device__ __forceinline__ float wave_max(float v)
{
    v = fmaxf(v, dpp_f<0xb1>(v));
    v = fmaxf(v, dpp_f<0x4e>(v));
    v = fmaxf(v, dpp_f<0x141>(v));
    v = fmaxf(v, dpp_f<0x140>(v));
    const float r0 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 0));
    const float r1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 16));
    const float r2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 32));
    const float r3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), 48));
    return fmaxf(fmaxf(r0, r1), fmaxf(r2, r3));
}

// Integer data-parallel-primitive move for scans: lanes whose source lies outside their row of 16, and rows not
// named in ROW_MASK, receive 0.
template <int CTRL, int ROW_MASK = 0xf>
__device__ __forceinline__ int dpp_i0(int v)
{
    return __builtin_amdgcn_update_dpp(0, v, CTRL, ROW_MASK, 0xf, false);
}

// Inclusive prefix sum over the 64 lanes of a wave, entirely in the vector ALU: four shifted adds inside each
// row of 16 lanes (row_shr 1, 2, 4, 8), then lane 15 of a row is added to the following row (rows 1 and 3), then
// lane 31 to rows 2 and 3.  Must be called with all 64 lanes active.
__device__ __forceinline__ int wave_inclusive_scan(int v, int /*lane*/)
{
    v += dpp_i0<0x111>(v);
    v += dpp_i0<0x112>(v);
    v += dpp_i0<0x114>(v);
    v += dpp_i0<0x118>(v);
    v += dpp_i0<0x142, 0xa>(v);   // row_bcast:15
    v += dpp_i0<0x143, 0xc>(v);   // row_bcast:31
    return v;
}

// Sum over the wave (all 64 lanes active); every lane gets the result.
__device__ __forceinline__ int wave_sum_i(int v)
{
    return __builtin_amdgcn_readlane(wave_inclusive_scan(v, 0), 63);
}

// Sets bit `id` of a bit mask (LDS or global memory) for every lane with `keep`, called by a whole wave.  Candidates
// are listed in
// ascending id order and the children of a kept cluster are consecutive, so the kept lanes of a wave usually hold
// ids base + lane: their ballot, shifted by base % 32, IS the content of at most three mask words, written by three
// lanes -- instead of up to 32 lanes contending for one word.  Any other pattern falls back to one atomic per lane.
__device__ __forceinline__ void wave_mask_or(uint32_t *mask, int id, bool keep, int lane)
{
    const unsigned long long bal = __ballot(keep);
    if (bal == 0ull) return;                                  // wave-uniform
    const int first = __ffsll((long long)bal) - 1;
    const int base = __builtin_amdgcn_readlane(id, first) - first;
    if (__ballot(keep && id != base + lane) == 0ull) {
        const int s = base & 31, w0 = base >> 5;              // floor division: base may be negative (unkept low lanes)
        uint32_t v = 0u;
        if (lane == 0) v = (uint32_t)(bal << s);
        else if (lane == 1) v = s ? (uint32_t)(bal >> (32 - s)) : (uint32_t)(bal >> 32);
        else if (lane == 2) v = s ? (uint32_t)(bal >> (64 - s)) : 0u;
        if (lane < 3 && v != 0u) atomicOr(&mask[w0 + lane], v);   // (a word below 0 would hold no bit: v == 0)
    } else if (keep) {
        atomicOr(&mask[id >> 5], 1u << (id & 31));
    }
}

// fp32 dot product of two 8-element fp16 vectors (exact products, fp32 accumulation).
__device__ __forceinline__ float dot8(h8 a, h8 b, float acc)
{
    acc = __builtin_amdgcn_fdot2(h2{a[0], a[1]}, h2{b[0], b[1]}, acc, false);
    acc = __builtin_amdgcn_fdot2(h2{a[2], a[3]}, h2{b[2], b[3]}, acc, false);
    acc = __builtin_amdgcn_fdot2(h2{a[4], a[5]}, h2{b[4], b[5]}, acc, false);
    acc = __builtin_amdgcn_fdot2(h2{a[6], a[7]}, h2{b[6], b[7]}, acc, false);
    return acc;
}

// Rows of one chunk from its run-length records (position of a record's first key relative to the
// chunk, row of that key minus that position): slot t lies in the last record whose position is <= t
// and reads row t + delta.  Positions ascend and the first is <= 0.  Called by a whole workgroup of at
// least CH threads (contains a barrier); thread t < CH passes record t and gets s_rows[t] = its row
// clamped to [0, limit), or -1 for slots past `nvalid`.
template <int CH>
__device__ __forceinline__ void chunk_rows_from_records(int rec_pos, int rec_delta, int nrec, int nvalid, int limit,
                                                        int *s_pos, int *s_delta, int *s_rows, int tid)
{
    if (tid < CH) {
        s_pos[tid] = rec_pos;
        s_delta[tid] = rec_delta;
    }
    __syncthreads();
    if (tid < CH) {
        int lo = 0;
#pragma unroll
        for (int step = CH / 2; step > 0; step >>= 1)
            if (lo + step < nrec && s_pos[lo + step] <= tid) lo += step;
        const int r = tid + s_delta[lo];
        s_rows[tid] = tid < nvalid ? max(0, min(r, limit - 1)) : -1;   // malformed input stays in the tensor
    }
}

// Row statistics of Eq. 1 in max-subtracted form, computed by ONE wave for one query row:
//   m = max over clusters with N > 0 of x;  D = sum_i N_i * exp(x_i - m).
// The library has ONE summation order for D, chosen so that a 1024-thread workgroup can produce it in
// parallel: virtual thread v (0..1023) adds clusters v, v+1024, ... in ascending order; the 64 threads of
// each of the 16 groups are combined with an xor butterfly; the 16 group sums are added in ascending
// order.  This function walks the 16 groups one after the other, the selection kernel computes them
// side by side: the results are bit-identical.  Every implementation adds a term as ONE fused multiply-add
// (__fmaf_rn(N, e, sum); a thread's first term is then the rounded product), so the bits do not depend on what the
// compiler chooses to contract.
__device__ __forceinline__ void wave_row_stats(const float *x, const int32_t *N, int n, int lane, float &m_out,
                                               float &D_out)
{
    constexpr int UN = 8;
    float m = SQ_NEG_INF;
    for (int i0 = 0; i0 < n; i0 += 64 * UN) {
        float xv[UN];
        int nv[UN];
#pragma unroll
        for (int u = 0; u < UN; ++u) {
            const int i = i0 + u * 64 + lane;
            nv[u] = i < n ? N[i] : 0;
            xv[u] = i < n ? x[i] : 0.0f;
        }
#pragma unroll
        for (int u = 0; u < UN; ++u)
            if (nv[u] > 0) m = fmaxf(m, xv[u]);
    }
    m = wave_max(m);
    // One accumulator per group; a pass over 1024 clusters issues its 16 loads together.
    float loc[16];
#pragma unroll
    for (int g = 0; g < 16; ++g) loc[g] = 0.0f;
    for (int i0 = 0; i0 < n; i0 += 1024) {
        float xv[16];
        int nv[16];
#pragma unroll
        for (int g = 0; g < 16; ++g) {
            const int i = i0 + g * 64 + lane;
            nv[g] = i < n ? N[i] : 0;
            xv[g] = i < n ? x[i] : 0.0f;
        }
#pragma unroll
        for (int g = 0; g < 16; ++g)
            if (nv[g] > 0) loc[g] = __fmaf_rn((float)nv[g], expf(xv[g] - m), loc[g]);   // (fused, everywhere)
    }
    float Dsum = 0.0f;
#pragma unroll
    for (int g = 0; g < 16; ++g) Dsum += wave_sum(loc[g]);
    m_out = m;
    D_out = Dsum;
}

// A-operand of O^T += V^T P^T from a ROW-MAJOR V tile in LDS, with the CDNA4 transposing LDS read: within each
// group of 16 lanes, lane i receives element i % 4 of the four halves addressed by lanes i/4, 4 + i/4, 8 + i/4 and
// 12 + i/4.  With lane 4r + c of a group pointing at V[key0 + r][d0 + 4c .. +4], lane i gets V[key0 + 0..3][d0 + i]:
// four consecutive keys of one dimension, which is what the operand wants, and no transposed copy is ever written.
typedef __fp16 tr_h4 __attribute__((__vector_size__(4 * sizeof(__fp16))));
__device__ __forceinline__ h4 lds_read_tr16(const _Float16 *p)
{
    typedef __attribute__((address_space(3))) tr_h4 *lds_ptr_t;
    return __builtin_bit_cast(h4, __builtin_amdgcn_ds_read_tr16_b64_v4f16((lds_ptr_t)(p)));
}

}  // namespace sq
