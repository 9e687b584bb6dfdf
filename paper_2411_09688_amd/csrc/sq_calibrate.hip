// Threshold calibration (Appendix C): per head, the threshold T for which the rule S_i > T retrieves a target number
// of keys over a set of calibration queries.  The cluster scores S_i = exp(x_i - m) / D (Eq. 1, fp32) of all
// calibration queries of a head are pooled, each weighing N_i keys; s_k is the lowest score that still has to be
// kept so that the pooled weight of the scores >= s_k reaches the target, and T is the geometric mean of s_k and the
// highest score strictly below it (s_k / 2 if there is none or it is 0).
//
// No sort: for non-negative floats the bit pattern orders like the value, and the pooled weight W(t) of the scores
// >= t falls as t rises, so s_k -- the largest t with W(t) >= target -- is found by a radix selection over the 31
// value bits, four passes over the pooled scores (they stay in the last-level cache between passes).
#include "sq_common.hpp"
#include "sq_internal.hpp"

namespace sq {

// S[h, b * Lq + t, i] = exp(x - m) / D of row (b, h, t), 0 for clusters without keys.
__global__ __launch_bounds__(256) void calib_scores_kernel(const float *__restrict__ logits,
                                                           const float *__restrict__ row_max,
                                                           const float *__restrict__ denom,
                                                           const int32_t *__restrict__ sizes, float *__restrict__ S,
                                                           int B, int H, int Lq, int C)
{
    const int r = blockIdx.y;                                   // row of the [B, H, Lq] tensors
    const int b = r / (H * Lq), h = (r / Lq) % H, t = r % Lq;
    const int i = blockIdx.x * 256 + threadIdx.x;
    if (i >= C) return;
    const float s = sizes[(size_t)h * C + i] > 0 ? expf(logits[(size_t)r * C + i] - row_max[r]) / denom[r] : 0.0f;
    S[(((size_t)h * B + b) * Lq + t) * C + i] = s;
}

__global__ __launch_bounds__(1024) void calib_select_kernel(const float *__restrict__ S,
                                                            const int32_t *__restrict__ sizes,
                                                            float *__restrict__ thresh, int n_rows, int C, int target)
{
    __shared__ int s_hist[256];
    __shared__ int s_part[16];
    __shared__ float s_fpart[16];
    __shared__ uint32_t s_prefix;
    __shared__ int s_above;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int h = blockIdx.x;
    const float *Sh = S + (size_t)h * n_rows * C;
    const int32_t *Nh = sizes + (size_t)h * C;

    // Everything the head's queries can retrieve: every score is >= 0.
    int acc = 0;
    for (int i = tid; i < C; i += 1024) acc += Nh[i];
    acc = wave_sum_i(acc);
    if (lane == 0) s_part[wave] = acc;
    if (tid == 0) {
        s_prefix = 0u;
        s_above = 0;
    }
    __syncthreads();
    int reachable = 0;
#pragma unroll
    for (int w = 0; w < 16; ++w) reachable += s_part[w];
    reachable *= n_rows;
    const int want = max(min(target, reachable), 1);           // a budget of 0 still keeps the best score

    // s_k = the largest t with W(t) >= want, W(t) = pooled weight of the scores >= t, found digit by digit from the
    // top of the 31 value bits (7 + 8 + 8 + 8): a histogram of pooled weight over the next digit of the scores that
    // share the digits fixed so far, then the highest digit at which the weight above it plus its own reaches the
    // budget.  A thread sums runs of equal digits in a register before it touches the histogram.
    for (int shift = 24; shift >= 0; shift -= 8) {
        for (int b = tid; b < 256; b += 1024) s_hist[b] = 0;
        __syncthreads();
        const uint32_t prefix = s_prefix;
        int run_bin = -1, run_sum = 0;
        for (int i = tid; i < C; i += 1024) {
            const int N = Nh[i];
            for (int r = 0; r < n_rows; ++r) {
                const uint32_t bits = __float_as_uint(Sh[(size_t)r * C + i]);
                if ((bits >> 8 >> shift) != prefix) continue;   // (two shifts: shift + 8 may be 32)
                const int bin = (int)((bits >> shift) & 255u);
                if (bin != run_bin) {
                    if (run_sum) atomicAdd(&s_hist[run_bin], run_sum);
                    run_bin = bin;
                    run_sum = 0;
                }
                run_sum += N;
            }
        }
        if (run_sum) atomicAdd(&s_hist[run_bin], run_sum);
        __syncthreads();
        if (tid == 0) {
            int above = s_above, bin = 255;
            while (bin > 0 && above + s_hist[bin] < want) above += s_hist[bin--];
            s_above = above;
            s_prefix = (prefix << 8) | (uint32_t)bin;
        }
        __syncthreads();
    }
    const float s_k = __uint_as_float(s_prefix);
    float below = -1.0f;
    for (int i = tid; i < C; i += 1024)
        for (int r = 0; r < n_rows; ++r) {
            const float s = Sh[(size_t)r * C + i];
            if (s < s_k) below = fmaxf(below, s);
        }
    below = wave_max(below);
    if (lane == 0) s_fpart[wave] = below;
    __syncthreads();
    if (tid == 0) {
#pragma unroll
        for (int w = 0; w < 16; ++w) below = fmaxf(below, s_fpart[w]);
        thresh[h] = below > 0.0f ? sqrtf(s_k) * sqrtf(below) : 0.5f * s_k;
    }
}

hipError_t launch_calibrate(const float *logits, const float *row_max, const float *denom, const int32_t *sizes,
                            float *S, float *thresh, int target, int B, int H, int Lq, int C, hipStream_t s)
{
    hipLaunchKernelGGL(calib_scores_kernel, dim3((C + 255) / 256, B * H * Lq), dim3(256), 0, s, logits, row_max, denom,
                       sizes, S, B, H, Lq, C);
    hipLaunchKernelGGL(calib_select_kernel, dim3(H), dim3(1024), 0, s, (const float *)S, sizes, thresh, B * Lq, C,
                       target);
    return hipGetLastError();
}

}  // namespace sq
