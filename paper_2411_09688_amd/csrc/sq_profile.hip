// Measurement hook: every launch of the dominant kernel of a step (the split-KV partial kernel, which moves
// almost all of the bytes of a decode step; the attention kernel of a prefill step) carries a pair of HIP events
// attached to its dispatch on the launch stream (start and end time of the kernel), so a benchmark can read that
// kernel's duration from inside the process.  Off by default; not thread-safe by design.
#include <vector>

#include "../../include/squeezed_attention.h"
#include "sq_internal.hpp"

namespace sq {

namespace {
struct Profiler {
    bool on = false;
    std::vector<hipEvent_t> ev;   // 2 per launch
    size_t used = 0;
} g_prof;
}  // namespace

bool profile_pair(hipEvent_t *start, hipEvent_t *stop)
{
    if (!g_prof.on || g_prof.used + 2 > g_prof.ev.size()) return false;
    *start = g_prof.ev[g_prof.used];
    *stop = g_prof.ev[g_prof.used + 1];
    g_prof.used += 2;
    return true;
}

}  // namespace sq

namespace sq {
// Plain streaming read: every lane loads 16 bytes per step (non-temporal loads, what a kernel that reads its data
// once would use), grid-stride, and folds them into one word per workgroup so the loads cannot be dropped.  The
// ceiling an HBM-bound kernel can approach.
typedef unsigned u4v __attribute__((ext_vector_type(4)));

__global__ __launch_bounds__(256) void stream_read_kernel(const u4v *__restrict__ src, size_t n16,
                                                          unsigned *__restrict__ sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
    unsigned acc = 0;
    for (; i + 3 * stride < n16; i += 4 * stride) {
        const u4v a = __builtin_nontemporal_load(src + i), b = __builtin_nontemporal_load(src + i + stride),
                  c = __builtin_nontemporal_load(src + i + 2 * stride), d = __builtin_nontemporal_load(src + i + 3 * stride);
        acc ^= a.x ^ a.y ^ a.z ^ a.w ^ b.x ^ b.y ^ b.z ^ b.w ^ c.x ^ c.y ^ c.z ^ c.w ^ d.x ^ d.y ^ d.z ^ d.w;
    }
    for (; i < n16; i += stride) {
        const u4v a = __builtin_nontemporal_load(src + i);
        acc ^= a.x ^ a.y ^ a.z ^ a.w;
    }
    if (acc == 0x9e3779b9u) sink[blockIdx.x & 255] = acc;     // practically never true; keeps the loads live
}
}  // namespace sq

extern "C" {

int sq_probe_stream_read(const void *buf, size_t bytes, void *sink, int workgroups, void *stream)
{
    if (!buf || !sink || bytes < 16 || workgroups <= 0 || (reinterpret_cast<uintptr_t>(buf) & 15u))
        return SQ_ERR_INVALID_ARG;
    hipLaunchKernelGGL(sq::stream_read_kernel, dim3(workgroups), dim3(256), 0, static_cast<hipStream_t>(stream),
                       static_cast<const sq::u4v *>(buf), bytes / 16, static_cast<unsigned *>(sink));
    return hipGetLastError() == hipSuccess ? SQ_OK : SQ_ERR_HIP;
}

int sq_profile_begin(int max_launches)
{
    using sq::g_prof;
    if (g_prof.on || max_launches <= 0 || max_launches > (1 << 20)) return SQ_ERR_INVALID_ARG;
    g_prof.ev.resize((size_t)max_launches * 2);
    for (auto &e : g_prof.ev)
        if (hipEventCreate(&e) != hipSuccess) return SQ_ERR_HIP;
    g_prof.used = 0;
    g_prof.on = true;
    return SQ_OK;
}

int sq_profile_end(float *avg_us, float *min_us, float *max_us)
{
    using sq::g_prof;
    if (!g_prof.on) return 0;
    g_prof.on = false;
    int n = 0;
    double sum = 0.0;
    float mn = 1e30f, mx = 0.0f;
    for (size_t i = 0; i + 1 < g_prof.used; i += 2) {
        float ms = 0.0f;
        if (hipEventSynchronize(g_prof.ev[i + 1]) != hipSuccess) continue;
        if (hipEventElapsedTime(&ms, g_prof.ev[i], g_prof.ev[i + 1]) != hipSuccess) continue;
        const float us = ms * 1000.0f;
        sum += us;
        mn = us < mn ? us : mn;
        mx = us > mx ? us : mx;
        ++n;
    }
    for (auto &e : g_prof.ev) (void)hipEventDestroy(e);
    g_prof.ev.clear();
    g_prof.used = 0;
    if (avg_us) *avg_us = n ? (float)(sum / n) : 0.0f;
    if (min_us) *min_us = n ? mn : 0.0f;
    if (max_us) *max_us = mx;
    return n;
}

}  // extern "C"
