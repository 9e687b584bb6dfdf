// A decode step for callers that cannot allocate device memory (code under HIP graph capture, tight serving loops,
// harnesses that forbid hipMalloc): sq_decode_step with the workspace taken from a fixed device array that is part
// of the library's code object instead of from the caller.
//
// The array lives once per GPU the library runs on, until the process ends.  Every call on a GPU shares that GPU's
// array and finds the previous call's contents in it: nothing in it is assumed to be zero (the step's kernels clear
// the counters they use), and two calls that overlap in time on one GPU -- on different streams or from different
// threads -- race on it.
#include <hip/hip_runtime.h>

#include <atomic>

#include "../../include/squeezed_attention.h"
#include "sq_internal.hpp"

namespace {

// Device memory for the step's intermediate state: logits, range records, work list, partial results.
static __device__ __align__(256) unsigned char scratch[SQ_NOALLOC_SCRATCH_BYTES];

// `scratch` above is, in host code, only a handle for the symbol.  Its address in device memory differs from GPU to
// GPU and is looked up once per device; host code uses nothing but these pointers.
constexpr int MAX_DEVICES = 64;
std::atomic<void *> g_scratch_ptr[MAX_DEVICES];

}  // namespace

extern "C" int sq_decode_step_noalloc(const sq_shape_t *sh, const void *q, const void *centroids, const int32_t *sizes,
                                      const int32_t *offsets, const float *thresh, const void *K_fixed,
                                      const void *V_fixed, const void *K_user, const void *V_user, void *out, float *lse,
                                      uint32_t *keep_mask, int32_t *n_keys, void *stream)
{
    // Size check first, on the host alone (an invalid shape needs no workspace and is reported by sq_decode_step).
    const size_t need = sq_workspace_bytes(sh, SQ_CALL_DECODE_STEP);
    if (need > (size_t)SQ_NOALLOC_SCRATCH_BYTES)
        return sq::set_error(SQ_ERR_WORKSPACE,
                             "sq_decode_step_noalloc: this shape needs %zu bytes of intermediate state, the built-in "
                             "buffer holds %zu; use sq_decode_step with a workspace of the caller's",
                             need, (size_t)SQ_NOALLOC_SCRATCH_BYTES);
    int dev = -1;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return sq::set_error(SQ_ERR_HIP, "sq_decode_step_noalloc: hipGetDevice -> %s", hipGetErrorString(e));
    if (dev < 0 || dev >= MAX_DEVICES)
        return sq::set_error(SQ_ERR_UNSUPPORTED, "sq_decode_step_noalloc: device index %d not supported", dev);
    void *ptr = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (!ptr) {                                              // first call on this device (which is current)
        e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
        if (e != hipSuccess || !ptr)
            return sq::set_error(SQ_ERR_HIP, "sq_decode_step_noalloc: hipGetSymbolAddress -> %s", hipGetErrorString(e));
        g_scratch_ptr[dev].store(ptr, std::memory_order_release);   // (two threads racing here store the same address)
    }
    return sq_decode_step(sh, q, centroids, sizes, offsets, thresh, K_fixed, V_fixed, K_user, V_user, out, lse, keep_mask,
                          n_keys, ptr, (size_t)SQ_NOALLOC_SCRATCH_BYTES, stream);
}
