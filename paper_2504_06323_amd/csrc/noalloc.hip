// prune_stats_norms with its scratch built into the library: for callers that cannot allocate
// device memory (code under HIP graph capture, tight serving loops, harnesses that forbid it).
//
// The per-stripe partial sums that prune_stats_norms keeps in the caller's workspace live in a
// file-scope device array here.  Every GPU the library runs on holds its own copy of that array
// (2 MiB, until the process ends) at its own address; the address is looked up once per device and
// handed to the kernels as an ordinary pointer argument, exactly like a caller's workspace.
#include <atomic>

#include "common.hpp"

namespace mp {
namespace {

constexpr size_t kStaticScratchBytes = PRUNE_STATIC_SCRATCH_BYTES;
constexpr int kMaxDevices = 64;

static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

// device address of `scratch` on each GPU (0 = not looked up yet).  Two threads racing through the
// first call on a device store the same value.
std::atomic<void *> g_scratch_ptr[kMaxDevices];

// The address of this device's copy of the array, or nullptr if the runtime refuses to give it.
void *static_scratch_for_current_device() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    void *p = g_scratch_ptr[dev].load(std::memory_order_acquire);
    if (p) return p;
    if (hipGetSymbolAddress(&p, HIP_SYMBOL(scratch)) != hipSuccess || !p) {
        (void)hipGetLastError();
        return nullptr;
    }
    g_scratch_ptr[dev].store(p, std::memory_order_release);
    return p;
}

}  // namespace
}  // namespace mp

extern "C" int prune_stats_norms_static(const void *x, int dtype, int64_t n_tokens, int64_t n_channels, int64_t ld_x,
                                        float *sumsq, float *norms, void *stream) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_tokens < 0 || n_channels <= 0 || ld_x < n_channels) return PRUNE_ERR_SHAPE;
    if (!sumsq || !norms || (n_tokens > 0 && !x)) return PRUNE_ERR_NULL;
    if ((x && !aligned_to(x, elem_size(dtype))) || !aligned_to(sumsq, 4) || !aligned_to(norms, 4))
        return PRUNE_ERR_ALIGNMENT;
    // the partial sums of this shape must fit the built-in array
    if (colsum_workspace_bytes(n_tokens > 0 ? n_tokens : 1, n_channels) > kStaticScratchBytes)
        return PRUNE_ERR_WORKSPACE;
    void *ws = static_scratch_for_current_device();
    if (!ws) return PRUNE_ERR_DEVICE;
    // Nothing has to be cleared: every partial the reduction reads is written by this call's first kernel.
    return launch_colsum(x, dtype, n_tokens, n_channels, ld_x, sumsq, ws, static_cast<hipStream_t>(stream), false,
                         norms);
}
