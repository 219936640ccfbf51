// Streaming ceilings of the device, measured with the plainest kernels there are: a read-only pass
// and a copy, both in 128-bit accesses.  The benchmark runs them next to the pruning kernels so that
// every pass can be held against what the memory system of this very card delivers on this very
// day, beside the published peak.  Nothing of the method is computed here.
#include "common.hpp"

namespace mp {
namespace {

constexpr int kProbeBlock = 256;
constexpr int kProbeUnroll = 8;

// Every thread reads kProbeUnroll packets of 16 bytes per trip (a block covers 32 KB contiguous per trip) and
// folds them into one word, so that the loads cannot be dropped; one word per thread is written at the end.
__global__ __launch_bounds__(kProbeBlock) void probe_read(const u32x4 *__restrict__ src, int64_t n_packets,
                                                          uint32_t *__restrict__ sink) {
    const int64_t per_trip = static_cast<int64_t>(kProbeBlock) * kProbeUnroll;
    uint32_t acc = 0;
    for (int64_t base = static_cast<int64_t>(blockIdx.x) * per_trip; base < n_packets;
         base += static_cast<int64_t>(gridDim.x) * per_trip) {
        u32x4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            const int64_t i = base + u * kProbeBlock + threadIdx.x;
            v[u] = i < n_packets ? __builtin_nontemporal_load(src + i) : u32x4{0u, 0u, 0u, 0u};
        }
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) acc ^= (v[u][0] ^ v[u][1]) ^ (v[u][2] ^ v[u][3]);
    }
    sink[static_cast<int64_t>(blockIdx.x) * kProbeBlock + threadIdx.x] = acc;
}

__global__ __launch_bounds__(kProbeBlock) void probe_copy(const u32x4 *__restrict__ src, u32x4 *__restrict__ dst,
                                                          int64_t n_packets) {
    const int64_t per_trip = static_cast<int64_t>(kProbeBlock) * kProbeUnroll;
    for (int64_t base = static_cast<int64_t>(blockIdx.x) * per_trip; base < n_packets;
         base += static_cast<int64_t>(gridDim.x) * per_trip) {
        u32x4 v[kProbeUnroll];
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            const int64_t i = base + u * kProbeBlock + threadIdx.x;
            if (i < n_packets) v[u] = __builtin_nontemporal_load(src + i);
        }
#pragma unroll
        for (int u = 0; u < kProbeUnroll; ++u) {
            const int64_t i = base + u * kProbeBlock + threadIdx.x;
            if (i < n_packets) __builtin_nontemporal_store(v[u], dst + i);
        }
    }
}

}  // namespace
}  // namespace mp

extern "C" size_t prune_bandwidth_probe_sink_bytes(int blocks) {
    return blocks > 0 ? static_cast<size_t>(blocks) * mp::kProbeBlock * sizeof(uint32_t) : 0;
}

extern "C" int prune_bandwidth_probe(const void *src, void *dst, size_t bytes, int mode, int blocks, void *stream) {
    using namespace mp;
    if (mode != PRUNE_PROBE_READ && mode != PRUNE_PROBE_COPY) return PRUNE_ERR_RANGE;
    if (blocks <= 0 || blocks > (1 << 20)) return PRUNE_ERR_RANGE;
    if (bytes == 0 || bytes % 16 != 0) return PRUNE_ERR_SHAPE;
    if (!src || !dst) return PRUNE_ERR_NULL;
    if (!aligned_to(src, 16) || !aligned_to(dst, 16)) return PRUNE_ERR_ALIGNMENT;
    const int64_t n = static_cast<int64_t>(bytes / 16);
    if (mode == PRUNE_PROBE_READ)
        hipLaunchKernelGGL(probe_read, dim3(static_cast<unsigned>(blocks)), dim3(kProbeBlock), 0,
                           static_cast<hipStream_t>(stream), static_cast<const u32x4 *>(src), n,
                           static_cast<uint32_t *>(dst));
    else
        hipLaunchKernelGGL(probe_copy, dim3(static_cast<unsigned>(blocks)), dim3(kProbeBlock), 0,
                           static_cast<hipStream_t>(stream), static_cast<const u32x4 *>(src),
                           static_cast<u32x4 *>(dst), n);
    return launch_status();
}
