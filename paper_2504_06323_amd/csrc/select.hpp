// Block-wide exact selection of the k smallest (value, index) pairs.
//
// Every item is a 31-bit non-negative key (the bit pattern of a non-negative
// float orders like the float) and a unique index.  The two are glued into one
// composite integer  comp = key << index_bits | index,  which makes all items
// distinct and puts equal keys in ascending index order.  A most-significant-
// digit-first radix search (11-bit digits, histogram in LDS) finds the bound B
// with exactly k items <= B.  The search stops as soon as the digit bin that
// contains the k-th item is needed in full, which for real-valued data is
// usually after two digits; index digits are only visited when the k-th key
// has duplicates.
#pragma once

#include "common.hpp"

namespace mp {

constexpr int kSelBins = 2048;
constexpr int kSelDigit = 11;

template <int BLOCK>
struct SelectSmem {
    alignas(16) uint32_t hist[kSelBins];
    uint32_t wave_tot[BLOCK / kWave];
    uint32_t sel_bin, sel_before, sel_count;
};

__device__ __forceinline__ uint64_t composite(uint32_t key, uint32_t idx, int idx_bits) {
    return (static_cast<uint64_t>(key) << idx_bits) | idx;
}

__device__ __forceinline__ uint32_t key_of(float metric_value) { return __float_as_uint(metric_value) & 0x7fffffffu; }

inline int index_bits_for(int64_t n) {  // bits needed for indices 0 .. n-1 (at least 1)
    int b = 1;
    while ((int64_t(1) << b) < n) ++b;
    return b;
}

// for_each(f) must call f(key, idx) once for every item the calling thread owns
// and must visit the same items on every call.  1 <= k <= number of items.
// All threads of the block must call this; returns the same bound to all.
template <int BLOCK, class ForEach>
__device__ uint64_t block_select_bound(ForEach for_each, uint32_t k, int idx_bits, SelectSmem<BLOCK> &sm) {
    constexpr int BPT = kSelBins / BLOCK;  // histogram bins scanned per thread
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    int pos = 31 + idx_bits;  // bits [pos, top) of comp are already fixed to `prefix`
    uint64_t prefix = 0;
    uint32_t need = k;
    for (;;) {
        const int left = pos > idx_bits ? pos - idx_bits : pos;  // finish the key digits before the index digits
        const int width = left < kSelDigit ? left : kSelDigit;
        const int shift = pos - width;
        const uint32_t dmask = (1u << width) - 1u;

        for (int b = tid; b < kSelBins; b += BLOCK) sm.hist[b] = 0u;
        __syncthreads();
        for_each([&](uint32_t key, uint32_t idx) {
            const uint64_t comp = composite(key, idx, idx_bits);
            if ((comp >> pos) == prefix) atomicAdd(&sm.hist[static_cast<uint32_t>(comp >> shift) & dmask], 1u);
        });
        __syncthreads();

        uint32_t h[BPT], s = 0;
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            h[i] = sm.hist[tid * BPT + i];
            s += h[i];
        }
        const uint32_t incl = wave_inclusive_scan(s);
        if (lane == kWave - 1) sm.wave_tot[wv] = incl;
        __syncthreads();
        uint32_t excl = incl - s;
        for (int i = 0; i < wv; ++i) excl += sm.wave_tot[i];
        if (excl < need && need <= excl + s) {  // exactly one thread: its bins hold the k-th item
            uint32_t run = excl;
#pragma unroll
            for (int i = 0; i < BPT; ++i) {
                if (run < need && need <= run + h[i]) {
                    sm.sel_bin = static_cast<uint32_t>(tid * BPT + i);
                    sm.sel_before = run;
                    sm.sel_count = h[i];
                }
                run += h[i];
            }
        }
        __syncthreads();
        const uint32_t bin = sm.sel_bin, before = sm.sel_before, cnt = sm.sel_count;
        prefix = (prefix << width) | bin;
        need -= before;
        pos = shift;
        if (pos == 0) return prefix;                           // all digits fixed: comp is unique
        if (need == cnt) return ((prefix + 1) << pos) - 1;     // the whole bin goes
    }
}

}  // namespace mp
