// Block-wide exact selection of the k smallest (value, index) pairs.
//
// Every item is a 31-bit non-negative key (the bit pattern of a non-negative
// float orders like the float) and a unique index.  Items are ordered by key,
// then by index, so the k smallest are unique even when keys repeat.  A
// most-significant-digit-first radix search with an LDS histogram walks the key
// in digits of 11, 11 and 9 bits; it stops as soon as the bin that holds the
// k-th item is needed in full, which for real-valued data is usually after two
// digits.  Only when the k-th key itself has duplicates that must be split does
// the search continue over the index bits of the items carrying that key.
// Everything is 32-bit arithmetic; a one-wave block needs no hardware barrier.
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

// An item is selected (is among the k smallest) iff
//   key < bound.key  ||  (key == bound.key && idx <= bound.idx)
struct SelectBound {
    uint32_t key;
    uint32_t idx;
};

__device__ __forceinline__ bool is_selected(uint32_t key, uint32_t idx, SelectBound b) {
    return key < b.key || (key == b.key && idx <= b.idx);
}

__device__ __forceinline__ uint32_t key_of(float metric_value) { return __float_as_uint(metric_value) & 0x7fffffffu; }

inline int index_bits_for(int64_t n) {  // bits needed for indices 0 .. n-1 (at least 1)
    int b = 1;
    while ((int64_t(1) << b) < n) ++b;
    return b;
}

// The histogram is complete and visible.  Finds the bin holding the `need`-th item (1-based,
// counted from bin 0), returns how many items lie in lower bins and how many in that bin, and
// leaves the histogram zeroed for the next digit.
template <int BLOCK>
__device__ __forceinline__ void locate_bin(SelectSmem<BLOCK> &sm, uint32_t need, uint32_t &bin, uint32_t &before,
                                           uint32_t &count) {
    constexpr int BPT = kSelBins / BLOCK;  // bins owned by a thread
    static_assert(BPT % 4 == 0 || BPT == 2, "bins per thread");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    uint32_t *mine = &sm.hist[tid * BPT];
    uint32_t s = 0;
    if constexpr (BPT >= 4) {
#pragma unroll
        for (int i = 0; i < BPT; i += 4) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(mine + i);
            s += (v[0] + v[1]) + (v[2] + v[3]);
        }
    } else {
        s = mine[0] + mine[1];
    }
    const uint32_t incl = wave_inclusive_scan(s);
    uint32_t excl = incl - s;
    if constexpr (BLOCK > kWave) {
        if (lane == kWave - 1) sm.wave_tot[wv] = incl;
        __syncthreads();
        for (int i = 0; i < wv; ++i) excl += sm.wave_tot[i];
    }
    if (excl < need && need <= excl + s) {  // exactly one thread: its bins hold the item
        uint32_t run = excl;
        for (int i = 0; i < BPT; ++i) {
            const uint32_t h = mine[i];
            if (need <= run + h) {
                sm.sel_bin = static_cast<uint32_t>(tid * BPT + i);
                sm.sel_before = run;
                sm.sel_count = h;
                break;
            }
            run += h;
        }
    }
    if constexpr (BPT >= 4) {
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < BPT; i += 4) *reinterpret_cast<u32x4 *>(mine + i) = z;
    } else {
        mine[0] = 0u;
        mine[1] = 0u;
    }
    __syncthreads();
    bin = sm.sel_bin;
    before = sm.sel_before;
    count = sm.sel_count;
}

// for_each(f, salt) must call f(key, idx) once for every item the calling thread owns and must
// visit the same items on every call; keys are below 2^31 and indices below 2^idx_bits.  salt is
// always zero, but opaque to the compiler inside the rarely taken tie loop: a caller that derives
// its indices from (thread id + salt) keeps them from being hoisted out of that loop into
// registers that the common path would then have to carry.
// 1 <= k <= number of items.  All threads of the block call this; all get the same bound.
template <int BLOCK, class ForEach>
__device__ SelectBound block_select_bound(ForEach for_each, uint32_t k, int idx_bits, SelectSmem<BLOCK> &sm) {
    for (int b = threadIdx.x; b < kSelBins; b += BLOCK) sm.hist[b] = 0u;
    __syncthreads();
    uint32_t need = k, bin, before, count;

    // key bits 30..20
    for_each([&](uint32_t key, uint32_t) { atomicAdd(&sm.hist[key >> 20], 1u); }, 0u);
    __syncthreads();
    locate_bin<BLOCK>(sm, need, bin, before, count);
    need -= before;
    uint32_t prefix = bin;
    if (need == count) return {(prefix << 20) | 0xfffffu, 0xffffffffu};

    // key bits 19..9
    for_each([&](uint32_t key, uint32_t) {
        if ((key >> 20) == prefix) atomicAdd(&sm.hist[(key >> 9) & 0x7ffu], 1u);
    }, 0u);
    __syncthreads();
    locate_bin<BLOCK>(sm, need, bin, before, count);
    need -= before;
    prefix = (prefix << 11) | bin;
    if (need == count) return {(prefix << 9) | 0x1ffu, 0xffffffffu};

    // key bits 8..0
    for_each([&](uint32_t key, uint32_t) {
        if ((key >> 9) == prefix) atomicAdd(&sm.hist[key & 0x1ffu], 1u);
    }, 0u);
    __syncthreads();
    locate_bin<BLOCK>(sm, need, bin, before, count);
    need -= before;
    const uint32_t v = (prefix << 9) | bin;
    if (need == count) return {v, 0xffffffffu};

    // the k-th key is v and only some of its copies are selected: lowest indices first
    int pos = idx_bits;  // index bits [pos, idx_bits) are fixed to ipre
    uint32_t ipre = 0;
    for (;;) {
        const int width = pos < kSelDigit ? pos : kSelDigit;
        const int shift = pos - width;
        const uint32_t dmask = (1u << width) - 1u;
        uint32_t salt = 0u, vv = v;
        asm volatile("" : "+v"(salt), "+v"(vv));  // redefined every iteration: nothing below is loop-invariant
        for_each([&](uint32_t key, uint32_t idx) {
            const uint32_t hi = pos >= 32 ? 0u : (idx >> pos);
            if (key == vv && hi == ipre) atomicAdd(&sm.hist[(idx >> shift) & dmask], 1u);
        }, salt);
        __syncthreads();
        locate_bin<BLOCK>(sm, need, bin, before, count);
        need -= before;
        ipre = (ipre << width) | bin;
        pos = shift;
        if (pos == 0) return {v, ipre};
        if (need == count) return {v, static_cast<uint32_t>(((static_cast<uint64_t>(ipre) + 1) << pos) - 1)};
    }
}

}  // namespace mp
