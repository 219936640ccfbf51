// Block-wide exact selection of the k smallest (value, index) pairs.
//
// Every item is a 31-bit non-negative key (the bit pattern of a non-negative
// float orders like the float) and a unique index.  Items are ordered by key,
// then by index, so the k smallest are unique even when keys repeat.  A
// most-significant-digit-first radix search with an LDS histogram walks the key
// in digits of 11, 8, 8 and 4 bits; it stops as soon as the bin that holds the
// k-th item is needed in full, which for real-valued data is usually after two
// or three digits.  Only when the k-th key itself has duplicates that must be split does
// the search continue over the index bits of the items carrying that key.
// Everything is 32-bit arithmetic; a one-wave block needs no hardware barrier.
#pragma once

#include "common.hpp"

namespace mp {

constexpr int kSelBins = 2048;

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

// The histogram over bins [0, BINS) is complete and visible.  Finds the bin holding the `need`-th item
// (1-based, counted from bin 0), returns how many items lie in lower bins and how many in that bin,
// and leaves those bins zeroed for the next digit.
template <int BLOCK, int BINS>
__device__ __forceinline__ void locate_bin(SelectSmem<BLOCK> &sm, uint32_t need, uint32_t &bin, uint32_t &before,
                                           uint32_t &count) {
    constexpr int BPT = BINS >= BLOCK ? BINS / BLOCK : 1;  // bins owned by a thread
    static_assert(BPT < 4 || BPT % 4 == 0, "bins per thread");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    const bool owner = BINS >= BLOCK || tid < BINS;
    uint32_t *mine = &sm.hist[tid * BPT];
    uint32_t s = 0;
    if (owner) {
        if constexpr (BPT >= 4) {
#pragma unroll
            for (int i = 0; i < BPT; i += 4) {
                const u32x4 v = *reinterpret_cast<const u32x4 *>(mine + i);
                s += (v[0] + v[1]) + (v[2] + v[3]);
            }
        } else {
#pragma unroll
            for (int i = 0; i < BPT; ++i) s += mine[i];
        }
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
    if (owner) {
        if constexpr (BPT >= 4) {
            const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
            for (int i = 0; i < BPT; i += 4) *reinterpret_cast<u32x4 *>(mine + i) = z;
        } else {
#pragma unroll
            for (int i = 0; i < BPT; ++i) mine[i] = 0u;
        }
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
// The histogram must be all zero (and visible to the block) on entry; it is all zero again on return.
//
// Digits: key bits 30..20 first (2048 bins: the exponent and three mantissa bits, which is where
// the values of a row spread), then 8 bits at a time (256 bins: few candidates are left, so the
// per-digit cost is what matters), the last key digit being 4 bits.
template <int BLOCK, class ForEach>
__device__ SelectBound block_select_bound(ForEach for_each, uint32_t k, int idx_bits, SelectSmem<BLOCK> &sm) {
    uint32_t need = k, bin, before, count;

    for_each([&](uint32_t key, uint32_t) { atomicAdd(&sm.hist[key >> 20], 1u); }, 0u);
    __syncthreads();
    locate_bin<BLOCK, kSelBins>(sm, need, bin, before, count);
    need -= before;
    uint32_t prefix = bin;  // key bits above `pos`
    if (need == count) return {(prefix << 20) | 0xfffffu, 0xffffffffu};

    int pos = 20;
#pragma unroll 1
    while (pos > 0) {
        const int width = pos >= 8 ? 8 : pos;  // 8, 8, 4
        const int shift = pos - width;
        const uint32_t dmask = (1u << width) - 1u;
        for_each([&](uint32_t key, uint32_t) {
            if ((key >> pos) == prefix) atomicAdd(&sm.hist[(key >> shift) & dmask], 1u);
        }, 0u);
        __syncthreads();
        locate_bin<BLOCK, 256>(sm, need, bin, before, count);
        need -= before;
        prefix = (prefix << width) | bin;
        pos = shift;
        if (need == count) return {pos ? (((prefix + 1u) << pos) - 1u) : prefix, 0xffffffffu};
    }
    const uint32_t v = prefix;

    // the k-th key is v and only some of its copies are selected: lowest indices first
    pos = idx_bits;  // index bits [pos, idx_bits) are fixed to ipre
    uint32_t ipre = 0;
    for (;;) {
        const int width = pos < 8 ? pos : 8;
        const int shift = pos - width;
        const uint32_t dmask = (1u << width) - 1u;
        uint32_t salt = 0u, vv = v;
        asm volatile("" : "+v"(salt), "+v"(vv));  // redefined every iteration: nothing below is loop-invariant
        for_each([&](uint32_t key, uint32_t idx) {
            const uint32_t hi = pos >= 32 ? 0u : (idx >> pos);
            if (key == vv && hi == ipre) atomicAdd(&sm.hist[(idx >> shift) & dmask], 1u);
        }, salt);
        __syncthreads();
        locate_bin<BLOCK, 256>(sm, need, bin, before, count);
        need -= before;
        ipre = (ipre << width) | bin;
        pos = shift;
        if (pos == 0) return {v, ipre};
        if (need == count) return {v, static_cast<uint32_t>(((static_cast<uint64_t>(ipre) + 1) << pos) - 1)};
    }
}

}  // namespace mp
