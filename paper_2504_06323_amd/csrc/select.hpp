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

// First digit: the histogram over all kSelBins bins is complete and visible.  The threads share the
// scan: each owns kSelBins / BLOCK consecutive bins.  Finds the bin holding the `need`-th item (1-based,
// counted from bin 0), returns how many items lie in lower bins and how many in that bin, and leaves
// the whole histogram zeroed (and visible) for the later digits.
template <int BLOCK>
__device__ __forceinline__ void locate_first_digit(SelectSmem<BLOCK> &sm, uint32_t need, uint32_t &bin,
                                                   uint32_t &before, uint32_t &count) {
    constexpr int BPT = kSelBins / BLOCK;  // bins owned by a thread
    constexpr int NW = BLOCK / kWave;
    static_assert(BPT < 4 || BPT % 4 == 0, "bins per thread");
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    uint32_t *mine = &sm.hist[tid * BPT];
    uint32_t s = 0;
    uint32_t h[BPT <= 8 ? BPT : 1];  // a short run of bins stays in registers for the walk below
    if constexpr (BPT >= 4) {
#pragma unroll
        for (int i = 0; i < BPT; i += 4) {
            const u32x4 v = *reinterpret_cast<const u32x4 *>(mine + i);
            s += (v[0] + v[1]) + (v[2] + v[3]);
            if constexpr (BPT <= 8) {
                h[i] = v[0];
                h[i + 1] = v[1];
                h[i + 2] = v[2];
                h[i + 3] = v[3];
            }
        }
    } else {
#pragma unroll
        for (int i = 0; i < BPT; ++i) {
            h[i] = mine[i];
            s += h[i];
        }
    }
    const uint32_t incl = wave_inclusive_scan(s);
    uint32_t excl = incl - s;
    if constexpr (NW > 1) {
        if (lane == kWave - 1) sm.wave_tot[wv] = incl;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NW - 1; ++i) {  // independent loads, masked adds: no dependent LDS round trips
            const uint32_t t = sm.wave_tot[i];
            excl += i < wv ? t : 0u;
        }
    }
    if (excl < need && need <= excl + s) {  // exactly one thread: its bins hold the item
        if constexpr (BPT <= 8) {
            uint32_t run = excl, b = 0, bef = excl, cnt = h[0];
#pragma unroll
            for (int i = 1; i < BPT; ++i) {
                run += h[i - 1];
                const bool later = need > run;  // the item lies in bin i or beyond
                b = later ? static_cast<uint32_t>(i) : b;
                bef = later ? run : bef;
                cnt = later ? h[i] : cnt;
            }
            sm.sel_bin = static_cast<uint32_t>(tid * BPT) + b;
            sm.sel_before = bef;
            sm.sel_count = cnt;
        } else {
            uint32_t run = excl;
            for (int i = 0; i < BPT; ++i) {
                const uint32_t hi = mine[i];
                if (need <= run + hi) {
                    sm.sel_bin = static_cast<uint32_t>(tid * BPT + i);
                    sm.sel_before = run;
                    sm.sel_count = hi;
                    break;
                }
                run += hi;
            }
        }
    }
    if constexpr (BPT >= 4) {
        const u32x4 z = {0u, 0u, 0u, 0u};
#pragma unroll
        for (int i = 0; i < BPT; i += 4) *reinterpret_cast<u32x4 *>(mine + i) = z;
    } else {
#pragma unroll
        for (int i = 0; i < BPT; ++i) mine[i] = 0u;
    }
    __syncthreads();
    bin = sm.sel_bin;
    before = sm.sel_before;
    count = sm.sel_count;
}

// Later digits: a 256-bin histogram (`region`) is complete and visible.  Every wave scans all of it on
// its own (four bins per lane, scan and pick in registers), so no data is exchanged between waves and
// all arrive at the same answer.  The region is left as it is: every later digit uses a fresh one.
__device__ __forceinline__ void locate_later_digit(const uint32_t *region, uint32_t need, uint32_t &bin,
                                                   uint32_t &before, uint32_t &count) {
    const int lane = threadIdx.x & (kWave - 1);
    const u32x4 v = *reinterpret_cast<const u32x4 *>(region + lane * 4);
    const uint32_t s = (v[0] + v[1]) + (v[2] + v[3]);
    const uint32_t incl = wave_inclusive_scan(s);
    const uint32_t c0 = incl - s, c1 = c0 + v[0], c2 = c1 + v[1], c3 = c2 + v[2];
    const bool hit = c0 < need && need <= incl;  // exactly one lane
    const uint32_t j = (need > c1 ? 1u : 0u) + (need > c2 ? 1u : 0u) + (need > c3 ? 1u : 0u);
    const uint32_t bef = j == 0 ? c0 : j == 1 ? c1 : j == 2 ? c2 : c3;
    const uint32_t cnt = j == 0 ? v[0] : j == 1 ? v[1] : j == 2 ? v[2] : v[3];
    const unsigned long long where = __ballot(hit);
    const int src = __builtin_amdgcn_readfirstlane(__ffsll(static_cast<long long>(where)) - 1);
    bin = static_cast<uint32_t>(src) * 4u + static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(j), src));
    before = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(bef), src));
    count = static_cast<uint32_t>(__builtin_amdgcn_readlane(static_cast<int>(cnt), src));
}

// for_each(f, salt) must call f(key, idx) once for every item the calling thread owns and must
// visit the same items on every call; keys are below 2^31 and indices below 2^idx_bits.  salt is
// always zero, but opaque to the compiler inside the rarely taken tie loop: a caller that derives
// its indices from (thread id + salt) keeps them from being hoisted out of that loop into
// registers that the common path would then have to carry.
// 1 <= k <= number of items.  All threads of the block call this; all get the same bound.
// The histogram must be all zero (and visible to the block) on entry.
//
// Digits: key bits 30..20 first (2048 bins: the exponent and three mantissa bits, which is where
// the values of a row spread), then 8 bits at a time (few candidates are left, so the per-digit cost
// is what matters), the last key digit being 4 bits; index digits of 8 bits if a tie must be split.
// The first digit leaves the histogram zeroed; each later digit counts into its own 256-bin slice of
// it, so later digits need neither zeroing nor more than one barrier (at most 3 + 4 slices are used).
//
// A caller that knows that all its keys agree in the bits above bit first_shift + 10 passes those common
// bits as hi_common (= key >> (first_shift + 11)) and a first_shift below 20: the first digit then starts
// at the first bit where keys can differ, which keeps keys of nearly equal magnitude from piling into a
// single bin (LDS atomics on one address are serialised).
template <int BLOCK, class ForEach>
__device__ SelectBound block_select_bound(ForEach for_each, uint32_t k, int idx_bits, SelectSmem<BLOCK> &sm,
                                          int first_shift = 20, uint32_t hi_common = 0u) {
    uint32_t need = k, bin, before, count;

    // (the digit is masked so that a key with bit 31 set -- only a NaN metric can have it -- stays inside the
    // histogram; such a key matches no later digit and is never selected)
    for_each([&](uint32_t key, uint32_t) { atomicAdd(&sm.hist[(key >> first_shift) & 0x7ffu], 1u); }, 0u);
    __syncthreads();
    locate_first_digit<BLOCK>(sm, need, bin, before, count);
    need -= before;
    uint32_t prefix = (hi_common << 11) | bin;  // key bits above `pos`
    int pos = first_shift;
    if (need == count) return {pos ? (((prefix + 1u) << pos) - 1u) : prefix, 0xffffffffu};

    uint32_t *region = sm.hist;  // next fresh 256-bin slice
#pragma unroll 1
    while (pos > 0) {
        const int width = pos >= 8 ? 8 : pos;  // 8, 8, 4
        const int shift = pos - width;
        // key matches the digits fixed so far iff clearing them leaves less than 2^pos
        const uint32_t fixed = prefix << pos, limit = 1u << pos;
        for_each([&](uint32_t key, uint32_t) {
            const uint32_t rest = key ^ fixed;
            if (rest < limit) atomicAdd(&region[rest >> shift], 1u);
        }, 0u);
        __syncthreads();
        locate_later_digit(region, need, bin, before, count);
        region += 256;
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
            if (key == vv && hi == ipre) atomicAdd(&region[(idx >> shift) & dmask], 1u);
        }, salt);
        __syncthreads();
        locate_later_digit(region, need, bin, before, count);
        region += 256;
        need -= before;
        ipre = (ipre << width) | bin;
        pos = shift;
        if (pos == 0) return {v, ipre};
        if (need == count) return {v, static_cast<uint32_t>(((static_cast<uint64_t>(ipre) + 1) << pos) - 1)};
    }
}

}  // namespace mp
