// Shared device helpers for the gfx950 pruning kernels: 128-bit row packets,
// exact bf16 widening, wave/block reductions.  Wavefront size is 64 throughout.
#pragma once

#include <hip/hip_runtime.h>
#include <stddef.h>
#include <stdint.h>

#include "mosaic_prune.h"

namespace mp {

constexpr int kWave = 64;

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

using bf16_t = uint16_t;  // bfloat16 storage: the high half of a float

__device__ __forceinline__ float bf16_to_float(bf16_t h) { return __uint_as_float(static_cast<uint32_t>(h) << 16); }
__device__ __forceinline__ float widen(bf16_t h) { return bf16_to_float(h); }
__device__ __forceinline__ float widen(float f) { return f; }

// One IEEE float multiply, never fused with a neighbouring add: every kernel
// that forms the weight metric goes through this so the bits agree everywhere.
__device__ __forceinline__ float metric(float w, float norm) { return __fmul_rn(fabsf(w), norm); }

// ---------------------------------------------------------------------------
// Packet<T, VEC>: VEC consecutive elements of a row held in registers in their
// storage format.  VEC == 8 moves 128-bit words (one for bf16, two for float);
// VEC == 1 is the scalar fallback for rows that cannot be accessed that way.
// ---------------------------------------------------------------------------
template <typename T, int VEC>
struct Packet;

template <>
struct Packet<bf16_t, 8> {
    u32x4 raw;
    template <bool NT = false>
    __device__ __forceinline__ void load(const bf16_t *p) {
        const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
        raw = NT ? __builtin_nontemporal_load(q) : *q;
    }
    __device__ __forceinline__ void store(bf16_t *p) const { *reinterpret_cast<u32x4 *>(p) = raw; }
    __device__ __forceinline__ void to_float(float (&v)[8]) const {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            v[2 * i] = __uint_as_float(raw[i] << 16);
            v[2 * i + 1] = __uint_as_float(raw[i] & 0xffff0000u);
        }
    }
    // keep element e iff bit e of `keep` is set; others become +0
    __device__ __forceinline__ void apply_keep(uint32_t keep) {
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            uint32_t m = ((keep >> (2 * i)) & 1u ? 0x0000ffffu : 0u) | ((keep >> (2 * i + 1)) & 1u ? 0xffff0000u : 0u);
            raw[i] &= m;
        }
    }
    // the same with one all-ones / all-zeros word per element
    __device__ __forceinline__ void apply_keep_words(const uint32_t (&km)[8]) {
#pragma unroll
        for (int i = 0; i < 4; ++i) raw[i] &= (km[2 * i] & 0x0000ffffu) | (km[2 * i + 1] & 0xffff0000u);
    }
    // acc + sum of the squares of the eight elements, in element order (products of bf16 are exact in float; the
    // two-element dot-product instruction is not used: its sum does not keep float precision)
    __device__ __forceinline__ float add_squares(float acc) const {
        float v[8];
        to_float(v);
#pragma unroll
        for (int i = 0; i < 8; ++i) acc = fmaf(v[i], v[i], acc);
        return acc;
    }
};

template <>
struct Packet<float, 8> {
    u32x4 raw[2];
    template <bool NT = false>
    __device__ __forceinline__ void load(const float *p) {
        const u32x4 *q = reinterpret_cast<const u32x4 *>(p);
        raw[0] = NT ? __builtin_nontemporal_load(q) : q[0];
        raw[1] = NT ? __builtin_nontemporal_load(q + 1) : q[1];
    }
    __device__ __forceinline__ void store(float *p) const {
        u32x4 *q = reinterpret_cast<u32x4 *>(p);
        q[0] = raw[0];
        q[1] = raw[1];
    }
    __device__ __forceinline__ void to_float(float (&v)[8]) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) v[i] = __uint_as_float(raw[i >> 2][i & 3]);
    }
    __device__ __forceinline__ void apply_keep(uint32_t keep) {
#pragma unroll
        for (int i = 0; i < 8; ++i)
            if (!((keep >> i) & 1u)) raw[i >> 2][i & 3] = 0u;
    }
    __device__ __forceinline__ void apply_keep_words(const uint32_t (&km)[8]) {
#pragma unroll
        for (int i = 0; i < 8; ++i) raw[i >> 2][i & 3] &= km[i];
    }
    __device__ __forceinline__ float add_squares(float acc) const {
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const float v = __uint_as_float(raw[i >> 2][i & 3]);
            acc = fmaf(v, v, acc);
        }
        return acc;
    }
};

template <typename T>
struct Packet<T, 1> {
    T raw;
    template <bool NT = false>
    __device__ __forceinline__ void load(const T *p) {
        raw = *p;
    }
    __device__ __forceinline__ void store(T *p) const { *p = raw; }
    __device__ __forceinline__ void to_float(float (&v)[1]) const { v[0] = widen(raw); }
    __device__ __forceinline__ void apply_keep(uint32_t keep) {
        if (!(keep & 1u)) raw = T(0);
    }
};

__device__ __forceinline__ void store_floats(float *p, const float (&v)[8]) {
    f32x4 a = {v[0], v[1], v[2], v[3]}, b = {v[4], v[5], v[6], v[7]};
    reinterpret_cast<f32x4 *>(p)[0] = a;
    reinterpret_cast<f32x4 *>(p)[1] = b;
}
__device__ __forceinline__ void store_floats(float *p, const float (&v)[1]) { p[0] = v[0]; }

__device__ __forceinline__ void load_floats(const float *p, float (&v)[8]) {
    f32x4 a = reinterpret_cast<const f32x4 *>(p)[0], b = reinterpret_cast<const f32x4 *>(p)[1];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
        v[i] = a[i];
        v[4 + i] = b[i];
    }
}
__device__ __forceinline__ void load_floats(const float *p, float (&v)[1]) { v[0] = p[0]; }

// ---------------------------------------------------------------------------
// reductions (fixed shapes => fixed summation order => reproducible results)
// ---------------------------------------------------------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    return v;  // valid in lane 0
}
__device__ __forceinline__ uint32_t wave_sum(uint32_t v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int off = kWave / 2; off > 0; off >>= 1) v += __shfl_down(v, off, kWave);
    return v;
}

// inclusive prefix sum across the 64 lanes of a wave, in registers (data-parallel primitives, no LDS):
// a Hillis-Steele scan inside every row of 16 lanes, then the row totals are carried forward.
__device__ __forceinline__ uint32_t wave_inclusive_scan(uint32_t v) {
    // update_dpp(old, src, ctrl, row_mask, bank_mask, bound_ctrl): lanes without a valid source, and
    // lanes of rows that row_mask switches off, receive `old` (zero here)
    v += __builtin_amdgcn_update_dpp(0u, v, 0x111, 0xf, 0xf, false);  // row_shr:1
    v += __builtin_amdgcn_update_dpp(0u, v, 0x112, 0xf, 0xf, false);  // row_shr:2
    v += __builtin_amdgcn_update_dpp(0u, v, 0x114, 0xf, 0xf, false);  // row_shr:4
    v += __builtin_amdgcn_update_dpp(0u, v, 0x118, 0xf, 0xf, false);  // row_shr:8
    v += __builtin_amdgcn_update_dpp(0u, v, 0x142, 0xa, 0xf, false);  // row_bcast:15 into rows 1 and 3
    v += __builtin_amdgcn_update_dpp(0u, v, 0x143, 0xc, 0xf, false);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Sum over a block of BLOCK threads; every thread must call it; result valid in thread 0.
template <int BLOCK, typename V>
__device__ __forceinline__ V block_sum(V v, V *smem /* BLOCK / 64 entries */) {
    constexpr int NW = BLOCK / kWave;
    v = wave_sum(v);
    if constexpr (NW == 1) return v;
    const int lane = threadIdx.x & (kWave - 1), wv = threadIdx.x / kWave;
    if (lane == 0) smem[wv] = v;
    __syncthreads();
    V t = V(0);
    if (threadIdx.x == 0) {
#pragma unroll
        for (int i = 0; i < NW; ++i) t += smem[i];
    }
    return t;
}

// ---------------------------------------------------------------------------
// host-side helpers
// ---------------------------------------------------------------------------
inline int64_t ceil_div(int64_t a, int64_t b) { return (a + b - 1) / b; }
inline size_t elem_size(int dtype) { return dtype == PRUNE_BF16 ? 2 : 4; }
inline bool aligned_to(const void *p, size_t a) { return (reinterpret_cast<uintptr_t>(p) % a) == 0; }
inline bool valid_dtype(int dtype) { return dtype == PRUNE_F32 || dtype == PRUNE_BF16; }

// rows can be moved as 8-element packets: base 16-byte aligned, width and pitch multiples of 8
inline bool packet_ok(const void *base, int64_t cols, int64_t ld) {
    return aligned_to(base, 16) && (cols % 8 == 0) && (ld % 8 == 0);
}

inline int launch_status() { return hipGetLastError() == hipSuccess ? PRUNE_OK : PRUNE_ERR_DEVICE; }

// ---- column sum-of-squares (used for activation statistics and for the down projection's channel magnitudes)
struct ColsumPlan {
    int tiles_vec;           // blocks along channels on the packet path (2048 channels each)
    int tiles_scalar;        // blocks along channels on the scalar path (256 channels each)
    int stripes;             // blocks along rows
    int64_t rows_per_block;  // rows each stripe covers
};
ColsumPlan plan_colsum(int64_t n_rows, int64_t n_cols);
size_t colsum_workspace_bytes(int64_t n_rows, int64_t n_cols);
// sumsq[j] (+)= sum_t x[t, j]^2 (accumulate picks += or =); norms (optional) = sqrt of the result;
// ws holds the per-stripe partials
int launch_colsum(const void *x, int dtype, int64_t n_rows, int64_t n_cols, int64_t ld, float *sumsq, void *ws,
                  hipStream_t stream, bool accumulate = true, float *norms = nullptr);

size_t score_workspace_bytes(int64_t rows, int64_t cols);
size_t select_workspace_bytes(int64_t rows, int64_t cols);
size_t struct_workspace_bytes(int64_t inter, int64_t hidden);
size_t rank_batch_workspace_bytes();
int launch_rank_groups(const float *group_mag, int64_t n, uint32_t r, int32_t *kept_idx, hipStream_t stream);

}  // namespace mp
