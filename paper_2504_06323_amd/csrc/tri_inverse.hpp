// Inverse of a 128 x 128 upper triangle held in LDS, by 256 threads.
#pragma once

#include "common.hpp"

namespace mp {

constexpr int kTriN = 128;
constexpr int kTriPitch = kTriN + 1;

// d holds the triangle R (sz x sz live part, zeros elsewhere, visible to the block); u is all zero.  On exit u holds
// R^-1 in its live sz x sz part and zeros elsewhere (visible to the block); d is used as scratch below its diagonal
// and gets a unit diagonal past sz.  All 256 threads of the block must call.
// HAVE_DIAG: the caller has already put the inverses of the eight 16 x 16 diagonal blocks into u (and a unit
// diagonal past sz into d and u); the first level is then skipped.
template <bool HAVE_DIAG = false>
__device__ __forceinline__ void invert_upper_triangle(float (&d)[kTriN][kTriPitch], float (&u)[kTriN][kTriPitch], int sz,
                                                      int tid) {
    constexpr int kNB = kTriN;
    // Inverse of the triangle by doubling.  The eight 16 x 16 diagonal blocks are inverted directly, one column
    // per thread (u_jj = 1 / r_jj, u_ij = -(sum_{k = i+1..j} r_ik u_kj) / r_ii); then blocks are merged pairwise:
    //   inv [A B; 0 D] = [inv A, -inv A * B * inv D; 0, inv D]
    // with the intermediate B * inv D parked in the unused lower triangle of d.  Rows and columns past sz carry a
    // unit diagonal, which leaves the live part unchanged.
    if constexpr (!HAVE_DIAG) {
        if (tid < kNB && tid >= sz) d[tid][tid] = 1.f;
        __syncthreads();
        if (tid < kNB) {
            const int j = tid, lo = j & ~15;
            u[j][j] = 1.f / d[j][j];
            for (int i = j - 1; i >= lo; --i) {
                float acc = 0.f;
                for (int k = i + 1; k <= j; ++k) acc = fmaf(d[i][k], u[k][j], acc);
                u[i][j] = -acc / d[i][i];
            }
        }
        __syncthreads();
    }
    // The first merge (16 -> 32: sixteen-wide products, 64 threads) runs on the vector units below; the merges to 64
    // and to 128 are products of 32 x 32 tiles on the matrix cores, one tile per wave.
    for (int s = 16, ls = 4; s < 32; s *= 2, ++ls) {
        // Every pair of this level is an s x s product, cut into 4 x 4 micro-tiles: (kNB / 2s) (s / 4)^2 = 8 s
        // micro-tiles, one per thread (s = 64 uses all 256).  Zeros below the diagonals of inv(A) and inv(D)
        // make the plain products right.
        const int q4 = ls - 2;                       // log2 of micro-tiles per row of a pair
        const bool active = tid < 8 * s;
        const int pair = tid >> (2 * q4), tr = (tid >> q4) & ((1 << q4) - 1), tc = tid & ((1 << q4) - 1);
        const int p = 2 * s * pair, r0 = 4 * tr, cc0 = 4 * tc;
        float acc[4][4];
        // T = B * inv(D): element (r, c) -> d[p + s + r][p + c]
        if (active) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) acc[i][jj] = 0.f;
#pragma unroll 4
            for (int k = 0; k < s; ++k) {
                float av[4], bv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    av[i] = d[p + r0 + i][p + s + k];
                    bv[i] = u[p + s + k][p + s + cc0 + i];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) acc[i][jj] = fmaf(av[i], bv[jj], acc[i][jj]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) d[p + s + r0 + i][p + cc0 + jj] = acc[i][jj];
        }
        __syncthreads();
        // inv(B-part) = -inv(A) * T
        if (active) {
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) acc[i][jj] = 0.f;
#pragma unroll 4
            for (int k = 0; k < s; ++k) {
                float av[4], bv[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    av[i] = u[p + r0 + i][p + k];
                    bv[i] = d[p + s + k][p + cc0 + i];
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int jj = 0; jj < 4; ++jj) acc[i][jj] = fmaf(av[i], bv[jj], acc[i][jj]);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int jj = 0; jj < 4; ++jj) u[p + r0 + i][p + s + cc0 + jj] = -acc[i][jj];
        }
        __syncthreads();
    }
    typedef __attribute__((ext_vector_type(16))) float tri_f32x16;
    const int lane = tid & 63, wave = tid >> 6;
    for (int s = 32; s < kNB; s *= 2) {
        const int tpd = s / 32;                                   // 32-wide tiles along a side of a pair's product
        const bool active = wave < (kNB / (2 * s)) * tpd * tpd;   // two tiles at s = 32, four at s = 64
        const int pair = wave / (tpd * tpd), tr = (wave / tpd) % tpd, tc = wave % tpd;
        const int p = 2 * s * pair, hl = lane >> 5, ll = lane & 31;
        // T = B * inv(D); inv(D) is upper triangular: column tile tc needs the inner indices below 32 (tc + 1)
        if (active) {
            tri_f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            const int k_end = 32 * (tc + 1);
            for (int kc = 0; kc < k_end; kc += 32) {  // 32 inner indices at a time: all operands asked for at once
                float a[16], b[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    a[q] = d[p + 32 * tr + ll][p + s + kc + 2 * q + hl];
                    b[q] = u[p + s + kc + 2 * q + hl][p + s + 32 * tc + ll];
                }
#pragma unroll
                for (int q = 0; q < 16; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q], b[q], acc, 0, 0, 0);
            }
            // accumulator element v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of the tile
#pragma unroll
            for (int v = 0; v < 16; ++v)
                d[p + s + 32 * tr + 8 * (v >> 2) + 4 * hl + (v & 3)][p + 32 * tc + ll] = acc[v];
        }
        __syncthreads();
        // inv(B-part) = -inv(A) * T; inv(A) is upper triangular: row tile tr needs the inner indices from 32 tr on
        if (active) {
            tri_f32x16 acc;
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[v] = 0.f;
            for (int kc = 32 * tr; kc < s; kc += 32) {
                float a[16], b[16];
#pragma unroll
                for (int q = 0; q < 16; ++q) {
                    a[q] = u[p + 32 * tr + ll][p + kc + 2 * q + hl];
                    b[q] = d[p + s + kc + 2 * q + hl][p + 32 * tc + ll];
                }
#pragma unroll
                for (int q = 0; q < 16; ++q) acc = __builtin_amdgcn_mfma_f32_32x32x2f32(a[q], b[q], acc, 0, 0, 0);
            }
#pragma unroll
            for (int v = 0; v < 16; ++v)
                u[p + 32 * tr + 8 * (v >> 2) + 4 * hl + (v & 3)][p + s + 32 * tc + ll] = -acc[v];
        }
        __syncthreads();
    }
    // only the live sz x sz part is handed on; the rest of dinv is zero
    for (int e = tid; e < kNB * kNB; e += 256) {
        const int i = e / kNB, k = e % kNB;
        if (i >= sz || k >= sz) u[i][k] = 0.f;
    }
    __syncthreads();
}

}  // namespace mp
