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
    for (int s = 16, ls = 4; s < kNB; s *= 2, ++ls) {
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
    // only the live sz x sz part is handed on; the rest of dinv is zero
    for (int e = tid; e < kNB * kNB; e += 256) {
        const int i = e / kNB, k = e % kNB;
        if (i >= sz || k >= sz) u[i][k] = 0.f;
    }
    __syncthreads();
}

}  // namespace mp
