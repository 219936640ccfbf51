// fp32 matrix product on the matrix cores, the workhorse of the Hessian factorisation and of the
// compensated sweep:   C = beta * C + alpha * A * op(B)
// A [M, K] row-major; op(B) = B for B [K, N] row-major (kBKN) or B^T for B [N, K] row-major (kBNK);
// C [M, N] row-major.  K and every leading dimension are multiples of 4 and all bases 16-byte aligned
// (checked by the callers), M and N are arbitrary.  A block of four waves owns a 128 x 128 tile of C
// (64 x 64 per wave, four 32 x 32 x 2 MFMA accumulators) or, for small products, a 64 x 128 tile (32 x 64 per
// wave); K is walked 32 at a time through a two-stage LDS buffer
// with both operands stored k-major so that a wave reads 32 consecutive floats per MFMA operand.  One owner per
// output element and a fixed order over K: results are reproducible.  C may be the same memory as A when N <= 128
// (a block then reads all of its rows of A before it writes them).
#pragma once

#include "common.hpp"

namespace mp {

enum GemmB { kBKN = 0, kBNK = 1 };

namespace gemm_detail {

typedef __attribute__((ext_vector_type(16))) float f32x16;
constexpr int kTileMN = 128, kTileK = 32, kPitch = kTileMN + 4;

template <int BL, int TM>
__global__ __launch_bounds__(256) void gemm_f32_kernel(int M, int N, int K, float alpha, const float *A, int64_t lda,
                                                       const float *B, int64_t ldb, float beta, float *C,
                                                       int64_t ldc,
                                                       int upper_from) {
    // two stages of both operand slices: a slice is parked in one stage while the matrix cores read the other
    __shared__ __attribute__((aligned(16))) float smem[2][2][kTileK][kPitch];
    static_assert(TM == 128 || TM == 64, "rows of C per block");
    constexpr int TI = TM / 64;  // 32-row tiles of a wave
    const int m0 = blockIdx.y * TM, n0 = blockIdx.x * kTileMN;
    // upper_from >= 0: column j of C is column upper_from + j of a square matrix whose row i is row i of C, and
    // tiles strictly below that matrix's diagonal are not needed
    if (upper_from >= 0 && upper_from + n0 + kTileMN <= m0) return;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = (wave >> 1) * (TM / 2), wn = (wave & 1) * 64;
    f32x16 acc[TI][2];
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    // The next 32-deep slice of both operands is fetched into registers while the matrix cores work on the
    // current one, and parked in LDS afterwards.
    f32x4 ra[4], rbv[4];
    auto fetch = [&](int k0) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = (tid >> 3) + 32 * p, kk = (tid & 7) * 4;
            const f32x4 zero = {0.f, 0.f, 0.f, 0.f};
            if (p < TM / 32)
                ra[p] = (m0 + r < M && k0 + kk < K) ? *reinterpret_cast<const f32x4 *>(A + (m0 + r) * lda + k0 + kk) : zero;
            if (BL == kBNK) {
                rbv[p] = (n0 + r < N && k0 + kk < K) ? *reinterpret_cast<const f32x4 *>(B + (n0 + r) * ldb + k0 + kk)
                                                     : zero;
            } else {
                const int kb = (tid >> 5) + 8 * p, c = (tid & 31) * 4;
                f32x4 v = zero;
                if (k0 + kb < K) {
                    const float *src = B + (k0 + kb) * ldb + n0 + c;
                    if (n0 + c + 4 <= N) {
                        v = *reinterpret_cast<const f32x4 *>(src);
                    } else {
#pragma unroll
                        for (int e = 0; e < 4; ++e)
                            if (n0 + c + e < N) v[e] = src[e];
                    }
                }
                rbv[p] = v;
            }
        }
    };
    auto park = [&](int stage) {
        float (&sa)[kTileK][kPitch] = smem[stage][0];
        float (&sb)[kTileK][kPitch] = smem[stage][1];
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int r = (tid >> 3) + 32 * p, kk = (tid & 7) * 4;
            if (p < TM / 32) {
#pragma unroll
                for (int e = 0; e < 4; ++e) sa[kk + e][r] = ra[p][e];
            }
            if (BL == kBNK) {
#pragma unroll
                for (int e = 0; e < 4; ++e) sb[kk + e][r] = rbv[p][e];
            } else {
                const int kb = (tid >> 5) + 8 * p, c = (tid & 31) * 4;
                *reinterpret_cast<f32x4 *>(&sb[kb][c]) = rbv[p];
            }
        }
    };
    fetch(0);
    park(0);
    __syncthreads();
    int stage = 0;
    for (int k0 = 0; k0 < K; k0 += kTileK, stage ^= 1) {
        const bool more = k0 + kTileK < K;
        if (more) fetch(k0 + kTileK);
        float (&sa)[kTileK][kPitch] = smem[stage][0];
        float (&sb)[kTileK][kPitch] = smem[stage][1];
#pragma unroll
        for (int kk = 0; kk < kTileK; kk += 2) {
            const int k = kk + (lane >> 5), c = lane & 31;
            float a[TI], b[2];
#pragma unroll
            for (int i = 0; i < TI; ++i) a[i] = sa[k][wm + 32 * i + c];
#pragma unroll
            for (int j = 0; j < 2; ++j) b[j] = sb[k][wn + 32 * j + c];
#pragma unroll
            for (int i = 0; i < TI; ++i)
#pragma unroll
                for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x2f32(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        // the other stage was last read before the barrier that ended the previous step: it can be written now,
        // while the matrix cores still work on this one
        if (more) park(stage ^ 1);
        __syncthreads();
    }
    // Accumulator element v of lane l: row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of its 32 x 32 tile.
    // When C allows 16-byte accesses, a wave passes its tile through LDS eight rows at a time (the operand
    // slices are dead by now), so that the update of C runs in 256-byte runs of 16 bytes per lane instead of
    // 4-byte accesses: with K as short as it is here, reading and writing C is most of the memory traffic.
    const bool wide = (ldc % 4 == 0) && (reinterpret_cast<uintptr_t>(C) % 16 == 0);
    if (wide) {
        constexpr int kEpPitch = 64 + 4;
        float *ep = &smem[0][0][0][0] + wave * (8 * kEpPitch);
        static_assert(4 * 8 * kEpPitch <= 2 * kTileK * kPitch, "the epilogue buffer fits in the operand slices");
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
            for (int vq = 0; vq < 4; ++vq) {
#pragma unroll
                for (int j = 0; j < 2; ++j)
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        ep[(4 * (lane >> 5) + e) * kEpPitch + 32 * j + (lane & 31)] = acc[i][j][4 * vq + e];
                // (only this wave touches its part of the buffer: LDS operations of a wave complete in order)
#pragma unroll
                for (int q = 0; q < 2; ++q) {
                    const int rr = (lane + 64 * q) >> 4, c4 = ((lane + 64 * q) & 15) * 4;
                    const f32x4 mine = *reinterpret_cast<const f32x4 *>(&ep[rr * kEpPitch + c4]);
                    const int row = m0 + wm + 32 * i + 8 * vq + rr, col = n0 + wn + c4;
                    if (row < M && col < N) {
                        float *dst = C + row * ldc + col;
                        if (col + 4 <= N) {
                            f32x4 out;
                            if (beta == 0.f) {
#pragma unroll
                                for (int e = 0; e < 4; ++e) out[e] = alpha * mine[e];
                            } else {
                                const f32x4 old = *reinterpret_cast<const f32x4 *>(dst);
#pragma unroll
                                for (int e = 0; e < 4; ++e) out[e] = beta * old[e] + alpha * mine[e];
                            }
                            *reinterpret_cast<f32x4 *>(dst) = out;
                        } else {
#pragma unroll
                            for (int e = 0; e < 4; ++e)
                                if (col + e < N) dst[e] = beta == 0.f ? alpha * mine[e] : beta * dst[e] + alpha * mine[e];
                        }
                    }
                }
            }
        return;
    }
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = m0 + wm + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int col = n0 + wn + 32 * j + (lane & 31);
                if (row < M && col < N) {
                    float *dst = C + row * ldc + col;
                    const float prod = alpha * acc[i][j][v];
                    *dst = beta == 0.f ? prod : beta * *dst + prod;
                }
            }
}

}  // namespace gemm_detail

inline bool gemm_operands_ok(const void *a, int64_t lda, const void *b, int64_t ldb, const void *c, int64_t K) {
    return aligned_to(a, 16) && aligned_to(b, 16) && aligned_to(c, 4) && lda % 4 == 0 && ldb % 4 == 0 && K % 4 == 0;
}

// C = beta * C + alpha * A * op(B) on `stream`; upper_tiles_only skips the 128 x 128 tiles strictly below
// the diagonal of C (for symmetric updates of which only the upper triangle is used); when C is a block of
// columns of a square matrix that starts at column upper_col0 (and at row 0), the diagonal meant is that
// matrix's.  M, N < 2^31 / 128.
template <int BL>
inline int launch_gemm_f32(int M, int N, int K, float alpha, const float *A, int64_t lda, const float *B, int64_t ldb,
                           float beta, float *C, int64_t ldc, bool upper_tiles_only, hipStream_t stream,
                           int upper_col0 = 0) {
    if (M <= 0 || N <= 0) return PRUNE_OK;
    const int64_t tiles_n = ceil_div(N, gemm_detail::kTileMN), tiles_m = ceil_div(M, gemm_detail::kTileMN);
    // A product with fewer 128-row tiles than the chip has compute units is a link in a chain of short kernels:
    // 64-row tiles halve the time of each block and double their number (same operations on every element).
    const bool small = tiles_n * tiles_m <= 256;
    const dim3 grid(static_cast<unsigned>(tiles_n), static_cast<unsigned>(small ? ceil_div(M, 64) : tiles_m));
    if (grid.y > 65535) return PRUNE_ERR_SHAPE;
    if (small)
        hipLaunchKernelGGL((gemm_detail::gemm_f32_kernel<BL, 64>), grid, dim3(256), 0, stream, M, N, K, alpha, A, lda, B,
                           ldb, beta, C, ldc, upper_tiles_only ? upper_col0 : -1);
    else
        hipLaunchKernelGGL((gemm_detail::gemm_f32_kernel<BL, 128>), grid, dim3(256), 0, stream, M, N, K, alpha, A, lda,
                           B, ldb, beta, C, ldc, upper_tiles_only ? upper_col0 : -1);
    return launch_status();
}

}  // namespace mp
