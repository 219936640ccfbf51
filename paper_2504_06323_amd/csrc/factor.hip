// Factor of the damped Hessian for the Hessian-based one-shot pruner (Section 4.1.3, "Pruning
// Methods").  The published algorithm works with U, the upper Cholesky factor of
// H^-1 (H^-1 = U^T U).  Its inverse R = U^-1 is upper triangular too and satisfies H = R R^T, so it is a
// Cholesky factorisation of H taken from the last row and column upwards -- one factorisation, no explicit
// inverse of the n x n matrix -- and the sweep can be written in terms of R (see sweep.hip).
//
// Steps: (1) channels that never fired (H_jj == 0) get H_jj = 1 and are reported; damp * mean(diag H) is added
// to the diagonal; (2) blocked right-looking factorisation from the last 128-column block to the first: factor
// the diagonal block in LDS (and invert that 128 x 128 triangle), turn the column panel above it into R's
// panel with one product, and downdate the leading part with the panel's outer product.  The products run on
// the fp32 matrix cores.  R overwrites the upper triangle of h; the strictly lower triangle is left as it was.
#include "gemm_f32.hpp"
#include "tri_inverse.hpp"

namespace mp {

namespace {

constexpr int kNB = kTriN;          // block size of the factorisation
constexpr int kDiagPitch = kTriPitch;

// dead[j] = (h_jj == 0); those get h_jj = 1; then h_jj += damp * mean(diag).  One block; the mean is a double sum in
// a fixed order.
__global__ __launch_bounds__(1024) void damp_diagonal(float *__restrict__ h, int64_t n, int64_t ld, double damp,
                                                      uint8_t *__restrict__ dead, int *__restrict__ info) {
    __shared__ double part[1024];
    const int tid = threadIdx.x;
    double s = 0.0;
    for (int64_t j = tid; j < n; j += 1024) {
        const float d = h[j * ld + j];
        const bool is_dead = d == 0.f;
        if (dead) dead[j] = is_dead ? 1 : 0;
        s += is_dead ? 1.0 : static_cast<double>(d);
    }
    part[tid] = s;
    __syncthreads();
    for (int w = 512; w > 0; w >>= 1) {
        if (tid < w) part[tid] += part[tid + w];
        __syncthreads();
    }
    const double add = damp * (part[0] / static_cast<double>(n));
    for (int64_t j = tid; j < n; j += 1024) {
        const float d = h[j * ld + j];
        h[j * ld + j] = static_cast<float>((d == 0.f ? 1.0 : static_cast<double>(d)) + add);
    }
    if (tid == 0 && info) *info = 0;
}

// One block.  D = h[c0 : c0 + sz, c0 : c0 + sz] (its upper triangle) -> R_bb with D = R_bb R_bb^T, written back
// over the upper triangle, and inv(R_bb) (upper triangular, zeros below) to dinv [kNB x kNB] (pitch kNB, the part
// beyond sz zero-filled).  A pivot that is not positive is reported in *info (1-based column) and poisons the
// block with NaN rather than stopping.
__global__ __launch_bounds__(256) void factor_diagonal_block(float *__restrict__ h, int64_t ld, int64_t c0, int sz,
                                                             float *__restrict__ dinv, int *__restrict__ info) {
    __shared__ float d[kNB][kDiagPitch];
    __shared__ float u[kNB][kDiagPitch];
    __shared__ float col[kNB];
    __shared__ float piv;
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    // The factorisation keeps the block in registers: thread (ty, tx) of a 16 x 16 grid owns the entries
    // (ty + 16 a, tx + 16 b), a, b = 0..7; only the scaled column of a step travels through LDS, so no step waits
    // on a read-modify-write of LDS.
    float t[8][8];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b2 = 0; b2 < 8; ++b2) {
            const int i = ty + 16 * a, k = tx + 16 * b2;
            t[a][b2] = (i < sz && k < sz && i <= k) ? h[(c0 + i) * ld + c0 + k] : 0.f;
        }
    for (int e = tid; e < kNB * kDiagPitch; e += 256) {
        (&d[0][0])[e] = 0.f;
        (&u[0][0])[e] = 0.f;
    }
    if (tid < kNB) col[tid] = 0.f;
    __syncthreads();
    // last column first: r_jj = sqrt(d_jj); R[i][j] = d[i][j] / r_jj (i < j); d[i][k] -= R[i][j] R[k][j] (i <= k < j).
    // The 16-wide group jb of column j is a compile-time constant of the unrolled outer loop, so every register
    // of t is addressed statically; jt = j % 16 runs inside.
    const int last = sz - 1;
#pragma unroll
    for (int jb = 7; jb >= 0; --jb) {
        if (jb > (last >> 4)) continue;  // uniform: groups past the live part
        for (int jt = (jb == (last >> 4) ? (last & 15) : 15); jt >= 0; --jt) {
            const int j = 16 * jb + jt;
            if (ty == jt && tx == jt) {
                const float pivot = t[jb][jb];
                if (!(pivot > 0.f) && info) atomicMax(info, static_cast<int>(c0) + j + 1);
                piv = sqrtf(pivot);
            }
            __syncthreads();
            const float rjj = piv;
            if (tx == jt) {
#pragma unroll
                for (int a = 0; a <= jb; ++a) {
                    const int i = ty + 16 * a;
                    if (i < j) t[a][jb] = t[a][jb] / rjj;
                    if (i == j) t[a][jb] = rjj;
                    if (i <= j) col[i] = t[a][jb];
                }
            }
            __syncthreads();
            // Entries (i <= k < j) must be downdated.  Entries below the diagonal are never read, so they may be
            // updated along with the rest (with whatever col holds for them); the one condition left is k < j in
            // the column group of j itself.
            float ci[8], ck[8];
#pragma unroll
            for (int a = 0; a <= jb; ++a) {
                ci[a] = col[ty + 16 * a];
                ck[a] = col[tx + 16 * a];
            }
            ck[jb] = tx < jt ? ck[jb] : 0.f;
#pragma unroll
            for (int b2 = 0; b2 <= jb; ++b2)
#pragma unroll
                for (int a = 0; a <= jb; ++a) t[a][b2] = fmaf(-ci[a], ck[b2], t[a][b2]);
            // (the next step's writes to col and piv come after its first barrier, which every thread reaches only
            // after these reads)
        }
    }
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b2 = 0; b2 < 8; ++b2) {
            const int i = ty + 16 * a, k = tx + 16 * b2;
            if (i < sz && k < sz && i <= k) {
                h[(c0 + i) * ld + c0 + k] = t[a][b2];
                d[i][k] = t[a][b2];
            }
        }
    __syncthreads();
    invert_upper_triangle(d, u, sz, tid);
    for (int e = tid; e < kNB * kNB; e += 256) dinv[e] = u[e / kNB][e % kNB];
}

}  // namespace

size_t factor_workspace_bytes() { return static_cast<size_t>(kNB) * kNB * sizeof(float); }

}  // namespace mp

extern "C" size_t prune_hessian_factor_workspace_bytes(int64_t n) {
    return n > 0 ? (mp::factor_workspace_bytes() + 255) / 256 * 256 : 0;
}

extern "C" int prune_hessian_factor(float *h, int64_t n, int64_t ld_h, double damp, uint8_t *dead, int *info, void *ws,
                                    size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (n <= 0 || ld_h < n || n > (int64_t(1) << 20)) return PRUNE_ERR_SHAPE;
    if (n % 4 != 0 || ld_h % 4 != 0) return PRUNE_ERR_SHAPE;
    if (!h || !ws) return PRUNE_ERR_NULL;
    if (!(damp >= 0.0)) return PRUNE_ERR_RANGE;
    if (!aligned_to(h, 16) || !aligned_to(ws, 16) || (info && !aligned_to(info, 4))) return PRUNE_ERR_ALIGNMENT;
    if (ws_bytes < factor_workspace_bytes()) return PRUNE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    float *dinv = static_cast<float *>(ws);
    hipLaunchKernelGGL(damp_diagonal, dim3(1), dim3(1024), 0, stream, h, n, ld_h, damp, dead, info);
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    const int64_t n_blocks = ceil_div(n, kNB);
    for (int64_t b = n_blocks - 1; b >= 0; --b) {
        const int64_t c0 = b * kNB;
        const int sz = static_cast<int>(n - c0 < kNB ? n - c0 : kNB);
        hipLaunchKernelGGL(factor_diagonal_block, dim3(1), dim3(256), 0, stream, h, ld_h, c0, sz, dinv, info);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        if (c0 == 0) break;
        const int m = static_cast<int>(c0);
        // panel: R[0:m, block] = H[0:m, block] * inv(R_bb)^T, in place (a block of the product owns whole rows)
        int st = launch_gemm_f32<kBNK>(m, sz, sz, 1.f, h + c0, ld_h, dinv, kNB, 0.f, h + c0, ld_h, false, stream);
        if (st != PRUNE_OK) return st;
        // downdate: H[0:m, 0:m] -= P P^T (upper tiles)
        st = launch_gemm_f32<kBNK>(m, m, sz, -1.f, h + c0, ld_h, h + c0, ld_h, 1.f, h, ld_h, true, stream);
        if (st != PRUNE_OK) return st;
    }
    return PRUNE_OK;
}
