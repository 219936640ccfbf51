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
// the fp32 matrix cores.  R overwrites the upper triangle of h; what the strictly lower triangle holds afterwards is
// unspecified.
#include "gemm_f32.hpp"
#include "tri_inverse.hpp"

namespace mp {

namespace {

constexpr int kNB = kTriN;          // block size of the factorisation
constexpr int kDiagPitch = kTriPitch;
constexpr int kFactorGroup = 4;     // panels whose downdates of the far part of H are applied together

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
//
// The 128 columns are taken in eight groups of 16, last group first.  For a group: sixteen lanes of the first wave
// factor its 16 x 16 diagonal block and invert it, a row per lane, exchanging values lane to lane (no memory, no
// barrier: 16 dependent steps of a square root and a division each, the latency-bound core of the whole
// factorisation); then all threads turn the 16 columns above the block into R's columns with that inverse and
// downdate the groups to the left with the outer product of those columns.  Three barriers per group instead of
// two per column.
__global__ __launch_bounds__(256) void factor_diagonal_block(float *__restrict__ h, int64_t ld, int64_t c0, int sz,
                                                             float *__restrict__ dinv, int *__restrict__ info) {
    __shared__ float d[kNB][kDiagPitch];
    __shared__ float u[kNB][kDiagPitch];
    constexpr int kG = 16, kPanelPitch = 20;  // 80-byte rows: 16-byte aligned, eight rows cover all banks
    static_assert(3 * kG * kG + 2 * kNB * kPanelPitch <= kNB * kDiagPitch, "the scratch fits into u");
    // u is not needed before the inversion at the end: until then it holds what the groups exchange
    float *scratch = &u[0][0];
    float (*blk)[kG] = reinterpret_cast<float (*)[kG]>(scratch);                     // a group's diagonal block
    float (*rb)[kG] = reinterpret_cast<float (*)[kG]>(scratch + kG * kG);            // its factor
    float (*ub)[kG] = reinterpret_cast<float (*)[kG]>(scratch + 2 * kG * kG);        // the factor's inverse
    float (*pd)[kPanelPitch] = reinterpret_cast<float (*)[kPanelPitch]>(scratch + 3 * kG * kG);   // columns above it
    float (*pp)[kPanelPitch] = reinterpret_cast<float (*)[kPanelPitch]>(scratch + 3 * kG * kG + kNB * kPanelPitch);
    const int tid = threadIdx.x, ty = tid >> 4, tx = tid & 15;
    // Thread (ty, tx) of a 16 x 16 grid owns the entries (ty + 16 a, tx + 16 b), a, b = 0..7, in registers.  Rows
    // and columns past sz carry a unit diagonal, which leaves the live part as it is.
    float t[8][8];
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b2 = 0; b2 < 8; ++b2) {
            const int i = ty + 16 * a, k = tx + 16 * b2;
            t[a][b2] = (i < sz && k < sz && i <= k) ? h[(c0 + i) * ld + c0 + k] : (i == k && i >= sz) ? 1.f : 0.f;
        }
    for (int e = tid; e < kNB * kDiagPitch; e += 256) (&d[0][0])[e] = 0.f;
    float uinv[8];  // this thread's entry of the inverse of every group's diagonal block
#pragma unroll
    for (int jb = 7; jb >= 0; --jb) {
        blk[ty][tx] = ty <= tx ? t[jb][jb] : 0.f;
#pragma unroll
        for (int a = 0; a < jb; ++a) pd[ty + 16 * a][tx] = t[a][jb];
        __syncthreads();
        if (tid < kG) {
            // lane i holds row i of the block; last column first: r_jj = sqrt(d_jj), R[i][j] = d[i][j] / r_jj (i < j),
            // d[i][k] -= R[i][j] R[k][j] (i <= k < j).  Entries below the diagonal are carried along and never read.
            const int lane = tid;
            float r[kG], w[kG], rinv_of[kG];  // rinv_of[j] = 1 / r_jj (uniform over the lanes)
#pragma unroll
            for (int q = 0; q < kG; q += 4) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(&blk[lane][q]);
                r[q] = v[0];
                r[q + 1] = v[1];
                r[q + 2] = v[2];
                r[q + 3] = v[3];
            }
#pragma unroll
            for (int j = kG - 1; j >= 0; --j) {
                const float pivot = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r[j]), j));
                if (!(pivot > 0.f) && info && lane == 0) atomicMax(info, static_cast<int>(c0) + 16 * jb + j + 1);
                // 1 / sqrt(pivot) from the hardware approximation and one Newton step (a relative error of a few
                // 2^-24, like a correctly rounded square root followed by a division, in a fifth of the dependent
                // instructions: this chain of 16 steps per group is what the whole block waits for); a pivot that is
                // not positive gives NaN here as it would there
                const float y0 = __builtin_amdgcn_rsqf(pivot);
                const float y1 = fmaf(0.5f * y0, fmaf(-pivot * y0, y0, 1.f), y0);
                rinv_of[j] = y1;
                r[j] = lane < j ? r[j] * y1 : lane == j ? pivot * y1 : 0.f;
#pragma unroll
                for (int k = 0; k < j; ++k) {
                    const float rkj = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r[j]), k));
                    r[k] = fmaf(-r[j], rkj, r[k]);
                }
            }
            // row i of W = R^-1 from W R = I, column by column: w_ik = (delta_ik - sum_{m < k} w_im r_mk) / r_kk
            // (zero for k < i by itself)
#pragma unroll
            for (int k = 0; k < kG; ++k) {
                float acc = lane == k ? 1.f : 0.f;
#pragma unroll
                for (int m = 0; m < k; ++m) {
                    const float rmk = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, r[k]), m));
                    acc = fmaf(-w[m], rmk, acc);
                }
                w[k] = acc * rinv_of[k];
            }
#pragma unroll
            for (int q = 0; q < kG; q += 4) {
                *reinterpret_cast<f32x4 *>(&rb[lane][q]) = f32x4{r[q], r[q + 1], r[q + 2], r[q + 3]};
                *reinterpret_cast<f32x4 *>(&ub[lane][q]) = f32x4{w[q], w[q + 1], w[q + 2], w[q + 3]};
            }
        }
        __syncthreads();
        t[jb][jb] = rb[ty][tx];
        uinv[jb] = ub[ty][tx];
        if (jb > 0) {
            // R[i][c] = sum_m D[i][m] W[c][m] for the rows i above the block (W is zero left of its diagonal)
            float wrow[kG];
#pragma unroll
            for (int q = 0; q < kG; q += 4) {
                const f32x4 v = *reinterpret_cast<const f32x4 *>(&ub[tx][q]);
                wrow[q] = v[0];
                wrow[q + 1] = v[1];
                wrow[q + 2] = v[2];
                wrow[q + 3] = v[3];
            }
#pragma unroll
            for (int a = 0; a < jb; ++a) {
                float acc = 0.f;
#pragma unroll
                for (int q = 0; q < kG; q += 4) {
                    const f32x4 v = *reinterpret_cast<const f32x4 *>(&pd[ty + 16 * a][q]);
#pragma unroll
                    for (int e = 0; e < 4; ++e) acc = fmaf(v[e], wrow[q + e], acc);
                }
                t[a][jb] = acc;
                pp[ty + 16 * a][tx] = acc;
            }
            __syncthreads();
            // d[i][k] -= sum_m R[i][m] R[k][m] for the groups to the left (entries below the diagonal are never
            // read, so they are updated along with the rest)
#pragma unroll
            for (int q = 0; q < kG; q += 4) {
                f32x4 ci[7], ck[7];
#pragma unroll
                for (int a = 0; a < jb; ++a) {
                    ci[a] = *reinterpret_cast<const f32x4 *>(&pp[ty + 16 * a][q]);
                    ck[a] = *reinterpret_cast<const f32x4 *>(&pp[tx + 16 * a][q]);
                }
#pragma unroll
                for (int a = 0; a < jb; ++a)
#pragma unroll
                    for (int b2 = 0; b2 < jb; ++b2)
#pragma unroll
                        for (int e = 0; e < 4; ++e) t[a][b2] = fmaf(-ci[a][e], ck[b2][e], t[a][b2]);
            }
        }
        // (the next group's writes to blk and pd come before its first barrier; blk was last read before this
        // group's second barrier and pd before its third, which every thread has passed by then)
    }
    __syncthreads();  // all reads of the scratch are done: u can be cleared
    for (int e = tid; e < kNB * kDiagPitch; e += 256) (&u[0][0])[e] = 0.f;
    __syncthreads();
#pragma unroll
    for (int a = 0; a < 8; ++a)
#pragma unroll
        for (int b2 = 0; b2 < 8; ++b2) {
            const int i = ty + 16 * a, k = tx + 16 * b2;
            if (i <= k) {
                d[i][k] = t[a][b2];
                if (i < sz && k < sz) h[(c0 + i) * ld + c0 + k] = t[a][b2];
            }
            if (a == b2) u[i][k] = uinv[a];
        }
    __syncthreads();
    invert_upper_triangle<true>(d, u, sz, tid);
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
    // Panels are taken in groups of kFactorGroup (aligned in the matrix).  A finished panel downdates at once only
    // the columns of its own group that are still to be factored; the part left of the group receives the whole
    // group's outer products in one product with a four times longer inner dimension once the group is done.  The
    // downdate is a read-modify-write of the leading part of H with little arithmetic per byte, so this cuts most of
    // the factorisation's memory traffic by four.  (The panels of a group lie side by side in h, so the long product
    // reads them in place.)
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
        const int64_t g0 = (b - b % kFactorGroup) * kNB;  // first column of the panel's group
        if (g0 < c0) {
            // H[0:m, g0:m] -= P P[g0:m]^T: the columns of the group still to come (upper tiles)
            st = launch_gemm_f32<kBNK>(m, static_cast<int>(c0 - g0), sz, -1.f, h + c0, ld_h, h + g0 * ld_h + c0, ld_h, 1.f,
                                       h + g0, ld_h, true, stream, static_cast<int>(g0));
            if (st != PRUNE_OK) return st;
        } else if (g0 > 0) {
            // the group is complete: H[0:g0, 0:g0] -= P_group P_group^T (upper tiles), P_group = R[0:g0, g0:group end)
            const int64_t group_end = g0 + kFactorGroup * kNB < n ? g0 + kFactorGroup * kNB : n;
            st = launch_gemm_f32<kBNK>(static_cast<int>(g0), static_cast<int>(g0), static_cast<int>(group_end - g0), -1.f,
                                       h + g0, ld_h, h + g0, ld_h, 1.f, h, ld_h, true, stream);
            if (st != PRUNE_OK) return st;
        }
    }
    return PRUNE_OK;
}
