// The compensated left-to-right sweep of the Hessian-based one-shot pruner with weight compensation
// (Section 4.1.3, "Pruning Methods"), with the sparsity target that the Projection Planner gives the
// projection (Section 3.3).
//
// The published algorithm is written with U, the upper Cholesky factor of H^-1: in column j the error
// e = (w_j - w'_j) / U_jj is spread to the right with row j of U.  Here it runs on R = U^-1 (H = R R^T, from
// prune_hessian_factor), which needs no n x n inverse.  Summing the updates, W - W' = E U, hence E = (W - W') R:
// with D = W - W' (the change of every finished column) and G_j = sum_{i<j} D_i R_ij,
//     V_j = w_j R_jj + G_j
// is, once every column before j is finished, the current weight of column j divided by U_jj = 1 / R_jj: a kept
// entry becomes w' = V_j / R_jj, a pruned one 0, and finishing column j adds D_j R_j,j' to every later G_j'.
// The selection, however, looks at a whole block when only the columns before the block are finished.  The
// published sweep's weights at that moment are W_block + G_block inv(R_bb) (R_bb the diagonal block of R; this is
// the block form of U = R^-1), so the saliencies (w / U_jj)^2 of a block need one 128 x 128 triangular inverse and
// one small product per block.
// Per block of 128 columns: (1) T = G_block inv(R_bb), saliency ((w + T) R_jj)^2, in one kernel; (2) the
// floor(s * rows * width) smallest saliencies of the block are found exactly by a radix search over all rows
// together (ties by row-major position); (3) the 128 columns are walked in order, a lane per row with the block of
// R in LDS (or, for ragged blocks, a wave per two rows); (4) fp32 matrix-core products add D R[finished, later] to G: after every block for the rest
// of its group of four blocks, after every group for everything beyond it.
#include "gemm_f32.hpp"
#include "tri_inverse.hpp"

namespace mp {

namespace {

constexpr int kSB = 128;  // columns per block
constexpr int kGroup = 4; // blocks per group: columns beyond the group receive a group's changes in one product
constexpr int kSBPitch = kSB + 1;
constexpr int kHistBins = 2048;

struct SweepState {
    uint32_t prefix, need, key, need_eq, count_eq, pad0, pad1, pad2;
};

__device__ __forceinline__ uint32_t saliency_key(float saliency) { return __float_as_uint(saliency) & 0x7fffffffu; }

__device__ __forceinline__ bf16_t narrow_bf16(float f) {  // round to nearest, ties to even
    const uint32_t b = __float_as_uint(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>(0x7fc0u);
    return static_cast<bf16_t>((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ void store_as(bf16_t *p, float f) { *p = narrow_bf16(f); }
__device__ __forceinline__ void store_as(float *p, float f) { *p = f; }

__global__ __launch_bounds__(256) void sweep_zero(float *__restrict__ g, int64_t n) {
    for (int64_t e = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; e < n;
         e += static_cast<int64_t>(gridDim.x) * 256)
        g[e] = 0.f;
}

// inv(R_bb) of the diagonal blocks first_block + blockIdx.x of R, each to a dense [128 x 128] slot (zero padded)
__global__ __launch_bounds__(256) void invert_diagonal_blocks(const float *__restrict__ r, int64_t ld_r, int64_t cols,
                                                              int64_t first_block, float *__restrict__ dinv_all) {
    __shared__ float d[kTriN][kTriPitch];
    __shared__ float u[kTriN][kTriPitch];
    const int tid = threadIdx.x;
    const int64_t c0 = (first_block + blockIdx.x) * kSB;
    const int sz = static_cast<int>(cols - c0 < kSB ? cols - c0 : kSB);
    for (int e = tid; e < kTriN * kTriN; e += 256) {
        const int i = e >> 7, k = e & (kTriN - 1);
        d[i][k] = (i < sz && k < sz && i <= k) ? r[(c0 + i) * ld_r + c0 + k] : 0.f;
        u[i][k] = 0.f;
    }
    __syncthreads();
    invert_upper_triangle(d, u, sz, tid);
    float *out = dinv_all + static_cast<int64_t>(blockIdx.x) * (kSB * kSB);
    for (int e = tid; e < kSB * kSB; e += 256) out[e] = u[e >> 7][e & (kSB - 1)];
}

// the search's global histogram is all zero between passes; this clears it once per call
__global__ __launch_bounds__(1024) void select_reset(uint32_t *hist) {
    for (int b = threadIdx.x; b < kHistBins; b += 1024) hist[b] = 0u;
}

// Saliency of the block's entries at the moment the block starts, ((w + t) * R_jj)^2 with t = G_block inv(R_bb),
// stored for the later passes and for the sweep, and the first pass of the radix search over them.  A block takes
// 16 rows: their part of G goes to LDS, a thread owns one column for eight of the rows and walks the column of
// inv(R_bb) once (sums in ascending order of the inner index, fused multiply-adds).
template <typename T>
__global__ __launch_bounds__(256) void saliency_first_pass(const T *__restrict__ w, int64_t ld_w,
                                                           const float *__restrict__ r, int64_t ld_r,
                                                           const uint8_t *__restrict__ dead, const float *__restrict__ g,
                                                           int64_t ldg, const float *__restrict__ dinv, int64_t rows,
                                                           int64_t c0, int width, float *__restrict__ sal,
                                                           int64_t ld_sal, uint32_t *__restrict__ hist) {
    __shared__ uint32_t h[kHistBins];
    __shared__ __attribute__((aligned(16))) float gs[16][kSB];
    const int tid = threadIdx.x;
    for (int b = tid; b < kHistBins; b += 256) h[b] = 0u;
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * 16;
    for (int e = tid; e < 16 * kSB; e += 256) {
        const int64_t row = r0 + (e >> 7);
        const int col = e & (kSB - 1);
        gs[e >> 7][col] = (row < rows && col < width) ? g[row * ldg + c0 + col] : 0.f;
    }
    __syncthreads();
    const int col = tid & (kSB - 1), rh = tid >> 7;  // rows r0 + rh + 2 q, q = 0..7
    float acc[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    // inv(R_bb) is upper triangular and zero padded: the terms past the column's own index add nothing, and the
    // width is a multiple of four
#pragma unroll 2
    for (int m = 0; m < width; m += 4) {
        float dv[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) dv[u] = dinv[(m + u) * kSB + col];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const f32x4 gv = *reinterpret_cast<const f32x4 *>(&gs[rh + 2 * q][m]);
#pragma unroll
            for (int u = 0; u < 4; ++u) acc[q] = fmaf(gv[u], dv[u], acc[q]);
        }
    }
    if (col < width) {
        const bool off = dead && dead[c0 + col];
        const float rjj = r[(c0 + col) * ld_r + c0 + col];
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const int64_t row = r0 + rh + 2 * q;
            if (row < rows) {
                const float current = (off ? 0.f : widen(w[row * ld_w + c0 + col])) + acc[q];
                const float scaled = __fmul_rn(current, rjj);
                const float s2 = __fmul_rn(scaled, scaled);
                sal[row * ld_sal + col] = s2;
                atomicAdd(&h[saliency_key(s2) >> 20], 1u);
            }
        }
    }
    __syncthreads();
    for (int b = tid; b < kHistBins; b += 256)
        if (h[b]) atomicAdd(&hist[b], h[b]);
}

// digits of the 31-bit key: bits 30..20, 19..10, 9..0
template <int PASS>
__global__ __launch_bounds__(256) void select_hist(const float *__restrict__ v, int64_t ldv, int64_t c0, int width,
                                                   int64_t rows, const SweepState *__restrict__ state,
                                                   uint32_t *__restrict__ hist) {
    constexpr int kBins = PASS == 0 ? 2048 : 1024;
    __shared__ uint32_t h[kBins];
    const int tid = threadIdx.x;
    for (int b = tid; b < kBins; b += 256) h[b] = 0u;
    const uint32_t prefix = state->prefix;
    __syncthreads();
    const int64_t r0 = static_cast<int64_t>(blockIdx.x) * 16;
    for (int e = tid; e < 16 * kSB; e += 256) {
        const int64_t row = r0 + (e >> 7);
        const int col = e & (kSB - 1);
        if (row < rows && col < width) {
            const uint32_t key = saliency_key(v[row * ldv + c0 + col]);
            if (PASS == 0)
                atomicAdd(&h[key >> 20], 1u);
            else if (PASS == 1) {
                if ((key >> 20) == prefix) atomicAdd(&h[(key >> 10) & 1023u], 1u);
            } else {
                if ((key >> 10) == prefix) atomicAdd(&h[key & 1023u], 1u);
            }
        }
    }
    __syncthreads();
    for (int b = tid; b < kBins; b += 256)
        if (h[b]) atomicAdd(&hist[b], h[b]);
}

// One block: find the bin of the `need`-th smallest key, extend the prefix, clear the histogram.
template <int PASS>
__global__ __launch_bounds__(1024) void select_locate(SweepState *state, uint32_t *hist, uint32_t k) {
    constexpr int kBins = PASS == 0 ? 2048 : 1024;
    constexpr int kPer = kBins / 1024;
    constexpr int kBits = PASS == 0 ? 11 : 10;
    __shared__ uint32_t wave_tot[16];
    __shared__ uint32_t found[3];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const uint32_t need = PASS == 0 ? k : state->need, prefix = PASS == 0 ? 0u : state->prefix;  // pass 0 starts the search
    uint32_t mine[kPer], s = 0;
#pragma unroll
    for (int i = 0; i < kPer; ++i) {
        mine[i] = hist[tid * kPer + i];
        s += mine[i];
    }
    const uint32_t incl = wave_inclusive_scan(s);
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    uint32_t excl = incl - s;
    for (int i = 0; i < wv; ++i) excl += wave_tot[i];
    if (excl < need && need <= excl + s) {
        uint32_t run = excl;
#pragma unroll
        for (int i = 0; i < kPer; ++i) {
            if (run < need && need <= run + mine[i]) {
                found[0] = static_cast<uint32_t>(tid * kPer + i);
                found[1] = run;
                found[2] = mine[i];
            }
            run += mine[i];
        }
    }
#pragma unroll
    for (int i = 0; i < kPer; ++i) hist[tid * kPer + i] = 0u;
    __syncthreads();
    if (tid == 0) {
        const uint32_t np = (prefix << kBits) | found[0], nn = need - found[1];
        state->prefix = np;
        state->need = nn;
        if (PASS == 2) {
            state->key = np;
            state->need_eq = nn;
            state->count_eq = found[2];
        }
    }
}

// number of entries of each row of the block that carry the threshold key (only needed when not all of them go)
__global__ __launch_bounds__(256) void tie_count(const float *__restrict__ v, int64_t ldv, int64_t c0, int width,
                                                 int64_t rows, const SweepState *__restrict__ state,
                                                 uint32_t *__restrict__ row_eq) {
    if (state->need_eq == state->count_eq) return;
    const int lane = threadIdx.x & 63;
    const uint32_t skey = state->key;
    for (int64_t row = static_cast<int64_t>(blockIdx.x) * 4 + (threadIdx.x >> 6); row < rows;
         row += static_cast<int64_t>(gridDim.x) * 4) {
        uint32_t n = 0;
        for (int col = lane; col < width; col += 64) n += saliency_key(v[row * ldv + c0 + col]) == skey ? 1u : 0u;
        n = wave_sum(n);
        if (lane == 0) row_eq[row] = n;
    }
}

// row_before[i] = sum of row_eq over rows before i (one block)
__global__ __launch_bounds__(1024) void tie_scan(const uint32_t *__restrict__ row_eq, uint32_t *__restrict__ row_before,
                                                 int64_t rows, const SweepState *__restrict__ state) {
    if (state->need_eq == state->count_eq) return;
    __shared__ uint32_t wave_tot[16];
    const int tid = threadIdx.x, lane = tid & 63, wv = tid >> 6;
    const int64_t per = (rows + 1023) / 1024, lo = tid * per < rows ? tid * per : rows, hi = lo + per < rows ? lo + per : rows;
    uint32_t s = 0;
    for (int64_t i = lo; i < hi; ++i) s += row_eq[i];
    const uint32_t incl = wave_inclusive_scan(s);
    if (lane == 63) wave_tot[wv] = incl;
    __syncthreads();
    uint32_t run = incl - s;
    for (int i = 0; i < wv; ++i) run += wave_tot[i];
    for (int64_t i = lo; i < hi; ++i) {
        row_before[i] = run;
        run += row_eq[i];
    }
}

__device__ __forceinline__ float lane_value(float x, int lane) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(x), lane));
}

// A wave walks the columns of the block in order for NR rows at once (the rows are independent chains of
// dependent operations, so they hide each other's latency).  mode: 0 nothing is pruned, 1 by the searched
// threshold, 2 everything.  Lane l owns columns l and l + 64 of the block.
// Eight waves share a block's copy of R in LDS (two blocks fit a compute unit: four waves per SIMD); two rows per
// wave measured best for every row count of the model shapes.
constexpr int kSweepThreads = 512, kSweepWaves = kSweepThreads / 64, kSweepRows = 2;

template <typename T, int NR>
__global__ __launch_bounds__(kSweepThreads) void sweep_block(const T *w, int64_t ld_w, T *w_out, int64_t ld_out,
                                                   const float *__restrict__ r, int64_t ld_r,
                                                   const uint8_t *__restrict__ dead, const float *__restrict__ g, int64_t ldg,
                                                   const float *__restrict__ sal, int64_t ld_sal, int64_t rows,
                                                   int64_t c0, int width, int mode,
                                                   const SweepState *__restrict__ state,
                                                   const uint32_t *__restrict__ row_before, float *__restrict__ dblk,
                                                   int64_t ld_d,
                                                   uint32_t *__restrict__ mask_bits, int64_t words_per_row,
                                                   int64_t cols) {
    __shared__ float rb[kSB][kSBPitch];
    __shared__ float rinv[kSB];
    const int tid = threadIdx.x, lane = tid & 63;
    for (int e = tid; e < kSB * kSB; e += kSweepThreads) {
        const int i = e >> 7, k = e & (kSB - 1);
        rb[i][k] = (i <= k && k < width) ? r[(c0 + i) * ld_r + c0 + k] : 0.f;
    }
    if (tid < kSB) rinv[tid] = tid < width ? 1.f / r[(c0 + tid) * ld_r + c0 + tid] : 0.f;
    __syncthreads();
    uint32_t skey = 0u, need_eq = 0u;
    bool all_eq = true;
    if (mode == 1) {
        skey = state->key;
        need_eq = state->need_eq;
        all_eq = need_eq == state->count_eq;
    }
    const bool valid0 = lane < width, valid1 = lane + 64 < width;
    const bool dead0 = valid0 && dead && dead[c0 + lane], dead1 = valid1 && dead && dead[c0 + lane + 64];
    const int n0 = width < 64 ? width : 64;
    const float rd0 = valid0 ? rb[lane][lane] : 0.f, rd1 = valid1 ? rb[lane + 64][lane + 64] : 0.f;
    const unsigned long long live0 = __ballot(valid0), live1 = __ballot(valid1);
    for (int64_t base = (static_cast<int64_t>(blockIdx.x) * kSweepWaves + (tid >> 6)) * NR; base < rows;
         base += static_cast<int64_t>(gridDim.x) * kSweepWaves * NR) {
        float v0[NR], v1[NR], w0[NR], w1[NR], o0[NR], o1[NR], d0[NR], d1[NR];
        unsigned long long pm0[NR], pm1[NR];  // which columns of the row are pruned (uniform over the wave)
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            const int64_t row = base + q;
            const bool live = row < rows;
            w0[q] = (live && valid0 && !dead0) ? widen(w[row * ld_w + c0 + lane]) : 0.f;
            w1[q] = (live && valid1 && !dead1) ? widen(w[row * ld_w + c0 + lane + 64]) : 0.f;
            v0[q] = (live && valid0) ? fmaf(w0[q], rd0, g[row * ldg + c0 + lane]) : 0.f;
            v1[q] = (live && valid1) ? fmaf(w1[q], rd1, g[row * ldg + c0 + lane + 64]) : 0.f;
            bool p0 = mode == 2 && valid0, p1 = mode == 2 && valid1;
            if (mode == 1) {
                const uint32_t k0 = (live && valid0) ? saliency_key(sal[row * ld_sal + lane]) : 0xffffffffu;
                const uint32_t k1 = (live && valid1) ? saliency_key(sal[row * ld_sal + lane + 64]) : 0xffffffffu;
                const bool e0 = k0 == skey, e1 = k1 == skey;
                if (all_eq) {
                    p0 = k0 <= skey;
                    p1 = k1 <= skey;
                } else {  // of the entries with the threshold key, the first need_eq in row-major order go
                    const unsigned long long b0 = __ballot(e0), b1 = __ballot(e1);
                    const unsigned long long below = (1ull << lane) - 1ull;
                    const uint32_t before = live ? row_before[row] : 0u;
                    const uint32_t rank0 = before + __popcll(b0 & below);
                    const uint32_t rank1 = before + __popcll(b0) + __popcll(b1 & below);
                    p0 = k0 < skey || (e0 && rank0 < need_eq);
                    p1 = k1 < skey || (e1 && rank1 < need_eq);
                }
            }
            pm0[q] = __ballot(p0);
            pm1[q] = __ballot(p1);
            o0[q] = o1[q] = d0[q] = d1[q] = 0.f;
        }
        // columns 0..63 of the block; the rows of R for four columns are fetched from LDS before the first of them is
        // needed, so that a column's chain of dependent operations does not start with an LDS round trip
        auto col_lo = [&](int j, float ri, float rl0, float rl1) {
#pragma unroll
            for (int q = 0; q < NR; ++q) {
                const float vj = lane_value(v0[q], j), wj = lane_value(w0[q], j);
                const float wnew = ((pm0[q] >> j) & 1ull) ? 0.f : __fmul_rn(vj, ri);
                const float dj = wj - wnew;
                if (lane == j) {
                    o0[q] = wnew;
                    d0[q] = dj;
                }
                v0[q] = fmaf(dj, rl0, v0[q]);
                v1[q] = fmaf(dj, rl1, v1[q]);
            }
        };
        auto col_hi = [&](int j, float ri, float rl1) {  // columns 64..127
#pragma unroll
            for (int q = 0; q < NR; ++q) {
                const float vj = lane_value(v1[q], j - 64), wj = lane_value(w1[q], j - 64);
                const float wnew = ((pm1[q] >> (j - 64)) & 1ull) ? 0.f : __fmul_rn(vj, ri);
                const float dj = wj - wnew;
                if (lane + 64 == j) {
                    o1[q] = wnew;
                    d1[q] = dj;
                }
                v1[q] = fmaf(dj, rl1, v1[q]);
            }
        };
        int j = 0;
        for (; j + 4 <= n0; j += 4) {
            float ri[4], rl0[4], rl1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ri[u] = rinv[j + u];
                rl0[u] = lane > j + u ? rb[j + u][lane] : 0.f;
                rl1[u] = rb[j + u][lane + 64];
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) col_lo(j + u, ri[u], rl0[u], rl1[u]);
        }
        for (; j < n0; ++j) col_lo(j, rinv[j], lane > j ? rb[j][lane] : 0.f, rb[j][lane + 64]);
        for (j = 64; j + 4 <= width; j += 4) {
            float ri[4], rl1[4];
#pragma unroll
            for (int u = 0; u < 4; ++u) {
                ri[u] = rinv[j + u];
                rl1[u] = lane + 64 > j + u ? rb[j + u][lane + 64] : 0.f;
            }
#pragma unroll
            for (int u = 0; u < 4; ++u) col_hi(j + u, ri[u], rl1[u]);
        }
        for (; j < width; ++j) col_hi(j, rinv[j], lane + 64 > j ? rb[j][lane + 64] : 0.f);
#pragma unroll
        for (int q = 0; q < NR; ++q) {
            const int64_t row = base + q;
            if (row >= rows) break;  // uniform
            if (valid0) store_as(w_out + row * ld_out + c0 + lane, o0[q]);
            if (valid1) store_as(w_out + row * ld_out + c0 + lane + 64, o1[q]);
            dblk[row * ld_d + lane] = d0[q];
            dblk[row * ld_d + lane + 64] = d1[q];
            if (mask_bits && lane < 4) {  // keep-bits of the block's four words (bit set = kept); bits past cols stay 0
                const int64_t word = c0 / 32 + lane;
                if (word * 32 < cols) {
                    const unsigned long long src = lane < 2 ? (live0 & ~pm0[q]) : (live1 & ~pm1[q]);
                    mask_bits[row * words_per_row + word] = static_cast<uint32_t>(src >> (32 * (lane & 1)));
                }
            }
        }
    }
}

struct SweepLayout {
    size_t v, d, sal, dinv, hist, state, row_eq, row_before, total;
};

SweepLayout sweep_layout(int64_t rows, int64_t cols, bool own_v) {
    auto up = [](size_t n) { return (n + 255) / 256 * 256; };
    SweepLayout l;
    size_t at = 0;
    l.v = at;
    at += own_v ? up(static_cast<size_t>(rows) * cols * 4) : 0;
    l.d = at;
    at += up(static_cast<size_t>(rows) * kGroup * kSB * 4);
    l.sal = at;
    at += up(static_cast<size_t>(rows) * kSB * 4);
    l.dinv = at;
    at += up(static_cast<size_t>(ceil_div(cols, kSB)) * kSB * kSB * 4);
    l.hist = at;
    at += up(kHistBins * 4);
    l.state = at;
    at += up(sizeof(SweepState));
    l.row_eq = at;
    at += up(static_cast<size_t>(rows) * 4);
    l.row_before = at;
    at += up(static_cast<size_t>(rows) * 4);
    l.total = at;
    return l;
}

// eight consecutive entries of a row (16-byte aligned), widened to fp32 / narrowed from it
__device__ __forceinline__ void load_row_run(const bf16_t *p, float (&out)[8]) {
    const u32x4 raw = *reinterpret_cast<const u32x4 *>(p);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        out[2 * e] = __uint_as_float(raw[e] << 16);
        out[2 * e + 1] = __uint_as_float(raw[e] & 0xffff0000u);
    }
}
__device__ __forceinline__ void load_row_run(const float *p, float (&out)[8]) {
    const f32x4 a = *reinterpret_cast<const f32x4 *>(p), b = *reinterpret_cast<const f32x4 *>(p + 4);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        out[e] = a[e];
        out[4 + e] = b[e];
    }
}
__device__ __forceinline__ void store_row_run(bf16_t *p, const float *v) {
    u32x4 raw;
#pragma unroll
    for (int e = 0; e < 4; ++e)
        raw[e] = static_cast<uint32_t>(narrow_bf16(v[2 * e])) | (static_cast<uint32_t>(narrow_bf16(v[2 * e + 1])) << 16);
    *reinterpret_cast<u32x4 *>(p) = raw;
}
__device__ __forceinline__ void store_row_run(float *p, const float *v) {
    f32x4 a, b;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
        a[e] = v[e];
        b[e] = v[4 + e];
    }
    *reinterpret_cast<f32x4 *>(p) = a;
    *reinterpret_cast<f32x4 *>(p + 4) = b;
}

// The same walk with a lane per row, for full blocks whose rows allow 16-byte accesses.  A workgroup of four waves
// takes 64 rows; the block's 16 runs of eight columns are dealt to the waves round robin (wave x owns runs x, x + 4,
// x + 8, x + 12), a lane holds its row's entries of its wave's 32 columns in registers.  The owner of a run walks
// its eight columns (a multiplication, a subtraction and the updates inside the run per column) and publishes the
// eight changes d of every row through LDS; after the one barrier per run, every wave adds d R[run, later] to the
// later columns it owns, the entries of R being uniform over the wave (one LDS address per read, no conflicts).  The owner of the next run
// brings that run up to date first, walks and publishes it, and only then updates its other columns, so that the
// chain run -> barrier -> next run is as short as the arithmetic allows.  Every column receives its updates in
// ascending order of the source column, as in the wave-per-two-rows form: the results are the same bits.
constexpr int kRowLanes = 64, kRunCols = 8, kRuns = kSB / kRunCols, kRunsPerWave = kRuns / 4;

template <typename T>
__global__ __launch_bounds__(256) void sweep_block_rows(const T *__restrict__ w, int64_t ld_w, T *__restrict__ w_out,
                                                        int64_t ld_out, const float *__restrict__ r, int64_t ld_r,
                                                        const uint8_t *__restrict__ dead, const float *__restrict__ g,
                                                        int64_t ldg, const float *__restrict__ sal, int64_t ld_sal,
                                                        int64_t rows, int64_t c0, int mode,
                                                        const SweepState *__restrict__ state,
                                                        const uint32_t *__restrict__ row_before,
                                                        float *__restrict__ dblk, int64_t ld_d,
                                                        uint8_t *__restrict__ mask_bytes, int64_t words_per_row) {
    __shared__ __attribute__((aligned(16))) float rs[kSB][kSB];  // the block of R (read with one address per wave)
    __shared__ float rinv[kSB];
    __shared__ float xch[2][kRunCols][kRowLanes];
    __shared__ uint32_t eq_bits[4][kRowLanes];
    const int tid = threadIdx.x, lane = tid & 63;
    const int wv = __builtin_amdgcn_readfirstlane(tid >> 6);
    const float *__restrict__ rb = r + c0 * ld_r + c0;  // the block of R: entry (i, k) at rb[i * ld_r + k]
    if (tid < kSB) rinv[tid] = 1.f / rb[tid * ld_r + tid];
    for (int e = tid; e < kSB * kSB / 4; e += 256) {
        const int i = e >> 5, k4 = (e & 31) * 4;
        *reinterpret_cast<f32x4 *>(&rs[i][k4]) = *reinterpret_cast<const f32x4 *>(rb + i * ld_r + k4);
    }
    const int64_t row_raw = static_cast<int64_t>(blockIdx.x) * kRowLanes + lane;
    const bool live = row_raw < rows;
    const int64_t row = live ? row_raw : rows - 1;  // lanes past the end compute on the last row and store nothing

    // this lane's entries: register q = 8 i + jj holds column 8 (wv + 4 i) + jj of the block
    float wq[32], vq[32];
    uint32_t pruned = mode == 2 ? 0xffffffffu : 0u, equal = 0u;
    uint32_t skey = 0u, need_eq = 0u;
    bool all_eq = true;
    if (mode == 1) {
        skey = state->key;
        need_eq = state->need_eq;
        all_eq = need_eq == state->count_eq;
    }
#pragma unroll
    for (int i = 0; i < kRunsPerWave; ++i) {
        const int col = kRunCols * (wv + 4 * i);
        float wf[8], gf[8];
        load_row_run(w + row * ld_w + c0 + col, wf);
        const f32x4 g0 = *reinterpret_cast<const f32x4 *>(g + row * ldg + c0 + col);
        const f32x4 g1 = *reinterpret_cast<const f32x4 *>(g + row * ldg + c0 + col + 4);
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            gf[e] = g0[e];
            gf[4 + e] = g1[e];
        }
        if (mode == 1) {
            const f32x4 s0 = *reinterpret_cast<const f32x4 *>(sal + row * ld_sal + col);
            const f32x4 s1 = *reinterpret_cast<const f32x4 *>(sal + row * ld_sal + col + 4);
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const uint32_t key = saliency_key(e < 4 ? s0[e] : s1[e - 4]);
                pruned |= (key < skey || (all_eq && key == skey) ? 1u : 0u) << (8 * i + e);
                equal |= (key == skey ? 1u : 0u) << (8 * i + e);
            }
        }
        // (the flags of the run's eight columns in one uniform load)
        const uint64_t dead8 = dead ? *reinterpret_cast<const uint64_t *>(dead + c0 + col) : 0ull;
#pragma unroll
        for (int e = 0; e < 8; ++e) {
            const bool is_dead = ((dead8 >> (8 * e)) & 0xffull) != 0ull;
            wq[8 * i + e] = is_dead ? 0.f : wf[e];
            vq[8 * i + e] = fmaf(wq[8 * i + e], rb[(col + e) * ld_r + col + e], gf[e]);  // (uniform address)
        }
    }
    if (mode == 1 && !all_eq) {
        // Of the entries with the threshold key, the first need_eq in row-major order go.  The waves exchange
        // which of their columns hold that key; word k of a row's 128 flags is made of byte k of each wave's 32.
        eq_bits[wv][lane] = equal;
        __syncthreads();
        uint32_t word[4];
#pragma unroll
        for (int k = 0; k < 4; ++k) {
            word[k] = 0u;
#pragma unroll
            for (int x = 0; x < 4; ++x) word[k] |= ((eq_bits[x][lane] >> (8 * k)) & 0xffu) << (8 * x);
        }
        const uint32_t before = row_before[row];
#pragma unroll
        for (int i = 0; i < kRunsPerWave; ++i) {
            uint32_t ahead = before;  // equal keys of this row in earlier words, then in this word before the run
#pragma unroll
            for (int k = 0; k < 4; ++k) ahead += k < i ? __popc(word[k]) : 0u;
#pragma unroll
            for (int e = 0; e < 8; ++e) {
                const int bit = 8 * wv + e;  // position of the column inside word i
                const uint32_t rank = ahead + __popc(word[i] & ((1u << bit) - 1u));
                const bool goes = ((equal >> (8 * i + e)) & 1u) && rank < need_eq;
                pruned |= (goes ? 1u : 0u) << (8 * i + e);
            }
        }
    }
    __syncthreads();  // rinv, rs

    // Eight rows of R (those of run `run`) at eight columns from `col`: fetched in one batch, so that a single LDS
    // round trip is waited for and not one per row
    struct RowRun {
        f32x4 lo[kRunCols], hi[kRunCols];
        __device__ __forceinline__ float at(int jj, int e) const { return e < 4 ? lo[jj][e] : hi[jj][e - 4]; }
    };
    auto fetch = [&](int run, int col, RowRun &rr) {
#pragma unroll
        for (int jj = 0; jj < kRunCols; ++jj) {
            rr.lo[jj] = *reinterpret_cast<const f32x4 *>(&rs[kRunCols * run + jj][col]);
            rr.hi[jj] = *reinterpret_cast<const f32x4 *>(&rs[kRunCols * run + jj][col + 4]);
        }
    };
    // columns of run `run` (owned by this wave, registers 8 i ...): walk them and publish the changes; rw holds the
    // run's own rows of R at its own columns, ri the reciprocals of its diagonal
    auto walk = [&](int run, int i, const RowRun &rw, const float (&ri)[kRunCols]) {
#pragma unroll
        for (int jj = 0; jj < kRunCols; ++jj) {
            const int q = 8 * i + jj;
            const float prod = __fmul_rn(vq[q], ri[jj]);
            const float wnew = ((pruned >> q) & 1u) ? 0.f : prod;
            const float dj = wq[q] - wnew;
            vq[q] = wnew;  // from here on the register holds the column's new weight ...
            wq[q] = dj;    // ... and this one its change
            xch[run & 1][jj][lane] = dj;
#pragma unroll
            for (int j2 = jj + 1; j2 < kRunCols; ++j2) vq[8 * i + j2] = fmaf(dj, rw.at(jj, j2), vq[8 * i + j2]);
        }
    };
    // add d R[run, columns of own run i] for the eight changes d of a run, rr holding those rows of R
    auto apply = [&](int i, const float (&d)[kRunCols], const RowRun &rr) {
#pragma unroll
        for (int jj = 0; jj < kRunCols; ++jj)
#pragma unroll
            for (int e = 0; e < kRunCols; ++e) vq[8 * i + e] = fmaf(d[jj], rr.at(jj, e), vq[8 * i + e]);
    };
    if (wv == 0) {
        RowRun rw;
        float ri[kRunCols];
        fetch(0, 0, rw);
#pragma unroll
        for (int jj = 0; jj < kRunCols; ++jj) ri[jj] = rinv[jj];
        walk(0, 0, rw, ri);
    }
#pragma clang loop unroll(full)
    for (int run = 0; run + 1 < kRuns; ++run) {
        const int next = run + 1, next_i = next >> 2;
        const bool owner_of_next = wv == (next & 3);  // uniform
        __builtin_amdgcn_sched_barrier(0);  // (reads of R are not to be moved up across trips: they would pile up in registers)
        __syncthreads();  // the changes of `run` are in xch[run & 1]
        float d[kRunCols];
#pragma unroll
        for (int jj = 0; jj < kRunCols; ++jj) d[jj] = xch[run & 1][jj][lane];
        if (owner_of_next) {
            RowRun ra, rw;
            float ri[kRunCols];
            fetch(run, kRunCols * next, ra);
            fetch(next, kRunCols * next, rw);
#pragma unroll
            for (int jj = 0; jj < kRunCols; ++jj) ri[jj] = rinv[kRunCols * next + jj];
            apply(next_i, d, ra);
            walk(next, next_i, rw, ri);
        }
#pragma unroll
        for (int i = 0; i < kRunsPerWave; ++i) {
            // own run wv + 4 i lies after `run`, and is not the one just brought up to date
            if (wv + 4 * i > run && !(owner_of_next && i == next_i)) {
                RowRun rr;
                __builtin_amdgcn_sched_barrier(0);
                fetch(run, kRunCols * (wv + 4 * i), rr);
                apply(i, d, rr);
            }
        }
    }

    if (!live) return;
#pragma unroll
    for (int i = 0; i < kRunsPerWave; ++i) {
        const int col = kRunCols * (wv + 4 * i);
        store_row_run(w_out + row * ld_out + c0 + col, &vq[8 * i]);
        f32x4 d0, d1;
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            d0[e] = wq[8 * i + e];
            d1[e] = wq[8 * i + 4 + e];
        }
        *reinterpret_cast<f32x4 *>(dblk + row * ld_d + col) = d0;
        *reinterpret_cast<f32x4 *>(dblk + row * ld_d + col + 4) = d1;
        // keep-bits (bit set = kept): byte wv of word c0 / 32 + i of the row
        if (mask_bytes) mask_bytes[(row * words_per_row + c0 / 32 + i) * 4 + wv] = static_cast<uint8_t>(~(pruned >> (8 * i)) & 0xffu);
    }
}

template <typename T>
int sweep_run(const T *w, T *w_out, int64_t rows, int64_t cols, int64_t ld_w, int64_t ld_out, const float *r,
              int64_t ld_r, const uint8_t *dead, double sparsity, int64_t first_block, int64_t n_blocks, float *g,
              float *saliency, uint32_t *mask_bits, char *ws, const SweepLayout &l, hipStream_t stream) {
    float *dgroup = reinterpret_cast<float *>(ws + l.d);  // D of the current group of blocks, [rows, kGroup * kSB]
    constexpr int64_t ld_d = kGroup * kSB;
    float *dinv_all = reinterpret_cast<float *>(ws + l.dinv);
    uint32_t *hist = reinterpret_cast<uint32_t *>(ws + l.hist);
    SweepState *state = reinterpret_cast<SweepState *>(ws + l.state);
    uint32_t *row_eq = reinterpret_cast<uint32_t *>(ws + l.row_eq);
    uint32_t *row_before = reinterpret_cast<uint32_t *>(ws + l.row_before);
    const int64_t words = ceil_div(cols, 32);
    if (n_blocks == 0) return PRUNE_OK;
    if (first_block == 0) {
        hipLaunchKernelGGL(sweep_zero, dim3(2048), dim3(256), 0, stream, g, rows * cols);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    }
    hipLaunchKernelGGL(select_reset, dim3(1), dim3(1024), 0, stream, hist);
    hipLaunchKernelGGL(invert_diagonal_blocks, dim3(static_cast<unsigned>(n_blocks)), dim3(256), 0, stream, r, ld_r, cols,
                       first_block, dinv_all);
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    const unsigned row_tiles = static_cast<unsigned>(ceil_div(rows, 16));
    const unsigned row_quads = static_cast<unsigned>(ceil_div(rows, 4) < 512 ? ceil_div(rows, 4) : 512);
    const unsigned row_groups = static_cast<unsigned>(ceil_div(rows, kSweepWaves * kSweepRows) < 1024
                                                          ? ceil_div(rows, kSweepWaves * kSweepRows) : 1024);
    for (int64_t b = first_block; b < first_block + n_blocks; ++b) {
        const int64_t c0 = b * kSB;
        const int width = static_cast<int>(cols - c0 < kSB ? cols - c0 : kSB);
        const double quota = floor(sparsity * static_cast<double>(rows) * static_cast<double>(width));
        const int64_t n_el = rows * width;
        const int64_t k = quota < 0 ? 0 : static_cast<int64_t>(quota);
        const int mode = k <= 0 ? 0 : k >= n_el ? 2 : 1;
        float *sal = saliency ? saliency + c0 : reinterpret_cast<float *>(ws + l.sal);
        const int64_t ld_sal = saliency ? cols : kSB;
        if (mode == 1 || saliency) {
            // the weights of the block as the published sweep holds them when the block starts: W + G inv(R_bb)
            const uint32_t k32 = static_cast<uint32_t>(mode == 1 ? k : 1);
            hipLaunchKernelGGL(saliency_first_pass<T>, dim3(row_tiles), dim3(256), 0, stream, w, ld_w, r, ld_r, dead, g, cols,
                               dinv_all + (b - first_block) * (kSB * kSB), rows, c0, width, sal, ld_sal, hist);
            hipLaunchKernelGGL(select_locate<0>, dim3(1), dim3(1024), 0, stream, state, hist, k32);
        }
        if (mode == 1) {
            hipLaunchKernelGGL(select_hist<1>, dim3(row_tiles), dim3(256), 0, stream, sal, ld_sal, int64_t(0), width, rows, state, hist);
            hipLaunchKernelGGL(select_locate<1>, dim3(1), dim3(1024), 0, stream, state, hist, 0u);
            hipLaunchKernelGGL(select_hist<2>, dim3(row_tiles), dim3(256), 0, stream, sal, ld_sal, int64_t(0), width, rows, state, hist);
            hipLaunchKernelGGL(select_locate<2>, dim3(1), dim3(1024), 0, stream, state, hist, 0u);
            hipLaunchKernelGGL(tie_count, dim3(row_quads), dim3(256), 0, stream, sal, ld_sal, int64_t(0), width, rows, state, row_eq);
            hipLaunchKernelGGL(tie_scan, dim3(1), dim3(1024), 0, stream, row_eq, row_before, rows, state);
            if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        }
        // Blocks are taken in groups of kGroup (aligned in the matrix, so that a sweep split over several calls does
        // the same operations): a finished block updates the rest of its group at once, and the columns beyond the
        // group receive the whole group's changes in one product with a four times longer inner dimension, which
        // cuts the read-modify-write traffic on G -- the bulk of the sweep's memory traffic -- by four.
        const int slot = static_cast<int>(b % kGroup);
        const int64_t group0 = (b - slot) * kSB;
        const int64_t group_end = group0 + ld_d < cols ? group0 + ld_d : cols;
        float *dblk = dgroup + slot * kSB;
        // full blocks whose rows can be read and written 16 bytes at a time take the lane-per-row form
        const bool by_rows = width == kSB && aligned_to(w + c0, 16) && aligned_to(w_out + c0, 16) &&
                             (ld_w * sizeof(T)) % 16 == 0 && (ld_out * sizeof(T)) % 16 == 0 && aligned_to(g + c0, 16) &&
                             cols % 4 == 0 && aligned_to(sal, 16) && ld_sal % 4 == 0 && aligned_to(dblk, 16) &&
                             (!dead || aligned_to(dead + c0, 8));
        if (by_rows) {
            hipLaunchKernelGGL(sweep_block_rows<T>, dim3(static_cast<unsigned>(ceil_div(rows, kRowLanes))), dim3(256), 0,
                               stream, w, ld_w, w_out, ld_out, r, ld_r, dead, g, cols, sal, ld_sal, rows, c0, mode, state,
                               row_before, dblk, ld_d, reinterpret_cast<uint8_t *>(mask_bits), words);
        } else {
            hipLaunchKernelGGL((sweep_block<T, kSweepRows>), dim3(row_groups), dim3(kSweepThreads), 0, stream, w, ld_w,
                               w_out, ld_out, r, ld_r, dead, g, cols, sal, ld_sal, rows, c0, width, mode, state, row_before,
                               dblk, ld_d, mask_bits, words, cols);
        }
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        const int64_t c1 = c0 + width;
        if (c1 < group_end) {
            const int st = launch_gemm_f32<kBKN>(static_cast<int>(rows), static_cast<int>(group_end - c1), width, 1.f, dblk,
                                                 ld_d, r + c0 * ld_r + c1, ld_r, 1.f, g + c1, cols, false, stream);
            if (st != PRUNE_OK) return st;
        } else if (group_end < cols) {
            const int st = launch_gemm_f32<kBKN>(static_cast<int>(rows), static_cast<int>(cols - group_end),
                                                 static_cast<int>(group_end - group0), 1.f, dgroup, ld_d,
                                                 r + group0 * ld_r + group_end, ld_r, 1.f, g + group_end, cols, false, stream);
            if (st != PRUNE_OK) return st;
        }
    }
    return PRUNE_OK;
}

}  // namespace

}  // namespace mp

extern "C" size_t prune_obs_sweep_workspace_bytes(int64_t rows, int64_t cols, int own_v) {
    if (rows <= 0 || cols <= 0) return 0;
    return mp::sweep_layout(rows, cols, own_v != 0).total;
}

extern "C" int prune_obs_sweep(const void *w, void *w_out, int dtype, int64_t rows, int64_t cols, int64_t ld_w,
                               int64_t ld_out, const float *r, int64_t ld_r, const uint8_t *dead, double sparsity,
                               int64_t first_block, int64_t n_blocks, float *v, float *saliency, uint32_t *mask_bits,
                               void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (rows <= 0 || cols <= 0 || ld_w < cols || ld_out < cols || ld_r < cols || rows > (int64_t(1) << 22) ||
        cols > (int64_t(1) << 20) || rows * kSB >= (int64_t(1) << 32))
        return PRUNE_ERR_SHAPE;
    if (cols % 4 != 0 || ld_r % 4 != 0) return PRUNE_ERR_SHAPE;
    if (w_out == w && ld_out != ld_w) return PRUNE_ERR_SHAPE;
    if (!w || !w_out || !r || !ws) return PRUNE_ERR_NULL;
    if (!(sparsity >= 0.0 && sparsity < 1.0)) return PRUNE_ERR_RANGE;
    const int64_t total_blocks = ceil_div(cols, kSB);
    if (n_blocks < 0) n_blocks = total_blocks - first_block;
    if (first_block < 0 || n_blocks < 0 || first_block + n_blocks > total_blocks) return PRUNE_ERR_RANGE;
    const size_t es = elem_size(dtype);
    if (!aligned_to(w, es) || !aligned_to(w_out, es) || !aligned_to(r, 16) || !aligned_to(ws, 256) ||
        (v && !aligned_to(v, 16)) || (saliency && !aligned_to(saliency, 4)) || (mask_bits && !aligned_to(mask_bits, 4)))
        return PRUNE_ERR_ALIGNMENT;
    const SweepLayout l = sweep_layout(rows, cols, v == nullptr);
    if (ws_bytes < l.total) return PRUNE_ERR_WORKSPACE;
    char *base = static_cast<char *>(ws);
    float *vv = v ? v : reinterpret_cast<float *>(base + l.v);
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (dtype == PRUNE_BF16)
        return sweep_run(static_cast<const bf16_t *>(w), static_cast<bf16_t *>(w_out), rows, cols, ld_w, ld_out, r, ld_r,
                         dead, sparsity, first_block, n_blocks, vv, saliency, mask_bits, base, l, stream);
    return sweep_run(static_cast<const float *>(w), static_cast<float *>(w_out), rows, cols, ld_w, ld_out, r, ld_r, dead,
                     sparsity, first_block, n_blocks, vv, saliency, mask_bits, base, l, stream);
}
