// Forward pass of the feed-forward block whose projections are pruned (LLaMA-style layers of Table 2,
// Section 4.1.1):  h = silu(x gate^T) * (x up^T),  y = h down^T.  It serves two purposes of the method:
// the input of the down projection -- the activation behind its weight metric (Eq. 5) -- comes from a real
// forward pass, with its per-channel sums of squares accumulated in the epilogue of the product that creates
// it; and the block can be timed at full and at structurally pruned size (Section 4.1.3, categories 2 and 3:
// removing coupled channels makes the projections smaller, which is where the inference speed-up comes from).
//
// bf16 projections on the matrix cores: y[t, n] = sum_k x[t, k] w[n, k], both operands contiguous along k.
// A block of four waves owns a 256 x 256 tile of y (128 x 128 per wave, sixteen 32 x 32 x 16 MFMA accumulators) and
// walks k 32 at a time; the two [256 rows x 32 k] slabs of a stage go from global memory straight into a
// four-stage LDS ring.  A slab row is 64 bytes (four 16-byte packets); packet c of row r sits at position
// c ^ ((r / 4) % 4), which makes the 16-byte operand reads of a wave conflict-free.  For the gate / up pair the
// weight slab holds 128 gate rows and 128 up rows of the same channels, so both products of a channel end up in the
// same lanes and silu(gate) * up is formed in registers.
// fp32 data, or shapes the packets do not fit, take a plain tiled FMA kernel.
#include "mfma_bf16.hpp"

namespace mp {

namespace {

constexpr int kLinTile = 256, kLinStep = 32, kLinRing = 4, kLinBlock = 256;
constexpr int kLinSlabBytes = kLinTile * kLinStep * 2;  // 16 KB

// eight consecutive k (8 (lane / 32) ... within the 16 at kk) of row row_base + lane % 32 of a slab
__device__ __forceinline__ bf16x8 operand_rows(const unsigned char *slab, int row_base, int kk, int lane) {
    const int row = row_base + (lane & 31);
    const int chunk = (kk >> 3) + (lane >> 5);
    const u32x4 v = *reinterpret_cast<const u32x4 *>(slab + row * 64 + ((chunk ^ ((row >> 2) & 3)) << 4));
    return __builtin_bit_cast(bf16x8, v);
}

__device__ __forceinline__ float silu(float a) { return a / (1.f + __expf(-a)); }

// Output tiles are numbered patch by patch (4 row tiles x 8 column tiles: 32 tiles that need only 12 operand
// slabs), patches row band by row band; tile `item` -> (mt, nt).
__device__ __forceinline__ void tile_of(int item, int m_tiles, int n_tiles, int &mt, int &nt) {
    mt = nt = 0;
    for (int r0 = 0; r0 < m_tiles; r0 += 4) {
        const int rows = m_tiles - r0 < 4 ? m_tiles - r0 : 4;
        for (int c0 = 0; c0 < n_tiles; c0 += 8) {
            const int cols = n_tiles - c0 < 8 ? n_tiles - c0 : 8;
            if (item < rows * cols) {
                mt = r0 + item / cols;
                nt = c0 + item % cols;
                return;
            }
            item -= rows * cols;
        }
    }
}

// DUAL = false: y[M, N] = x w0^T.   DUAL = true: y[M, N] = silu(x w0^T) * (x w1^T), N channels, and
// sq_partial[2 * (row tile) + {0, 1}][n] = sum over 128 rows of y^2 (of the rounded values), when non-null.
template <bool DUAL>
__global__ __launch_bounds__(kLinBlock, 1) void linear_tiles_bf16(const bf16_t *__restrict__ x, int64_t ld_x,
                                                                  const bf16_t *__restrict__ w0,
                                                                  const bf16_t *__restrict__ w1, int64_t ld_w, int M,
                                                                  int N, int K, bf16_t *__restrict__ y, int64_t ld_y,
                                                                  float *__restrict__ sq_partial) {
    __shared__ __attribute__((aligned(1024))) unsigned char ring[kLinRing][2][kLinSlabBytes];
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    constexpr int kChannels = DUAL ? kLinTile / 2 : kLinTile;  // output channels of a block
    const int m_tiles = (M + kLinTile - 1) / kLinTile, n_tiles = (N + kChannels - 1) / kChannels;
    int item, mt, nt;
    if (!item_of_block(blockIdx.x, m_tiles * n_tiles, item)) return;  // the whole block, before any barrier
    tile_of(item, m_tiles, n_tiles, mt, nt);
    const int m0 = mt * kLinTile;
    const int n0 = nt * kChannels;  // first output channel of the block
    const int n_stages = K / kLinStep;

    // Load instruction p of this wave fills LDS window 4 p + wave (16 rows of 64 bytes) of a slab: row
    // 16 (4 p + wave) + lane / 4, position lane % 4, i.e. packet (lane % 4) ^ ((row / 4) % 4).  Rows past the edge
    // of a matrix are clamped to its last row: they only feed outputs that are never stored.
    // The address of a load is a uniform base (the block's first row of x, or of the weight matrix the rows of load
    // p come from, plus the stage's offset along K: scalar arithmetic) plus a per-lane byte offset that never
    // changes -- no vector instruction per load (64-bit vector additions between the matrix instructions cost a wave
    // that has its SIMD to itself a tenth of the kernel's time).
    uint32_t offa[4], offb[4];
    const char *base_b[4];
    const char *const base_a = reinterpret_cast<const char *>(x + static_cast<int64_t>(m0) * ld_x);
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        const int row = 16 * (4 * p + wave) + (lane >> 2);
        const int c = (lane & 3) ^ ((row >> 2) & 3);
        const int xr = m0 + row < M ? row : M - 1 - m0;  // relative to m0
        offa[p] = static_cast<uint32_t>((static_cast<int64_t>(xr) * ld_x + 8 * c) * 2);
        const bf16_t *wsrc = w0;
        int wr = row;
        if (DUAL) {  // slab rows 0..127: gate channels n0 .. n0 + 127, rows 128..255: the same channels of up
            wsrc = p < 2 ? w0 : w1;  // (rows 16 (4 p + wave) ... + 15: below 128 exactly for p = 0, 1)
            wr = row & 127;
        }
        wr = n0 + wr < N ? wr : N - 1 - n0;  // relative to n0
        offb[p] = static_cast<uint32_t>((static_cast<int64_t>(wr) * ld_w + 8 * c) * 2);
        base_b[p] = reinterpret_cast<const char *>(wsrc + static_cast<int64_t>(n0) * ld_w);
    }
    auto issue_part = [&](int stage_index, int p) {
        const uint32_t dst = __builtin_amdgcn_readfirstlane(
            static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte *)&ring[stage_index & (kLinRing - 1)][0][0])) +
            static_cast<uint32_t>(wave) * 1024u);
        // stages past the end re-read the last one (into a buffer nobody reads any more)
        const int64_t koff = static_cast<int64_t>(stage_index < n_stages ? stage_index : n_stages - 1) * (kLinStep * 2);
        load_to_lds(base_a + koff, offa[p], dst + 4096u * p);
        load_to_lds(base_b[p] + koff, offb[p], dst + kLinSlabBytes + 4096u * p);
    };
    auto issue = [&](int stage_index) {
#pragma unroll
        for (int p = 0; p < 4; ++p) issue_part(stage_index, p);
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    bf16x8 a[2][4], b[2][4];
    auto read_a = [&](int set, int stage_index, int kk) {
        const unsigned char *slab = &ring[stage_index & (kLinRing - 1)][0][0];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[set][i] = operand_rows(slab, wm * 128 + 32 * i, kk, lane);
    };
    auto read_b = [&](int set, int stage_index, int kk) {
        const unsigned char *slab = &ring[stage_index & (kLinRing - 1)][1][0];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            // plain: columns wn * 128 + 32 j; gate / up pair: j = 0, 1 gate and j = 2, 3 up of channels wn * 64 + 32 (j % 2)
            const int base = DUAL ? (j >> 1) * 128 + wn * 64 + 32 * (j & 1) : wn * 128 + 32 * j;
            b[set][j] = operand_rows(slab, base, kk, lane);
        }
    };
    auto mfma_one = [&](int set, int i, int j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[set][i], b[set][j], acc[i][j], 0, 0, 0);
    };

    // Same pipeline as the Hessian kernel: the loads of stage s + 4 are issued in the middle of stage s into that
    // stage's own buffer, behind the one barrier per stage; every LDS read is issued in the shadow of MFMAs.
    issue(0);
    issue(1);
    issue(2);
    issue(3);
    MP_WAIT_VMCNT(24);
    __syncthreads();
    read_a(0, 0, 0);
    read_b(0, 0, 0);
    for (int s = 0; s < n_stages; ++s) {
        __builtin_amdgcn_sched_barrier(0);
        read_a(1, s, 16);
        read_b(1, s, 16);
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) mfma_one(0, i, j);
#pragma unroll
        for (int g = 0; g < 12; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
            __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_barrier(0);
        MP_WAIT_VMCNT(16);
        __syncthreads();
        // The remaining 20 MFMAs of the trip go in four groups of five, each behind two of the eight load
        // instructions and interleaved with the reads of two of the next stage's eight operands (a load
        // instruction holds the wave for some 40 cycles: spread out, less of that falls on idle matrix cores).
        {
            const unsigned char *slab_a = &ring[(s + 1) & (kLinRing - 1)][0][0], *slab_b = &ring[(s + 1) & (kLinRing - 1)][1][0];
            auto b_base = [&](int j) { return DUAL ? (j >> 1) * 128 + wn * 64 + 32 * (j & 1) : wn * 128 + 32 * j; };
            issue_part(s + 4, 0);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(0, 3, 0);
            mfma_one(0, 3, 1);
            mfma_one(0, 3, 2);
            mfma_one(0, 3, 3);
            mfma_one(1, 0, 0);
            a[0][0] = operand_rows(slab_a, wm * 128, 0, lane);
            a[0][1] = operand_rows(slab_a, wm * 128 + 32, 0, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue_part(s + 4, 1);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(1, 0, 1);
            mfma_one(1, 0, 2);
            mfma_one(1, 0, 3);
            mfma_one(1, 1, 0);
            mfma_one(1, 1, 1);
            a[0][2] = operand_rows(slab_a, wm * 128 + 64, 0, lane);
            a[0][3] = operand_rows(slab_a, wm * 128 + 96, 0, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue_part(s + 4, 2);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(1, 1, 2);
            mfma_one(1, 1, 3);
            mfma_one(1, 2, 0);
            mfma_one(1, 2, 1);
            mfma_one(1, 2, 2);
            b[0][0] = operand_rows(slab_b, b_base(0), 0, lane);
            b[0][1] = operand_rows(slab_b, b_base(1), 0, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue_part(s + 4, 3);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(1, 2, 3);
            mfma_one(1, 3, 0);
            mfma_one(1, 3, 1);
            mfma_one(1, 3, 2);
            mfma_one(1, 3, 3);
            b[0][2] = operand_rows(slab_b, b_base(2), 0, lane);
            b[0][3] = operand_rows(slab_b, b_base(3), 0, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    }
    MP_WAIT_VMCNT(0);  // nothing may still be landing in this block's LDS when it ends

    // accumulator element v of lane l sits at row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of its 32 x 32 tile
    if (!DUAL) {
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm * 128 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    const int col = n0 + wn * 128 + 32 * j + (lane & 31);
                    if (row < M && col < N) y[static_cast<int64_t>(row) * ld_y + col] = narrow_to_bf16(acc[i][j][v]);
                }
    } else {
#pragma unroll
        for (int j = 0; j < 2; ++j) {
            const int col = n0 + wn * 64 + 32 * j + (lane & 31);
            float sq = 0.f;
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int v = 0; v < 16; ++v) {
                    const int row = m0 + wm * 128 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                    const bf16_t hb = narrow_to_bf16(silu(acc[i][j][v]) * acc[i][j + 2][v]);
                    if (row < M && col < N) {
                        y[static_cast<int64_t>(row) * ld_y + col] = hb;
                        const float hv = widen(hb);
                        sq = fmaf(hv, hv, sq);
                    }
                }
            // lanes l and l + 32 hold the other rows of the same column
            sq += __shfl_xor(sq, 32);
            if (sq_partial && lane < 32 && col < N)
                sq_partial[(2 * static_cast<int64_t>(mt) + wm) * N + col] = sq;
        }
    }
}

// sumsq[n] += sum over the row groups of the partial sums (double accumulation in a fixed order: a block takes 64
// channels, four quarters of the groups side by side, then the quarters in order)
__global__ __launch_bounds__(256) void fold_square_partials(const float *__restrict__ partial, int n_groups, int N,
                                                            float *__restrict__ sumsq) {
    __shared__ double quarter[4][64];
    const int c = threadIdx.x & 63, q = threadIdx.x >> 6;
    const int n = blockIdx.x * 64 + c;
    const int per = (n_groups + 3) / 4, g0 = q * per, g1 = g0 + per < n_groups ? g0 + per : n_groups;
    double s = 0.0;
    if (n < N)
        for (int g = g0; g < g1; ++g) s += static_cast<double>(partial[static_cast<int64_t>(g) * N + n]);
    quarter[q][c] = s;
    __syncthreads();
    if (q == 0 && n < N) {
        const double total = ((quarter[0][c] + quarter[1][c]) + quarter[2][c]) + quarter[3][c];
        sumsq[n] = static_cast<float>(static_cast<double>(sumsq[n]) + total);
    }
}

// Any element type and shape: a 64 x 64 output tile per block (16 x 16 threads, 4 x 4 outputs each), fp32 FMAs.
// sumsq (DUAL only): the squares are added with integer-free, order-fixed arithmetic by one block per 64 channels
// walking its row tiles in order, so this kernel is launched with gridDim.y == 1 when sumsq is wanted.
template <typename T, bool DUAL>
__global__ __launch_bounds__(256) void linear_generic(const T *__restrict__ x, int64_t ld_x, const T *__restrict__ w0,
                                                      const T *__restrict__ w1, int64_t ld_w, int64_t M, int64_t N,
                                                      int64_t K, T *__restrict__ y, int64_t ld_y,
                                                      float *__restrict__ sumsq) {
    __shared__ float xs[16][64 + 4], ws0[16][64 + 4], ws1[DUAL ? 16 : 1][64 + 4];
    __shared__ float colsq[16][64];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t n0 = static_cast<int64_t>(blockIdx.x) * 64;
    float keep_sq[4] = {0.f, 0.f, 0.f, 0.f};  // running sums of this thread's 4 columns over its rows (fixed order)
    for (int64_t m0 = static_cast<int64_t>(blockIdx.y) * 64; m0 < M; m0 += static_cast<int64_t>(gridDim.y) * 64) {
        float acc0[4][4] = {}, acc1[4][4] = {};
        for (int64_t k0 = 0; k0 < K; k0 += 16) {
            for (int e = threadIdx.x; e < 16 * 64; e += 256) {
                const int kk = e & 15, r = e >> 4;
                const bool kin = k0 + kk < K;
                xs[kk][r] = (kin && m0 + r < M) ? widen(x[(m0 + r) * ld_x + k0 + kk]) : 0.f;
                ws0[kk][r] = (kin && n0 + r < N) ? widen(w0[(n0 + r) * ld_w + k0 + kk]) : 0.f;
                if constexpr (DUAL) ws1[kk][r] = (kin && n0 + r < N) ? widen(w1[(n0 + r) * ld_w + k0 + kk]) : 0.f;
            }
            __syncthreads();
#pragma unroll
            for (int kk = 0; kk < 16; ++kk) {
                float xv[4], wv0[4], wv1[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    xv[i] = xs[kk][ty * 4 + i];
                    wv0[i] = ws0[kk][tx * 4 + i];
                    if constexpr (DUAL) wv1[i] = ws1[kk][tx * 4 + i]; else wv1[i] = 0.f;
                }
#pragma unroll
                for (int i = 0; i < 4; ++i)
#pragma unroll
                    for (int j = 0; j < 4; ++j) {
                        acc0[i][j] = fmaf(xv[i], wv0[j], acc0[i][j]);
                        if (DUAL) acc1[i][j] = fmaf(xv[i], wv1[j], acc1[i][j]);
                    }
            }
            __syncthreads();
        }
#pragma unroll
        for (int i = 0; i < 4; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int64_t row = m0 + ty * 4 + i, col = n0 + tx * 4 + j;
                if (row < M && col < N) {
                    const float val = DUAL ? silu(acc0[i][j]) * acc1[i][j] : acc0[i][j];
                    T out;
                    if constexpr (sizeof(T) == 2) out = narrow_to_bf16(val); else out = val;
                    y[row * ld_y + col] = out;
                    const float hv = widen(out);
                    keep_sq[j] = fmaf(hv, hv, keep_sq[j]);
                }
            }
    }
    if (DUAL && sumsq) {
#pragma unroll
        for (int j = 0; j < 4; ++j) colsq[ty][tx * 4 + j] = keep_sq[j];
        __syncthreads();
        if (threadIdx.x < 64 && n0 + threadIdx.x < N) {
            double s = 0.0;
            for (int r = 0; r < 16; ++r) s += static_cast<double>(colsq[r][threadIdx.x]);
            sumsq[n0 + threadIdx.x] = static_cast<float>(static_cast<double>(sumsq[n0 + threadIdx.x]) + s);
        }
    }
}

// blocks for n_items tiles: whole chunks of 32 per die
unsigned tiled_grid(int64_t n_items) {
    return static_cast<unsigned>(ceil_div(ceil_div(n_items, kChunk), kXcds) * kXcds * kChunk);
}

bool linear_tiles_ok(int dtype, const void *x, int64_t ld_x, const void *w0, const void *w1, int64_t ld_w, int64_t M,
                     int64_t N, int64_t K) {
    return dtype == PRUNE_BF16 && K >= kLinStep && K % kLinStep == 0 && ld_x % 8 == 0 && ld_w % 8 == 0 &&
           aligned_to(x, 16) && aligned_to(w0, 16) && (!w1 || aligned_to(w1, 16)) && M > 0 && N > 0 &&
           M < (int64_t(1) << 31) - kLinTile && N < (int64_t(1) << 31) - kLinTile &&
           ceil_div(M, kLinTile) * ceil_div(N, kLinTile / 2) < (int64_t(1) << 30);
}

template <typename T, bool DUAL>
int launch_generic(const void *x, int64_t ld_x, const void *w0, const void *w1, int64_t ld_w, int64_t M, int64_t N,
                   int64_t K, void *y, int64_t ld_y, float *sumsq, hipStream_t stream) {
    // one block walks all row tiles of its 64 channels when the sums of squares are wanted (fixed order, one owner)
    const int64_t row_blocks = (DUAL && sumsq) ? 1 : (ceil_div(M, 64) < 65535 ? ceil_div(M, 64) : 65535);
    const dim3 grid(static_cast<unsigned>(ceil_div(N, 64)), static_cast<unsigned>(row_blocks));
    hipLaunchKernelGGL((linear_generic<T, DUAL>), grid, dim3(256), 0, stream, static_cast<const T *>(x), ld_x,
                       static_cast<const T *>(w0), static_cast<const T *>(w1), ld_w, M, N, K, static_cast<T *>(y), ld_y,
                       sumsq);
    return launch_status();
}

int validate_linear(const void *x, const void *w, const void *y, int dtype, int64_t tokens, int64_t n, int64_t k,
                    int64_t ld_x, int64_t ld_w, int64_t ld_y) {
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (tokens <= 0 || n <= 0 || k <= 0 || ld_x < k || ld_w < k || ld_y < n) return PRUNE_ERR_SHAPE;
    if (!x || !w || !y) return PRUNE_ERR_NULL;
    const size_t es = elem_size(dtype);
    if (!aligned_to(x, es) || !aligned_to(w, es) || !aligned_to(y, es)) return PRUNE_ERR_ALIGNMENT;
    return PRUNE_OK;
}

}  // namespace

}  // namespace mp

extern "C" size_t prune_mlp_workspace_bytes(int64_t tokens, int64_t inter) {
    if (tokens <= 0 || inter <= 0) return 0;
    const size_t n = static_cast<size_t>(2 * mp::ceil_div(tokens, mp::kLinTile)) * static_cast<size_t>(inter) * sizeof(float);
    return (n + 255) / 256 * 256;
}

extern "C" int prune_linear(const void *x, const void *w, void *y, int dtype, int64_t tokens, int64_t n, int64_t k,
                            int64_t ld_x, int64_t ld_w, int64_t ld_y, void *stream_) {
    using namespace mp;
    const int st = validate_linear(x, w, y, dtype, tokens, n, k, ld_x, ld_w, ld_y);
    if (st != PRUNE_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (linear_tiles_ok(dtype, x, ld_x, w, nullptr, ld_w, tokens, n, k)) {
        const dim3 grid(tiled_grid(ceil_div(tokens, kLinTile) * ceil_div(n, kLinTile)));
        hipLaunchKernelGGL(linear_tiles_bf16<false>, grid, dim3(kLinBlock), 0, stream, static_cast<const bf16_t *>(x),
                           ld_x, static_cast<const bf16_t *>(w), static_cast<const bf16_t *>(nullptr), ld_w,
                           static_cast<int>(tokens), static_cast<int>(n), static_cast<int>(k), static_cast<bf16_t *>(y),
                           ld_y, static_cast<float *>(nullptr));
        return launch_status();
    }
    return dtype == PRUNE_BF16 ? launch_generic<bf16_t, false>(x, ld_x, w, nullptr, ld_w, tokens, n, k, y, ld_y, nullptr, stream)
                               : launch_generic<float, false>(x, ld_x, w, nullptr, ld_w, tokens, n, k, y, ld_y, nullptr, stream);
}

extern "C" int prune_mlp_gate_up(const void *x, const void *gate, const void *up, void *h, int dtype, int64_t tokens,
                                 int64_t hidden, int64_t inter, int64_t ld_x, int64_t ld_w, int64_t ld_h, float *sumsq,
                                 void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    const int st = validate_linear(x, gate, h, dtype, tokens, inter, hidden, ld_x, ld_w, ld_h);
    if (st != PRUNE_OK) return st;
    if (!up) return PRUNE_ERR_NULL;
    if (!aligned_to(up, elem_size(dtype)) || (sumsq && !aligned_to(sumsq, 4)) || (ws && !aligned_to(ws, 16)))
        return PRUNE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (linear_tiles_ok(dtype, x, ld_x, gate, up, ld_w, tokens, inter, hidden)) {
        float *partial = nullptr;
        const int n_groups = static_cast<int>(2 * ceil_div(tokens, kLinTile));
        if (sumsq) {
            if (!ws) return PRUNE_ERR_NULL;
            if (ws_bytes < static_cast<size_t>(n_groups) * inter * sizeof(float)) return PRUNE_ERR_WORKSPACE;
            partial = static_cast<float *>(ws);
        }
        const dim3 grid(tiled_grid(ceil_div(tokens, kLinTile) * ceil_div(inter, kLinTile / 2)));
        hipLaunchKernelGGL(linear_tiles_bf16<true>, grid, dim3(kLinBlock), 0, stream, static_cast<const bf16_t *>(x),
                           ld_x, static_cast<const bf16_t *>(gate), static_cast<const bf16_t *>(up), ld_w,
                           static_cast<int>(tokens), static_cast<int>(inter), static_cast<int>(hidden),
                           static_cast<bf16_t *>(h), ld_h, partial);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        if (sumsq) {
            hipLaunchKernelGGL(fold_square_partials, dim3(static_cast<unsigned>(ceil_div(inter, 64))), dim3(256), 0,
                               stream, partial, n_groups, static_cast<int>(inter), sumsq);
            return launch_status();
        }
        return PRUNE_OK;
    }
    return dtype == PRUNE_BF16
               ? launch_generic<bf16_t, true>(x, ld_x, gate, up, ld_w, tokens, inter, hidden, h, ld_h, sumsq, stream)
               : launch_generic<float, true>(x, ld_x, gate, up, ld_w, tokens, inter, hidden, h, ld_h, sumsq, stream);
}
