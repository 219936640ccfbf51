// Hessian of the layer-wise reconstruction problem of one projection input
// (Section 4.1.3, "Pruning Methods": the one-shot pruner works with the inverse
// Hessian; Section 4.1.4, "Calibration": it is computed from the calibration
// samples):  H += X^T X  over the tokens of a chunk.
//
// This is the one dense contraction of the path, so it runs on the matrix cores.
// bf16 activations: the output is cut into 256 x 256 tiles, only tiles on or above
// the diagonal are computed (H is symmetric), and the tokens are split over several
// blocks per tile so that the grid fills the chip.  A block of four waves holds a
// 256 x 256 fp32 accumulator tile in registers (128 x 128 per wave, sixteen
// 32 x 32 x 16 MFMA accumulators) and walks its tokens 32 at a time: the two
// [32 tokens x 256 channels] slabs of X go through LDS exactly as they lie in
// memory (token-major), double buffered, and the MFMA operands -- which want eight
// consecutive tokens of one channel per lane -- are formed by the LDS transpose
// read.  Per-split partial tiles go to the workspace and are added up in a fixed
// order (so the result is reproducible bit for bit), mirrored below the diagonal.
// Any other element type, width or alignment takes a plain tiled FMA kernel.
#include "common.hpp"

namespace mp {

namespace {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

constexpr int kTile = 256;        // output tile edge (channels)
constexpr int kStep = 32;         // tokens per LDS stage
constexpr int kPitch = 288;       // bf16 elements per LDS row: 576 bytes, so that four consecutive rows start 64 bytes
                                  // apart modulo 256 and the transpose reads of a half wave fall into distinct banks
constexpr int kGramBlock = 256;
constexpr int kTargetBlocks = 2048;
constexpr int kMaxSplits = 64;

// tile pair p (0-based, row by row over the upper triangle) -> (mt, nt), mt <= nt
__device__ __forceinline__ void pair_of(int p, int n_tiles, int &mt, int &nt) {
    mt = 0;
    while (p >= n_tiles - mt) {
        p -= n_tiles - mt;
        ++mt;
    }
    nt = mt + p;
}

// Eight consecutive tokens (k16 + 8 * (lane / 32) ...) of channel ch_base + lane % 32, as the MFMA wants them,
// out of a token-major LDS slab.  The transpose read hands lane i of a 16-lane group, as element j, the
// element i % 4 of the 64-bit row that lane 4 j + i / 4 of the group points at; so lane s' points at token
// row s' / 4, channel quad s' % 4, and lane s receives channel s of four consecutive tokens.
__device__ __forceinline__ bf16x8 operand_from_slab(const bf16_t *slab, int k16, int ch_base, int lane) {
    const int s = lane & 15, g = lane >> 4;
    const bf16_t *p = slab + (k16 + 8 * (g >> 1) + (s >> 2)) * kPitch + ch_base + 16 * (g & 1) + 4 * (s & 3);
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * kPitch));
    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
}

__global__ __launch_bounds__(kGramBlock, 1) void gram_tiles_bf16(const bf16_t *__restrict__ x, int64_t n_tokens,
                                                                 int channels, int64_t ld, int n_tiles, int n_pairs,
                                                                 int64_t tokens_per_split,
                                                                 float *__restrict__ partials) {
    __shared__ __attribute__((aligned(16))) bf16_t slab[2][2][kStep * kPitch];  // [stage][operand]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    const int pair = blockIdx.x % n_pairs, split = blockIdx.x / n_pairs;
    int mt, nt;
    pair_of(pair, n_tiles, mt, nt);
    const int m0 = mt * kTile, n0 = nt * kTile;
    const int64_t t_begin = split * tokens_per_split;
    int64_t t_end = t_begin + tokens_per_split;
    if (t_end > n_tokens) t_end = n_tokens;

    // staging: pass p moves token rows 8 p + tid / 32, channel packet tid % 32 of both slabs
    const int srow = tid >> 5, spkt = tid & 31;
    const int cha = m0 + spkt * 8, chb = n0 + spkt * 8;
    const bool a_ok = cha < channels, b_ok = chb < channels;
    u32x4 ra[4], rb[4];
    auto fetch = [&](int64_t t0) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int64_t t = t0 + srow + 8 * p;
            const bool in = t < t_end;
            const u32x4 zero = {0u, 0u, 0u, 0u};
            ra[p] = (in && a_ok) ? *reinterpret_cast<const u32x4 *>(x + t * ld + cha) : zero;
            rb[p] = (in && b_ok) ? *reinterpret_cast<const u32x4 *>(x + t * ld + chb) : zero;
        }
    };
    auto park = [&](int stage) {
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            const int off = (srow + 8 * p) * kPitch + spkt * 8;
            *reinterpret_cast<u32x4 *>(&slab[stage][0][off]) = ra[p];
            *reinterpret_cast<u32x4 *>(&slab[stage][1][off]) = rb[p];
        }
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;

    const int64_t n_steps = (t_end - t_begin + kStep - 1) / kStep;
    if (n_steps > 0) {
        fetch(t_begin);
        park(0);
    }
    __syncthreads();
    for (int64_t it = 0; it < n_steps; ++it) {
        const int cur = static_cast<int>(it & 1);
        const bool more = it + 1 < n_steps;
        if (more) fetch(t_begin + (it + 1) * kStep);  // in flight while the matrix cores work on this stage
#pragma unroll
        for (int k16 = 0; k16 < kStep; k16 += 16) {
            bf16x8 a[4], b[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                a[i] = operand_from_slab(slab[cur][0], k16, wm * 128 + 32 * i, lane);
                b[i] = operand_from_slab(slab[cur][1], k16, wn * 128 + 32 * i, lane);
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j)
                    acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
        }
        if (more) park(cur ^ 1);
        __syncthreads();
    }

    // accumulator element v of lane l sits at row 8 (v / 4) + 4 (l / 32) + v % 4, column l % 32 of its 32 x 32 tile
    float *out = partials + (static_cast<int64_t>(split) * n_pairs + pair) * (kTile * kTile);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wm * 128 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int col = wn * 128 + 32 * j + (lane & 31);
                out[row * kTile + col] = acc[i][j][v];
            }
}

// h[tile] += sum over splits (in split order, in double) of the partial tile; the mirror image goes below the diagonal
__global__ __launch_bounds__(256) void gram_reduce(const float *__restrict__ partials, int n_splits, int n_pairs,
                                                   int n_tiles, int channels, float *__restrict__ h, int64_t ld_h) {
    __shared__ float flip[32][33];
    const int pair = blockIdx.x;
    int mt, nt;
    pair_of(pair, n_tiles, mt, nt);
    const int m0 = mt * kTile, n0 = nt * kTile;
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;  // 32 x 8
    // blockIdx.y walks the 8 x 8 sub-tiles of 32 x 32
    const int sr = (blockIdx.y >> 3) * 32, sc = (blockIdx.y & 7) * 32;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        const int row = sr + ty + 8 * q, col = sc + tx;
        double s = 0.0;
        for (int sp = 0; sp < n_splits; ++sp)
            s += static_cast<double>(
                partials[(static_cast<int64_t>(sp) * n_pairs + pair) * (kTile * kTile) + row * kTile + col]);
        const float add = static_cast<float>(s);
        flip[ty + 8 * q][tx] = add;
        const int gi = m0 + row, gj = n0 + col;
        if (gi < channels && gj < channels) {  // (the rounded sum is what both triangles receive: h stays symmetric)
            float *dst = h + static_cast<int64_t>(gi) * ld_h + gj;
            *dst = static_cast<float>(static_cast<double>(*dst) + static_cast<double>(add));
        }
    }
    if (mt == nt) return;  // a diagonal tile holds both of its triangles already
    __syncthreads();
#pragma unroll
    for (int q = 0; q < 4; ++q) {
        // element (row, col) of the tile goes to h[n0 + col][m0 + row]: read the sub-tile transposed
        const int col = sc + ty + 8 * q, row = sr + tx;
        const int gi = n0 + col, gj = m0 + row;
        if (gi < channels && gj < channels) {
            float *dst = h + static_cast<int64_t>(gi) * ld_h + gj;
            *dst = static_cast<float>(static_cast<double>(*dst) + static_cast<double>(flip[tx][ty + 8 * q]));
        }
    }
}

// Any element type and shape: a 64 x 64 output tile per block (16 x 16 threads, 4 x 4 outputs each), the whole
// token range walked 16 tokens at a time, fp32 FMAs, one owner per output element.
template <typename T>
__global__ __launch_bounds__(256) void gram_generic(const T *__restrict__ x, int64_t n_tokens, int64_t channels,
                                                    int64_t ld, float *__restrict__ h, int64_t ld_h) {
    __shared__ float xa[16][64 + 4], xb[16][64 + 4];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t m0 = static_cast<int64_t>(blockIdx.y) * 64, n0 = static_cast<int64_t>(blockIdx.x) * 64;
    float acc[4][4] = {};
    for (int64_t t0 = 0; t0 < n_tokens; t0 += 16) {
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            const int r = e >> 6, c = e & 63;
            const int64_t t = t0 + r;
            xa[r][c] = (t < n_tokens && m0 + c < channels) ? widen(x[t * ld + m0 + c]) : 0.f;
            xb[r][c] = (t < n_tokens && n0 + c < channels) ? widen(x[t * ld + n0 + c]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                av[i] = xa[r][ty * 4 + i];
                bv[i] = xb[r][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t gi = m0 + ty * 4 + i, gj = n0 + tx * 4 + j;
            if (gi < channels && gj < channels) h[gi * ld_h + gj] += acc[i][j];
        }
}

struct GramPlan {
    bool mfma;
    int n_tiles, n_pairs, n_splits;
    int64_t tokens_per_split;
};

GramPlan plan_gram(const void *x, int dtype, int64_t n_tokens, int64_t channels, int64_t ld) {
    GramPlan g = {};
    g.mfma = dtype == PRUNE_BF16 && packet_ok(x, channels, ld) && channels <= 65536 && n_tokens > 0;
    if (!g.mfma) return g;
    g.n_tiles = static_cast<int>(ceil_div(channels, kTile));
    g.n_pairs = g.n_tiles * (g.n_tiles + 1) / 2;
    int64_t want = ceil_div(kTargetBlocks, g.n_pairs);
    if (want > kMaxSplits) want = kMaxSplits;
    int64_t per = ceil_div(ceil_div(n_tokens, want), kStep) * kStep;
    g.tokens_per_split = per;
    g.n_splits = static_cast<int>(ceil_div(n_tokens, per));
    return g;
}

}  // namespace

size_t hessian_workspace_bytes(int64_t n_tokens, int64_t channels) {
    // sized for the matrix-core path whether or not a particular call can take it
    if (n_tokens <= 0 || channels <= 0) return 0;
    const int64_t n_tiles = ceil_div(channels, kTile), n_pairs = n_tiles * (n_tiles + 1) / 2;
    int64_t want = ceil_div(kTargetBlocks, n_pairs);
    if (want > kMaxSplits) want = kMaxSplits;
    const int64_t per = ceil_div(ceil_div(n_tokens, want), kStep) * kStep;
    const int64_t n_splits = ceil_div(n_tokens, per);
    return static_cast<size_t>(n_splits * n_pairs) * kTile * kTile * sizeof(float);
}

}  // namespace mp

extern "C" size_t prune_hessian_workspace_bytes(int64_t n_tokens, int64_t channels) {
    const size_t n = mp::hessian_workspace_bytes(n_tokens, channels);
    return (n + 255) / 256 * 256;
}

extern "C" int prune_hessian_accumulate(const void *x, int dtype, int64_t n_tokens, int64_t channels, int64_t ld_x,
                                        float *h, int64_t ld_h, void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_tokens < 0 || channels <= 0 || ld_x < channels || ld_h < channels || channels > 0x7fffffff)
        return PRUNE_ERR_SHAPE;
    if (!h || (!x && n_tokens > 0)) return PRUNE_ERR_NULL;
    if (!aligned_to(x, elem_size(dtype)) || !aligned_to(h, 4) || (ws && !aligned_to(ws, 16)))
        return PRUNE_ERR_ALIGNMENT;
    if (n_tokens == 0) return PRUNE_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const GramPlan g = plan_gram(x, dtype, n_tokens, channels, ld_x);
    if (g.mfma) {
        const size_t need = static_cast<size_t>(g.n_splits) * g.n_pairs * kTile * kTile * sizeof(float);
        if (!ws) return PRUNE_ERR_NULL;
        if (ws_bytes < need) return PRUNE_ERR_WORKSPACE;
        float *partials = static_cast<float *>(ws);
        hipLaunchKernelGGL(gram_tiles_bf16, dim3(static_cast<unsigned>(g.n_splits * g.n_pairs)), dim3(kGramBlock), 0,
                           stream, static_cast<const bf16_t *>(x), n_tokens, static_cast<int>(channels), ld_x,
                           g.n_tiles, g.n_pairs, g.tokens_per_split, partials);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        hipLaunchKernelGGL(gram_reduce, dim3(static_cast<unsigned>(g.n_pairs), 64), dim3(256), 0, stream, partials,
                           g.n_splits, g.n_pairs, g.n_tiles, static_cast<int>(channels), h, ld_h);
        return launch_status();
    }
    const dim3 grid(static_cast<unsigned>(ceil_div(channels, 64)), static_cast<unsigned>(ceil_div(channels, 64)));
    if (grid.y > 65535) return PRUNE_ERR_SHAPE;
    if (dtype == PRUNE_BF16)
        hipLaunchKernelGGL(gram_generic<bf16_t>, grid, dim3(256), 0, stream, static_cast<const bf16_t *>(x), n_tokens,
                           channels, ld_x, h, ld_h);
    else
        hipLaunchKernelGGL(gram_generic<float>, grid, dim3(256), 0, stream, static_cast<const float *>(x), n_tokens,
                           channels, ld_x, h, ld_h);
    return launch_status();
}
