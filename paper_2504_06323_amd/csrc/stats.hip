// Activation statistics: per-input-channel sum of squares over the calibration
// tokens (the l2-norm term of Eq. 5, gathered over all samples as in
// Algorithm 1), and its square root.
//
// HBM-bound streaming reduction.  Each thread owns 8 adjacent channels (one
// 128-bit load per row for bf16) and walks down a stripe of rows keeping 8
// private float accumulators, so nothing crosses lanes while streaming.  A
// block covers 2048 adjacent channels (4 KB of every row it touches); the grid
// is (channel tiles) x (row stripes), one resident block per compute unit.  A
// thread sums at most 1024 rows in float before folding into a double, so the
// error does not grow with the number of calibration tokens.  Each block writes
// one row of partials; a second small kernel adds the stripes in a fixed order
// in double and folds them into the caller's running sums.
#include "common.hpp"

namespace mp {

namespace {

constexpr int kBlock = 256;
// One resident block per compute unit (MI355X has 256): measured fastest.  Long
// private stripes stream at ~7.1 TB/s; more, shorter blocks lose up to 25 % to the
// tail wave of blocks and to the extra partial rows.
constexpr int kTargetBlocks = 256;
constexpr int kMinRowsPerBlock = 32;
constexpr int kMaxStripes = 4096;
constexpr int kFoldRows = 1024;  // rows summed in single precision before a fold into double (multiple of 8)

template <typename T, int UNROLL, int BLOCK>
__global__ __launch_bounds__(BLOCK) void colsumsq_partial_vec(const T *__restrict__ x, int64_t n_rows,
                                                               int64_t n_cols, int64_t ld, int64_t rows_per_block,
                                                               float *__restrict__ partials) {
    const int64_t c0 = (static_cast<int64_t>(blockIdx.x) * BLOCK + threadIdx.x) * 8;
    if (c0 >= n_cols) return;  // n_cols is a multiple of 8 on this path; no barriers below
    const int64_t t0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
    int64_t t1 = t0 + rows_per_block;
    if (t1 > n_rows) t1 = n_rows;

    // Single-precision accumulation never runs over more than kFoldRows rows: after that the eight sums are
    // folded into doubles, so the rounding error of a channel does not grow with the length of the stripe.
    double tot[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) tot[e] = 0.0;

    const T *p = x + t0 * ld + c0;
    int64_t t = t0;
    while (t < t1) {
        const int64_t te = t + kFoldRows < t1 ? t + kFoldRows : t1;
        float acc[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) acc[e] = 0.f;
        for (; t + UNROLL <= te; t += UNROLL) {
            Packet<T, 8> pk[UNROLL];
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) pk[u].template load<true>(p + u * ld);
            float s[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) s[e] = 0.f;
#pragma unroll
            for (int u = 0; u < UNROLL; ++u) {
                float v[8];
                pk[u].to_float(v);
#pragma unroll
                for (int e = 0; e < 8; ++e) s[e] = fmaf(v[e], v[e], s[e]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] += s[e];
            p += UNROLL * ld;
        }
        for (; t < te; ++t) {
            Packet<T, 8> pk;
            pk.template load<true>(p);
            float v[8];
            pk.to_float(v);
#pragma unroll
            for (int e = 0; e < 8; ++e) acc[e] = fmaf(v[e], v[e], acc[e]);
            p += ld;
        }
#pragma unroll
        for (int e = 0; e < 8; ++e) tot[e] += static_cast<double>(acc[e]);
    }
    float out[8];
#pragma unroll
    for (int e = 0; e < 8; ++e) out[e] = static_cast<float>(tot[e]);
    store_floats(partials + static_cast<int64_t>(blockIdx.y) * n_cols + c0, out);
}

// any width / pitch / alignment: one channel per thread, lanes on adjacent channels
template <typename T>
__global__ __launch_bounds__(kBlock) void colsumsq_partial_scalar(const T *__restrict__ x, int64_t n_rows,
                                                                  int64_t n_cols, int64_t ld,
                                                                  int64_t rows_per_block,
                                                                  float *__restrict__ partials) {
    const int64_t c = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (c >= n_cols) return;
    const int64_t t0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
    int64_t t1 = t0 + rows_per_block;
    if (t1 > n_rows) t1 = n_rows;
    double tot = 0.0;  // folded every kFoldRows rows, as in the packet kernel
    const T *p = x + t0 * ld + c;
    int64_t t = t0;
    while (t < t1) {
        const int64_t te = t + kFoldRows < t1 ? t + kFoldRows : t1;
        float a0 = 0.f, a1 = 0.f, a2 = 0.f, a3 = 0.f;
        for (; t + 4 <= te; t += 4) {
            const float v0 = widen(p[0]), v1 = widen(p[ld]), v2 = widen(p[2 * ld]), v3 = widen(p[3 * ld]);
            a0 = fmaf(v0, v0, a0);
            a1 = fmaf(v1, v1, a1);
            a2 = fmaf(v2, v2, a2);
            a3 = fmaf(v3, v3, a3);
            p += 4 * ld;
        }
        for (; t < te; ++t) {
            const float v = widen(p[0]);
            a0 = fmaf(v, v, a0);
            p += ld;
        }
        tot += static_cast<double>((a0 + a1) + (a2 + a3));
    }
    partials[static_cast<int64_t>(blockIdx.y) * n_cols + c] = static_cast<float>(tot);
}

// sumsq[c] += sum over stripes of partials[s, c].  A block owns 64 adjacent channels; its 16 waves
// each add every 16th stripe (4 independent chains per thread keep loads in flight), then the 16
// per-wave sums of a channel are added in index order.
constexpr int kReduceBlock = 1024;
constexpr int kReduceGroups = kReduceBlock / kWave;

// accumulate == 0 overwrites sumsq instead; norms (optional) receives sqrt of the new sumsq.
__global__ __launch_bounds__(kReduceBlock) void colsumsq_reduce(const float *__restrict__ partials, int n_stripes,
                                                                int64_t n_cols, float *__restrict__ sumsq,
                                                                int accumulate, float *__restrict__ norms) {
    __shared__ double sm[kReduceGroups][kWave];
    const int lane = threadIdx.x & (kWave - 1), grp = threadIdx.x / kWave;
    const int64_t c = static_cast<int64_t>(blockIdx.x) * kWave + lane;
    double a0 = 0.0, a1 = 0.0, a2 = 0.0, a3 = 0.0;
    if (c < n_cols) {
        const float *p = partials + c;
        int s = grp;
        for (; s + 3 * kReduceGroups < n_stripes; s += 4 * kReduceGroups) {
            const float v0 = p[static_cast<int64_t>(s) * n_cols];
            const float v1 = p[static_cast<int64_t>(s + kReduceGroups) * n_cols];
            const float v2 = p[static_cast<int64_t>(s + 2 * kReduceGroups) * n_cols];
            const float v3 = p[static_cast<int64_t>(s + 3 * kReduceGroups) * n_cols];
            a0 += static_cast<double>(v0);
            a1 += static_cast<double>(v1);
            a2 += static_cast<double>(v2);
            a3 += static_cast<double>(v3);
        }
        for (; s < n_stripes; s += kReduceGroups) a0 += static_cast<double>(p[static_cast<int64_t>(s) * n_cols]);
    }
    sm[grp][lane] = (a0 + a1) + (a2 + a3);
    __syncthreads();
    if (grp == 0 && c < n_cols) {
        double tot = 0.0;
#pragma unroll
        for (int g = 0; g < kReduceGroups; ++g) tot += sm[g][lane];
        const float total = static_cast<float>((accumulate ? static_cast<double>(sumsq[c]) : 0.0) + tot);
        sumsq[c] = total;
        if (norms) norms[c] = sqrtf(total);  // correctly rounded (hipcc default)
    }
}

__global__ __launch_bounds__(kBlock) void sqrt_kernel(const float *__restrict__ sumsq, int64_t n,
                                                      float *__restrict__ norms) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n) norms[i] = sqrtf(sumsq[i]);  // correctly rounded (hipcc default)
}

template <typename T>
int launch_colsum_t(const T *x, int64_t n_rows, int64_t n_cols, int64_t ld, float *sumsq, float *partials,
                    hipStream_t stream, bool accumulate, float *norms) {
    const ColsumPlan pl = plan_colsum(n_rows, n_cols);
    if (n_rows == 0) {  // nothing to stream: the reduction alone writes zeros (or leaves the running sums)
        hipLaunchKernelGGL(colsumsq_reduce, dim3(static_cast<unsigned>(ceil_div(n_cols, kWave))), dim3(kReduceBlock),
                           0, stream, partials, 0, n_cols, sumsq, accumulate ? 1 : 0, norms);
        return launch_status();
    }
    if (packet_ok(x, n_cols, ld)) {
        dim3 grid(pl.tiles_vec, pl.stripes);
        hipLaunchKernelGGL((colsumsq_partial_vec<T, 8, kBlock>), grid, dim3(kBlock), 0, stream, x, n_rows, n_cols, ld,
                           pl.rows_per_block, partials);
    } else {
        dim3 grid(pl.tiles_scalar, pl.stripes);
        hipLaunchKernelGGL((colsumsq_partial_scalar<T>), grid, dim3(kBlock), 0, stream, x, n_rows, n_cols, ld,
                           pl.rows_per_block, partials);
    }
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    hipLaunchKernelGGL(colsumsq_reduce, dim3(static_cast<unsigned>(ceil_div(n_cols, kWave))), dim3(kReduceBlock), 0,
                       stream, partials, pl.stripes, n_cols, sumsq, accumulate ? 1 : 0, norms);
    return launch_status();
}

}  // namespace

ColsumPlan plan_colsum(int64_t n_rows, int64_t n_cols) {
    ColsumPlan pl;
    pl.tiles_vec = static_cast<int>(ceil_div(n_cols, kBlock * 8));
    pl.tiles_scalar = static_cast<int>(ceil_div(n_cols, kBlock));
    int64_t max_stripes = kTargetBlocks / pl.tiles_vec;
    if (max_stripes < 1) max_stripes = 1;
    if (max_stripes > kMaxStripes) max_stripes = kMaxStripes;
    int64_t rpb = ceil_div(n_rows, max_stripes);
    if (rpb < kMinRowsPerBlock) rpb = kMinRowsPerBlock;
    rpb = ceil_div(rpb, 8) * 8;
    pl.rows_per_block = rpb;
    pl.stripes = static_cast<int>(ceil_div(n_rows, rpb));
    if (pl.stripes < 1) pl.stripes = 1;
    return pl;
}

size_t colsum_workspace_bytes(int64_t n_rows, int64_t n_cols) {
    const ColsumPlan pl = plan_colsum(n_rows, n_cols);
    return static_cast<size_t>(pl.stripes) * static_cast<size_t>(n_cols) * sizeof(float);
}

int launch_colsum(const void *x, int dtype, int64_t n_rows, int64_t n_cols, int64_t ld, float *sumsq, void *ws,
                  hipStream_t stream, bool accumulate, float *norms) {
    float *partials = static_cast<float *>(ws);
    if (dtype == PRUNE_BF16)
        return launch_colsum_t(static_cast<const bf16_t *>(x), n_rows, n_cols, ld, sumsq, partials, stream, accumulate,
                               norms);
    return launch_colsum_t(static_cast<const float *>(x), n_rows, n_cols, ld, sumsq, partials, stream, accumulate,
                           norms);
}

}  // namespace mp

extern "C" int prune_stats_accumulate(const void *x, int dtype, int64_t n_tokens, int64_t n_channels, int64_t ld_x,
                                      float *sumsq, void *ws, size_t ws_bytes, void *stream) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_tokens < 0 || n_channels <= 0 || ld_x < n_channels) return PRUNE_ERR_SHAPE;
    if (!sumsq) return PRUNE_ERR_NULL;
    if (n_tokens == 0) return PRUNE_OK;
    if (!x || !ws) return PRUNE_ERR_NULL;
    if (!aligned_to(x, elem_size(dtype)) || !aligned_to(sumsq, 4) || !aligned_to(ws, 16)) return PRUNE_ERR_ALIGNMENT;
    if (ws_bytes < colsum_workspace_bytes(n_tokens, n_channels)) return PRUNE_ERR_WORKSPACE;
    return launch_colsum(x, dtype, n_tokens, n_channels, ld_x, sumsq, ws, static_cast<hipStream_t>(stream));
}

extern "C" int prune_stats_norms(const void *x, int dtype, int64_t n_tokens, int64_t n_channels, int64_t ld_x,
                                 float *sumsq, float *norms, void *ws, size_t ws_bytes, void *stream) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_tokens < 0 || n_channels <= 0 || ld_x < n_channels) return PRUNE_ERR_SHAPE;
    if (!sumsq || !norms || !ws || (n_tokens > 0 && !x)) return PRUNE_ERR_NULL;
    if ((x && !aligned_to(x, elem_size(dtype))) || !aligned_to(sumsq, 4) || !aligned_to(norms, 4) ||
        !aligned_to(ws, 16))
        return PRUNE_ERR_ALIGNMENT;
    if (ws_bytes < colsum_workspace_bytes(n_tokens > 0 ? n_tokens : 1, n_channels)) return PRUNE_ERR_WORKSPACE;
    return launch_colsum(x, dtype, n_tokens, n_channels, ld_x, sumsq, ws, static_cast<hipStream_t>(stream), false,
                         norms);
}

extern "C" int prune_stats_finalize(const float *sumsq, int64_t n_channels, float *norms, void *stream) {
    using namespace mp;
    if (n_channels <= 0) return PRUNE_ERR_SHAPE;
    if (!sumsq || !norms) return PRUNE_ERR_NULL;
    if (!aligned_to(sumsq, 4) || !aligned_to(norms, 4)) return PRUNE_ERR_ALIGNMENT;
    hipLaunchKernelGGL(sqrt_kernel, dim3(static_cast<unsigned>(ceil_div(n_channels, kBlock))), dim3(kBlock), 0,
                       static_cast<hipStream_t>(stream), sumsq, n_channels, norms);
    return launch_status();
}
