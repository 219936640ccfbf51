// Weight metric (Eq. 5) and projection outlier count (Eq. 6; Algorithm 1's
// C / O steps).
//
// Both passes stream the projection once.  A thread owns 8 adjacent input
// channels: it loads their 8 norms once and then walks down a stripe of output
// rows with 128-bit loads, so the norm vector costs almost no traffic.  The
// metric sum is kept per thread in float for a handful of rows, folded into a
// double, reduced over the block in a fixed tree and written as one partial per
// block; a one-block kernel adds the partials in index order.  The count pass
// compares every metric with tau = float(alpha * mean) and adds one integer
// per block to the result with an integer atomic.
#include "common.hpp"

namespace mp {

namespace {

constexpr int kBlock = 256;
constexpr int kTargetBlocks = 512;  // two resident blocks per compute unit: long stripes stream best
constexpr int kMinRowsPerBlock = 8;
constexpr int kUnroll = 4;

struct ScanPlan {
    int tiles_vec, tiles_scalar, stripes;
    int64_t rows_per_block;
};

ScanPlan plan_scan(int64_t rows, int64_t cols) {
    ScanPlan pl;
    pl.tiles_vec = static_cast<int>(ceil_div(cols, kBlock * 8));
    pl.tiles_scalar = static_cast<int>(ceil_div(cols, kBlock));
    int64_t max_stripes = kTargetBlocks / pl.tiles_vec;
    if (max_stripes < 1) max_stripes = 1;
    int64_t rpb = ceil_div(rows, max_stripes);
    if (rpb < kMinRowsPerBlock) rpb = kMinRowsPerBlock;
    rpb = ceil_div(rpb, kUnroll) * kUnroll;
    pl.rows_per_block = rpb;
    pl.stripes = static_cast<int>(ceil_div(rows, rpb));
    return pl;
}

__device__ __forceinline__ float threshold_from_sum(float alpha, const double *score_sum, int64_t numel) {
    return static_cast<float>(static_cast<double>(alpha) * (*score_sum) / static_cast<double>(numel));
}

// MODE 0: metric sum (+ optional materialisation);  MODE 1: count of metric > tau.
// FROM_SCORES: the rows hold precomputed float metrics instead of weights.
template <typename T, int VEC, int MODE, bool WRITE_SCORES, bool FROM_SCORES>
__global__ __launch_bounds__(kBlock) void metric_scan(const T *__restrict__ w, int64_t rows, int64_t cols,
                                                      int64_t ld, const float *__restrict__ norms,
                                                      float *__restrict__ scores, int64_t rows_per_block,
                                                      double *__restrict__ partials, float alpha,
                                                      const double *__restrict__ score_sum,
                                                      unsigned long long *__restrict__ count) {
    __shared__ double sm_d[kBlock / kWave];
    __shared__ uint32_t sm_u[kBlock / kWave];
    const int64_t c0 = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * VEC;
    const bool active = c0 < cols;
    const int64_t r0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
    int64_t r1 = r0 + rows_per_block;
    if (r1 > rows) r1 = rows;

    float nrm[VEC];
#pragma unroll
    for (int e = 0; e < VEC; ++e) nrm[e] = 1.f;
    if (active && !FROM_SCORES) load_floats(norms + c0, nrm);

    __shared__ float sm_tau;
    float tau = 0.f;
    if (MODE == 1) {  // one double division per block, not per thread
        if (threadIdx.x == 0) sm_tau = threshold_from_sum(alpha, score_sum, rows * cols);
        __syncthreads();
        tau = sm_tau;
    }

    double dsum = 0.0;
    uint32_t cnt = 0;
    if (active) {
        const T *p = w + r0 * ld + c0;
        float *sp = WRITE_SCORES ? scores + r0 * cols + c0 : nullptr;
        int64_t r = r0;
        for (; r + kUnroll <= r1; r += kUnroll) {
            Packet<T, VEC> pk[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) pk[u].template load<true>(p + u * ld);
            float fs = 0.f;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float v[VEC], om[VEC];
                pk[u].to_float(v);
#pragma unroll
                for (int e = 0; e < VEC; ++e) om[e] = FROM_SCORES ? v[e] : metric(v[e], nrm[e]);
                if (MODE == 0) {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) fs += om[e];
                    if (WRITE_SCORES) store_floats(sp + u * cols, om);
                } else {
#pragma unroll
                    for (int e = 0; e < VEC; ++e) cnt += (om[e] > tau) ? 1u : 0u;
                }
            }
            dsum += static_cast<double>(fs);
            p += kUnroll * ld;
            if (WRITE_SCORES) sp += kUnroll * cols;
        }
        for (; r < r1; ++r) {
            Packet<T, VEC> pk;
            pk.template load<true>(p);
            float v[VEC], om[VEC];
            pk.to_float(v);
            float fs = 0.f;
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                om[e] = FROM_SCORES ? v[e] : metric(v[e], nrm[e]);
                fs += om[e];
                cnt += (MODE == 1 && om[e] > tau) ? 1u : 0u;
            }
            if (MODE == 0 && WRITE_SCORES) store_floats(sp, om);
            dsum += static_cast<double>(fs);
            p += ld;
            if (WRITE_SCORES) sp += cols;
        }
    }
    if (MODE == 0) {
        const double tot = block_sum<kBlock>(dsum, sm_d);
        if (threadIdx.x == 0) partials[static_cast<int64_t>(blockIdx.y) * gridDim.x + blockIdx.x] = tot;
    } else {
        const uint32_t tot = block_sum<kBlock>(cnt, sm_u);
        if (threadIdx.x == 0 && tot) atomicAdd(count, static_cast<unsigned long long>(tot));
    }
}

// one block: out = sum of n partials, index order within each thread, fixed tree across threads
__global__ __launch_bounds__(kBlock) void sum_partials(const double *__restrict__ partials, int n,
                                                       double *__restrict__ out) {
    __shared__ double sm[kBlock];
    double a = 0.0;
    for (int i = threadIdx.x; i < n; i += kBlock) a += partials[i];
    sm[threadIdx.x] = a;
    __syncthreads();
    for (int s = kBlock / 2; s > 0; s >>= 1) {
        if (static_cast<int>(threadIdx.x) < s) sm[threadIdx.x] += sm[threadIdx.x + s];
        __syncthreads();
    }
    if (threadIdx.x == 0) *out = sm[0];
}

__global__ void outlier_prepare(float alpha, const double *__restrict__ score_sum, int64_t numel,
                                unsigned long long *__restrict__ count, float *__restrict__ tau) {
    if (threadIdx.x == 0 && blockIdx.x == 0) {
        *count = 0ull;
        if (tau) *tau = threshold_from_sum(alpha, score_sum, numel);
    }
}

template <typename T, int MODE, bool WRITE_SCORES, bool FROM_SCORES>
int launch_scan(const T *w, int64_t rows, int64_t cols, int64_t ld, const float *norms, float *scores,
                double *partials, float alpha, const double *score_sum, unsigned long long *count,
                hipStream_t stream, int *n_partials) {
    const ScanPlan pl = plan_scan(rows, cols);
    bool vec = packet_ok(w, cols, ld);
    if (!FROM_SCORES && !aligned_to(norms, 16)) vec = false;
    if (WRITE_SCORES && !aligned_to(scores, 16)) vec = false;
    const int tiles = vec ? pl.tiles_vec : pl.tiles_scalar;
    dim3 grid(tiles, pl.stripes);
    if (n_partials) *n_partials = tiles * pl.stripes;
    if (vec)
        hipLaunchKernelGGL((metric_scan<T, 8, MODE, WRITE_SCORES, FROM_SCORES>), grid, dim3(kBlock), 0, stream, w,
                           rows, cols, ld, norms, scores, pl.rows_per_block, partials, alpha, score_sum, count);
    else
        hipLaunchKernelGGL((metric_scan<T, 1, MODE, WRITE_SCORES, FROM_SCORES>), grid, dim3(kBlock), 0, stream, w,
                           rows, cols, ld, norms, scores, pl.rows_per_block, partials, alpha, score_sum, count);
    return launch_status();
}

}  // namespace

size_t score_workspace_bytes(int64_t rows, int64_t cols) {
    const ScanPlan pl = plan_scan(rows, cols);
    const size_t tiles = static_cast<size_t>(pl.tiles_scalar > pl.tiles_vec ? pl.tiles_scalar : pl.tiles_vec);
    return tiles * static_cast<size_t>(pl.stripes) * sizeof(double);
}

}  // namespace mp

extern "C" int prune_score(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld_w, const float *norms,
                           float *scores, double *score_sum, void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (rows <= 0 || cols <= 0 || ld_w < cols) return PRUNE_ERR_SHAPE;
    if (!w || !norms || !score_sum || !ws) return PRUNE_ERR_NULL;
    if (!aligned_to(w, elem_size(dtype)) || !aligned_to(norms, 4) || !aligned_to(score_sum, 8) ||
        !aligned_to(ws, 16) || (scores && !aligned_to(scores, 4)))
        return PRUNE_ERR_ALIGNMENT;
    if (ws_bytes < score_workspace_bytes(rows, cols)) return PRUNE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    double *partials = static_cast<double *>(ws);
    int n_partials = 0, st;
    if (dtype == PRUNE_BF16) {
        const bf16_t *wp = static_cast<const bf16_t *>(w);
        st = scores ? launch_scan<bf16_t, 0, true, false>(wp, rows, cols, ld_w, norms, scores, partials, 0.f, nullptr,
                                                          nullptr, stream, &n_partials)
                    : launch_scan<bf16_t, 0, false, false>(wp, rows, cols, ld_w, norms, nullptr, partials, 0.f,
                                                           nullptr, nullptr, stream, &n_partials);
    } else {
        const float *wp = static_cast<const float *>(w);
        st = scores ? launch_scan<float, 0, true, false>(wp, rows, cols, ld_w, norms, scores, partials, 0.f, nullptr,
                                                         nullptr, stream, &n_partials)
                    : launch_scan<float, 0, false, false>(wp, rows, cols, ld_w, norms, nullptr, partials, 0.f,
                                                          nullptr, nullptr, stream, &n_partials);
    }
    if (st != PRUNE_OK) return st;
    hipLaunchKernelGGL(sum_partials, dim3(1), dim3(kBlock), 0, stream, partials, n_partials, score_sum);
    return launch_status();
}

extern "C" int prune_outlier_ratio(const void *w, int dtype, int64_t rows, int64_t cols, int64_t ld_w,
                                   const float *norms, const float *scores, float alpha, const double *score_sum,
                                   unsigned long long *count, float *tau, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (rows <= 0 || cols <= 0 || (!scores && ld_w < cols)) return PRUNE_ERR_SHAPE;
    if (!score_sum || !count) return PRUNE_ERR_NULL;
    if (!scores && (!w || !norms)) return PRUNE_ERR_NULL;
    if (!(alpha >= 0.f)) return PRUNE_ERR_RANGE;
    if ((w && !aligned_to(w, elem_size(dtype))) || (norms && !aligned_to(norms, 4)) ||
        (scores && !aligned_to(scores, 4)) || !aligned_to(score_sum, 8) || !aligned_to(count, 8) ||
        (tau && !aligned_to(tau, 4)))
        return PRUNE_ERR_ALIGNMENT;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    hipLaunchKernelGGL(outlier_prepare, dim3(1), dim3(kWave), 0, stream, alpha, score_sum, rows * cols, count, tau);
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    if (scores)
        return launch_scan<float, 1, false, true>(scores, rows, cols, cols, nullptr, nullptr, nullptr, alpha,
                                                  score_sum, count, stream, nullptr);
    if (dtype == PRUNE_BF16)
        return launch_scan<bf16_t, 1, false, false>(static_cast<const bf16_t *>(w), rows, cols, ld_w, norms, nullptr,
                                                    nullptr, alpha, score_sum, count, stream, nullptr);
    return launch_scan<float, 1, false, false>(static_cast<const float *>(w), rows, cols, ld_w, norms, nullptr,
                                               nullptr, alpha, score_sum, count, stream, nullptr);
}
