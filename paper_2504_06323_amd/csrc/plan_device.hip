// The projection planner (Algorithm 1's normalize(R_LLM) and the Projection
// Planner of Section 3.3) as one small kernel, so that ranking, planning and
// pruning can be enqueued back to back without the host ever reading the
// outlier counts.  The arithmetic and its order are those of the host planner:
// every per-projection expression is evaluated independently, the one sum (the
// mean of the normalised ratios) is accumulated by a single thread in index
// order, and min / max do not depend on order.
#include "common.hpp"

namespace mp {

namespace {

constexpr int kPlanBlock = 256;
constexpr int kPlanStage = 2048;  // entries of a group that are staged in LDS for the ordered sum

__device__ __forceinline__ double block_min_max(double v, bool take_max, double *scratch) {
    const int tid = threadIdx.x;
    scratch[tid] = v;
    __syncthreads();
    for (int s = kPlanBlock / 2; s > 0; s >>= 1) {
        if (tid < s) {
            const double a = scratch[tid], b = scratch[tid + s];
            scratch[tid] = take_max ? fmax(a, b) : fmin(a, b);
        }
        __syncthreads();
    }
    const double out = scratch[0];
    __syncthreads();
    return out;
}

// One block.  Groups are the sets over which the ratios are normalised: all entries (n_groups == 1),
// or, per projection type m, the entries l * n_proj + m (n_groups == n_proj).  by_layer (layer pruning; n_groups
// == n_proj then): the ratio of a layer's pooled counts sits in the slot of the layer's first projection, only
// group 0 -- those slots -- is normalised and spread, and the layer's other projections copy the result.
__global__ __launch_bounds__(kPlanBlock) void plan_kernel(const unsigned long long *__restrict__ counts,
                                                          const unsigned long long *__restrict__ numels,
                                                          const int64_t *__restrict__ cols, int n, int n_groups,
                                                          int by_layer, double p, double lambda,
                                                          double *__restrict__ sparsity,
                                                          uint32_t *__restrict__ zeros_per_row,
                                                          int *__restrict__ flags) {
    __shared__ double scratch[kPlanBlock];
    __shared__ double stage[kPlanStage];
    __shared__ double mean_sh;
    __shared__ int clamped_sh, invalid_sh;
    const int tid = threadIdx.x;
    if (tid == 0) {
        clamped_sh = 0;
        invalid_sh = 0;
    }
    __syncthreads();
    // R = O / C * 100, parked in the output array
    for (int i = tid; i < n; i += kPlanBlock) {
        const unsigned long long c = counts[i], e = numels[i];
        if (e == 0 || c > e || cols[i] <= 0) invalid_sh = 1;
        sparsity[i] = e ? 100.0 * static_cast<double>(c) / static_cast<double>(e) : 0.0;
    }
    __syncthreads();
    const int per_group = n / n_groups;
    if (by_layer) {
        for (int l = tid; l < per_group; l += kPlanBlock) {
            unsigned long long c = 0, e = 0;
            for (int m = 0; m < n_groups; ++m) {
                c += counts[l * n_groups + m];
                e += numels[l * n_groups + m];
            }
            sparsity[l * n_groups] = e ? 100.0 * static_cast<double>(c) / static_cast<double>(e) : 0.0;
        }
        __syncthreads();
    }
    for (int g = 0; g < (by_layer ? 1 : n_groups); ++g) {
        // entry j of group g sits at g + j * n_groups (n_groups == 1: all entries in order)
        double lo = INFINITY, hi = -INFINITY;
        for (int j = tid; j < per_group; j += kPlanBlock) {
            const double r = sparsity[g + j * n_groups];
            lo = fmin(lo, r);
            hi = fmax(hi, r);
        }
        lo = block_min_max(lo, false, scratch);
        hi = block_min_max(hi, true, scratch);
        if (hi == lo) {
            for (int j = tid; j < per_group; j += kPlanBlock) sparsity[g + j * n_groups] = p;
            __syncthreads();
            continue;
        }
        // the normalised ratios also go to LDS when the group fits, so that the one thread that adds them up
        // in index order reads them at LDS latency, eight loads at a time, not one global load per addition
        const bool staged = per_group <= kPlanStage;
        for (int j = tid; j < per_group; j += kPlanBlock) {
            const int i = g + j * n_groups;
            const double v = (sparsity[i] - lo) / (hi - lo);
            sparsity[i] = v;
            if (staged) stage[j] = v;
        }
        __syncthreads();
        if (tid == 0) {
            double mean_hat = 0.0;
            if (staged) {
                int j = 0;
                for (; j + 8 <= per_group; j += 8) {
                    double v[8];
#pragma unroll
                    for (int u = 0; u < 8; ++u) v[u] = stage[j + u];
#pragma unroll
                    for (int u = 0; u < 8; ++u) mean_hat += v[u];
                }
                for (; j < per_group; ++j) mean_hat += stage[j];
            } else {
                for (int j = 0; j < per_group; ++j) mean_hat += sparsity[g + j * n_groups];
            }
            mean_sh = mean_hat / static_cast<double>(per_group);
        }
        __syncthreads();
        const double mean_hat = mean_sh;
        for (int j = tid; j < per_group; j += kPlanBlock) {
            const int i = g + j * n_groups;
            sparsity[i] = p + 2.0 * lambda * (mean_hat - sparsity[i]);
        }
        __syncthreads();
    }
    if (by_layer) {  // (the sources, slots l * n_groups, are not written here)
        for (int i = tid; i < n; i += kPlanBlock)
            if (i % n_groups) sparsity[i] = sparsity[i - i % n_groups];
        __syncthreads();
    }
    for (int i = tid; i < n; i += kPlanBlock) {
        const double width = static_cast<double>(cols[i] > 0 ? cols[i] : 1);
        const double hi = 1.0 - 1.0 / width;
        const double s0 = sparsity[i];
        double s = s0;
        if (s < 0.0) s = 0.0;
        if (s > hi) s = hi;
        if (s != s0) clamped_sh = 1;
        sparsity[i] = s;
        zeros_per_row[i] = static_cast<uint32_t>(floor(s * width));
    }
    __syncthreads();
    if (tid == 0) {
        flags[0] = clamped_sh;
        flags[1] = invalid_sh;
    }
}

}  // namespace

}  // namespace mp

extern "C" int prune_plan_sparsity_device(const unsigned long long *counts, const unsigned long long *numels,
                                          const int64_t *cols, int n_layers, int n_proj, double p, double lambda,
                                          int scope, double *sparsity_out, uint32_t *zeros_per_row_out, int *flags_out,
                                          void *stream_) {
    using namespace mp;
    if (!counts || !numels || !cols || !sparsity_out || !zeros_per_row_out || !flags_out) return PRUNE_ERR_NULL;
    if (n_layers <= 0 || n_proj <= 0 || static_cast<int64_t>(n_layers) * n_proj > (1 << 20)) return PRUNE_ERR_SHAPE;
    if (!(p >= 0.0 && p < 1.0) || !(lambda >= 0.0)) return PRUNE_ERR_RANGE;
    if (scope != PRUNE_SCOPE_GLOBAL && scope != PRUNE_SCOPE_CATEGORY && scope != PRUNE_SCOPE_LAYER) return PRUNE_ERR_RANGE;
    if (!aligned_to(counts, 8) || !aligned_to(numels, 8) || !aligned_to(cols, 8) || !aligned_to(sparsity_out, 8) ||
        !aligned_to(zeros_per_row_out, 4) || !aligned_to(flags_out, 4))
        return PRUNE_ERR_ALIGNMENT;
    const int n = n_layers * n_proj;
    const int n_groups = scope == PRUNE_SCOPE_GLOBAL ? 1 : n_proj;
    hipLaunchKernelGGL(plan_kernel, dim3(1), dim3(kPlanBlock), 0, static_cast<hipStream_t>(stream_), counts, numels,
                       cols, n, n_groups, scope == PRUNE_SCOPE_LAYER ? 1 : 0, p, lambda, sparsity_out, zeros_per_row_out,
                       flags_out);
    return launch_status();
}
