// Ranking of several projections in one go (Algorithm 1's loop over the
// projections of a layer: weight metric, mean, outlier count for each).
//
// Launching the metric-sum and count passes once per projection leaves the GPU
// with seven short kernels per pass and their ramp-up, tail and launch gaps;
// here one launch covers every projection of the batch.  The block index is
// mapped to (projection, channel tile, row stripe) through a small table in the
// kernel arguments; blocks are shared out in proportion to the projections'
// sizes so that every block streams about the same number of bytes.
// Three launches per batch: metric sums -> mean / threshold -> outlier counts.
// With per-projection thresholds (Eq. 6) the results are what prune_score
// followed by prune_outlier_ratio give (sums in a different, but still fixed,
// order); with one threshold for the whole batch the outliers are those of the
// layer-level rule (Eq. 3, Eq. 4) when the batch is one layer.
#include "common.hpp"

namespace mp {

namespace {

constexpr int kBlock = 256;
constexpr int kUnroll = 8;
constexpr int kMaxBatch = 16;
constexpr int kTargetBlocks = 512;  // two resident blocks per compute unit: measured fastest (long stripes)
constexpr int kMaxBlocks = 65536;  // partial sums the workspace holds (scalar path of very wide projections)

struct BatchDesc {
    const void *w;
    const float *norms;
    int64_t rows, ld;
    uint32_t cols, tiles, stripes, rows_per_block;
    uint32_t block0;  // first block of this projection
    uint32_t pad;
};

struct BatchArgs {
    BatchDesc d[kMaxBatch];
    int n;
};

// MODE 0: partial metric sums; MODE 1: outlier counts against tau[p].
// VEC 8: 128-bit row packets; VEC 1: scalar accesses for rows that cannot be moved as packets.
template <typename T, int VEC, int MODE>
__global__ __launch_bounds__(kBlock) void batch_metric_scan(const BatchArgs args, double *__restrict__ partials,
                                                            const float *__restrict__ tau,
                                                            unsigned long long *__restrict__ counts) {
    __shared__ double sm_d[kBlock / kWave];
    __shared__ uint32_t sm_u[kBlock / kWave];
    int p = 0;
    for (int i = 1; i < args.n; ++i)
        if (blockIdx.x >= args.d[i].block0) p = i;
    const BatchDesc &d = args.d[p];
    const uint32_t local = blockIdx.x - d.block0;
    const uint32_t tile = local % d.tiles, stripe = local / d.tiles;
    const uint32_t c0 = (tile * kBlock + threadIdx.x) * VEC;
    const bool active = c0 < d.cols;
    const int64_t r0 = static_cast<int64_t>(stripe) * d.rows_per_block;
    int64_t r1 = r0 + d.rows_per_block;
    if (r1 > d.rows) r1 = d.rows;

    const float th = MODE == 1 ? tau[p] : 0.f;
    double dsum = 0.0;
    uint32_t cnt = 0;
    if (active) {
        float nrm[VEC];
        load_floats(d.norms + c0, nrm);
        const T *ptr = static_cast<const T *>(d.w) + r0 * d.ld + c0;
        int64_t r = r0;
        for (; r + kUnroll <= r1; r += kUnroll) {
            Packet<T, VEC> pk[kUnroll];
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) pk[u].template load<true>(ptr + u * d.ld);
            float fs = 0.f;
#pragma unroll
            for (int u = 0; u < kUnroll; ++u) {
                float v[VEC];
                pk[u].to_float(v);
#pragma unroll
                for (int e = 0; e < VEC; ++e) {
                    const float om = metric(v[e], nrm[e]);
                    if (MODE == 0) fs += om;
                    else cnt += (om > th) ? 1u : 0u;
                }
            }
            dsum += static_cast<double>(fs);
            ptr += kUnroll * d.ld;
        }
        for (; r < r1; ++r) {
            Packet<T, VEC> pk;
            pk.template load<true>(ptr);
            float v[VEC], fs = 0.f;
            pk.to_float(v);
#pragma unroll
            for (int e = 0; e < VEC; ++e) {
                const float om = metric(v[e], nrm[e]);
                if (MODE == 0) fs += om;
                else cnt += (om > th) ? 1u : 0u;
            }
            dsum += static_cast<double>(fs);
            ptr += d.ld;
        }
    }
    if (MODE == 0) {
        const double tot = block_sum<kBlock>(dsum, sm_d);
        if (threadIdx.x == 0) partials[blockIdx.x] = tot;
    } else {
        const uint32_t tot = block_sum<kBlock>(cnt, sm_u);
        if (threadIdx.x == 0 && tot) atomicAdd(counts + p, static_cast<unsigned long long>(tot));
    }
}

// Block p: score_sums[p] = sum of projection p's partials (fixed order); its threshold; zeroed count.
// per_layer == 0: tau[p] = alpha * mean of projection p (Eq. 6).
// per_layer != 0: one tau for all = alpha * mean over every parameter of the batch (Eq. 4); every
// block then adds up all projections itself, in index order, so all blocks get the same value.
__global__ __launch_bounds__(kBlock) void batch_finalize(const BatchArgs args, const double *__restrict__ partials,
                                                         float alpha, int per_layer, double *__restrict__ score_sums,
                                                         float *__restrict__ tau_ws, float *__restrict__ taus,
                                                         unsigned long long *__restrict__ counts) {
    __shared__ double sm[kBlock];
    const int me = blockIdx.x;
    double mine = 0.0, layer_sum = 0.0, layer_numel = 0.0;
    for (int p = per_layer ? 0 : me; p < (per_layer ? args.n : me + 1); ++p) {
        const BatchDesc &d = args.d[p];
        const int n = static_cast<int>(d.tiles * d.stripes);
        double a = 0.0;
        for (int i = threadIdx.x; i < n; i += kBlock) a += partials[d.block0 + i];
        sm[threadIdx.x] = a;
        __syncthreads();
        for (int s = kBlock / 2; s > 0; s >>= 1) {
            if (static_cast<int>(threadIdx.x) < s) sm[threadIdx.x] += sm[threadIdx.x + s];
            __syncthreads();
        }
        const double total = sm[0];
        __syncthreads();
        if (p == me) mine = total;
        layer_sum += total;
        layer_numel += static_cast<double>(d.rows * static_cast<int64_t>(d.cols));
    }
    if (threadIdx.x == 0) {
        const float th = static_cast<float>(static_cast<double>(alpha) * layer_sum / layer_numel);
        score_sums[me] = mine;
        tau_ws[me] = th;
        if (taus) taus[me] = th;
        counts[me] = 0ull;
    }
}

template <typename T, int VEC>
int launch_batch(const BatchArgs &args, int total_blocks, float alpha, int per_layer, double *score_sums,
                 unsigned long long *counts, float *taus, void *ws, hipStream_t stream) {
    double *partials = static_cast<double *>(ws);
    float *tau_ws = reinterpret_cast<float *>(partials + kMaxBlocks);
    hipLaunchKernelGGL((batch_metric_scan<T, VEC, 0>), dim3(total_blocks), dim3(kBlock), 0, stream, args, partials,
                       nullptr, nullptr);
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    hipLaunchKernelGGL(batch_finalize, dim3(args.n), dim3(kBlock), 0, stream, args, partials, alpha, per_layer, score_sums,
                       tau_ws, taus, counts);
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    hipLaunchKernelGGL((batch_metric_scan<T, VEC, 1>), dim3(total_blocks), dim3(kBlock), 0, stream, args, nullptr,
                       tau_ws, counts);
    return launch_status();
}

}  // namespace

size_t rank_batch_workspace_bytes() { return kMaxBlocks * sizeof(double) + kMaxBatch * sizeof(float); }

}  // namespace mp

extern "C" int prune_score_outlier_batch(const prune_projection *projs, int n_proj, int dtype, float alpha,
                                         int outlier_scope, double *score_sums, unsigned long long *counts,
                                         float *taus, void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_proj <= 0) return PRUNE_ERR_SHAPE;
    if (!projs || !score_sums || !counts || !ws) return PRUNE_ERR_NULL;
    if (!(alpha >= 0.f)) return PRUNE_ERR_RANGE;
    if (outlier_scope != PRUNE_OUTLIERS_PER_PROJECTION && outlier_scope != PRUNE_OUTLIERS_PER_LAYER)
        return PRUNE_ERR_RANGE;
    if (outlier_scope == PRUNE_OUTLIERS_PER_LAYER && n_proj > kMaxBatch) return PRUNE_ERR_RANGE;
    if (!aligned_to(score_sums, 8) || !aligned_to(counts, 8) || (taus && !aligned_to(taus, 4)) || !aligned_to(ws, 16))
        return PRUNE_ERR_ALIGNMENT;
    bool packets = true;
    for (int i = 0; i < n_proj; ++i) {
        const prune_projection &q = projs[i];
        if (q.rows <= 0 || q.cols <= 0 || q.ld_w < q.cols || q.cols > 0x7fffffff) return PRUNE_ERR_SHAPE;
        if (!q.w || !q.norms) return PRUNE_ERR_NULL;
        if (!aligned_to(q.w, elem_size(dtype)) || !aligned_to(q.norms, 4)) return PRUNE_ERR_ALIGNMENT;
        if (!packet_ok(q.w, q.cols, q.ld_w) || !aligned_to(q.norms, 16)) packets = false;
    }
    if (ws_bytes < rank_batch_workspace_bytes()) return PRUNE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const int vec = packets ? 8 : 1;

    // plan every launch first so that nothing runs if some part of the batch cannot be planned
    for (int pass = 0; pass < 2; ++pass) {
        for (int first = 0; first < n_proj; first += kMaxBatch) {
            const int n = n_proj - first < kMaxBatch ? n_proj - first : kMaxBatch;
            double total_elems = 0.0;
            for (int i = 0; i < n; ++i)
                total_elems += static_cast<double>(projs[first + i].rows) * projs[first + i].cols;
            BatchArgs args;
            args.n = n;
            uint64_t block0 = 0;
            for (int i = 0; i < n; ++i) {
                const prune_projection &q = projs[first + i];
                BatchDesc &d = args.d[i];
                d.w = q.w;
                d.norms = q.norms;
                d.rows = q.rows;
                d.ld = q.ld_w;
                d.cols = static_cast<uint32_t>(q.cols);
                d.tiles = static_cast<uint32_t>(ceil_div(q.cols, kBlock * vec));
                // this projection's share of the blocks, in whole stripes of at least kUnroll rows
                const double share = kTargetBlocks * (static_cast<double>(q.rows) * q.cols) / total_elems;
                int64_t stripes = static_cast<int64_t>(share / d.tiles + 0.5);
                if (stripes < 1) stripes = 1;
                int64_t rpb = ceil_div(q.rows, stripes);
                rpb = ceil_div(rpb, kUnroll) * kUnroll;
                d.rows_per_block = static_cast<uint32_t>(rpb < 0x7fffffff ? rpb : 0x7fffffff);
                d.stripes = static_cast<uint32_t>(ceil_div(q.rows, static_cast<int64_t>(d.rows_per_block)));
                d.block0 = static_cast<uint32_t>(block0);
                d.pad = 0;
                block0 += static_cast<uint64_t>(d.tiles) * d.stripes;
            }
            if (block0 > static_cast<uint64_t>(kMaxBlocks)) return PRUNE_ERR_RANGE;  // absurdly wide, unaligned rows
            if (pass == 0) continue;
            const int per_layer = outlier_scope == PRUNE_OUTLIERS_PER_LAYER;
            int st;
            if (dtype == PRUNE_BF16)
                st = packets ? launch_batch<bf16_t, 8>(args, static_cast<int>(block0), alpha, per_layer,
                                                       score_sums + first, counts + first,
                                                       taus ? taus + first : nullptr, ws, stream)
                             : launch_batch<bf16_t, 1>(args, static_cast<int>(block0), alpha, per_layer,
                                                       score_sums + first, counts + first,
                                                       taus ? taus + first : nullptr, ws, stream);
            else
                st = packets ? launch_batch<float, 8>(args, static_cast<int>(block0), alpha, per_layer,
                                                      score_sums + first, counts + first,
                                                      taus ? taus + first : nullptr, ws, stream)
                             : launch_batch<float, 1>(args, static_cast<int>(block0), alpha, per_layer,
                                                      score_sums + first, counts + first,
                                                      taus ? taus + first : nullptr, ws, stream);
            if (st != PRUNE_OK) return st;
        }
    }
    return PRUNE_OK;
}
