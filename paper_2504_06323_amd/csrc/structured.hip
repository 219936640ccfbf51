// Structured removal of MLP intermediate channels (Section 4.1.3, categories 2
// and 3; Fig. 4).  Channel c couples row c of gate, row c of up and column c of
// down.  Its magnitude is the squared l2 norm of the three pieces; the r
// channels with the lowest magnitude are removed and the three matrices are
// compacted by gathering the kept rows / columns.
//
// Kernels: (1) one wave per channel adds the gate and up row sums of squares;
// (2) the column sum-of-squares kernel shared with the activation statistics
// adds down's columns on top; (3) one 1024-thread block runs the same exact
// radix selection as the unstructured pass over the channel magnitudes and
// emits the kept indices in ascending order; (4) row / column gathers.
#include "select.hpp"

namespace mp {

namespace {

constexpr int kBlock = 256;
constexpr int kRankBlock = 1024;

// g[c] = sum_j gate[c, j]^2 + sum_j up[c, j]^2 ; one wave per channel, fixed shuffle tree
template <typename T, int VEC>
__global__ __launch_bounds__(kBlock) void row_sumsq_pair(const T *__restrict__ gate, const T *__restrict__ up,
                                                         int64_t inter, int64_t hidden, float *__restrict__ g) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t c = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + threadIdx.x / kWave;
    if (c >= inter) return;  // whole waves leave together; no block barrier below
    float sg = 0.f, su = 0.f;
    const T *pg = gate + c * hidden, *pu = up + c * hidden;
    for (int64_t j = static_cast<int64_t>(lane) * VEC; j < hidden; j += kWave * VEC) {
        Packet<T, VEC> a, b;
        a.template load<true>(pg + j);
        b.template load<true>(pu + j);
        float va[VEC], vb[VEC];
        a.to_float(va);
        b.to_float(vb);
#pragma unroll
        for (int e = 0; e < VEC; ++e) {
            sg = fmaf(va[e], va[e], sg);
            su = fmaf(vb[e], vb[e], su);
        }
    }
    sg = wave_sum(sg);
    su = wave_sum(su);
    if (lane == 0) g[c] = sg + su;
}

// One block: select the r smallest (g, c) pairs, write the other channels' indices ascending.
__global__ __launch_bounds__(kRankBlock) void rank_channels(const float *__restrict__ g, int64_t inter, uint32_t r,
                                                            int idx_bits, int32_t *__restrict__ kept_idx,
                                                            int64_t n_kept) {
    __shared__ SelectSmem<kRankBlock> sm;
    __shared__ uint32_t wave_cnt[kRankBlock / kWave];
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    bool have_bound = false;
    SelectBound bound = {0u, 0u};
    if (r > 0) {
        for (int b = tid; b < kSelBins; b += kRankBlock) sm.hist[b] = 0u;
        __syncthreads();
        bound = block_select_bound<kRankBlock>(
            [&](auto f, uint32_t) {
                for (int64_t c = tid; c < inter; c += kRankBlock) f(key_of(g[c]), static_cast<uint32_t>(c));
            },
            r, idx_bits, sm);
        have_bound = true;
    }
    // ordered compaction, 1024 consecutive channels per round
    uint32_t base = 0;
    for (int64_t c0 = 0; c0 < inter; c0 += kRankBlock) {
        const int64_t c = c0 + tid;
        bool keep = false;
        if (c < inter) keep = !have_bound || !is_selected(key_of(g[c]), static_cast<uint32_t>(c), bound);
        const unsigned long long ballot = __ballot(keep);
        const uint32_t before_in_wave = __popcll(ballot & ((1ull << lane) - 1ull));
        if (lane == 0) wave_cnt[wv] = __popcll(ballot);
        __syncthreads();
        uint32_t off = base, total = 0;
        for (int i = 0; i < kRankBlock / kWave; ++i) {
            const uint32_t n = wave_cnt[i];
            if (i < wv) off += n;
            total += n;
        }
        const uint32_t slot = off + before_in_wave;
        if (keep && slot < n_kept) kept_idx[slot] = static_cast<int32_t>(c);
        base += total;
        __syncthreads();
    }
}

// dst[n, :] = src[kept[n], :]
template <typename T, int VEC>
__global__ __launch_bounds__(kBlock) void gather_rows(const T *__restrict__ src, T *__restrict__ dst,
                                                      const int32_t *__restrict__ kept, int64_t width) {
    const int64_t n = blockIdx.x;
    const T *s = src + static_cast<int64_t>(kept[n]) * width;
    T *d = dst + n * width;
    for (int64_t j = static_cast<int64_t>(threadIdx.x) * VEC; j < width; j += kBlock * VEC) {
        Packet<T, VEC> pk;
        pk.template load<true>(s + j);
        pk.store(d + j);
    }
}

// dst[i, n] = src[i, kept[n]] ; lanes on adjacent output columns, blockIdx.y walks rows
template <typename T>
__global__ __launch_bounds__(kBlock) void gather_cols(const T *__restrict__ src, T *__restrict__ dst,
                                                      const int32_t *__restrict__ kept, int64_t n_rows,
                                                      int64_t src_cols, int64_t n_kept, int64_t rows_per_block) {
    const int64_t n = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (n >= n_kept) return;
    const int64_t c = kept[n];
    const int64_t i0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
    int64_t i1 = i0 + rows_per_block;
    if (i1 > n_rows) i1 = n_rows;
    for (int64_t i = i0; i < i1; ++i) dst[i * n_kept + n] = src[i * src_cols + c];
}

}  // namespace

// kept_idx = ascending indices of the n - r groups left after dropping the r lowest magnitudes
int launch_rank_groups(const float *group_mag, int64_t n, uint32_t r, int32_t *kept_idx, hipStream_t stream) {
    hipLaunchKernelGGL(rank_channels, dim3(1), dim3(kRankBlock), 0, stream, group_mag, n, r, index_bits_for(n),
                       kept_idx, n - static_cast<int64_t>(r));
    return launch_status();
}

namespace {

template <typename T>
int struct_dispatch(const T *gate, const T *up, const T *down, int64_t inter, int64_t hidden, uint32_t r,
                    float *group_mag, int32_t *kept_idx, T *gate_out, T *up_out, T *down_out, void *ws,
                    hipStream_t stream) {
    const int waves_per_block = kBlock / kWave;
    const dim3 rgrid(static_cast<unsigned>(ceil_div(inter, waves_per_block)));
    if (packet_ok(gate, hidden, hidden) && packet_ok(up, hidden, hidden))
        hipLaunchKernelGGL((row_sumsq_pair<T, 8>), rgrid, dim3(kBlock), 0, stream, gate, up, inter, hidden, group_mag);
    else
        hipLaunchKernelGGL((row_sumsq_pair<T, 1>), rgrid, dim3(kBlock), 0, stream, gate, up, inter, hidden, group_mag);
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;

    const int dtype = sizeof(T) == 2 ? PRUNE_BF16 : PRUNE_F32;
    int st = launch_colsum(down, dtype, hidden, inter, inter, group_mag, ws, stream);
    if (st != PRUNE_OK) return st;

    if (launch_rank_groups(group_mag, inter, r, kept_idx, stream) != PRUNE_OK) return PRUNE_ERR_DEVICE;
    if (!gate_out) return PRUNE_OK;

    const int64_t n_kept = inter - r;
    const dim3 ggrid(static_cast<unsigned>(n_kept));
    if (packet_ok(gate, hidden, hidden) && packet_ok(up, hidden, hidden) && packet_ok(gate_out, hidden, hidden) &&
        packet_ok(up_out, hidden, hidden)) {
        hipLaunchKernelGGL((gather_rows<T, 8>), ggrid, dim3(kBlock), 0, stream, gate, gate_out, kept_idx, hidden);
        hipLaunchKernelGGL((gather_rows<T, 8>), ggrid, dim3(kBlock), 0, stream, up, up_out, kept_idx, hidden);
    } else {
        hipLaunchKernelGGL((gather_rows<T, 1>), ggrid, dim3(kBlock), 0, stream, gate, gate_out, kept_idx, hidden);
        hipLaunchKernelGGL((gather_rows<T, 1>), ggrid, dim3(kBlock), 0, stream, up, up_out, kept_idx, hidden);
    }
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    const int64_t rows_per_block = 16;
    const dim3 cgrid(static_cast<unsigned>(ceil_div(n_kept, kBlock)),
                     static_cast<unsigned>(ceil_div(hidden, rows_per_block)));
    hipLaunchKernelGGL(gather_cols<T>, cgrid, dim3(kBlock), 0, stream, down, down_out, kept_idx, hidden, inter, n_kept,
                       rows_per_block);
    return launch_status();
}

}  // namespace

size_t struct_workspace_bytes(int64_t inter, int64_t hidden) { return colsum_workspace_bytes(hidden, inter); }

}  // namespace mp

extern "C" int prune_struct_compact(const void *gate, const void *up, const void *down, int dtype, int64_t inter,
                                    int64_t hidden, uint32_t r, float *group_mag, int32_t *kept_idx, void *gate_out,
                                    void *up_out, void *down_out, void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (inter <= 0 || hidden <= 0 || inter > 0x7fffffff || ceil_div(hidden, 16) > 65535) return PRUNE_ERR_SHAPE;
    if (!gate || !up || !down || !group_mag || !kept_idx || !ws) return PRUNE_ERR_NULL;
    const int n_out = (gate_out ? 1 : 0) + (up_out ? 1 : 0) + (down_out ? 1 : 0);
    if (n_out != 0 && n_out != 3) return PRUNE_ERR_NULL;
    if (static_cast<int64_t>(r) >= inter) return PRUNE_ERR_RANGE;
    const size_t es = elem_size(dtype);
    if (!aligned_to(gate, es) || !aligned_to(up, es) || !aligned_to(down, es) || !aligned_to(group_mag, 4) ||
        !aligned_to(kept_idx, 4) || !aligned_to(ws, 16) ||
        (n_out && (!aligned_to(gate_out, es) || !aligned_to(up_out, es) || !aligned_to(down_out, es))))
        return PRUNE_ERR_ALIGNMENT;
    if (ws_bytes < struct_workspace_bytes(inter, hidden)) return PRUNE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (dtype == PRUNE_BF16)
        return struct_dispatch(static_cast<const bf16_t *>(gate), static_cast<const bf16_t *>(up),
                               static_cast<const bf16_t *>(down), inter, hidden, r, group_mag, kept_idx,
                               static_cast<bf16_t *>(gate_out), static_cast<bf16_t *>(up_out),
                               static_cast<bf16_t *>(down_out), ws, stream);
    return struct_dispatch(static_cast<const float *>(gate), static_cast<const float *>(up),
                           static_cast<const float *>(down), inter, hidden, r, group_mag, kept_idx,
                           static_cast<float *>(gate_out), static_cast<float *>(up_out),
                           static_cast<float *>(down_out), ws, stream);
}
