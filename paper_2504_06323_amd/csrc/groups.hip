// Structured removal of coupled groups that span several projections (Section
// 4.1.3, categories 2 and 3: attention heads and feed-forward channels are
// removed; Fig. 4: the nodes between projections are pruned as a group).
//
// A group g owns `rows_per_group` consecutive rows in each row-grouped matrix
// and `cols_per_group` consecutive columns in each column-grouped matrix:
//   attention with grouped queries, one group per key/value head:
//     q rows (heads of the group), k rows, v rows; o columns
//   feed-forward channel: one gate row, one up row; one down column
// Group magnitude = sum of squares of everything the group owns; the r lowest
// go, the matrices are compacted by gathering what the kept groups own.
//
// Kernels: per-row sums of squares (one wave per row), the shared column
// sum-of-squares kernels, a per-group reduction in a fixed order, the exact
// radix ranking shared with the other structured pass, and packet gathers of
// whole row / column groups.
#include "common.hpp"

namespace mp {

namespace {

constexpr int kBlock = 256;
constexpr int kMaxMats = 8;

template <typename T, int VEC>
__global__ __launch_bounds__(kBlock) void rows_sumsq(const T *__restrict__ m, int64_t rows, int64_t width,
                                                     float *__restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t r = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + threadIdx.x / kWave;
    if (r >= rows) return;  // whole waves leave together; no block barrier below
    float s = 0.f;
    const T *p = m + r * width;
    for (int64_t j = static_cast<int64_t>(lane) * VEC; j < width; j += kWave * VEC) {
        Packet<T, VEC> a;
        a.template load<true>(p + j);
        float v[VEC];
        a.to_float(v);
#pragma unroll
        for (int e = 0; e < VEC; ++e) s = fmaf(v[e], v[e], s);
    }
    s = wave_sum(s);
    if (lane == 0) out[r] = s;
}

struct GroupTerms {
    const float *sq[2 * kMaxMats];  // per-row (or per-column) sums of squares of each matrix
    int64_t per_group[2 * kMaxMats];
    int n;
};

// one wave per group: add the group's entries of every matrix, matrices in order, fixed lane tree
__global__ __launch_bounds__(kBlock) void group_reduce(const GroupTerms terms, int64_t n_groups,
                                                       float *__restrict__ group_mag) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t g = static_cast<int64_t>(blockIdx.x) * (kBlock / kWave) + threadIdx.x / kWave;
    if (g >= n_groups) return;
    float total = 0.f;
    for (int m = 0; m < terms.n; ++m) {
        const int64_t per = terms.per_group[m];
        const float *p = terms.sq[m] + g * per;
        float s = 0.f;
        for (int64_t i = lane; i < per; i += kWave) s += p[i];
        total += wave_sum(s);
    }
    if (lane == 0) group_mag[g] = total;
}

// dst row n = src row kept[n / per] * per + n % per
template <typename T, int VEC>
__global__ __launch_bounds__(kBlock) void gather_row_groups(const T *__restrict__ src, T *__restrict__ dst,
                                                            const int32_t *__restrict__ kept, int64_t per,
                                                            int64_t width) {
    const int64_t n = blockIdx.x;
    const int64_t srow = static_cast<int64_t>(kept[n / per]) * per + n % per;
    const T *s = src + srow * width;
    T *d = dst + n * width;
    for (int64_t j = static_cast<int64_t>(threadIdx.x) * VEC; j < width; j += kBlock * VEC) {
        Packet<T, VEC> pk;
        pk.template load<true>(s + j);
        pk.store(d + j);
    }
}

// dst[i, n .. n+VEC) = src[i, kept[n / per] * per + n % per ..); a packet never straddles a group when VEC | per
template <typename T, int VEC>
__global__ __launch_bounds__(kBlock) void gather_col_groups(const T *__restrict__ src, T *__restrict__ dst,
                                                            const int32_t *__restrict__ kept, int64_t per,
                                                            int64_t height, int64_t src_cols, int64_t dst_cols,
                                                            int64_t rows_per_block) {
    const int64_t n = (static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x) * VEC;
    if (n >= dst_cols) return;
    const int64_t c = static_cast<int64_t>(kept[n / per]) * per + n % per;
    const int64_t i0 = static_cast<int64_t>(blockIdx.y) * rows_per_block;
    int64_t i1 = i0 + rows_per_block;
    if (i1 > height) i1 = height;
    for (int64_t i = i0; i < i1; ++i) {
        Packet<T, VEC> pk;
        pk.template load<true>(src + i * src_cols + c);
        pk.store(dst + i * dst_cols + n);
    }
}

struct GroupsLayout {
    size_t partials_bytes;  // column sum-of-squares partials (largest column-grouped matrix)
    size_t total_bytes;
};

GroupsLayout groups_layout(const int64_t *row_per, const int64_t *, int n_row, const int64_t *col_per,
                           const int64_t *col_height, int n_col, int64_t n_groups) {
    GroupsLayout l;
    l.partials_bytes = 0;
    size_t floats = 0;
    for (int i = 0; i < n_row; ++i) floats += static_cast<size_t>(n_groups * row_per[i]);
    for (int i = 0; i < n_col; ++i) {
        floats += static_cast<size_t>(n_groups * col_per[i]);
        const size_t pb = colsum_workspace_bytes(col_height[i], n_groups * col_per[i]);
        if (pb > l.partials_bytes) l.partials_bytes = pb;
    }
    l.partials_bytes = (l.partials_bytes + 255) / 256 * 256;
    l.total_bytes = l.partials_bytes + floats * sizeof(float);
    return l;
}

template <typename T>
int groups_dispatch(const void *const *row_mats, const int64_t *row_per, const int64_t *row_width, int n_row,
                    const void *const *col_mats, const int64_t *col_per, const int64_t *col_height, int n_col,
                    int dtype, int64_t n_groups, uint32_t r, float *group_mag, int32_t *kept_idx,
                    void *const *row_outs, void *const *col_outs, void *ws, hipStream_t stream) {
    const GroupsLayout lay = groups_layout(row_per, row_width, n_row, col_per, col_height, n_col, n_groups);
    float *temp = reinterpret_cast<float *>(static_cast<char *>(ws) + lay.partials_bytes);
    GroupTerms terms;
    terms.n = 0;
    const int wpb = kBlock / kWave;
    for (int i = 0; i < n_row; ++i) {
        const T *m = static_cast<const T *>(row_mats[i]);
        const int64_t rows = n_groups * row_per[i], width = row_width[i];
        const dim3 grid(static_cast<unsigned>(ceil_div(rows, wpb)));
        if (packet_ok(m, width, width))
            hipLaunchKernelGGL((rows_sumsq<T, 8>), grid, dim3(kBlock), 0, stream, m, rows, width, temp);
        else
            hipLaunchKernelGGL((rows_sumsq<T, 1>), grid, dim3(kBlock), 0, stream, m, rows, width, temp);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        terms.sq[terms.n] = temp;
        terms.per_group[terms.n++] = row_per[i];
        temp += rows;
    }
    for (int i = 0; i < n_col; ++i) {
        const int64_t cols = n_groups * col_per[i];
        const int st = launch_colsum(col_mats[i], dtype, col_height[i], cols, cols, temp, ws, stream, false, nullptr);
        if (st != PRUNE_OK) return st;
        terms.sq[terms.n] = temp;
        terms.per_group[terms.n++] = col_per[i];
        temp += cols;
    }
    hipLaunchKernelGGL(group_reduce, dim3(static_cast<unsigned>(ceil_div(n_groups, wpb))), dim3(kBlock), 0, stream,
                       terms, n_groups, group_mag);
    if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    if (launch_rank_groups(group_mag, n_groups, r, kept_idx, stream) != PRUNE_OK) return PRUNE_ERR_DEVICE;
    if (!row_outs && !col_outs) return PRUNE_OK;

    const int64_t n_kept = n_groups - r;
    for (int i = 0; i < n_row; ++i) {
        const T *m = static_cast<const T *>(row_mats[i]);
        T *o = static_cast<T *>(row_outs[i]);
        const int64_t width = row_width[i];
        const dim3 grid(static_cast<unsigned>(n_kept * row_per[i]));
        if (packet_ok(m, width, width) && packet_ok(o, width, width))
            hipLaunchKernelGGL((gather_row_groups<T, 8>), grid, dim3(kBlock), 0, stream, m, o, kept_idx, row_per[i],
                               width);
        else
            hipLaunchKernelGGL((gather_row_groups<T, 1>), grid, dim3(kBlock), 0, stream, m, o, kept_idx, row_per[i],
                               width);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    }
    for (int i = 0; i < n_col; ++i) {
        const T *m = static_cast<const T *>(col_mats[i]);
        T *o = static_cast<T *>(col_outs[i]);
        const int64_t per = col_per[i], src_cols = n_groups * per, dst_cols = n_kept * per;
        const int64_t rows_per_block = 16;
        const bool vec = per % 8 == 0 && packet_ok(m, src_cols, src_cols) && packet_ok(o, dst_cols, dst_cols);
        const dim3 grid(static_cast<unsigned>(ceil_div(vec ? dst_cols / 8 : dst_cols, kBlock)),
                        static_cast<unsigned>(ceil_div(col_height[i], rows_per_block)));
        if (vec)
            hipLaunchKernelGGL((gather_col_groups<T, 8>), grid, dim3(kBlock), 0, stream, m, o, kept_idx, per,
                               col_height[i], src_cols, dst_cols, rows_per_block);
        else
            hipLaunchKernelGGL((gather_col_groups<T, 1>), grid, dim3(kBlock), 0, stream, m, o, kept_idx, per,
                               col_height[i], src_cols, dst_cols, rows_per_block);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
    }
    return PRUNE_OK;
}

int validate_groups(const void *const *row_mats, const int64_t *row_per, const int64_t *row_width, int n_row,
                    const void *const *col_mats, const int64_t *col_per, const int64_t *col_height, int n_col,
                    int dtype, int64_t n_groups, uint32_t r, const float *group_mag, const int32_t *kept_idx,
                    void *const *row_outs, void *const *col_outs, const void *ws) {
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_row < 0 || n_col < 0 || n_row > kMaxMats || n_col > kMaxMats || n_row + n_col == 0 || n_groups <= 0 ||
        n_groups > 0x7fffffff)
        return PRUNE_ERR_SHAPE;
    if ((n_row && (!row_mats || !row_per || !row_width)) || (n_col && (!col_mats || !col_per || !col_height)) ||
        !group_mag || !kept_idx || !ws)
        return PRUNE_ERR_NULL;
    if (static_cast<int64_t>(r) >= n_groups) return PRUNE_ERR_RANGE;
    const bool want_out = row_outs || col_outs;
    if (want_out && ((n_row && !row_outs) || (n_col && !col_outs))) return PRUNE_ERR_NULL;
    const size_t es = elem_size(dtype);
    for (int i = 0; i < n_row; ++i) {
        if (row_per[i] <= 0 || row_width[i] <= 0 || n_groups * row_per[i] > 0x7fffffff) return PRUNE_ERR_SHAPE;
        if (!row_mats[i] || (want_out && !row_outs[i])) return PRUNE_ERR_NULL;
        if (!aligned_to(row_mats[i], es) || (want_out && !aligned_to(row_outs[i], es))) return PRUNE_ERR_ALIGNMENT;
    }
    for (int i = 0; i < n_col; ++i) {
        if (col_per[i] <= 0 || col_height[i] <= 0 || n_groups * col_per[i] > 0x7fffffff ||
            ceil_div(col_height[i], 16) > 65535)
            return PRUNE_ERR_SHAPE;
        if (!col_mats[i] || (want_out && !col_outs[i])) return PRUNE_ERR_NULL;
        if (!aligned_to(col_mats[i], es) || (want_out && !aligned_to(col_outs[i], es))) return PRUNE_ERR_ALIGNMENT;
    }
    if (!aligned_to(group_mag, 4) || !aligned_to(kept_idx, 4) || !aligned_to(ws, 16)) return PRUNE_ERR_ALIGNMENT;
    return PRUNE_OK;
}

}  // namespace

}  // namespace mp

extern "C" size_t prune_struct_groups_workspace_bytes(const int64_t *row_per, const int64_t *row_width, int n_row,
                                                      const int64_t *col_per, const int64_t *col_height, int n_col,
                                                      int64_t n_groups) {
    using namespace mp;
    if (n_row < 0 || n_col < 0 || n_row > kMaxMats || n_col > kMaxMats || n_groups <= 0) return 0;
    if ((n_row && (!row_per || !row_width)) || (n_col && (!col_per || !col_height))) return 0;
    for (int i = 0; i < n_row; ++i)
        if (row_per[i] <= 0 || row_width[i] <= 0) return 0;
    for (int i = 0; i < n_col; ++i)
        if (col_per[i] <= 0 || col_height[i] <= 0) return 0;
    const size_t n = groups_layout(row_per, row_width, n_row, col_per, col_height, n_col, n_groups).total_bytes;
    return (n + 255) / 256 * 256;
}

extern "C" int prune_struct_groups(const void *const *row_mats, const int64_t *row_per, const int64_t *row_width,
                                   int n_row, const void *const *col_mats, const int64_t *col_per,
                                   const int64_t *col_height, int n_col, int dtype, int64_t n_groups, uint32_t r,
                                   float *group_mag, int32_t *kept_idx, void *const *row_outs, void *const *col_outs,
                                   void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    const int st = validate_groups(row_mats, row_per, row_width, n_row, col_mats, col_per, col_height, n_col, dtype,
                                   n_groups, r, group_mag, kept_idx, row_outs, col_outs, ws);
    if (st != PRUNE_OK) return st;
    if (ws_bytes < groups_layout(row_per, row_width, n_row, col_per, col_height, n_col, n_groups).total_bytes)
        return PRUNE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (dtype == PRUNE_BF16)
        return groups_dispatch<bf16_t>(row_mats, row_per, row_width, n_row, col_mats, col_per, col_height, n_col, dtype,
                                       n_groups, r, group_mag, kept_idx, row_outs, col_outs, ws, stream);
    return groups_dispatch<float>(row_mats, row_per, row_width, n_row, col_mats, col_per, col_height, n_col, dtype,
                                  n_groups, r, group_mag, kept_idx, row_outs, col_outs, ws, stream);
}
