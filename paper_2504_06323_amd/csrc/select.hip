// Unstructured projection pruning (Section 4.1.3, category 1): in every output
// row the k entries with the smallest weight metric (Eq. 5) are set to zero,
// lower column first among equal metrics.
//
// One block per row.  The row is loaded once with 128-bit loads and stays in
// registers in its storage format; the metric keys live in registers too, the
// radix search runs over them with its histogram in LDS, and the row is written
// back once (plus one keep-bit per element).  HBM traffic is one read and one
// write of the projection.
#include "select.hpp"

namespace mp {

namespace {

template <typename T, int BLOCK, int NCHUNK, bool FROM_SCORES>
__global__ __launch_bounds__(BLOCK, 4) void select_rows_vec(const T *w, T *w_out, uint32_t cols, int64_t ld,
                                                            int64_t ld_out, const float *__restrict__ norms,
                                                            const float *__restrict__ scores, uint32_t k,
                                                            int idx_bits, uint8_t *__restrict__ mask_bytes,
                                                            uint32_t mask_row_bytes) {
    __shared__ SelectSmem<BLOCK> sm;
    const int64_t row = blockIdx.x;
    const uint32_t tid = threadIdx.x;
    const T *wrow = w + row * ld;  // uniform row bases; per-lane offsets stay 32-bit
    T *orow = w_out + row * ld_out;

    Packet<T, 8> pk[NCHUNK];
    uint32_t key[NCHUNK][8];
#pragma unroll
    for (int c = 0; c < NCHUNK; ++c) {
        const uint32_t col0 = (c * BLOCK + tid) * 8;
        if (col0 < cols) {
            pk[c].template load<true>(wrow + col0);
            float om[8];
            if (FROM_SCORES) {
                load_floats(scores + row * cols + col0, om);
            } else {
                float v[8], nrm[8];
                pk[c].to_float(v);
                load_floats(norms + col0, nrm);
#pragma unroll
                for (int e = 0; e < 8; ++e) om[e] = metric(v[e], nrm[e]);
            }
#pragma unroll
            for (int e = 0; e < 8; ++e) key[c][e] = key_of(om[e]);
        }
    }

    SelectBound bound = {0xffffffffu, 0xffffffffu};  // k == cols: everything goes
    if (k < cols) {
        for (int b = tid; b < kSelBins; b += BLOCK) sm.hist[b] = 0u;
        __syncthreads();
        bound = block_select_bound<BLOCK>(
            [&](auto f, uint32_t salt) {
#pragma unroll
                for (int c = 0; c < NCHUNK; ++c) {
                    const uint32_t col0 = (c * BLOCK + tid + salt) * 8;
                    if (col0 < cols) {
#pragma unroll
                        for (int e = 0; e < 8; ++e) f(key[c][e], col0 + e);
                    }
                }
            },
            k, idx_bits, sm);
    }

    const bool whole_bins = bound.idx == 0xffffffffu;  // uniform: no tie to split by column
#pragma unroll
    for (int c = 0; c < NCHUNK; ++c) {
        const uint32_t col0 = (c * BLOCK + tid) * 8;
        if (col0 < cols) {
            uint32_t keep = 0;
            if (whole_bins) {
#pragma unroll
                for (int e = 0; e < 8; ++e) keep |= (key[c][e] > bound.key ? 1u : 0u) << e;
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) keep |= (is_selected(key[c][e], col0 + e, bound) ? 0u : 1u) << e;
            }
            pk[c].apply_keep(keep);
            pk[c].store(orow + col0);
            if (mask_bytes) {
                uint8_t *mrow = mask_bytes + row * mask_row_bytes;
                mrow[col0 >> 3] = static_cast<uint8_t>(keep);
                if (col0 + 8 == cols)  // owner of the last packet clears the padding of the last word
                    for (uint32_t b = (cols >> 3); b < mask_row_bytes; ++b) mrow[b] = 0;
            }
        }
    }
}

// any width / pitch / alignment; keys are recomputed from memory on every digit pass
template <typename T, int BLOCK, bool FROM_SCORES>
__global__ __launch_bounds__(BLOCK) void select_rows_generic(const T *w, T *w_out, int64_t cols, int64_t ld, int64_t ld_out,
                                                             const float *__restrict__ norms,
                                                             const float *__restrict__ scores, uint32_t k,
                                                             int idx_bits, uint32_t *__restrict__ mask_words,
                                                             int64_t words_per_row) {
    __shared__ SelectSmem<BLOCK> sm;
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const T *wr = w + row * ld;
    auto key_at = [&](int64_t j) -> uint32_t {
        const float om = FROM_SCORES ? scores[row * cols + j] : metric(widen(wr[j]), norms[j]);
        return key_of(om);
    };
    SelectBound bound = {0xffffffffu, 0xffffffffu};
    if (k < cols) {
        for (int b = tid; b < kSelBins; b += BLOCK) sm.hist[b] = 0u;
        __syncthreads();
        bound = block_select_bound<BLOCK>(
            [&](auto f, uint32_t) {
                for (int64_t j = tid; j < cols; j += BLOCK) f(key_at(j), static_cast<uint32_t>(j));
            },
            k, idx_bits, sm);
    }
    T *orow = w_out + row * ld_out;
    for (int64_t q = tid; q < words_per_row; q += BLOCK) {
        uint32_t word = 0;
        for (int b = 0; b < 32; ++b) {
            const int64_t j = q * 32 + b;
            if (j < cols) {
                const bool keep = !is_selected(key_at(j), static_cast<uint32_t>(j), bound);
                const T v = wr[j];
                orow[j] = keep ? v : T(0);
                word |= (keep ? 1u : 0u) << b;
            }
        }
        if (mask_words) mask_words[row * words_per_row + q] = word;
    }
}

template <typename T>
__global__ __launch_bounds__(256) void copy_rows(const T *__restrict__ src, T *__restrict__ dst, int64_t rows,
                                                 int64_t cols, int64_t ld, int64_t ld_out) {
    const int64_t n = rows * cols;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t r = i / cols, c = i - r * cols;
        dst[r * ld_out + c] = src[r * ld + c];
    }
}

// keep-bits all ones over the live columns, zero in the padding of the last word
__global__ __launch_bounds__(256) void fill_keep_all(uint32_t *__restrict__ mask_words, int64_t rows, int64_t cols,
                                                     int64_t words_per_row) {
    const int64_t n = rows * words_per_row;
    for (int64_t i = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; i < n;
         i += static_cast<int64_t>(gridDim.x) * 256) {
        const int64_t q = i % words_per_row;
        const int64_t live = cols - q * 32;
        mask_words[i] = live >= 32 ? 0xffffffffu : ((1u << live) - 1u);
    }
}

template <typename T, bool FROM_SCORES>
int launch_select(const T *w, T *w_out, int64_t rows, int64_t cols, int64_t ld, int64_t ld_out, const float *norms,
                  const float *scores, uint32_t k, uint32_t *mask_bits, hipStream_t stream) {
    const int idx_bits = index_bits_for(cols);
    const int64_t words = ceil_div(cols, 32);
    const dim3 grid(static_cast<unsigned>(rows));
    bool vec = packet_ok(w, cols, ld) && packet_ok(w_out, cols, ld_out) && cols <= 16384;
    if (FROM_SCORES ? !aligned_to(scores, 16) : !aligned_to(norms, 16)) vec = false;
    if (!vec) {
        hipLaunchKernelGGL((select_rows_generic<T, 256, FROM_SCORES>), grid, dim3(256), 0, stream, w, w_out, cols,
                           ld, ld_out, norms, scores, k, idx_bits, mask_bits, words);
        return launch_status();
    }
    uint8_t *mb = reinterpret_cast<uint8_t *>(mask_bits);
    const int64_t mrb = words * 4;
#define MP_SELECT_CASE(BLOCK, NCHUNK)                                                                              \
    hipLaunchKernelGGL((select_rows_vec<T, BLOCK, NCHUNK, FROM_SCORES>), grid, dim3(BLOCK), 0, stream, w, w_out,   \
                       static_cast<uint32_t>(cols), ld, ld_out, norms, scores, k, idx_bits, mb,                   \
                       static_cast<uint32_t>(mrb))
    const int64_t packets = cols / 8;
    // waves per row grow with the row width so that a thread holds at most 4 packets (32 keys)
    const int block = packets <= 128 ? 64 : packets <= 256 ? 128 : packets <= 1024 ? 256 : 512;
    const int nchunk = static_cast<int>(ceil_div(packets, block));
#define MP_SELECT_BLOCK(BLOCK)                   \
    switch (nchunk) {                            \
        case 1: MP_SELECT_CASE(BLOCK, 1); break; \
        case 2: MP_SELECT_CASE(BLOCK, 2); break; \
        case 3: MP_SELECT_CASE(BLOCK, 3); break; \
        default: MP_SELECT_CASE(BLOCK, 4); break; \
    }
    if (block == 64) { MP_SELECT_BLOCK(64) }
    else if (block == 128) { MP_SELECT_BLOCK(128) }
    else if (block == 256) { MP_SELECT_BLOCK(256) }
    else { MP_SELECT_BLOCK(512) }
#undef MP_SELECT_BLOCK
#undef MP_SELECT_CASE
    return launch_status();
}

template <typename T>
int select_dispatch(const T *w, T *w_out, int64_t rows, int64_t cols, int64_t ld, int64_t ld_out, const float *norms,
                    const float *scores, uint32_t k, uint32_t *mask_bits, hipStream_t stream) {
    if (k == 0) {  // nothing to prune: copy through, every bit kept
        if (w_out != w) {
            hipLaunchKernelGGL(copy_rows<T>, dim3(2048), dim3(256), 0, stream, w, w_out, rows, cols, ld, ld_out);
            if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        }
        if (mask_bits) {
            hipLaunchKernelGGL(fill_keep_all, dim3(1024), dim3(256), 0, stream, mask_bits, rows, cols,
                               ceil_div(cols, 32));
            return launch_status();
        }
        return PRUNE_OK;
    }
    return scores ? launch_select<T, true>(w, w_out, rows, cols, ld, ld_out, norms, scores, k, mask_bits, stream)
                  : launch_select<T, false>(w, w_out, rows, cols, ld, ld_out, norms, scores, k, mask_bits, stream);
}

}  // namespace

size_t select_workspace_bytes(int64_t, int64_t) { return 0; }  // the row lives in registers and LDS

}  // namespace mp

extern "C" int prune_select_mask(const void *w, void *w_out, int dtype, int64_t rows, int64_t cols, int64_t ld_w,
                                 int64_t ld_out, const float *norms, const float *scores, uint32_t k, uint32_t *mask_bits, void *ws,
                                 size_t ws_bytes, void *stream_) {
    using namespace mp;
    (void)ws;
    (void)ws_bytes;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (rows <= 0 || cols <= 0 || ld_w < cols || ld_out < cols || cols > (int64_t(1) << 32) || rows > 0x7fffffff)
        return PRUNE_ERR_SHAPE;
    if (w_out == w && ld_out != ld_w) return PRUNE_ERR_SHAPE;
    if (!w || !w_out || (!scores && !norms)) return PRUNE_ERR_NULL;
    if (static_cast<int64_t>(k) > cols) return PRUNE_ERR_RANGE;
    const size_t es = elem_size(dtype);
    if (!aligned_to(w, es) || !aligned_to(w_out, es) || (norms && !aligned_to(norms, 4)) ||
        (scores && !aligned_to(scores, 4)) || (mask_bits && !aligned_to(mask_bits, 4)))
        return PRUNE_ERR_ALIGNMENT;
    if (w_out != w) {  // separate output must not partially overlap the input
        const uintptr_t a = reinterpret_cast<uintptr_t>(w), b = reinterpret_cast<uintptr_t>(w_out);
        const uintptr_t span_a = static_cast<uintptr_t>((rows - 1) * ld_w + cols) * es;
        const uintptr_t span_b = static_cast<uintptr_t>((rows - 1) * ld_out + cols) * es;
        if ((a < b && a + span_a > b) || (b < a && b + span_b > a)) return PRUNE_ERR_RANGE;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (dtype == PRUNE_BF16)
        return select_dispatch(static_cast<const bf16_t *>(w), static_cast<bf16_t *>(w_out), rows, cols, ld_w, ld_out, norms,
                               scores, k, mask_bits, stream);
    return select_dispatch(static_cast<const float *>(w), static_cast<float *>(w_out), rows, cols, ld_w, ld_out, norms, scores,
                           k, mask_bits, stream);
}
