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

// One row: load it, form the metric keys, search the bound, write the masked row and its keep-bits.
// wrow / orow / srow / mrow are the row's base addresses (uniform over the block).
template <typename T, int BLOCK, int NCHUNK, bool FROM_SCORES>
__device__ __forceinline__ void select_one_row(const T *wrow, T *orow, uint32_t cols,
                                               const float *__restrict__ norms, const float *__restrict__ srow,
                                               uint32_t k, int idx_bits, uint8_t *__restrict__ mrow,
                                               uint32_t mask_row_bytes, SelectSmem<BLOCK> &sm,
                                               float *__restrict__ row_sumsq = nullptr) {
    const uint32_t tid = threadIdx.x;
    // All loads of the row are issued before anything waits on them.  A packet past the end of a
    // ragged row re-reads packet 0 (always valid) and is ignored later, so no load sits behind a branch.
    Packet<T, 8> pk[NCHUNK];
#pragma unroll
    for (int c = 0; c < NCHUNK; ++c) {
        const uint32_t col0 = (c * BLOCK + tid) * 8;
        pk[c].load(wrow + (col0 < cols ? col0 : 0u));
    }
    // clear the histogram: the stores overlap the latency of the loads.  Nothing up to here depends on k,
    // which may itself still be on its way from device memory.
    for (int b = tid; b < kSelBins; b += BLOCK) sm.hist[b] = 0u;
    const bool nothing = k == 0;        // uniform: no entry of the row goes
    const bool everything = k >= cols;  // uniform: the whole row goes
    const bool search = !nothing && !everything;
    uint32_t key[NCHUNK][8];
#pragma unroll
    for (int c = 0; c < NCHUNK; ++c) {
        const uint32_t col0 = (c * BLOCK + tid) * 8;
        float aux[8];  // the norms of this packet's columns, or the row's precomputed scores
        load_floats((FROM_SCORES ? srow : norms) + (col0 < cols ? col0 : 0u), aux);
        if (FROM_SCORES) {
            // scores handed in by a caller get the sign bit cleared
#pragma unroll
            for (int e = 0; e < 8; ++e) key[c][e] = key_of(aux[e]);
        } else {
            // a metric recomputed here is |w| * norm: non-negative, its bits are the key
            float v[8];
            pk[c].to_float(v);
#pragma unroll
            for (int e = 0; e < 8; ++e) key[c][e] = __float_as_uint(metric(v[e], aux[e]));
        }
    }

    SelectBound bound = {0xffffffffu, 0xffffffffu};  // no search: decided by the two flags alone
    if (search) {
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
    const uint32_t force_keep = nothing ? 0xffffffffu : 0u;  // without a search the flags decide
    float sq = 0.f;  // squares of what this thread leaves in the row
#pragma unroll
    for (int c = 0; c < NCHUNK; ++c) {
        const uint32_t col0 = (c * BLOCK + tid) * 8;
        if (col0 < cols) {
            uint32_t keep = 0;
            if constexpr (sizeof(T) == 2) {
                if (whole_bins && search) {
                    // The common case, eight elements in 24 instructions: a compare of the key with the bound
                    // (kept iff key > bound; a NaN key, bit 31 set, counts as kept), a conditional move that
                    // zeroes the element's half of its word in place, and an add-with-carry that shifts the
                    // compare's result into the keep-bits (elements 7 ... 0, so that element e lands in bit e).
                    uint32_t r0 = pk[c].raw[0], r1 = pk[c].raw[1], r2 = pk[c].raw[2], r3 = pk[c].raw[3];
                    const uint32_t zero = 0u, b = __builtin_amdgcn_readfirstlane(bound.key);
#define MP_KEEP_STEP(KEY, REG, HALF)                                                                              \
    "v_cmp_lt_u32_e32 vcc, %[b], " KEY "\n\t"                                                                      \
    "v_cndmask_b32_sdwa " REG ", %[z], " REG ", vcc dst_sel:" HALF " dst_unused:UNUSED_PRESERVE src0_sel:" HALF    \
    " src1_sel:" HALF "\n\t"                                                                                       \
    "v_addc_co_u32_e32 %[kp], vcc, %[kp], %[kp], vcc\n\t"
                    asm volatile(MP_KEEP_STEP("%[k7]", "%[r3]", "WORD_1") MP_KEEP_STEP("%[k6]", "%[r3]", "WORD_0")
                                 MP_KEEP_STEP("%[k5]", "%[r2]", "WORD_1") MP_KEEP_STEP("%[k4]", "%[r2]", "WORD_0")
                                 MP_KEEP_STEP("%[k3]", "%[r1]", "WORD_1") MP_KEEP_STEP("%[k2]", "%[r1]", "WORD_0")
                                 MP_KEEP_STEP("%[k1]", "%[r0]", "WORD_1") MP_KEEP_STEP("%[k0]", "%[r0]", "WORD_0")
                                 : [kp] "+&v"(keep), [r0] "+&v"(r0), [r1] "+&v"(r1), [r2] "+&v"(r2), [r3] "+&v"(r3)
                                 : [b] "s"(b), [z] "v"(zero), [k0] "v"(key[c][0]), [k1] "v"(key[c][1]),
                                   [k2] "v"(key[c][2]), [k3] "v"(key[c][3]), [k4] "v"(key[c][4]),
                                   [k5] "v"(key[c][5]), [k6] "v"(key[c][6]), [k7] "v"(key[c][7])
                                 : "vcc");
#undef MP_KEEP_STEP
                    pk[c].raw[0] = r0;
                    pk[c].raw[1] = r1;
                    pk[c].raw[2] = r2;
                    pk[c].raw[3] = r3;
                }
            }
            if (sizeof(T) == 2 && whole_bins && search) {
                // done above
            } else if (whole_bins) {
                // key > bound  <=>  bound - key is negative (keys and bound are below 2^31, or a NaN key
                // with bit 31, which then counts as kept): the sign, spread over the word, is the mask
                uint32_t km[8];
                if (search) {
#pragma unroll
                    for (int e = 0; e < 8; ++e)
                        km[e] = static_cast<uint32_t>(static_cast<int32_t>(bound.key - key[c][e]) >> 31);
                } else {
#pragma unroll
                    for (int e = 0; e < 8; ++e) km[e] = force_keep;
                }
#pragma unroll
                for (int e = 0; e < 8; ++e) keep |= km[e] & (1u << e);
                pk[c].apply_keep_words(km);
            } else {
#pragma unroll
                for (int e = 0; e < 8; ++e) keep |= (is_selected(key[c][e], col0 + e, bound) ? 0u : 1u) << e;
                pk[c].apply_keep(keep);
            }
            pk[c].store(orow + col0);
            if (row_sumsq) sq = pk[c].add_squares(sq);
            if (mrow) {
                mrow[col0 >> 3] = static_cast<uint8_t>(keep);
                if (col0 + 8 == cols)  // owner of the last packet clears the padding of the last word
                    for (uint32_t b = (cols >> 3); b < mask_row_bytes; ++b) mrow[b] = 0;
            }
        }
    }
    if (row_sumsq) {
        // Sum of squares of the masked row, as stored: thread sums in packet order, a fixed tree inside each
        // wave, the waves in index order.  The waves meet once more for it, at the very end of the row, where
        // the block would wait for its last wave anyway.
        constexpr int NW = BLOCK / kWave;
        sq = wave_sum(sq);
        if constexpr (NW == 1) {
            if (tid == 0) *row_sumsq = sq;
        } else {
            if ((tid & (kWave - 1)) == 0) sm.wave_tot[tid / kWave] = __float_as_uint(sq);
            __syncthreads();
            if (tid == 0) {
                float total = 0.f;
#pragma unroll
                for (int i = 0; i < NW; ++i) total += __uint_as_float(sm.wave_tot[i]);
                *row_sumsq = total;
            }
        }
    }
}

template <typename T, int BLOCK, int NCHUNK, bool FROM_SCORES>
__global__ __launch_bounds__(BLOCK, (BLOCK == 64 ? 4 : NCHUNK <= 3 ? 8 : NCHUNK == 4 ? 6 : 4)) void select_rows_vec(const T *w, T *w_out, uint32_t cols, int64_t ld,
                                                            int64_t ld_out, const float *__restrict__ norms,
                                                            const float *__restrict__ scores, uint32_t k,
                                                            int idx_bits, uint8_t *__restrict__ mask_bytes,
                                                            uint32_t mask_row_bytes) {
    __shared__ SelectSmem<BLOCK> sm;
    const int64_t row = blockIdx.x;
    select_one_row<T, BLOCK, NCHUNK, FROM_SCORES>(w + row * ld, w_out + row * ld_out, cols, norms,
                                                  FROM_SCORES ? scores + row * cols : nullptr, k, idx_bits,
                                                  mask_bytes ? mask_bytes + row * mask_row_bytes : nullptr,
                                                  mask_row_bytes, sm);
}

// Several projections of equal width class in one launch: the block index is mapped to
// (projection, row) through a small table in the kernel arguments.
constexpr int kMaxSelectBatch = 16;

struct SelectItem {
    const void *w;
    void *w_out;
    const float *norms;
    uint8_t *mask_bytes;
    int64_t ld, ld_out;
    uint32_t cols, k, mask_row_bytes, row0;  // row0: first block of this projection
    int idx_bits, pad;
    const uint32_t *k_dev;  // when set: k is read from here (and capped at cols)
    float *row_sumsq;       // when set: [rows], receives the sum of squares of every masked row
};

struct SelectArgs {
    SelectItem it[kMaxSelectBatch];
    int n;
};

template <typename T, int BLOCK, int NCHUNK>
__global__ __launch_bounds__(BLOCK, (BLOCK == 64 ? 4 : NCHUNK <= 3 ? 8 : NCHUNK == 4 ? 6 : 4)) void select_rows_batch(const SelectArgs args) {
    __shared__ SelectSmem<BLOCK> sm;
    int p = 0;
    for (int i = 1; i < args.n; ++i)
        if (blockIdx.x >= args.it[i].row0) p = i;
    const SelectItem &it = args.it[p];
    const int64_t row = blockIdx.x - it.row0;
    const uint32_t k = it.k_dev ? *it.k_dev : it.k;
    select_one_row<T, BLOCK, NCHUNK, false>(static_cast<const T *>(it.w) + row * it.ld,
                                            static_cast<T *>(it.w_out) + row * it.ld_out, it.cols, it.norms, nullptr,
                                            k, it.idx_bits,
                                            it.mask_bytes ? it.mask_bytes + row * it.mask_row_bytes : nullptr,
                                            it.mask_row_bytes, sm,
                                            // (the host never pairs row sums with more than 4 packets per thread)
                                            NCHUNK > 4 ? nullptr : it.row_sumsq ? it.row_sumsq + row : nullptr);
}

// any width / pitch / alignment; keys are recomputed from memory on every digit pass
template <typename T, int BLOCK, bool FROM_SCORES>
__global__ __launch_bounds__(BLOCK) void select_rows_generic(const T *w, T *w_out, int64_t cols, int64_t ld, int64_t ld_out,
                                                             const float *__restrict__ norms,
                                                             const float *__restrict__ scores, uint32_t k_arg,
                                                             const uint32_t *__restrict__ k_dev, int idx_bits,
                                                             uint32_t *__restrict__ mask_words, int64_t words_per_row) {
    __shared__ SelectSmem<BLOCK> sm;
    const int64_t row = blockIdx.x;
    const int tid = threadIdx.x;
    const uint32_t k = k_dev ? *k_dev : k_arg;
    const bool nothing = k == 0;
    const T *wr = w + row * ld;
    auto key_at = [&](int64_t j) -> uint32_t {
        const float om = FROM_SCORES ? scores[row * cols + j] : metric(widen(wr[j]), norms[j]);
        return key_of(om);
    };
    SelectBound bound = {0xffffffffu, 0xffffffffu};
    if (k < cols && !nothing) {
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
                const bool keep = nothing || !is_selected(key_at(j), static_cast<uint32_t>(j), bound);
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

// sum of squares of every row of a matrix (for projections that do not go through the packet kernels)
template <typename T>
__global__ __launch_bounds__(256) void rows_sumsq_plain(const T *__restrict__ w, int64_t rows, int64_t cols, int64_t ld,
                                                        float *__restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = static_cast<int64_t>(blockIdx.x) * (256 / kWave) + threadIdx.x / kWave;
    if (row >= rows) return;  // whole waves leave together
    float acc = 0.f;
    for (int64_t j = lane; j < cols; j += kWave) {
        const float v = widen(w[row * ld + j]);
        acc = fmaf(v, v, acc);
    }
    acc = wave_sum(acc);
    if (lane == 0) out[row] = acc;
}

template <typename T>
int launch_rows_sumsq_plain(const void *w, int64_t rows, int64_t cols, int64_t ld, float *out, hipStream_t stream) {
    hipLaunchKernelGGL(rows_sumsq_plain<T>, dim3(static_cast<unsigned>(ceil_div(rows, 256 / kWave))), dim3(256), 0, stream,
                       static_cast<const T *>(w), rows, cols, ld, out);
    return launch_status();
}

// Waves per row grow with the row width so that a thread holds at most 4 packets (32 keys).  Rows of more than
// 1024 packets take eight waves, unless four waves with up to 7 packets per thread leave fewer thread slots
// without a packet (14336 columns are 7 x 256 packets exactly but only 3.5 x 512): idle slots cost registers and
// lanes, which is worth more here than the shorter per-thread chains of the wider block.  (Not when the row's sum
// of squares is wanted as well: with that the seven-packet form no longer fits its registers.)
inline void select_variant(int64_t cols, int elem_bytes, bool row_sums, int &block, int &nchunk) {
    const int64_t packets = cols / 8;
    block = packets <= 128 ? 64 : packets <= 256 ? 128 : packets <= 1024 ? 256 : 512;
    nchunk = static_cast<int>(ceil_div(packets, block));
    if (block == 512 && !row_sums) {
        const int64_t n256 = ceil_div(packets, 256);
        // (n256 is 5 or 7 then; seven packets of 4-byte elements and their keys do not fit a thread's registers)
        if (n256 <= (elem_bytes == 2 ? 7 : 5) && 256 * n256 < 512 * static_cast<int64_t>(nchunk)) {
            block = 256;
            nchunk = static_cast<int>(n256);
        }
    }
}

inline bool select_packets_ok(const void *w, const void *w_out, int64_t cols, int64_t ld, int64_t ld_out,
                              const float *norms) {
    return packet_ok(w, cols, ld) && packet_ok(w_out, cols, ld_out) && cols <= 16384 && aligned_to(norms, 16);
}

template <typename T>
int launch_select_batch(const SelectArgs &args, int total_rows, int block, int nchunk, hipStream_t stream) {
    const dim3 grid(static_cast<unsigned>(total_rows));
#define MP_BATCH_CASE(BLOCK, NCHUNK) \
    hipLaunchKernelGGL((select_rows_batch<T, BLOCK, NCHUNK>), grid, dim3(BLOCK), 0, stream, args)
#define MP_BATCH_BLOCK(BLOCK)                   \
    switch (nchunk) {                           \
        case 1: MP_BATCH_CASE(BLOCK, 1); break; \
        case 2: MP_BATCH_CASE(BLOCK, 2); break; \
        case 3: MP_BATCH_CASE(BLOCK, 3); break; \
        default: MP_BATCH_CASE(BLOCK, 4); break; \
    }
    if (block == 64) { MP_BATCH_BLOCK(64) }
    else if (block == 128) { MP_BATCH_BLOCK(128) }
    else if (block == 256 && nchunk == 5) { MP_BATCH_CASE(256, 5); }
    else if (block == 256 && nchunk == 7) { MP_BATCH_CASE(256, 7); }
    else if (block == 256) { MP_BATCH_BLOCK(256) }
    else { MP_BATCH_BLOCK(512) }
#undef MP_BATCH_BLOCK
#undef MP_BATCH_CASE
    return launch_status();
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
                           ld, ld_out, norms, scores, k, static_cast<const uint32_t *>(nullptr), idx_bits, mask_bits,
                           words);
        return launch_status();
    }
    uint8_t *mb = reinterpret_cast<uint8_t *>(mask_bits);
    const int64_t mrb = words * 4;
#define MP_SELECT_CASE(BLOCK, NCHUNK)                                                                              \
    hipLaunchKernelGGL((select_rows_vec<T, BLOCK, NCHUNK, FROM_SCORES>), grid, dim3(BLOCK), 0, stream, w, w_out,   \
                       static_cast<uint32_t>(cols), ld, ld_out, norms, scores, k, idx_bits, mb,                   \
                       static_cast<uint32_t>(mrb))
    int block, nchunk;
    select_variant(cols, static_cast<int>(sizeof(T)), false, block, nchunk);
#define MP_SELECT_BLOCK(BLOCK)                   \
    switch (nchunk) {                            \
        case 1: MP_SELECT_CASE(BLOCK, 1); break; \
        case 2: MP_SELECT_CASE(BLOCK, 2); break; \
        case 3: MP_SELECT_CASE(BLOCK, 3); break; \
        default: MP_SELECT_CASE(BLOCK, 4); break; \
    }
    if (block == 64) { MP_SELECT_BLOCK(64) }
    else if (block == 128) { MP_SELECT_BLOCK(128) }
    else if (block == 256 && nchunk == 5) { MP_SELECT_CASE(256, 5); }
    else if (block == 256 && nchunk == 7) { MP_SELECT_CASE(256, 7); }
    else if (block == 256) { MP_SELECT_BLOCK(256) }
    else { MP_SELECT_BLOCK(512) }
#undef MP_SELECT_BLOCK
#undef MP_SELECT_CASE
    return launch_status();
}

// a projection that cannot go through the packet kernels, with its k in device memory
template <typename T>
int launch_generic_device_k(const prune_select_item &q, hipStream_t stream) {
    hipLaunchKernelGGL((select_rows_generic<T, 256, false>), dim3(static_cast<unsigned>(q.rows)), dim3(256), 0, stream,
                       static_cast<const T *>(q.w), static_cast<T *>(q.w_out), q.cols, q.ld_w, q.ld_out, q.norms,
                       static_cast<const float *>(nullptr), 0u, q.k_dev, index_bits_for(q.cols), q.mask_bits,
                       ceil_div(q.cols, 32));
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

namespace mp {
namespace {
int validate_select(const void *w, const void *w_out, int dtype, int64_t rows, int64_t cols, int64_t ld_w,
                    int64_t ld_out, const float *norms, const float *scores, uint32_t k, const uint32_t *mask_bits) {
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
    return PRUNE_OK;
}
}  // namespace
}  // namespace mp

extern "C" int prune_select_mask(const void *w, void *w_out, int dtype, int64_t rows, int64_t cols, int64_t ld_w,
                                 int64_t ld_out, const float *norms, const float *scores, uint32_t k,
                                 uint32_t *mask_bits, void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    (void)ws;
    (void)ws_bytes;
    const int st = validate_select(w, w_out, dtype, rows, cols, ld_w, ld_out, norms, scores, k, mask_bits);
    if (st != PRUNE_OK) return st;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (dtype == PRUNE_BF16)
        return select_dispatch(static_cast<const bf16_t *>(w), static_cast<bf16_t *>(w_out), rows, cols, ld_w, ld_out,
                               norms, scores, k, mask_bits, stream);
    return select_dispatch(static_cast<const float *>(w), static_cast<float *>(w_out), rows, cols, ld_w, ld_out, norms,
                           scores, k, mask_bits, stream);
}

extern "C" int prune_select_mask_batch(const prune_select_item *items, int n_items, int dtype, void *ws,
                                       size_t ws_bytes, void *stream_) {
    using namespace mp;
    (void)ws;
    (void)ws_bytes;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_items <= 0) return PRUNE_ERR_SHAPE;
    if (!items) return PRUNE_ERR_NULL;
    for (int i = 0; i < n_items; ++i) {  // reject the whole batch before anything is launched
        const prune_select_item &q = items[i];
        const int st = validate_select(q.w, q.w_out, dtype, q.rows, q.cols, q.ld_w, q.ld_out, q.norms, nullptr,
                                       q.k_dev ? 0u : q.k, q.mask_bits);
        if (st != PRUNE_OK) return st;
        if (q.k_dev && !aligned_to(q.k_dev, 4)) return PRUNE_ERR_ALIGNMENT;
        if (q.row_sumsq && !aligned_to(q.row_sumsq, 4)) return PRUNE_ERR_ALIGNMENT;
    }
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    // projections that share a kernel variant go into one launch; the rest take the single-projection path
    bool done[1024];
    if (n_items > 1024) return PRUNE_ERR_RANGE;
    for (int i = 0; i < n_items; ++i) done[i] = false;
    for (int i = 0; i < n_items; ++i) {
        if (done[i]) continue;
        const prune_select_item &q = items[i];
        auto batchable_item = [](const prune_select_item &x) {
            return (x.k_dev || x.k > 0) && select_packets_ok(x.w, x.w_out, x.cols, x.ld_w, x.ld_out, x.norms);
        };
        if (!batchable_item(q)) {
            const int st = !q.k_dev ? prune_select_mask(q.w, q.w_out, dtype, q.rows, q.cols, q.ld_w, q.ld_out, q.norms,
                                                        nullptr, q.k, q.mask_bits, ws, ws_bytes, stream_)
                           : dtype == PRUNE_BF16 ? launch_generic_device_k<bf16_t>(q, stream)
                                                 : launch_generic_device_k<float>(q, stream);
            if (st != PRUNE_OK) return st;
            if (q.row_sumsq) {  // the sums of the rows just written
                const int st2 = dtype == PRUNE_BF16
                                    ? launch_rows_sumsq_plain<bf16_t>(q.w_out, q.rows, q.cols, q.ld_out, q.row_sumsq, stream)
                                    : launch_rows_sumsq_plain<float>(q.w_out, q.rows, q.cols, q.ld_out, q.row_sumsq, stream);
                if (st2 != PRUNE_OK) return st2;
            }
            done[i] = true;
            continue;
        }
        int block, nchunk;
        select_variant(q.cols, dtype == PRUNE_BF16 ? 2 : 4, q.row_sumsq != nullptr, block, nchunk);
        SelectArgs args;
        args.n = 0;
        int64_t total_rows = 0;
        auto flush = [&]() -> int {
            if (args.n == 0) return PRUNE_OK;
            const int st = dtype == PRUNE_BF16
                               ? launch_select_batch<bf16_t>(args, static_cast<int>(total_rows), block, nchunk, stream)
                               : launch_select_batch<float>(args, static_cast<int>(total_rows), block, nchunk, stream);
            args.n = 0;
            total_rows = 0;
            return st;
        };
        for (int j = i; j < n_items; ++j) {
            if (done[j]) continue;
            const prune_select_item &r = items[j];
            if (!batchable_item(r)) continue;
            int b2, c2;
            select_variant(r.cols, dtype == PRUNE_BF16 ? 2 : 4, r.row_sumsq != nullptr, b2, c2);
            if (b2 != block || c2 != nchunk) continue;
            if (args.n == kMaxSelectBatch || total_rows + r.rows > 0x7fffffff) {
                const int st = flush();
                if (st != PRUNE_OK) return st;
            }
            SelectItem &it = args.it[args.n++];
            it.w = r.w;
            it.w_out = r.w_out;
            it.norms = r.norms;
            it.mask_bytes = reinterpret_cast<uint8_t *>(r.mask_bits);
            it.ld = r.ld_w;
            it.ld_out = r.ld_out;
            it.cols = static_cast<uint32_t>(r.cols);
            it.k = r.k;
            it.mask_row_bytes = static_cast<uint32_t>(ceil_div(r.cols, 32) * 4);
            it.row0 = static_cast<uint32_t>(total_rows);
            it.idx_bits = index_bits_for(r.cols);
            it.pad = 0;
            it.k_dev = r.k_dev;
            it.row_sumsq = r.row_sumsq;
            total_rows += r.rows;
            done[j] = true;
        }
        const int st = flush();
        if (st != PRUNE_OK) return st;
    }
    return PRUNE_OK;
}
