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

// g[c] = a[c] + b[c]: the row terms of the group magnitude when the caller brings them along
__global__ __launch_bounds__(kBlock) void pair_sum(const float *__restrict__ a, const float *__restrict__ b, int64_t n,
                                                   float *__restrict__ g) {
    const int64_t i = static_cast<int64_t>(blockIdx.x) * kBlock + threadIdx.x;
    if (i < n) g[i] = a[i] + b[i];
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

// The same for up to Q * 4096 channels with the keys in registers, so no digit pass goes back to
// memory.  In round q (of Q) thread t owns the four consecutive channels 4096 q + 4 t ... + 3: the
// magnitudes are read as one 16-byte load per round when VEC_LOAD (g 16-byte aligned), and the ordered
// compaction is one block-wide scan of the per-round kept counts, after which neighbouring threads
// write neighbouring slots.
template <int Q, bool VEC_LOAD>
__global__ __launch_bounds__(kRankBlock) void rank_channels_owned(const float *__restrict__ g, uint32_t inter,
                                                                  uint32_t r, int idx_bits,
                                                                  int32_t *__restrict__ kept_idx, uint32_t n_kept) {
    constexpr int NW = kRankBlock / kWave;
    constexpr uint32_t kRound = 4 * kRankBlock;
    __shared__ SelectSmem<kRankBlock> sm;
    __shared__ uint32_t wave_cnt[Q][NW];
    __shared__ uint32_t wave_lo[NW], wave_hi[NW];
    const uint32_t tid = threadIdx.x, lane = tid & (kWave - 1), wv = tid / kWave;
    uint32_t key[Q][4];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const uint32_t c0 = q * kRound + 4 * tid;
        if (VEC_LOAD && c0 + 4 <= inter) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(g + c0);
#pragma unroll
            for (int e = 0; e < 4; ++e) key[q][e] = key_of(v[e]);
        } else {
#pragma unroll
            for (int e = 0; e < 4; ++e) key[q][e] = c0 + e < inter ? key_of(g[c0 + e]) : 0u;
        }
    }
    SelectBound bound = {0u, 0u};
    if (r > 0) {
        // Channel magnitudes of one layer are close to each other: most share their exponent and leading
        // mantissa bits.  The first radix digit therefore starts at the highest bit in which the smallest
        // and the largest key differ; the bits above it are common to all keys.
        uint32_t lo = 0xffffffffu, hi = 0u;
#pragma unroll
        for (int q = 0; q < Q; ++q)
#pragma unroll
            for (int e = 0; e < 4; ++e)
                if (q * kRound + 4 * tid + e < inter) {
                    lo = min(lo, key[q][e]);
                    hi = max(hi, key[q][e]);
                }
        for (int off = kWave / 2; off > 0; off >>= 1) {
            lo = min(lo, static_cast<uint32_t>(__shfl_xor(static_cast<int>(lo), off)));
            hi = max(hi, static_cast<uint32_t>(__shfl_xor(static_cast<int>(hi), off)));
        }
        if (lane == 0) {
            wave_lo[wv] = lo;
            wave_hi[wv] = hi;
        }
        for (int b = tid; b < kSelBins; b += kRankBlock) sm.hist[b] = 0u;
        __syncthreads();
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            lo = min(lo, wave_lo[i]);
            hi = max(hi, wave_hi[i]);
        }
        const uint32_t differ = lo ^ hi;
        const int top = differ ? 31 - __clz(static_cast<int>(differ)) : 0;  // keys are below 2^31: top <= 30
        const int first_shift = top > 10 ? top - 10 : 0;
        const uint32_t hi_common = lo >> (first_shift + 11);
        bound = block_select_bound<kRankBlock>(
            [&](auto f, uint32_t salt) {
#pragma unroll
                for (int q = 0; q < Q; ++q) {
                    const uint32_t c0 = q * kRound + 4 * (tid + salt);
#pragma unroll
                    for (int e = 0; e < 4; ++e)
                        if (c0 + e < inter) f(key[q][e], c0 + e);
                }
            },
            r, idx_bits, sm, first_shift, hi_common);
    }
    uint32_t keep[Q], before[Q];
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        const uint32_t c0 = q * kRound + 4 * tid;
        keep[q] = 0;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if (c0 + e < inter && (r == 0 || !is_selected(key[q][e], c0 + e, bound))) keep[q] |= 1u << e;
        const uint32_t mine = __popc(keep[q]);
        const uint32_t incl = wave_inclusive_scan(mine);
        if (lane == kWave - 1) wave_cnt[q][wv] = incl;
        before[q] = incl - mine;
    }
    __syncthreads();
    uint32_t base = 0;  // kept channels in earlier rounds, then in earlier waves of this round
#pragma unroll
    for (int q = 0; q < Q; ++q) {
        uint32_t earlier_waves = 0, round_total = 0;
#pragma unroll
        for (int i = 0; i < NW; ++i) {
            const uint32_t t = wave_cnt[q][i];
            earlier_waves += static_cast<uint32_t>(i) < wv ? t : 0u;
            round_total += t;
        }
        uint32_t slot = base + earlier_waves + before[q];
        const uint32_t c0 = q * kRound + 4 * tid;
#pragma unroll
        for (int e = 0; e < 4; ++e)
            if ((keep[q] >> e) & 1u) {
                if (slot < n_kept) kept_idx[slot] = static_cast<int32_t>(c0 + e);
                ++slot;
            }
        base += round_total;
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

// dst[i, n] = src[i, kept[n]] ; lanes on adjacent output columns, blockIdx.y walks rows.
// Any width and element type; two- or four-byte accesses.
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

// The same gather with every HBM access 16 bytes wide.  A block walks rows i = blockIdx.x, += gridDim.x.
// A source row is read with 128-bit loads into registers (the next row's loads are in flight while the
// current one is gathered), parked in LDS, and gathered from there through a 16-bit copy of the kept
// indices that also sits in LDS.  The compacted rows are dense, so a row starts at any element offset:
// its first few elements up to the next 16-byte boundary and its last few are stored one by one, all
// packets in between with 128-bit stores.
// Needs src_cols <= 65535, 16-byte aligned source rows, src_cols <= kGatherBlock * kGatherPackets * VEC.
constexpr int kGatherBlock = 512;
constexpr int kGatherPackets = 4;
constexpr size_t kGatherLdsMax = 64 * 1024;

template <typename T>
__global__ __launch_bounds__(kGatherBlock) void gather_cols_lds(const T *__restrict__ src, T *__restrict__ dst,
                                                                const int32_t *__restrict__ kept, int64_t n_rows,
                                                                uint32_t src_cols, uint32_t n_kept,
                                                                uint32_t row_buf_bytes) {
    constexpr int VEC = 16 / static_cast<int>(sizeof(T));
    extern __shared__ __align__(16) unsigned char gather_smem[];
    T *rowbuf = reinterpret_cast<T *>(gather_smem);
    uint16_t *idx = reinterpret_cast<uint16_t *>(gather_smem + row_buf_bytes);
    const uint32_t tid = threadIdx.x;
    for (uint32_t n = tid; n < n_kept; n += kGatherBlock) idx[n] = static_cast<uint16_t>(kept[n]);

    u32x4 pk[kGatherPackets];
    int64_t i = blockIdx.x;
    if (i < n_rows) {
#pragma unroll
        for (int c = 0; c < kGatherPackets; ++c) {
            const uint32_t col0 = (c * kGatherBlock + tid) * VEC;
            pk[c] = __builtin_nontemporal_load(
                reinterpret_cast<const u32x4 *>(src + i * src_cols + (col0 < src_cols ? col0 : 0u)));
        }
    }
    for (; i < n_rows; i += gridDim.x) {
#pragma unroll
        for (int c = 0; c < kGatherPackets; ++c) {
            const uint32_t col0 = (c * kGatherBlock + tid) * VEC;
            if (col0 < src_cols) *reinterpret_cast<u32x4 *>(rowbuf + col0) = pk[c];
        }
        __syncthreads();  // the row (and, the first time, the index copy) is visible
        const int64_t inext = i + gridDim.x;
        if (inext < n_rows) {
#pragma unroll
            for (int c = 0; c < kGatherPackets; ++c) {
                const uint32_t col0 = (c * kGatherBlock + tid) * VEC;
                pk[c] = __builtin_nontemporal_load(
                    reinterpret_cast<const u32x4 *>(src + inext * src_cols + (col0 < src_cols ? col0 : 0u)));
            }
        }
        T *d = dst + i * n_kept;
        uint32_t head = static_cast<uint32_t>((16u - (reinterpret_cast<uintptr_t>(d) & 15u)) & 15u) /
                        static_cast<uint32_t>(sizeof(T));
        if (head > n_kept) head = n_kept;
        const uint32_t n_body = (n_kept - head) / VEC;
        const uint32_t tail0 = head + n_body * VEC;
        if (tid < head) d[tid] = rowbuf[idx[tid]];
        for (uint32_t q = tid; q < n_body; q += kGatherBlock) {
            const uint32_t base = head + q * VEC;
            u32x4 out;
            if constexpr (sizeof(T) == 2) {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    out[e] = static_cast<uint32_t>(rowbuf[idx[base + 2 * e]]) |
                             (static_cast<uint32_t>(rowbuf[idx[base + 2 * e + 1]]) << 16);
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e) out[e] = __float_as_uint(rowbuf[idx[base + e]]);
            }
            *reinterpret_cast<u32x4 *>(d + base) = out;
        }
        if (tid < n_kept - tail0) d[tail0 + tid] = rowbuf[idx[tail0 + tid]];
        __syncthreads();  // everyone is done with the row before the next one replaces it
    }
}

}  // namespace

// kept_idx = ascending indices of the n - r groups left after dropping the r lowest magnitudes
int launch_rank_groups(const float *group_mag, int64_t n, uint32_t r, int32_t *kept_idx, hipStream_t stream) {
    const int bits = index_bits_for(n);
    const int64_t n_kept = n - static_cast<int64_t>(r);
    const dim3 one(1), block(kRankBlock);
    const uint32_t n32 = static_cast<uint32_t>(n), kept32 = static_cast<uint32_t>(n_kept);
    const bool vec = aligned_to(group_mag, 16);
    if (n <= 4 * kRankBlock) {
        if (vec)
            hipLaunchKernelGGL((rank_channels_owned<1, true>), one, block, 0, stream, group_mag, n32, r, bits, kept_idx,
                               kept32);
        else
            hipLaunchKernelGGL((rank_channels_owned<1, false>), one, block, 0, stream, group_mag, n32, r, bits, kept_idx,
                               kept32);
    } else if (n <= 16 * kRankBlock) {
        if (vec)
            hipLaunchKernelGGL((rank_channels_owned<4, true>), one, block, 0, stream, group_mag, n32, r, bits, kept_idx,
                               kept32);
        else
            hipLaunchKernelGGL((rank_channels_owned<4, false>), one, block, 0, stream, group_mag, n32, r, bits, kept_idx,
                               kept32);
    }
    else
        hipLaunchKernelGGL(rank_channels, one, block, 0, stream, group_mag, n, r, bits, kept_idx, n_kept);
    return launch_status();
}

namespace {

// down_out[i, n] = down[i, kept[n]] for a dense [n_rows, n_kept] result
template <typename T>
int launch_gather_cols(const T *src, T *dst, const int32_t *kept, int64_t n_rows, int64_t src_cols, int64_t n_kept,
                       hipStream_t stream) {
    constexpr int64_t vec = 16 / static_cast<int64_t>(sizeof(T));
    const size_t row_buf_bytes = static_cast<size_t>(ceil_div(src_cols, vec) * 16);
    const size_t lds_bytes = row_buf_bytes + static_cast<size_t>(n_kept) * 2;
    if (src_cols <= 65535 && src_cols <= kGatherBlock * kGatherPackets * vec && lds_bytes <= kGatherLdsMax &&
        packet_ok(src, src_cols, src_cols) && aligned_to(dst, sizeof(T))) {
        const int64_t blocks = n_rows < 1024 ? n_rows : 1024;
        hipLaunchKernelGGL(gather_cols_lds<T>, dim3(static_cast<unsigned>(blocks)), dim3(kGatherBlock), lds_bytes,
                           stream, src, dst, kept, n_rows, static_cast<uint32_t>(src_cols),
                           static_cast<uint32_t>(n_kept), static_cast<uint32_t>(row_buf_bytes));
        return launch_status();
    }
    const int64_t rows_per_block = 16;
    const dim3 cgrid(static_cast<unsigned>(ceil_div(n_kept, kBlock)),
                     static_cast<unsigned>(ceil_div(n_rows, rows_per_block)));
    hipLaunchKernelGGL(gather_cols<T>, cgrid, dim3(kBlock), 0, stream, src, dst, kept, n_rows, src_cols, n_kept,
                       rows_per_block);
    return launch_status();
}

template <typename T>
int struct_dispatch(const T *gate, const T *up, const T *down, int64_t inter, int64_t hidden, uint32_t r,
                    const float *gate_rowsq, const float *up_rowsq, float *group_mag, int32_t *kept_idx, T *gate_out,
                    T *up_out, T *down_out, void *ws, hipStream_t stream) {
    const int waves_per_block = kBlock / kWave;
    const dim3 rgrid(static_cast<unsigned>(ceil_div(inter, waves_per_block)));
    if (gate_rowsq)
        hipLaunchKernelGGL(pair_sum, dim3(static_cast<unsigned>(ceil_div(inter, kBlock))), dim3(kBlock), 0, stream,
                           gate_rowsq, up_rowsq, inter, group_mag);
    else if (packet_ok(gate, hidden, hidden) && packet_ok(up, hidden, hidden))
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
    return launch_gather_cols(down, down_out, kept_idx, hidden, inter, n_kept, stream);
}

}  // namespace

size_t struct_workspace_bytes(int64_t inter, int64_t hidden) { return colsum_workspace_bytes(hidden, inter); }

}  // namespace mp

extern "C" int prune_struct_compact(const void *gate, const void *up, const void *down, int dtype, int64_t inter,
                                    int64_t hidden, uint32_t r, const float *gate_rowsq, const float *up_rowsq,
                                    float *group_mag, int32_t *kept_idx, void *gate_out, void *up_out, void *down_out,
                                    void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (inter <= 0 || hidden <= 0 || inter > 0x7fffffff || ceil_div(hidden, 16) > 65535) return PRUNE_ERR_SHAPE;
    if (!gate || !up || !down || !group_mag || !kept_idx || !ws) return PRUNE_ERR_NULL;
    const int n_out = (gate_out ? 1 : 0) + (up_out ? 1 : 0) + (down_out ? 1 : 0);
    if (n_out != 0 && n_out != 3) return PRUNE_ERR_NULL;
    if ((gate_rowsq == nullptr) != (up_rowsq == nullptr)) return PRUNE_ERR_NULL;
    if (static_cast<int64_t>(r) >= inter) return PRUNE_ERR_RANGE;
    const size_t es = elem_size(dtype);
    if (!aligned_to(gate, es) || !aligned_to(up, es) || !aligned_to(down, es) || !aligned_to(group_mag, 4) ||
        !aligned_to(kept_idx, 4) || !aligned_to(ws, 16) || (gate_rowsq && !aligned_to(gate_rowsq, 4)) ||
        (up_rowsq && !aligned_to(up_rowsq, 4)) ||
        (n_out && (!aligned_to(gate_out, es) || !aligned_to(up_out, es) || !aligned_to(down_out, es))))
        return PRUNE_ERR_ALIGNMENT;
    if (ws_bytes < struct_workspace_bytes(inter, hidden)) return PRUNE_ERR_WORKSPACE;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    if (dtype == PRUNE_BF16)
        return struct_dispatch(static_cast<const bf16_t *>(gate), static_cast<const bf16_t *>(up),
                               static_cast<const bf16_t *>(down), inter, hidden, r, gate_rowsq, up_rowsq, group_mag, kept_idx,
                               static_cast<bf16_t *>(gate_out), static_cast<bf16_t *>(up_out),
                               static_cast<bf16_t *>(down_out), ws, stream);
    return struct_dispatch(static_cast<const float *>(gate), static_cast<const float *>(up),
                           static_cast<const float *>(down), inter, hidden, r, gate_rowsq, up_rowsq, group_mag, kept_idx,
                           static_cast<float *>(gate_out), static_cast<float *>(up_out),
                           static_cast<float *>(down_out), ws, stream);
}
