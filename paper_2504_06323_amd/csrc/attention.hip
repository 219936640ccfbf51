// Causal attention of one layer on the matrix cores (bf16, heads of width 128; grouped key / value heads):
//   o[s, h] = sum_{t <= s} softmax_t(q[s, h] . k[t, g] / sqrt(d)) v[t, g],   g = h / (heads / kv_heads).
// It produces the input of the o projection from the layer's own q, k, v (LLaMA-style layers of Table 2,
// Section 4.1.1), so that this activation too can come from a forward pass.
//
// A block of four waves takes 128 consecutive queries of one (sequence, head), 32 per wave, and walks the keys
// 64 at a time with the usual streaming softmax.  Both products are formed transposed, which keeps every step in
// registers:  S^T = K Q^T puts a query in a lane (column) and its keys in that lane's accumulator elements, so
// the running maximum and sum of a query are in-lane reductions plus one exchange with the lane 32 apart, and the
// 8 probabilities an MFMA operand wants per lane are 8 consecutive accumulator elements -- P never leaves the
// registers;  O^T = V^T P^T then needs V with the keys along the MFMA's inner dimension, which the LDS transpose
// read provides from the row-major tile.  Any permutation of the inner (key) index is fine as long as both
// operands use the same one; the one used is the accumulator's own element order.
// K and V tiles go from global memory straight into LDS (two stages), swizzled per row against bank conflicts.
#include "mfma_bf16.hpp"

namespace mp {

namespace {

constexpr int kHeadDim = 128, kQueriesPerBlock = 128, kKeysPerTile = 64;
constexpr int kTileBytes = kKeysPerTile * kHeadDim * 2;  // 16 KB
constexpr int kOutPitch = 272;                           // bytes per query row in the output staging (256 + 16)

// two floats -> two bf16 (round to nearest even) in one word, low half first
__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
    uint32_t r;
    asm("v_cvt_pk_bf16_f32 %0, %1, %2" : "=v"(r) : "v"(lo), "v"(hi));
    return r;
}

typedef __attribute__((address_space(3))) unsigned char lds_byte;
typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
typedef __attribute__((address_space(3))) u32x4 lds_u32x4;

// A operand of S^T = K Q^T: keys 32 mt + lane % 32, the 8 head dimensions 16 kk + 8 (lane / 32) ...  K tile rows are
// 256 bytes (16 packets); packet c of row r sits at position c ^ (r % 16).  The lane's byte offset for (mt = 0, kk);
// other mt are a constant 8192 bytes further (32 rows, and r % 16 does not change).
__device__ __forceinline__ uint32_t k_operand_offset(int kk, int lane) {
    const int row = lane & 31, chunk = 2 * kk + (lane >> 5);
    return static_cast<uint32_t>(row * 256 + ((chunk ^ (row & 15)) << 4));
}

// A operand of O^T = V^T P^T: head dimension 32 dt + lane % 32, and for the lane's half h = lane / 32 the keys
// row_base + 4 h + {0, 1, 2, 3} (first read) and + 8 (second read): the keys whose probabilities sit in accumulator
// elements v0 .. v0 + 7 of that half.  V tile rows are 256 bytes; packet c of row r at c ^ (4 (r % 4)).  The lane's
// byte offset of the first read for (row_base = 0, dt); row_base (a multiple of 8) adds 256 row_base bytes.
__device__ __forceinline__ uint32_t v_operand_offset(int dt, int lane) {
    const int s = lane & 15, g = lane >> 4;
    const int row = 4 * (g >> 1) + (s >> 2);
    const int col = 32 * dt + 16 * (g & 1) + 4 * (s & 3);
    return static_cast<uint32_t>(row * 256 + ((((col >> 3) ^ (4 * (row & 3)))) << 4) + (col & 4) * 2);
}

__device__ __forceinline__ bf16x8 read_k_operand(lds_byte *at) {
    return __builtin_bit_cast(bf16x8, *reinterpret_cast<lds_u32x4 *>(at));
}

__device__ __forceinline__ bf16x8 read_v_operand(lds_byte *at) {
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_s16x4 *>(at));
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(reinterpret_cast<lds_s16x4 *>(at + 8 * 256));
    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
}

template <int V>
struct Const {
    static constexpr int value = V;
};

__global__ __launch_bounds__(256, 2) void attention_tiles_bf16(const bf16_t *__restrict__ q, const bf16_t *__restrict__ k,
                                                            const bf16_t *__restrict__ v, bf16_t *__restrict__ o,
                                                            int seq_len, int heads, int kv_heads, int64_t ld_q,
                                                            int64_t ld_k, int64_t ld_v, int64_t ld_o, float scale_log2e, int n_units) {
    __shared__ __attribute__((aligned(1024))) unsigned char ring[2][2][kTileBytes];  // [stage][K, V]
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int q_tiles = (seq_len + kQueriesPerBlock - 1) / kQueriesPerBlock;
    // Workgroups go to the chip's eight dies round robin by their index, and a query tile's work grows with its
    // position in the sequence: were tile j of every (sequence, head) simply block j of its group of q_tiles, a die
    // would see the same few tile positions for the whole launch -- the heavy ones on some dies, the light ones on
    // others -- and the launch would end with most dies idle (measured: 1.3 to 1.6 times slower).  So a die takes
    // whole units -- a sequence's query heads that share one K / V head -- every eighth one: all positions, the
    // heaviest first, the heads of a unit side by side, and everything that reads the same K and V shares that
    // die's L2.
    const int per_kv = heads / kv_heads, unit_blocks = per_kv * q_tiles;
    const int die = static_cast<int>(blockIdx.x % kXcds), slot = static_cast<int>(blockIdx.x / kXcds);
    const int unit = (slot / unit_blocks) * kXcds + die;
    if (unit >= n_units) return;  // the whole block, before any barrier: padding of the last round of units
    const int r = slot % unit_blocks;
    const int qt = q_tiles - 1 - r / per_kv;
    const int head = (unit % kv_heads) * per_kv + r % per_kv;
    const int64_t seq = unit / kv_heads;
    const int kv_head = head / (heads / kv_heads);
    const int64_t t0 = seq * seq_len;
    const int q0 = qt * kQueriesPerBlock + 32 * wave;  // first query of this wave
    const int my_query = q0 + (lane & 31);
    const int n_tiles = (qt * kQueriesPerBlock + kQueriesPerBlock + kKeysPerTile - 1) / kKeysPerTile;

    // Q as the B operand, kept in registers: query lane % 32, head dimensions 16 kk + 8 (lane / 32) ...
    bf16x8 qreg[8];
    {
        const int qr = my_query < seq_len ? my_query : seq_len - 1;
        const bf16_t *src = q + (t0 + qr) * ld_q + head * kHeadDim + 8 * (lane >> 5);
#pragma unroll
        for (int kk = 0; kk < 8; ++kk)
            qreg[kk] = __builtin_bit_cast(bf16x8, *reinterpret_cast<const u32x4 *>(src + 16 * kk));
    }

    // load instruction p of this wave fills rows 4 (4 p + wave) ... + 3 of a tile: row 4 (4 p + wave) + lane / 16,
    // position lane % 16
    const char *pk[4], *pv[4];
    int lrow[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        lrow[p] = 4 * (4 * p + wave) + (lane >> 4);
        const int pos = lane & 15;
        pk[p] = reinterpret_cast<const char *>(k + t0 * ld_k + kv_head * kHeadDim + 8 * (pos ^ (lrow[p] & 15)));
        pv[p] = reinterpret_cast<const char *>(v + t0 * ld_v + kv_head * kHeadDim + 8 * (pos ^ (4 * (lrow[p] & 3))));
    }
    auto issue = [&](int tile) {
        const uint32_t dst = __builtin_amdgcn_readfirstlane(
            static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte *)&ring[tile & 1][0][0])) +
            static_cast<uint32_t>(wave) * 1024u);
#pragma unroll
        for (int p = 0; p < 4; ++p) {
            int key = tile * kKeysPerTile + lrow[p];
            key = key < seq_len ? key : seq_len - 1;  // keys past the end are masked by causality anyway
            load_to_lds(pk[p] + static_cast<int64_t>(key) * ld_k * 2, dst + 4096u * p);
            load_to_lds(pv[p] + static_cast<int64_t>(key) * ld_v * 2, dst + kTileBytes + 4096u * p);
        }
    };

    f32x16 acc_o[4];
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int e = 0; e < 16; ++e) acc_o[dt][e] = 0.f;
    float m_run = -INFINITY, l_run = 0.f;  // running maximum (in units of log2) and this lane's share of the sum

    // every LDS address below is a per-lane offset computed once plus a compile-time constant (the stage, the row
    // base): two trips of the loop are written out so that the stage is one
    lds_byte *const lds0 = (lds_byte *)&ring[0][0][0];
    uint32_t k_off[8], v_off[4];
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) k_off[kk] = k_operand_offset(kk, lane);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt) v_off[dt] = v_operand_offset(dt, lane);
    f32x16 zero16;
#pragma unroll
    for (int e = 0; e < 16; ++e) zero16[e] = 0.f;

    auto one_tile = [&](int tile, auto stage_c) {
        constexpr int kStage = decltype(stage_c)::value * 2 * kTileBytes;
        MP_WAIT_VMCNT(0);  // this thread's loads of the tile have landed
        __syncthreads();   // ... and everyone's; and every wave is done with the previous tile,
        if (tile + 1 < n_tiles) issue(tile + 1);  // whose buffer takes the next one while this one is worked on
        if (tile * kKeysPerTile > q0 + 31) return;  // uniform over the wave: every key is masked for all its queries

        // S^T for 64 keys x 32 queries
        f32x16 s[2];
#pragma unroll
        for (int mt = 0; mt < 2; ++mt) {
#pragma unroll
            for (int kk = 0; kk < 8; ++kk)
                s[mt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_k_operand(lds0 + k_off[kk] + (kStage + 8192 * mt)),
                                                                qreg[kk], kk == 0 ? zero16 : s[mt], 0, 0, 0);
        }
        // scale, causal mask (only the tiles that reach past this wave's first query need it: a uniform branch),
        // running maximum
        float m_new = m_run;
        if (tile * kKeysPerTile + kKeysPerTile - 1 > q0) {
            const int key0 = tile * kKeysPerTile + 4 * (lane >> 5);
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    const int key = key0 + 32 * mt + 8 * (e >> 2) + (e & 3);
                    const float x = key > my_query ? -INFINITY : s[mt][e] * scale_log2e;
                    s[mt][e] = x;
                    m_new = fmaxf(m_new, x);
                }
        } else {
#pragma unroll
            for (int mt = 0; mt < 2; ++mt)
#pragma unroll
                for (int e = 0; e < 16; ++e) {
                    s[mt][e] *= scale_log2e;
                    m_new = fmaxf(m_new, s[mt][e]);
                }
        }
        m_new = fmaxf(m_new, __shfl_xor(m_new, 32));  // the other half of the keys of this query
        // (m_new is finite: key 0 is visible to every query, and tile 0 is processed first)
        // The accumulated output is rescaled only when some query's maximum grew, which after the first few tiles
        // is rare: the multiply would otherwise cost more vector instructions than the softmax itself.
        if (__builtin_amdgcn_ballot_w64(m_new > m_run) != 0ull) {
            const float fix = __builtin_amdgcn_exp2f(m_run - m_new);
            m_run = m_new;
            l_run *= fix;
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
#pragma unroll
                for (int e = 0; e < 16; ++e) acc_o[dt][e] *= fix;
        }
        // probabilities, and O^T += V^T P^T sixteen keys at a time
#pragma unroll
        for (int step = 0; step < 4; ++step) {
            const int mt = step >> 1, e0 = 8 * (step & 1);
            float p[8];
#pragma unroll
            for (int i = 0; i < 8; ++i) {
                p[i] = __builtin_amdgcn_exp2f(s[mt][e0 + i] - m_new);  // the bare instruction: no denormal care needed
                l_run += p[i];
            }
            const u32x4 packed = {pack_bf16(p[0], p[1]), pack_bf16(p[2], p[3]), pack_bf16(p[4], p[5]),
                                  pack_bf16(p[6], p[7])};
            const bf16x8 pb = __builtin_bit_cast(bf16x8, packed);
            const int row_base = 32 * mt + 16 * (step & 1);
#pragma unroll
            for (int dt = 0; dt < 4; ++dt)
                acc_o[dt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(
                    read_v_operand(lds0 + v_off[dt] + (kStage + kTileBytes + 256 * row_base)), pb, acc_o[dt], 0, 0, 0);
        }
    };
    issue(0);
    for (int tile = 0; tile < n_tiles; tile += 2) {
        one_tile(tile, Const<0>{});
        if (tile + 1 < n_tiles) one_tile(tile + 1, Const<1>{});
    }
    __syncthreads();  // the tiles are dead: their memory stages the output

    // o[query][d] = O^T[d][query] / sum; staged through LDS so that a query's 256 bytes leave in 16-byte pieces
    const float inv = 1.f / (l_run + __shfl_xor(l_run, 32));
    unsigned char *stage = &ring[0][0][0] + wave * (32 * kOutPitch);
#pragma unroll
    for (int dt = 0; dt < 4; ++dt)
#pragma unroll
        for (int e = 0; e < 16; e += 2) {
            // elements e, e + 1 are head dimensions d, d + 1 of this lane's query
            const int d = 32 * dt + 8 * (e >> 2) + 4 * (lane >> 5) + (e & 3);
            *reinterpret_cast<uint32_t *>(stage + (lane & 31) * kOutPitch + d * 2) =
                pack_bf16(acc_o[dt][e] * inv, acc_o[dt][e + 1] * inv);
        }
    // (only this wave touches its part of the staging area: LDS operations of a wave complete in order)
#pragma unroll
    for (int r = 0; r < 8; ++r) {
        const int piece = lane + 64 * r, row = piece >> 4, c = piece & 15;
        const int query = q0 + row;
        if (query < seq_len)
            *reinterpret_cast<u32x4 *>(o + (t0 + query) * ld_o + head * kHeadDim + 8 * c) =
                *reinterpret_cast<const u32x4 *>(stage + row * kOutPitch + c * 16);
    }
}

}  // namespace

bool launch_attention_tiles(const void *q, const void *k, const void *v, void *o, int dtype, int64_t n_seqs,
                            int64_t seq_len, int64_t heads, int64_t kv_heads, int64_t head_dim, int64_t ld_q,
                            int64_t ld_k, int64_t ld_v, int64_t ld_o, hipStream_t stream) {
    const int64_t q_tiles = ceil_div(seq_len, kQueriesPerBlock);
    const int64_t n_units = n_seqs * kv_heads;
    const int64_t blocks = ceil_div(n_units, kXcds) * kXcds * (heads / kv_heads) * q_tiles;
    if (dtype != PRUNE_BF16 || head_dim != kHeadDim || seq_len > (1 << 24) || blocks >= (int64_t(1) << 31) ||
        ld_q % 8 != 0 || ld_k % 8 != 0 || ld_v % 8 != 0 || ld_o % 8 != 0 || !aligned_to(q, 16) || !aligned_to(k, 16) ||
        !aligned_to(v, 16) || !aligned_to(o, 16))
        return false;
    const float scale_log2e = 1.4426950408889634f / sqrtf(static_cast<float>(head_dim));
    hipLaunchKernelGGL(attention_tiles_bf16, dim3(static_cast<unsigned>(blocks)), dim3(256), 0, stream,
                       static_cast<const bf16_t *>(q), static_cast<const bf16_t *>(k), static_cast<const bf16_t *>(v),
                       static_cast<bf16_t *>(o), static_cast<int>(seq_len), static_cast<int>(heads),
                       static_cast<int>(kv_heads), ld_q, ld_k, ld_v, ld_o, scale_log2e, static_cast<int>(n_units));
    return true;
}

}  // namespace mp
