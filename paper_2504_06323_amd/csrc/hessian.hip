// Hessian of the layer-wise reconstruction problem of one projection input
// (Section 4.1.3, "Pruning Methods": the one-shot pruner works with the inverse
// Hessian; Section 4.1.4, "Calibration": it is computed from the calibration
// samples):  H += X^T X  over the tokens of a chunk.
//
// This is the one dense contraction of the path, so it runs on the matrix cores.
// bf16 activations: the output is cut into 256 x 256 tiles, only tiles on or above
// the diagonal are computed (H is symmetric), and the tokens are split over several
// blocks per tile so that the grid fills the chip.  A block of four waves holds a
// 256 x 256 fp32 accumulator tile in registers (128 x 128 per wave, sixteen
// 32 x 32 x 16 MFMA accumulators) and walks its tokens 32 at a time: the two
// [32 tokens x 256 channels] slabs of X are loaded from global memory directly
// into a four-stage LDS ring, token-major as they lie in memory, and the MFMA
// operands -- which want eight consecutive tokens of one channel per lane -- are
// formed by the LDS transpose read.  Per-split partial tiles go to the workspace
// and are added up in a fixed order (so the result is reproducible bit for bit),
// mirrored below the diagonal.  Any other element type, width or alignment takes
// a plain tiled FMA kernel.
#include "mfma_bf16.hpp"

namespace mp {

namespace {

constexpr int kTile = 256;        // output tile edge (channels)
constexpr int kStep = 32;         // tokens per LDS stage
constexpr int kGramBlock = 256;
constexpr int kMaxSplits = 64;

// Tile pairs (mt, nt), mt <= nt, are numbered patch by patch: a patch is 4 tile rows by 8 tile columns of the
// upper triangle (32 pairs that need only 12 of the 256-channel slabs of X), patches are walked row band by
// row band.  Pairs that are neighbours in this order share slabs.
constexpr int kPatchRows = 4, kPatchCols = 8;

__device__ __forceinline__ void pair_of(int p, int n_tiles, int &mt, int &nt) {
    mt = nt = 0;
    for (int r0 = 0; r0 < n_tiles; r0 += kPatchRows) {
        const int r1 = r0 + kPatchRows < n_tiles ? r0 + kPatchRows : n_tiles;
        for (int c0 = r0; c0 < n_tiles; c0 += kPatchCols) {
            const int c1 = c0 + kPatchCols < n_tiles ? c0 + kPatchCols : n_tiles;
            for (int r = r0; r < r1; ++r) {
                const int lo = c0 > r ? c0 : r;
                const int width = c1 - lo;
                if (width <= 0) continue;
                if (p < width) {
                    mt = r;
                    nt = lo + p;
                    return;
                }
                p -= width;
            }
        }
    }
}

// The slabs of X go from global memory straight into LDS (no staging registers, no LDS stores): a wave's load
// instruction drops 64 x 16 bytes at consecutive LDS addresses, so a slab row is 512
// bytes without padding and bank conflicts of the transpose reads are avoided by a swizzle instead: in token row r
// the 16-byte packet c sits at position c ^ (4 (r % 4)) -- which each lane implements simply by fetching the packet
// that belongs at its fixed position.  Four 32 KB stages form a ring; the loads of stage s + 4 are issued in the
// middle of stage s, right after the barrier behind which every wave has the operands of stage s in registers:
// they reuse that stage's own buffer.  Loads that land in LDS are counted by vmcnt; the waits are explicit.
constexpr int kRing = 4;
constexpr int kSlabBytes = kStep * kTile * 2;

template <int V>
struct Whole {
    static constexpr int value = V;
};

__device__ __forceinline__ bf16x8 operand_from_ring(const unsigned char *slab, int k16, int group, int i, int lane) {
    const int s = lane & 15, g = lane >> 4;
    const int row = k16 + 8 * (g >> 1) + (s >> 2);
    const int packet = 16 * group + 4 * (i ^ (s >> 2)) + 2 * (g & 1) + ((s & 3) >> 1);
    const unsigned char *p = slab + row * (kTile * 2) + packet * 16 + (s & 1) * 8;
    typedef __attribute__((address_space(3))) s16x4 lds_s16x4;
    const s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)p);
    const s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_s16x4 *)(p + 4 * kTile * 2));
    const s16x8 both = {lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
    return __builtin_bit_cast(bf16x8, both);
}

__global__ __launch_bounds__(kGramBlock, 1) void gram_tiles_bf16(const bf16_t *__restrict__ x, int64_t n_tokens,
                                                                     int channels, int64_t ld, int n_tiles, int n_pairs,
                                                                     int n_splits, int64_t tokens_per_split,
                                                                     float *__restrict__ partials) {
    __shared__ __attribute__((aligned(1024))) unsigned char ring[kRing][2][kSlabBytes];
    typedef __attribute__((address_space(3))) unsigned char lds_byte;
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6, wm = wave >> 1, wn = wave & 1;
    int item;
    if (!item_of_block(blockIdx.x, n_pairs * n_splits, item)) return;  // the whole block, before any barrier
    const int pair = item % n_pairs, split = item / n_pairs;
    int mt, nt;
    pair_of(pair, n_tiles, mt, nt);
    const int m0 = mt * kTile, n0 = nt * kTile;
    const int64_t t_begin = split * tokens_per_split;
    int64_t t_end = t_begin + tokens_per_split;
    if (t_end > n_tokens) t_end = n_tokens;
    const int64_t n_stages = (t_end - t_begin + kStep - 1) / kStep;
    const int64_t n_whole = (t_end - t_begin) / kStep;

    // load instruction p of this wave fills LDS window 4 p + wave of a slab: token rows 2 (4 p + wave) + lane / 32,
    // position lane % 32, i.e. packet (lane % 32) ^ (4 (row % 4)); channels past the edge are clamped to packet 0
    // of the slab (they only feed outputs that are never stored)
    int drow[4];
    uint32_t offa[4], offb[4];
#pragma unroll
    for (int p = 0; p < 4; ++p) {
        drow[p] = 2 * (4 * p + wave) + (lane >> 5);
        const int c = (lane & 31) ^ (4 * (drow[p] & 3));
        const int cha = m0 + 8 * c < channels ? m0 + 8 * c : 0, chb = n0 + 8 * c < channels ? n0 + 8 * c : 0;
        offa[p] = static_cast<uint32_t>((drow[p] * ld + cha) * 2);
        offb[p] = static_cast<uint32_t>((drow[p] * ld + chb) * 2);
    }
    // The address of a load is a uniform base, formed with scalar arithmetic, plus a per-lane byte offset that
    // never changes (offa / offb): no vector instruction per load.  (Per-lane 64-bit addresses advanced or formed
    // per stage cost 130 of a stage's 1600 cycles: the 64-bit vector additions run at a quarter of the rate and sit
    // between four matrix instructions.)  Only a stage that reaches past the last token needs per-lane addresses;
    // WHOLE says that the caller knows the stage to be whole, which keeps that code out of the steady-state loop.
    const char *const xb = reinterpret_cast<const char *>(x) + t_begin * ld * 2;
    const int64_t stage_bytes = static_cast<int64_t>(kStep) * ld * 2;
    auto issue_part = [&](int64_t stage_index, int p, auto whole_c) {  // load instruction p (one for each slab) of a stage
        constexpr bool kWhole = decltype(whole_c)::value != 0;
        // LDS byte address of this wave's first window in the stage's A slab (uniform over the wave)
        const uint32_t dst = __builtin_amdgcn_readfirstlane(
            static_cast<uint32_t>(reinterpret_cast<uintptr_t>((lds_byte *)&ring[stage_index & (kRing - 1)][0][0])) +
            static_cast<uint32_t>(wave) * 1024u);
        if (kWhole || stage_index < n_whole) {  // uniform: every token row of the stage exists
            const char *from = xb + stage_index * stage_bytes;
            load_to_lds(from, offa[p], dst + 4096u * p);
            load_to_lds(from, offb[p], dst + kSlabBytes + 4096u * p);
        } else {  // rows past the last token re-read the last one (zeroed after landing, or never used)
            int64_t t = t_begin + stage_index * kStep + drow[p];
            t = t < n_tokens ? t : n_tokens - 1;
            const char *from = reinterpret_cast<const char *>(x) + t * ld * 2 - static_cast<int64_t>(drow[p]) * ld * 2;
            load_to_lds(from + offa[p], dst + 4096u * p);
            load_to_lds(from + offb[p], dst + kSlabBytes + 4096u * p);
        }
    };
    auto issue = [&](int64_t stage_index) {
#pragma unroll
        for (int p = 0; p < 4; ++p) issue_part(stage_index, p, Whole<0>{});
    };
    // token rows past the end of a ragged last stage must count as zeros
    auto blank_tail = [&](int64_t stage_index) {
        const int valid = static_cast<int>(t_end - t_begin - stage_index * kStep);  // < kStep
        unsigned char *dst = &ring[stage_index & (kRing - 1)][0][0];
        const u32x4 zero = {0u, 0u, 0u, 0u};
        for (int e = tid; e < 2 * kStep * 32; e += kGramBlock) {
            const int op = e / (kStep * 32), row = (e / 32) % kStep, pos = e % 32;
            if (row >= valid) *reinterpret_cast<u32x4 *>(dst + op * kSlabBytes + row * 512 + pos * 16) = zero;
        }
        __syncthreads();
    };

    f32x16 acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) acc[i][j][v] = 0.f;
    bf16x8 a[2][4], b[2][4];
    auto read_a = [&](int set, int64_t stage_index, int k16) {
        const unsigned char *slab = &ring[stage_index & (kRing - 1)][0][0];
#pragma unroll
        for (int i = 0; i < 4; ++i) a[set][i] = operand_from_ring(slab, k16, wm, i, lane);
    };
    auto read_b = [&](int set, int64_t stage_index, int k16) {
        const unsigned char *slab = &ring[stage_index & (kRing - 1)][1][0];
#pragma unroll
        for (int i = 0; i < 4; ++i) b[set][i] = operand_from_ring(slab, k16, wn, i, lane);
    };

    issue(0);
    issue(1);
    issue(2);
    issue(3);
    MP_WAIT_VMCNT(24);
    __syncthreads();
    if (n_stages == 1 && n_whole == 0) blank_tail(0);
    read_a(0, 0, 0);
    read_b(0, 0, 0);
    // A wave has its SIMD to itself, so every instruction that is not an MFMA should issue in the shadow of one
    // (an MFMA keeps the pipe busy for 32 cycles, time for about eight other instructions).  The scheduler is told
    // to alternate: one MFMA, then a couple of LDS reads of the operands needed later.
    auto mfma_one = [&](int set, int i, int j) {
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[set][i], b[set][j], acc[i][j], 0, 0, 0);
    };
    auto trip = [&](int64_t s, auto whole_c) {  // stage s; whole_c: stage s + 4, whose loads are issued here, is known to be whole
        // first 12 MFMAs of the stage's first 16 tokens, interleaved with the 16 reads of its last 16 tokens
        __builtin_amdgcn_sched_barrier(0);
        read_a(1, s, 16);
        read_b(1, s, 16);
#pragma unroll
        for (int i = 0; i < 3; ++i)
#pragma unroll
            for (int j = 0; j < 4; ++j) mfma_one(0, i, j);
#pragma unroll
        for (int g = 0; g < 12; ++g) {
            __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);  // one MFMA
            __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);  // two LDS reads (there are 16: the last groups stay empty)
        }
        __builtin_amdgcn_sched_barrier(0);
        MP_WAIT_VMCNT(16);  // this thread's loads of stage s + 1 have landed (stages s + 2, s + 3 may be in flight)
        __syncthreads();    // ... and everyone's; and every wave has read all it needs of stage s from LDS:
        // its buffer takes the stage four ahead.
        if (s + 1 == n_stages - 1 && n_whole < n_stages) blank_tail(s + 1);  // uniform
        // The remaining 20 MFMAs of the trip (the last four of the first 16 tokens, the 16 of the last 16 tokens) go
        // in four groups of five, each behind two of the eight load instructions and interleaved with four of the 16
        // reads of the next stage's first 16 tokens: a load instruction holds the wave for some 40 cycles, and the
        // matrix cores only have the one instruction in flight to work on meanwhile.
        {
            const unsigned char *slab_a = &ring[(s + 1) & (kRing - 1)][0][0], *slab_b = &ring[(s + 1) & (kRing - 1)][1][0];
            issue_part(s + 4, 0, whole_c);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(0, 3, 0);
            mfma_one(0, 3, 1);
            mfma_one(0, 3, 2);
            mfma_one(0, 3, 3);
            mfma_one(1, 0, 0);
            a[0][0] = operand_from_ring(slab_a, 0, wm, 0, lane);
            a[0][1] = operand_from_ring(slab_a, 0, wm, 1, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue_part(s + 4, 1, whole_c);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(1, 0, 1);
            mfma_one(1, 0, 2);
            mfma_one(1, 0, 3);
            mfma_one(1, 1, 0);
            mfma_one(1, 1, 1);
            a[0][2] = operand_from_ring(slab_a, 0, wm, 2, lane);
            a[0][3] = operand_from_ring(slab_a, 0, wm, 3, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue_part(s + 4, 2, whole_c);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(1, 1, 2);
            mfma_one(1, 1, 3);
            mfma_one(1, 2, 0);
            mfma_one(1, 2, 1);
            mfma_one(1, 2, 2);
            b[0][0] = operand_from_ring(slab_b, 0, wn, 0, lane);
            b[0][1] = operand_from_ring(slab_b, 0, wn, 1, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
            issue_part(s + 4, 3, whole_c);
            __builtin_amdgcn_sched_barrier(0);
            mfma_one(1, 2, 3);
            mfma_one(1, 3, 0);
            mfma_one(1, 3, 1);
            mfma_one(1, 3, 2);
            mfma_one(1, 3, 3);
            b[0][2] = operand_from_ring(slab_b, 0, wn, 2, lane);
            b[0][3] = operand_from_ring(slab_b, 0, wn, 3, lane);
#pragma unroll
            for (int g = 0; g < 5; ++g) {
                __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
                __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
            }
            __builtin_amdgcn_sched_barrier(0);
        }
    };
    int64_t s = 0;
    for (; s + 4 < n_whole && s < n_stages; ++s) trip(s, Whole<1>{});  // the steady state
    for (; s < n_stages; ++s) trip(s, Whole<0>{});                     // the last few trips issue stages that may be ragged or absent
    MP_WAIT_VMCNT(0);  // nothing may still be landing in this block's LDS when it ends

    float *out = partials + (static_cast<int64_t>(split) * n_pairs + pair) * (kTile * kTile);
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
#pragma unroll
            for (int v = 0; v < 16; ++v) {
                const int row = wm * 128 + 32 * i + 8 * (v >> 2) + 4 * (lane >> 5) + (v & 3);
                const int col = wn * 128 + 32 * j + (lane & 31);
                out[row * kTile + col] = acc[i][j][v];
            }
}

// h[tile] += sum over splits (in split order, in double) of the partial tile; the mirror image goes below the
// diagonal.  A block takes 32 rows of a tile: 16-byte loads along the rows of the partials, and the transposed
// copy goes through LDS so that it is written in 128-byte runs as well.
__global__ __launch_bounds__(256) void gram_reduce(const float *__restrict__ partials, int n_splits, int n_pairs,
                                                   int n_tiles, int channels, float *__restrict__ h, int64_t ld_h) {
    __shared__ float flip[32][kTile + 1];
    const int pair = blockIdx.x;
    int mt, nt;
    pair_of(pair, n_tiles, mt, nt);
    const int m0 = mt * kTile, n0 = nt * kTile;
    const int r0 = blockIdx.y * 32;                           // first tile row of this block
    const int c4 = (threadIdx.x & 63) * 4, rr = threadIdx.x >> 6;  // 4 columns, row rr + 4 q
    const bool vec_ok = (ld_h % 4 == 0) && (reinterpret_cast<uintptr_t>(h) % 16 == 0);
#pragma unroll 2
    for (int q = 0; q < 8; ++q) {
        const int row = r0 + rr + 4 * q;
        double s[4] = {0.0, 0.0, 0.0, 0.0};
        for (int sp = 0; sp < n_splits; ++sp) {
            const f32x4 v = *reinterpret_cast<const f32x4 *>(
                partials + (static_cast<int64_t>(sp) * n_pairs + pair) * (kTile * kTile) + row * kTile + c4);
#pragma unroll
            for (int e = 0; e < 4; ++e) s[e] += static_cast<double>(v[e]);
        }
        float add[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) {
            add[e] = static_cast<float>(s[e]);  // the rounded sum is what both triangles receive: h stays symmetric
            flip[rr + 4 * q][c4 + e] = add[e];
        }
        const int gi = m0 + row, gj = n0 + c4;
        if (gi < channels) {
            float *dst = h + static_cast<int64_t>(gi) * ld_h + gj;
            if (vec_ok && gj + 4 <= channels) {
                f32x4 old = *reinterpret_cast<f32x4 *>(dst);
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    old[e] = static_cast<float>(static_cast<double>(old[e]) + static_cast<double>(add[e]));
                *reinterpret_cast<f32x4 *>(dst) = old;
            } else {
#pragma unroll
                for (int e = 0; e < 4; ++e)
                    if (gj + e < channels)
                        dst[e] = static_cast<float>(static_cast<double>(dst[e]) + static_cast<double>(add[e]));
            }
        }
    }
    if (mt == nt) return;  // a diagonal tile holds both of its triangles already
    __syncthreads();
    // element (row, col) of the tile goes to h[n0 + col][m0 + row]: 32 consecutive rows make one 128-byte run
    const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;
    for (int col = ty; col < kTile; col += 8) {
        const int gi = n0 + col, gj = m0 + r0 + tx;
        if (gi < channels && gj < channels) {
            float *dst = h + static_cast<int64_t>(gi) * ld_h + gj;
            *dst = static_cast<float>(static_cast<double>(*dst) + static_cast<double>(flip[tx][col]));
        }
    }
}

// Any element type and shape: a 64 x 64 output tile per block (16 x 16 threads, 4 x 4 outputs each), the whole
// token range walked 16 tokens at a time, fp32 FMAs, one owner per output element.
template <typename T>
__global__ __launch_bounds__(256) void gram_generic(const T *__restrict__ x, int64_t n_tokens, int64_t channels,
                                                    int64_t ld, float *__restrict__ h, int64_t ld_h) {
    __shared__ float xa[16][64 + 4], xb[16][64 + 4];
    const int tx = threadIdx.x & 15, ty = threadIdx.x >> 4;
    const int64_t m0 = static_cast<int64_t>(blockIdx.y) * 64, n0 = static_cast<int64_t>(blockIdx.x) * 64;
    float acc[4][4] = {};
    for (int64_t t0 = 0; t0 < n_tokens; t0 += 16) {
        for (int e = threadIdx.x; e < 16 * 64; e += 256) {
            const int r = e >> 6, c = e & 63;
            const int64_t t = t0 + r;
            xa[r][c] = (t < n_tokens && m0 + c < channels) ? widen(x[t * ld + m0 + c]) : 0.f;
            xb[r][c] = (t < n_tokens && n0 + c < channels) ? widen(x[t * ld + n0 + c]) : 0.f;
        }
        __syncthreads();
#pragma unroll
        for (int r = 0; r < 16; ++r) {
            float av[4], bv[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                av[i] = xa[r][ty * 4 + i];
                bv[i] = xb[r][tx * 4 + i];
            }
#pragma unroll
            for (int i = 0; i < 4; ++i)
#pragma unroll
                for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(av[i], bv[j], acc[i][j]);
        }
        __syncthreads();
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t gi = m0 + ty * 4 + i, gj = n0 + tx * 4 + j;
            if (gi < channels && gj < channels) h[gi * ld_h + gj] += acc[i][j];
        }
}

// Tokens per block.  The grid is (token splits) x (tile pairs) blocks of equal work on 256 compute units, one
// block each: the fewest splits that give at least four full rounds and leave the last round at least 97 %
// full (else the fullest last round), in whole stages.
int64_t tokens_per_split_for(int64_t n_tokens, int64_t n_pairs) {
    const int64_t max_splits = ceil_div(n_tokens, kStep) < kMaxSplits ? ceil_div(n_tokens, kStep) : kMaxSplits;
    int64_t best = 1;
    double best_fill = 0.0;
    for (int64_t sp = 1; sp <= max_splits; ++sp) {
        const double rounds = static_cast<double>(sp * n_pairs) / 256.0;
        const double fill = rounds / static_cast<double>(ceil_div(sp * n_pairs, 256));
        if (sp * n_pairs >= 4 * 256 && fill >= 0.97) {
            best = sp;
            break;
        }
        if (fill > best_fill + 1e-9) {
            best_fill = fill;
            best = sp;
        }
    }
    return ceil_div(ceil_div(n_tokens, best), kStep) * kStep;
}

struct GramPlan {
    bool mfma;
    int n_tiles, n_pairs, n_splits;
    int64_t tokens_per_split;
};

GramPlan plan_gram(const void *x, int dtype, int64_t n_tokens, int64_t channels, int64_t ld) {
    GramPlan g = {};
    g.mfma = dtype == PRUNE_BF16 && packet_ok(x, channels, ld) && channels <= 65536 && ld <= (1 << 24) && n_tokens > 0;
    if (!g.mfma) return g;
    g.n_tiles = static_cast<int>(ceil_div(channels, kTile));
    g.n_pairs = g.n_tiles * (g.n_tiles + 1) / 2;
    const int64_t per = tokens_per_split_for(n_tokens, g.n_pairs);
    g.tokens_per_split = per;
    g.n_splits = static_cast<int>(ceil_div(n_tokens, per));
    return g;
}

}  // namespace

size_t hessian_workspace_bytes(int64_t n_tokens, int64_t channels) {
    // sized for the matrix-core path whether or not a particular call can take it
    if (n_tokens <= 0 || channels <= 0) return 0;
    const int64_t n_tiles = ceil_div(channels, kTile), n_pairs = n_tiles * (n_tiles + 1) / 2;
    const int64_t per = tokens_per_split_for(n_tokens, n_pairs);
    const int64_t n_splits = ceil_div(n_tokens, per);
    return static_cast<size_t>(n_splits * n_pairs) * kTile * kTile * sizeof(float);
}

}  // namespace mp

extern "C" size_t prune_hessian_workspace_bytes(int64_t n_tokens, int64_t channels) {
    const size_t n = mp::hessian_workspace_bytes(n_tokens, channels);
    return (n + 255) / 256 * 256;
}

extern "C" int prune_hessian_accumulate(const void *x, int dtype, int64_t n_tokens, int64_t channels, int64_t ld_x,
                                        float *h, int64_t ld_h, void *ws, size_t ws_bytes, void *stream_) {
    using namespace mp;
    if (!valid_dtype(dtype)) return PRUNE_ERR_DTYPE;
    if (n_tokens < 0 || channels <= 0 || ld_x < channels || ld_h < channels || channels > 0x7fffffff)
        return PRUNE_ERR_SHAPE;
    if (!h || (!x && n_tokens > 0)) return PRUNE_ERR_NULL;
    if (!aligned_to(x, elem_size(dtype)) || !aligned_to(h, 4) || (ws && !aligned_to(ws, 16)))
        return PRUNE_ERR_ALIGNMENT;
    if (n_tokens == 0) return PRUNE_OK;
    hipStream_t stream = static_cast<hipStream_t>(stream_);
    const GramPlan g = plan_gram(x, dtype, n_tokens, channels, ld_x);
    if (g.mfma) {
        const size_t need = static_cast<size_t>(g.n_splits) * g.n_pairs * kTile * kTile * sizeof(float);
        if (!ws) return PRUNE_ERR_NULL;
        if (ws_bytes < need) return PRUNE_ERR_WORKSPACE;
        float *partials = static_cast<float *>(ws);
        const int64_t n_chunks = ceil_div(ceil_div(static_cast<int64_t>(g.n_splits) * g.n_pairs, kChunk), kXcds) * kXcds;
        hipLaunchKernelGGL(gram_tiles_bf16, dim3(static_cast<unsigned>(n_chunks * kChunk)), dim3(kGramBlock), 0,
                           stream, static_cast<const bf16_t *>(x), n_tokens, static_cast<int>(channels), ld_x,
                           g.n_tiles, g.n_pairs, g.n_splits, g.tokens_per_split, partials);
        if (launch_status() != PRUNE_OK) return PRUNE_ERR_DEVICE;
        hipLaunchKernelGGL(gram_reduce, dim3(static_cast<unsigned>(g.n_pairs), kTile / 32), dim3(256), 0, stream, partials,
                           g.n_splits, g.n_pairs, g.n_tiles, static_cast<int>(channels), h, ld_h);
        return launch_status();
    }
    const dim3 grid(static_cast<unsigned>(ceil_div(channels, 64)), static_cast<unsigned>(ceil_div(channels, 64)));
    if (grid.y > 65535) return PRUNE_ERR_SHAPE;
    if (dtype == PRUNE_BF16)
        hipLaunchKernelGGL(gram_generic<bf16_t>, grid, dim3(256), 0, stream, static_cast<const bf16_t *>(x), n_tokens,
                           channels, ld_x, h, ld_h);
    else
        hipLaunchKernelGGL(gram_generic<float>, grid, dim3(256), 0, stream, static_cast<const float *>(x), n_tokens,
                           channels, ld_x, h, ld_h);
    return launch_status();
}
