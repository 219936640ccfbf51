// Pieces shared by the bf16 matrix-core kernels: operand vector types, the global -> LDS load and the explicit
// wait that goes with it.
#pragma once

#include "common.hpp"

namespace mp {

typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;

// One global -> LDS load of 16 bytes per lane: lane l's packet lands at lds_addr + 16 l (lds_addr uniform, in M0).
// Written as an instruction rather than through the builtin on purpose: the compiler would otherwise guard every
// later LDS read with a wait for all such loads in flight (it cannot tell the ring's stages apart), which undoes
// the prefetch; the waits are placed by hand below.
__device__ __forceinline__ void load_to_lds(const void *src, uint32_t lds_addr) {
    // (one wait state between the scalar write of M0 and the load that reads it).  M0 is declared as written:
    // the compiler keeps values of its own there (the index of a dynamically indexed register array, the
    // operand of its own LDS-DMA and message instructions) and must not assume they survive this statement.
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                 :
                 : "s"(lds_addr), "v"(src)
                 : "memory", "m0");
}

// The same with the address as a uniform 64-bit base (in scalar registers) plus a 32-bit byte offset per lane.  A
// wave that has its SIMD to itself pays for every vector instruction between two matrix instructions, and 64-bit
// vector additions run at a quarter of the rate: a caller whose per-lane part does not change from call to call
// advances the base with scalar arithmetic and spends no vector instruction per load.
__device__ __forceinline__ void load_to_lds(const void *base, uint32_t lane_offset, uint32_t lds_addr) {
    asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                 :
                 : "s"(lds_addr), "v"(lane_offset), "s"(base)
                 : "memory", "m0");
}

// s_waitcnt with only the vector-memory counter set (6 bits: [3:0] and [15:14]); the others left at "no wait"
#define MP_WAIT_VMCNT(n) __builtin_amdgcn_s_waitcnt((((n) & 15) | (((n) >> 4) << 14)) | 0x0F70)

constexpr int kChunk = 32, kXcds = 8;

// Work item of a block of a tiled matrix-core kernel.  Workgroups go to the chip's eight dies round robin, each
// die has its own L2, and a die runs 32 of these blocks at a time: so die x takes items in chunks of 32
// consecutive ones (the kernels number their items so that neighbours share operand slabs), and the blocks that
// share an L2 share slabs.
// Returns false for the padding blocks at the end of the grid.
__device__ __forceinline__ bool item_of_block(int block, int n_items, int &item) {
    const int die = block % kXcds, j = block / kXcds;
    item = ((j / kChunk) * kXcds + die) * kChunk + j % kChunk;
    return item < n_items;
}

__device__ __forceinline__ bf16_t narrow_to_bf16(float f) {  // round to nearest, ties to even
    const uint32_t b = __float_as_uint(f);
    if ((b & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>(0x7fc0u);
    return static_cast<bf16_t>((b + 0x7fffu + ((b >> 16) & 1u)) >> 16);
}

}  // namespace mp
