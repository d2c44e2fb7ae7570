// Pieces shared by the bf16 MFMA attention kernels: vector types, the LDS chunk swizzles, the
// asynchronous global -> LDS tile copy and the partner-lane exchange.
#pragma once

#include "kernels.h"

namespace ca {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) short shortx4;

// Tables that no kernel ever writes are read through the constant address space, which lets the
// compiler keep wave-uniform reads on the scalar unit even after the loop has issued LDS DMA.
#define CONST_PTR(T, p) ((const __attribute__((address_space(4))) T*)(p))
#define LDS_PTR(p) ((__attribute__((address_space(3))) void*)(p))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMinusInf = -__builtin_inff();
constexpr float kLazyLog2 = 8.0f;          // the exponent reference may lag the row max by 2^8
constexpr int kXcdChunk = 32;              // consecutive launch-order entries handed to one XCD

template <int B_, int D_>
struct Shape {
  static constexpr int B = B_, D = D_;
  static constexpr int kWaves = B / 32;           // one wave per 32 queries
  static constexpr int kThreads = kWaves * 64;
  static constexpr int kKeyBlocks = B / 32;       // 32-key blocks of a key tile
  static constexpr int kQkSteps = D / 16;         // contraction steps of S^T = K Q^T
  static constexpr int kDBlocks = D / 32;         // 32-wide blocks of the head dim in O^T
  static constexpr int kRowBytes = D * 2;
  static constexpr int kChunksPerRow = D / 8;     // 16-byte chunks
  static constexpr int kTileBytes = B * D * 2;
  static constexpr int kLoadsPerThread = kTileBytes / (kThreads * 16);
  static constexpr int kRowsPerLoad = 1024 / kRowBytes;  // rows covered by one wave-wide 16-byte load
  static_assert(kLoadsPerThread * kThreads * 16 == kTileBytes, "tile must split evenly");
};

// Chunk swizzles: logical 16-byte chunk `c` of row `row` lives at physical chunk c ^ f(row).
// K is read by 16 consecutive rows at one logical chunk: f must take 16 (D=128) or 8x2 (D=64)
// distinct values.  V is read four rows at a time, 64 contiguous bytes per row: f moves each of
// the four rows to a different 64-byte group.
template <int D>
__device__ __forceinline__ int k_swizzle(int row) {
  return D == 128 ? (row & 15) : ((row >> 1) & 7);
}
template <int D>
__device__ __forceinline__ int v_swizzle(int row) {
  return D == 128 ? ((row & 3) << 2) : (((row >> 1) & 1) << 2);
}

// Asynchronous copy of one B x D tile from global memory into LDS (global_load_lds_dwordx4: each
// lane moves 16 bytes, the wave's 64 chunks land contiguously at M0 + offset).  Wave `w` fills the
// KiB blocks [w*L, (w+1)*L) of the tile, L = kLoadsPerThread.  The swizzle is applied on the global
// side: the lane that fills physical chunk p of LDS row r fetches logical chunk p ^ f(r).
// Written as inline assembly on purpose: the compiler then does not track these copies and leaves
// the waiting to the explicit s_waitcnt vmcnt(n) below, which is what lets a copy stay in flight
// across the matrix products of the other operand.  The instruction offset moves the global and
// the LDS address together, so a group of four loads shares one M0 value and one scalar base.
template <class S, bool kIsV>
struct TileLoader {
  static constexpr int kGroups = (S::kLoadsPerThread + 3) / 4;  // loads are issued four per M0 value
  static constexpr int kPerGroup = S::kLoadsPerThread / kGroups;
  static_assert(kPerGroup == 4, "four loads per group");
  uint32_t voff[4];  // per-lane byte offset inside the wave's slice for loads 0..3 of a group

  __device__ __forceinline__ TileLoader(int wave, int lane) {
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      // the swizzle depends on the row only through bits that repeat every four KiB blocks
      const int blk = wave * S::kLoadsPerThread + i;
      const int row = blk * S::kRowsPerLoad + lane / S::kChunksPerRow;
      const int phys = lane % S::kChunksPerRow;
      const int logical = phys ^ (kIsV ? v_swizzle<S::D>(row) : k_swizzle<S::D>(row));
      voff[i] = (uint32_t)((lane / S::kChunksPerRow) * S::kRowBytes + logical * 16);
    }
  }

  // gtile: global address of the tile (wave-uniform); lds_tile: LDS byte address of the buffer.
  __device__ __forceinline__ void issue(const char* gtile, uint32_t lds_tile, int wave) const {
#pragma unroll
    for (int grp = 0; grp < kGroups; ++grp) {
      const uint32_t slice = (uint32_t)(wave * S::kLoadsPerThread + grp * 4) * 1024u;
      const char* sbase = gtile + slice;
      const uint32_t m0 = lds_tile + slice;
      asm volatile(
          "s_mov_b32 m0, %[m0]\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %[v0], %[sb] offset:0\n\t"
          "global_load_lds_dwordx4 %[v1], %[sb] offset:1024\n\t"
          "global_load_lds_dwordx4 %[v2], %[sb] offset:2048\n\t"
          "global_load_lds_dwordx4 %[v3], %[sb] offset:3072\n\t"
          :
          : [m0] "s"(m0), [v0] "v"(voff[0]), [v1] "v"(voff[1]), [v2] "v"(voff[2]), [v3] "v"(voff[3]), [sb] "s"(sbase)
          : "memory");
    }
  }

  // The same copy with one global base per KiB block (a tile gathered from natural token order):
  // sb[i] is the address of the first row of the wave's i-th block.  The instruction offset moves the
  // global and the LDS address together, so each base is handed over minus that offset.
  __device__ __forceinline__ void issue_blocks(const char* const (&sb)[S::kLoadsPerThread], uint32_t lds_tile, int wave) const {
#pragma unroll
    for (int grp = 0; grp < kGroups; ++grp) {
      const uint32_t m0 = lds_tile + (uint32_t)(wave * S::kLoadsPerThread + grp * 4) * 1024u;
      asm volatile(
          "s_mov_b32 m0, %[m0]\n\t"
          "s_nop 0\n\t"
          "global_load_lds_dwordx4 %[v0], %[s0] offset:0\n\t"
          "global_load_lds_dwordx4 %[v1], %[s1] offset:1024\n\t"
          "global_load_lds_dwordx4 %[v2], %[s2] offset:2048\n\t"
          "global_load_lds_dwordx4 %[v3], %[s3] offset:3072\n\t"
          :
          : [m0] "s"(m0), [v0] "v"(voff[0]), [v1] "v"(voff[1]), [v2] "v"(voff[2]), [v3] "v"(voff[3]), [s0] "s"(sb[grp * 4]),
            [s1] "s"(sb[grp * 4 + 1] - 1024), [s2] "s"(sb[grp * 4 + 2] - 2048), [s3] "s"(sb[grp * 4 + 3] - 3072)
          : "memory");
    }
  }

  // One block whose rows may run past the end of the tensor: lane rows are clamped to `last_row`
  // (rows counted from `first`, which is inside the tensor).
  __device__ __forceinline__ void issue_clamped(const char* first, int32_t last_row, int i, uint32_t lds_tile, int wave, int lane) const {
    const int row = min(lane / S::kChunksPerRow, (int)last_row);
    const uint32_t v = (voff[i & 3] % (uint32_t)S::kRowBytes) + (uint32_t)row * S::kRowBytes;
    const uint32_t m0 = lds_tile + (uint32_t)(wave * S::kLoadsPerThread + i) * 1024u;
    asm volatile(
        "s_mov_b32 m0, %[m0]\n\t"
        "s_nop 0\n\t"
        "global_load_lds_dwordx4 %[v], %[sb] offset:0\n\t"
        :
        : [m0] "s"(m0), [v] "v"(v), [sb] "s"(first)
        : "memory");
  }
};

// Exchange with the partner lane (lane ^ 32) on the VALU: returns max / sum of x and partner's x.
__device__ __forceinline__ float max_with_partner(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return fmaxf(a, b);
}
__device__ __forceinline__ float sum_with_partner(float x) {
  float a = x, b = x;
  asm volatile("s_nop 1\n\tv_permlane32_swap_b32 %0, %1\n\ts_nop 1" : "+v"(a), "+v"(b));
  return a + b;
}

#define WAIT_VMCNT(n) asm volatile("s_waitcnt vmcnt(%0)" ::"n"(n) : "memory")
#define WAIT_LGKMCNT0() asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory")
#define BARRIER() asm volatile("s_barrier" ::: "memory")

}  // namespace
}  // namespace ca
