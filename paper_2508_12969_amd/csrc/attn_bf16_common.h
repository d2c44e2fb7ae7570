// Pieces shared by the bf16 MFMA attention kernels: vector types, the LDS chunk swizzles, the
// asynchronous global -> LDS tile copy (tile order and natural order), the partner-lane exchange,
// and the tile step itself: what one wave of 32 queries does with one key tile (S^T = K Q^T,
// padding mask, online softmax with a lazy exponent reference, O^T += V^T P^T) and its epilogue.
// The kernels differ only in how rows are mapped to workgroups and how the tile list is walked.
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
constexpr int kXcdChunk = 64;              // consecutive launch-order entries handed to one XCD

// Launch-order entry of a workgroup id.  Workgroup ids are dealt round-robin to the 8 XCDs, each
// with an L2 of its own; they are remapped so that the workgroups resident on one XCD at a time
// (64: two per CU) are kXcdChunk consecutive entries of the launch order (same head, neighbouring
// query tiles, equal list lengths) instead of every eighth entry: their key-tile lists overlap, so
// more of the K/V tile copies hit that L2.  The order is sorted by descending list length, so in a
// round of 8 chunks the first chunk is the longest; rounds are therefore dealt to the XCDs in
// alternating direction, which evens out the work per XCD (measured at the 130K-token layouts:
// 1.4 % faster at 65 % sparsity, 2.3 % at 80 %, against chunks of 32 always dealt in the same
// direction).  Ids past the last full round keep their place.
__device__ __forceinline__ int64_t xcd_launch_order(int64_t id, int64_t total) {
  const int64_t span = 8 * (int64_t)kXcdChunk;
  if (id >= total / span * span) return id;
  const int64_t xcd = id & 7, seq = id >> 3, round = seq / kXcdChunk;
  return round * span + ((round & 1) ? 7 - xcd : xcd) * kXcdChunk + seq % kXcdChunk;
}

// Launch-order entry of this workgroup, or -1 if it has none.  Workgroup ids below a.static_items are
// bound to entries through xcd_launch_order.  The XCDs of a card differ in speed by a few per cent,
// and ids are bound to XCDs, so the cheapest entries at the end of the order are left unbound: each
// of the a.pool_wgs workgroups after the static part draws a ticket, and takes entry static_items +
// ticket if there is one.  An XCD that is ahead reaches its pool workgroups earlier and draws more
// of them; about twice as many pool workgroups are launched as there are pool entries, so that no
// XCD runs out of draws, and the surplus ones return at once.  The workgroup that draws the last
// ticket puts the counter back to zero for the next launch.  `ticket`: one int of LDS.
__device__ __forceinline__ int64_t launch_entry(const AttnArgs& a, int* ticket) {
  if ((int64_t)blockIdx.x < a.static_items) return xcd_launch_order(blockIdx.x, a.static_items);
  if (threadIdx.x == 0) {
    const int t = atomicAdd(a.pool_counter, 1);
    if (t == a.pool_wgs - 1) __hip_atomic_store(a.pool_counter, 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    *ticket = t;
  }
  __syncthreads();
  const int t = *ticket;
  return t < a.pool_items ? a.static_items + t : -1;
}

// kWaves_: waves of a workgroup that share the tile copies (B / 32 when a workgroup owns one query
// tile, twice that when it owns two).
template <int B_, int D_, int kWaves_ = B_ / 32>
struct Shape {
  static constexpr int B = B_, D = D_;
  static constexpr int kWaves = kWaves_;
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

typedef __attribute__((address_space(3))) const char* LdsTile;

// Where a wave's share of a key tile comes from.  Tile order: the tile is one contiguous block.
// Natural order (kNat): a KiB block of a tile (kRowsPerLoad consecutive slots, inside one run of tw
// tokens) is contiguous there too, at row tile_origin[tile] + (dt*H + dy)*W + dx of the plane; a
// text tile is contiguous as a whole.  row_in_tile[i] is that offset for the i-th block this wave
// copies.
template <class S, bool kNat>
struct TileSource {
  int32_t row_in_tile[kNat ? S::kLoadsPerThread : 1];
  int32_t n_vid, N_real;
  int wave, lane;

  __device__ __forceinline__ TileSource(const AttnArgs& a, int wave_, int lane_) : wave(wave_), lane(lane_) {
    n_vid = (int32_t)a.n_vid;
    N_real = (int32_t)a.N_real;
    row_in_tile[0] = 0;
    if constexpr (kNat) {
#pragma unroll
      for (int i = 0; i < S::kLoadsPerThread; ++i) {
        const int slot0 = (wave * S::kLoadsPerThread + i) * S::kRowsPerLoad;
        const int dx = slot0 % a.tw, run = slot0 / a.tw, dy = run % a.th, dt = run / a.th;
        row_in_tile[i] = (dt * a.H + dy) * a.W + dx;
      }
    }
  }

  // base: the (batch, head) plane of K or V; origin: tile_origin[tile] (natural order only)
  template <class Loader>
  __device__ __forceinline__ void issue(const Loader& loader, const char* base, int tile, int32_t origin, uint32_t lds_addr) const {
    if constexpr (!kNat) {
      loader.issue(base + (int64_t)tile * S::kTileBytes, lds_addr, wave);
    } else {
      const bool text = tile >= n_vid;
      const char* sb[S::kLoadsPerThread];
      bool inside = true;
#pragma unroll
      for (int i = 0; i < S::kLoadsPerThread; ++i) {
        const int32_t row = origin + (text ? (wave * S::kLoadsPerThread + i) * S::kRowsPerLoad : row_in_tile[i]);
        inside = inside && row + S::kRowsPerLoad <= N_real;
        sb[i] = base + (int64_t)row * S::kRowBytes;
      }
      if (inside) {
        loader.issue_blocks(sb, lds_addr, wave);
      } else {
        // slots past the last token (padding of the last tiles): every lane is pointed at a row of the
        // tensor; what it fetches is never attended
#pragma unroll
        for (int i = 0; i < S::kLoadsPerThread; ++i) {
          const int32_t row = origin + (text ? (wave * S::kLoadsPerThread + i) * S::kRowsPerLoad : row_in_tile[i]);
          const int32_t first = min(row, N_real - 1);
          loader.issue_clamped(base + (int64_t)first * S::kRowBytes, N_real - 1 - first, i, lds_addr, wave, lane);
        }
      }
    }
  }

  // Natural-order row of slot `slot` of query tile `q_tile` (clamped into the tensor for a padding
  // slot, whose result is never stored).
  __device__ __forceinline__ int64_t query_row(const AttnArgs& a, int64_t q_tile, int slot) const {
    const int dx = slot % a.tw, run = slot / a.tw, dy = run % a.th, dt = run / a.th;
    const int64_t row = CONST_PTR(int32_t, a.tile_origin)[q_tile] + (q_tile >= a.n_vid ? slot : (dt * a.H + dy) * a.W + dx);
    return row < a.N_real ? row : a.N_real - 1;
  }
};

// Which slot of its query tile a lane works for.  Lanes take the tile's slots in the order of
// class_perm (the slots that hold a token first, then the padding slots), so the queries of a padded
// tile fill as few 32-query waves as possible and the remaining waves only move tiles.  Every lane
// still owns exactly one slot, i.e. one row of the output: a padding slot's row is written as zero.
struct QuerySlot {
  int slot;          // position in the tile, 0 .. B-1
  bool real;         // the slot holds a token
  bool wave_active;  // at least one lane of this wave holds a token (wave-uniform)
};
// first: index of the wave's first lane in that order (32 * wave for a tile of its own)
template <int B, class Args>
__device__ __forceinline__ QuerySlot query_slot(const Args& a, int64_t q_tile, int first, int qi) {
  const int cls = CONST_PTR(int32_t, a.tile_class)[q_tile];
  const auto mask = CONST_PTR(uint32_t, a.class_mask) + cls * 4;
  int valid = __builtin_popcount(mask[0]) + __builtin_popcount(mask[1]);
  if (B > 64) valid += __builtin_popcount(mask[2]) + __builtin_popcount(mask[3]);
  QuerySlot q;
  q.slot = first + qi;
  if (cls != 0) q.slot = a.class_perm[cls * 128 + first + qi];
  q.real = first + qi < valid;
  q.wave_active = first < valid;
  return q;
}

// One wave's 32 queries: operand fragments, accumulators and softmax state, and the tile step.
//
// Transposed formulation.  Scores are computed as S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so in
// the accumulator a lane holds ONE query (column lane%32) and 16 of the 32 keys of a block; its
// partner lane^32 holds the other 16.  Row max and row sum are register-local except for a single
// exchange with the partner lane, and the running max / sum / rescale factor are one scalar per
// lane.  The output is accumulated transposed as well, O^T = V^T P^T, whose B operand (P^T: keys
// along the contraction, queries across lanes) is exactly the bf16-rounded score accumulator,
// register for register: no shuffle and no LDS round trip between the two matrix products.  The
// contraction order over keys inside a 32-key block is permuted (a lane group owns keys {0-3,
// 8-11, 16-19, 24-27} + 4*group), and the V^T operand is fetched with the same permutation.
template <class S>
struct QueryWave {
  static constexpr int D = S::D;
  bf16x8 qf[S::kQkSteps];      // B operand of S^T: lane (qi, g) holds d = 16*step + 8*g .. +7 of its query
  floatx16 acc_o[S::kDBlocks];
  // Exponent reference of this lane's query (raw score units): the first tile's row maximum,
  // afterwards a lagging running maximum.  neg_m holds -m_run in all 16 registers and is the C
  // operand of the first contraction step, so the score accumulator comes out as (score - reference).
  floatx16 neg_m;
  float m_run, l_run;          // l_run: this lane's share of the running sum (partner lane holds the rest)
  float c2, lazy_raw;          // scale * log2(e); kLazyLog2 in raw score units
  int qi, g;
  // per-lane LDS read offsets
  int k_lane_row_off, k_lane_swz;                              // K: row (32*kb + qi), logical chunk 2*step + g
  int v_lane_row, v_lane_swz, v_lane_chunk, v_lane_half;       // V: transposing read, see read_v()

  __device__ __forceinline__ QueryWave(int lane, float scale) {
    qi = lane & 31;
    g = lane >> 5;
    c2 = scale * kLog2e;
    lazy_raw = kLazyLog2 / c2;
    m_run = 0.f;
    l_run = 0.f;
#pragma unroll
    for (int r = 0; r < 16; ++r) neg_m[r] = 0.f;
#pragma unroll
    for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
    k_lane_row_off = qi * S::kRowBytes;
    k_lane_swz = k_swizzle<D>(qi);  // 32*kb does not change the swizzle
    // V: lane covers key row 4*g + (lane%16)/4 (+ 32*kb + 16*t + 8*half) and the 8-byte half-chunk
    // that holds d = 32*db + 16*((lane/16)%2) + 4*(lane%4) .. +3
    v_lane_row = 4 * g + ((lane & 15) >> 2);
    v_lane_swz = v_swizzle<D>(v_lane_row);  // multiples of 8 rows keep it
    v_lane_chunk = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
    v_lane_half = (lane & 1) * 8;
  }

  // q_row_ptr: this lane's query row in global memory
  __device__ __forceinline__ void load_q(const char* q_row_ptr) {
    const char* Qp = q_row_ptr + g * 16;
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(Qp + s * 32);
    // Touch the fragments so that the compiler waits for these loads here, before the loop: inside
    // the loop the vector-memory counter must belong to the tile copies alone.
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) asm volatile("" : "+v"(qf[s]));
  }

  // ---- S^T = K Q^T for the key blocks [kKb0, kKb1) of the tile in lds_k ------------------------
  // One accumulator chain per key block, the contraction steps innermost: written in this order the
  // compiler requests the K fragments of step s + 1 before it issues the products of step s
  // (measured 2-3 % faster at 128-token tiles than the contraction step outermost).
  template <int kKb0, int kKb1>
  __device__ __forceinline__ void qk(LdsTile lds_k, floatx16 (&acc_s)[S::kKeyBlocks]) const {
#pragma unroll
    for (int kb = kKb0; kb < kKb1; ++kb) {
#pragma unroll
      for (int s = 0; s < S::kQkSteps; ++s) {
        const int off = kb * 32 * S::kRowBytes + k_lane_row_off + (((2 * s + g) ^ k_lane_swz) << 4);
        const bf16x8 kf = *reinterpret_cast<const __attribute__((address_space(3))) bf16x8*>(lds_k + off);
        acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? neg_m : acc_s[kb], 0, 0, 0);
      }
    }
  }

  // S^T of one tile.  `upper_keys` false: the upper half of the key slots is padding only (a tile on
  // a padded face of the grid along t); those key blocks are not multiplied, their scores are -inf.
  __device__ __forceinline__ void qk_tile(LdsTile lds_k, floatx16 (&acc_s)[S::kKeyBlocks], bool upper_keys) const {
    constexpr int kLower = S::kKeyBlocks / 2;
    qk<0, kLower>(lds_k, acc_s);
    if (upper_keys) {
      qk<kLower, S::kKeyBlocks>(lds_k, acc_s);
    } else {
#pragma unroll
      for (int kb = kLower; kb < S::kKeyBlocks; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_s[kb][r] = kMinusInf;
    }
  }

  // ---- padding keys never take part ------------------------------------------------------------
  // Only tiles on a padded face of the grid have invalid slots (cls != 0, wave-uniform).  The valid
  // bits of a 32-key block are one scalar word; the select mask of each score register is built on
  // the scalar unit (lanes 0-31 hold key 8*(r/4) + r%4 of the block, lanes 32-63 that key + 4) and
  // applied with one v_cndmask per register.
  template <class MaskPtr>
  __device__ __forceinline__ void mask_padding_keys(floatx16 (&acc_s)[S::kKeyBlocks], int cls, MaskPtr class_mask) const {
    if (cls == 0) return;
#pragma unroll
    for (int kb = 0; kb < S::kKeyBlocks; ++kb) {
      const uint32_t bits = class_mask[cls * 4 + kb];
      if (bits != 0xffffffffu) {
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int bit = 8 * (r / 4) + (r % 4);
          const uint32_t lo = 0u - ((bits >> bit) & 1u), hi = 0u - ((bits >> (bit + 4)) & 1u);
          const uint64_t keep = (uint64_t)lo | ((uint64_t)hi << 32);
          asm("v_cndmask_b32 %0, %1, %0, %2" : "+v"(acc_s[kb][r]) : "v"(kMinusInf), "s"(keep));
        }
      }
    }
  }

  // ---- online softmax (one query per lane) -------------------------------------------------------
  // acc_s holds score - reference in raw units.  The reference is set to the row maximum on the
  // first tile of the row (`first`, wave-uniform) and afterwards moves only for rows whose maximum
  // exceeds it by more than 2^kLazyLog2 (probabilities then stay below that factor, far inside fp32
  // and bf16 range); the accumulator rescale O *= alpha is then a rarely taken wave-uniform branch
  // and the common path per score is one multiply and one exp2.  The result is still the exact
  // softmax: numerator and denominator share the same reference.  Probabilities are rounded to bf16
  // (the B operand of the second product); the row sum adds up the rounded values, two per v_dot2, so
  // numerator and denominator see the same numbers.
  __device__ __forceinline__ void softmax(floatx16 (&acc_s)[S::kKeyBlocks], bool first, bf16x8 (&pf)[S::kKeyBlocks][2]) {
    float mx = acc_s[0][0];
#pragma unroll
    for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
      for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[kb][r]);
    mx = max_with_partner(mx);
    {
      const uint64_t over = __builtin_amdgcn_ballot_w64(mx > lazy_raw);
      if (first || __builtin_amdgcn_readfirstlane((uint32_t)over | (uint32_t)(over >> 32)) != 0) {
        float delta = (first || mx > lazy_raw) ? mx : 0.f;
        if (delta == kMinusInf) delta = 0.f;  // a row that has seen no real key yet keeps its reference
        const float alpha = first ? 1.0f : __builtin_amdgcn_exp2f(-delta * c2);
        m_run += delta;
        l_run *= alpha;
#pragma unroll
        for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_s[kb][r] -= delta;
#pragma unroll
        for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_o[db][r] *= alpha;
#pragma unroll
        for (int r = 0; r < 16; ++r) neg_m[r] = -m_run;
      }
    }
    bf16x2 ones;
    ones[0] = (__bf16)1.0f;
    ones[1] = (__bf16)1.0f;
#pragma unroll
    for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
      for (int t = 0; t < 2; ++t) {
        bf16x8 p8;
#pragma unroll
        for (int e = 0; e < 8; ++e) p8[e] = (__bf16)__builtin_amdgcn_exp2f(acc_s[kb][8 * t + e] * c2);
        pf[kb][t] = p8;
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p8, p8, 0, 1), ones, l_run, false);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p8, p8, 2, 3), ones, l_run, false);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p8, p8, 4, 5), ones, l_run, false);
        l_run = __builtin_amdgcn_fdot2_f32_bf16(__builtin_shufflevector(p8, p8, 6, 7), ones, l_run, false);
      }
  }

  // ---- O^T += V^T P^T ---------------------------------------------------------------------------
  // V stays row-major [key][d] in LDS and is read with ds_read_b64_tr_b16, which hands each lane
  // four consecutive keys of one d column, i.e. the A operand of O^T for the 16 keys of contraction
  // step (kb, t) and the d block db.
  __device__ __forceinline__ bf16x8 read_v(LdsTile lds_v, int kb, int t, int db) const {
    const int chunk = (db * 4 + v_lane_chunk) ^ v_lane_swz;
    const int base = (kb * 32 + t * 16 + v_lane_row) * S::kRowBytes + chunk * 16 + v_lane_half;
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(lds_v + base));
    const shortx4 hi =
        __builtin_amdgcn_ds_read_tr16_b64_v4i16((shortx4 __attribute__((address_space(3)))*)(lds_v + base + 8 * S::kRowBytes));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }

  // the key blocks [kKb0, kKb1) of the tile in lds_v
  template <int kKb0, int kKb1>
  __device__ __forceinline__ void pv(LdsTile lds_v, const bf16x8 (&pf)[S::kKeyBlocks][2]) {
#pragma unroll
    for (int kb = kKb0; kb < kKb1; ++kb)
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int db = 0; db < S::kDBlocks; ++db)
          acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(read_v(lds_v, kb, t, db), pf[kb][t], acc_o[db], 0, 0, 0);
  }

  // O^T += V^T P^T of one tile; the upper key blocks are skipped with their scores (see qk_tile):
  // their probabilities are exactly zero.
  __device__ __forceinline__ void pv_tile(LdsTile lds_v, const bf16x8 (&pf)[S::kKeyBlocks][2], bool upper_keys) {
    pv<0, S::kKeyBlocks / 2>(lds_v, pf);
    if (upper_keys) pv<S::kKeyBlocks / 2, S::kKeyBlocks>(lds_v, pf);
  }

  // ---- epilogue: O = O^T / l; a padding query (q_real false) and an empty row give zeros ---------
  // out_row: this lane's output row in global memory; `write` false: the layout has no row for this
  // lane's slot (a padding slot in natural order) and nothing is stored
  __device__ __forceinline__ void store(char* out_row, bool q_real, bool write) const {
    const float l_tot = sum_with_partner(l_run);
    const float inv = (q_real && l_tot > 0.f) ? 1.0f / l_tot : 0.f;
    if (!write) return;
#pragma unroll
    for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
      for (int r4 = 0; r4 < 4; ++r4) {
        bf16x4 o4;
#pragma unroll
        for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(acc_o[db][4 * r4 + e] * inv);
        const int d0 = db * 32 + 8 * r4 + 4 * g;
        *reinterpret_cast<bf16x4*>(out_row + d0 * 2) = o4;
      }
  }
};

}  // namespace
}  // namespace ca
