// Block-sparse attention forward on bf16 MFMA for gfx950 (Appendix D of the paper: a block loop
// with online softmax that visits only the kept key tiles of each query tile).
//
// Work decomposition.  One workgroup owns one (batch, head, query tile) row of the layout and
// walks that row's kept key tiles.  A wave owns 32 query tokens; the workgroup has B/32 waves.
//
// Transposed formulation.  Scores are computed as S^T = K Q^T with v_mfma_f32_32x32x16_bf16, so
// in the accumulator a lane holds ONE query (column lane%32) and 16 of the 32 keys of a block;
// its partner lane^32 holds the other 16.  Row max and row sum are therefore register-local
// except for a single exchange with the partner lane, and the running max / sum / rescale factor
// are one scalar per lane.  The output is accumulated transposed as well, O^T = V^T P^T, whose
// B operand (P^T: keys along the contraction, queries across lanes) is exactly the bf16-rounded
// score accumulator, register for register: no shuffle and no LDS round trip between the two
// matrix products.  The contraction order over keys inside a 32-key block is permuted (a lane
// group owns keys {0-3, 8-11, 16-19, 24-27} + 4*group), and the V^T operand is fetched with the
// same permutation.
//
// Operand staging.  K and V tiles go from HBM/L2 straight into LDS (global_load_lds, 16 bytes
// per lane, no VGPR staging), two buffers each.  K rows are read back as 16-byte row fragments
// (A operand of S^T).  V stays row-major [key][d] in LDS and is read with ds_read_b64_tr_b16,
// which hands each lane four consecutive keys of one d column, i.e. the A operand of O^T.  Both
// tiles are stored with an XOR swizzle of the 16-byte chunk index, applied on the global side of
// the copy (the LDS side of global_load_lds is lane-contiguous), so that both read patterns
// spread over all banks.
//
// Software pipeline.  On this hardware the matrix pipe and the vector ALU overlap only when their
// instructions alternate inside ONE wave's instruction stream: a second wave on the SIMD did not
// hide the softmax behind the other wave's MFMAs (measured).  So the kernel runs one wave per SIMD
// and step j of the loop issues, interleaved in one basic block,
//     MFMA:  O^T += V(j-1)^T P(j-1)^T   and   S(j+1)^T = K(j+1) Q^T
//     VALU:  P(j) = exp2(scale' * S(j) - m)   with the running max / sum update,
// which keeps three tiles in flight in registers (S(j+1) being produced, S(j) being exponentiated,
// P(j-1) being consumed).  The copies K(j+2) and V(j) are issued at the top of step j and waited
// for at the top of step j+1, with one workgroup barrier per step.
//
// Rescaling.  The reference value m of the exponent only moves when the row maximum exceeds it by
// more than 2^kLazyLog2 (probabilities then stay below that factor, far inside fp32 and bf16
// range); the accumulator rescale O *= alpha is a rarely taken wave-uniform branch between steps.
// The result is still the exact softmax: numerator and denominator share the same reference.
#include "kernels.h"

namespace ca {
namespace {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) __bf16 bf16x4;
typedef __attribute__((ext_vector_type(16))) float floatx16;
typedef __attribute__((ext_vector_type(4))) short shortx4;

// Tables that no kernel ever writes are read through the constant address space, which lets the
// compiler keep wave-uniform reads on the scalar unit even after the loop has issued LDS DMA.
#define CONST_PTR(T, p) ((const __attribute__((address_space(4))) T*)(p))
#define LDS_CAST(T, addr) ((T __attribute__((address_space(3)))*)(uintptr_t)(addr))

constexpr float kLog2e = 1.4426950408889634f;
constexpr float kMinusInf = -__builtin_inff();
constexpr float kRunningMaxInit = -1e30f;  // finite, so that (m_old - m_new) never forms inf - inf
constexpr float kLazyLog2 = 8.0f;          // the exponent reference may lag the row max by 2^8

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
  static constexpr int kUnitRows = 64;                   // keys per pipeline unit
  static constexpr int kUnits = B / kUnitRows;           // units per tile
  static constexpr int kUnitBytes = kUnitRows * kRowBytes;
  static constexpr int kLoadsPerThread = kUnitBytes / (kThreads * 16);  // 16-byte loads per lane per unit
  static constexpr int kRowsPerLoad = 1024 / kRowBytes;  // rows covered by one wave-wide 16-byte load
  static constexpr int kLdsBytes = 4 * kUnitBytes;       // two K slots and two V slots of one unit each
  static_assert(kLoadsPerThread * kThreads * 16 == kUnitBytes, "unit must split evenly");
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

// Asynchronous copy of one unit (64 rows of a B x D tile) from global memory into LDS (global_load_lds_dwordx4: each
// lane moves 16 bytes, the wave's 64 chunks land contiguously at M0 + offset).  Wave `w` fills the
// KiB blocks [w*L, (w+1)*L) of the unit, L = kLoadsPerThread.  The swizzle is applied on the global
// side: the lane that fills physical chunk p of LDS row r fetches logical chunk p ^ f(r).
// Written as inline assembly on purpose: the compiler then does not track these copies and leaves
// the waiting to the explicit s_waitcnt below.  The instruction offset moves the global and the
// LDS address together, so a group of four loads shares one M0 value and one scalar base.
template <class S, bool kIsV>
struct UnitLoader {
  static constexpr int kPerGroup = S::kLoadsPerThread < 4 ? S::kLoadsPerThread : 4;  // loads per M0 value
  static constexpr int kGroups = S::kLoadsPerThread / kPerGroup;
  static_assert(kPerGroup * kGroups == S::kLoadsPerThread && (kPerGroup == 2 || kPerGroup == 4), "2 or 4 loads per group");
  uint32_t voff[4];  // per-lane byte offset inside the wave's slice for loads 0..3 of a group

  __device__ __forceinline__ UnitLoader(int wave, int lane) {
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

  // gunit: global address of the unit's first row (wave-uniform); lds_slot: LDS byte address.
  __device__ __forceinline__ void issue(const char* gunit, uint32_t lds_slot, int wave) const {
#ifdef CA_EXP_NOLOAD
    return;
#endif
#pragma unroll
    for (int grp = 0; grp < kGroups; ++grp) {
      const uint32_t slice = (uint32_t)(wave * S::kLoadsPerThread + grp * kPerGroup) * 1024u;
      const char* sbase = gunit + slice;
      const uint32_t m0 = lds_slot + slice;
      if constexpr (kPerGroup == 4) {
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
      } else {
        asm volatile(
            "s_mov_b32 m0, %[m0]\n\t"
            "s_nop 0\n\t"
            "global_load_lds_dwordx4 %[v0], %[sb] offset:0\n\t"
            "global_load_lds_dwordx4 %[v1], %[sb] offset:1024\n\t"
            :
            : [m0] "s"(m0), [v0] "v"(voff[0]), [v1] "v"(voff[1]), [sb] "s"(sbase)
            : "memory");
      }
    }
  }
};

// all tile copies of this wave have landed and all of its LDS reads have returned
#define WAIT_VMCNT0() asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory")
#define BARRIER() asm volatile("s_barrier" ::: "memory")

// Exchange with the partner lane (lane ^ 32) on the VALU: returns max(x, partner's x).
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

// The pipeline advances in units of 64 keys (two 32-key blocks): a 128-token tile is two units, a
// 64-token tile one.  A unit's scores are 32 accumulator registers per lane.
//
// Instruction order.  This file is compiled with the machine schedulers switched off, so the
// order written here is the order issued.  pipeline_step() therefore spells the interleaving out:
// after each MFMA it emits the LDS reads of the MFMA two places ahead and a slice of the softmax
// arithmetic, sized so that the vector ALU work fits in the 32 cycles the matrix pipe is busy.
template <class S>
struct Wave {
  // per-lane constants
  int lane, wave, qi, g;
  uint32_t k_read_off;   // K fragment: row qi of a key block, before the chunk swizzle
  uint32_t k_swz;        // chunk swizzle of this lane's K rows
  uint32_t v_read_off[S::kDBlocks];  // V fragment address of d-block db for key row 4*g + (lane%16)/4
  float c2;              // softmax scale * log2(e)
  float lazy_raw;        // kLazyLog2 expressed in raw score units

  // softmax state of this lane's query
  float m_ref, l_run;

  // registers of the pipeline
  bf16x8 qf[S::kQkSteps];
  floatx16 acc_o[S::kDBlocks];

  __device__ __forceinline__ void init(int lane_, int wave_, float scale) {
    lane = lane_; wave = wave_; qi = lane & 31; g = lane >> 5;
    k_read_off = (uint32_t)(qi * S::kRowBytes);
    k_swz = (uint32_t)k_swizzle<S::D>(qi);  // 32*kb leaves the swizzle unchanged
    const int v_row = 4 * g + ((lane & 15) >> 2);          // + 32*kb + 16*t + 8*half
    const int v_swz = v_swizzle<S::D>(v_row);              // unchanged by multiples of 8 rows
    const int v_chunk = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
#pragma unroll
    for (int db = 0; db < S::kDBlocks; ++db)
      v_read_off[db] = (uint32_t)(v_row * S::kRowBytes + (((db * 4 + v_chunk) ^ v_swz) << 4) + (lane & 1) * 8);
    c2 = scale * kLog2e;
    lazy_raw = kLazyLog2 / c2;
    m_ref = kRunningMaxInit;
    l_run = 0.f;
#pragma unroll
    for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
  }

  // A operand of QK MFMA number i (i = 2*s + kb): K rows of block kb, d = 16*s + 8*g .. +7.
  __device__ __forceinline__ bf16x8 k_frag(uint32_t k_lds, int i) const {
    const int s = i >> 1, kb = i & 1;
    const uint32_t chunk = (((uint32_t)(2 * s + g)) ^ k_swz) << 4;
    return *LDS_CAST(const bf16x8, k_lds + k_read_off + chunk + kb * 32 * S::kRowBytes);
  }
  // A operand of PV MFMA number i (i = kk*kDBlocks + db): V^T, d-block db, 16-key slice kk.
  __device__ __forceinline__ bf16x8 v_frag(uint32_t v_lds, int i) const {
    const int kk = i / S::kDBlocks, db = i % S::kDBlocks;
    const uint32_t addr = v_lds + v_read_off[db] + kk * 16 * S::kRowBytes;
    const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_CAST(shortx4, addr));
    const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(LDS_CAST(shortx4, addr + 8 * S::kRowBytes));
    return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
  }
  __device__ __forceinline__ void qk_mfma(floatx16 (&s_next)[2], int i, bf16x8 kf) const {
    const int s = i >> 1, kb = i & 1;
    if (s == 0) {
      const floatx16 zero = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
      s_next[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], zero, 0, 0, 0);
    } else {
      s_next[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s_next[kb], 0, 0, 0);
    }
  }
  __device__ __forceinline__ void pv_mfma(const bf16x8 (&p)[2][2], int i, bf16x8 vf) {
    const int kk = i / S::kDBlocks, db = i % S::kDBlocks;
    acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, p[kk >> 1][kk & 1], acc_o[db], 0, 0, 0);
  }

  // Plain (not interleaved) forms, used to fill and drain the pipeline.
  __device__ __forceinline__ void qk_all(floatx16 (&s_next)[2], uint32_t k_lds) const {
#pragma unroll
    for (int i = 0; i < 2 * S::kQkSteps; ++i) qk_mfma(s_next, i, k_frag(k_lds, i));
  }
  __device__ __forceinline__ void pv_all(const bf16x8 (&p)[2][2], uint32_t v_lds) {
#pragma unroll
    for (int i = 0; i < 4 * S::kDBlocks; ++i) pv_mfma(p, i, v_frag(v_lds, i));
  }

  // Moves the exponent reference if the row maximum ran away from it; returns the factor by which
  // everything accumulated before this unit has to be multiplied (exactly 1 when it stays).
  __device__ __forceinline__ float update_reference(float row_max) {
    const float m_new = row_max > m_ref + lazy_raw ? row_max : m_ref;
    const float alpha = __builtin_amdgcn_exp2f((m_ref - m_new) * c2);
    m_ref = m_new;
    return alpha;
  }

  __device__ __forceinline__ void rescale_if_needed(float alpha) {
    const uint64_t moved = __builtin_amdgcn_ballot_w64(alpha != 1.0f);
    // a scalar condition, so that this stays a skipped branch and never runs under a lane mask
    if (__builtin_amdgcn_readfirstlane((uint32_t)moved | (uint32_t)(moved >> 32)) != 0) {
#pragma unroll
      for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
        for (int r = 0; r < 16; ++r) acc_o[db][r] *= alpha;
    }
  }

  // Padding keys never take part: their scores become -inf before the row max is taken.
  // valid0/1: validity bits of the 32 keys of block 0/1 of this unit.
  __device__ __forceinline__ void mask_padding(floatx16 (&s)[2], uint32_t valid0, uint32_t valid1) const {
#pragma unroll
    for (int kb = 0; kb < 2; ++kb) {
      const uint32_t bits = (kb ? valid1 : valid0) >> (4 * g);
#pragma unroll
      for (int r = 0; r < 16; ++r) {
        const int bit = 8 * (r / 4) + (r % 4);  // key 32*kb + 8*(r/4) + 4*g + r%4
        if (!((bits >> bit) & 1u)) s[kb][r] = kMinusInf;
      }
    }
  }
};

// One step of the software pipeline (see the file header), on units of 64 keys.  kPV: there is a
// previous unit whose probabilities p_prev are multiplied into O from the V rows at v_lds.  kQK:
// there is a next unit with its K rows at k_lds whose scores go to s_next.  Returns the factor
// by which O (as it is after this step's PV) has to be rescaled.
//
// Softmax of the current unit, in issue order between the MFMAs:
//   slots 0..3    row maximum of the lane's 32 scores (4 chains of max), then the exchange with
//                 the partner lane and the reference update
//   slots 4..     per score: x = fma(s, c2, -m*c2), p = exp2(x)  (exp2 is 2 issue slots), and two
//                 scores later: sum += p, and for every second score the packed bf16 conversion
template <class S, bool kPV, bool kQK>
__device__ __forceinline__ float pipeline_step(Wave<S>& w, const floatx16 (&s_cur)[2], floatx16 (&s_next)[2],
                                               const bf16x8 (&p_prev)[2][2], bf16x8 (&p_cur)[2][2], uint32_t k_lds,
                                               uint32_t v_lds) {
  constexpr int kNumPv = kPV ? 4 * S::kDBlocks : 0, kNumQk = kQK ? 2 * S::kQkSteps : 0;
  constexpr int kNum = kNumPv + kNumQk;     // MFMAs of this step
#ifndef CA_EXP_AHEAD
#define CA_EXP_AHEAD 2
#endif
  constexpr int kAhead = CA_EXP_AHEAD;      // operand reads run this many MFMAs ahead
  constexpr int kMaxSlots = 4;              // MFMAs that shadow the row maximum
  bf16x8 frag[kNum > 0 ? kNum : 1];
  auto fetch = [&](int i) {
#ifdef CA_EXP_NOLDS
    frag[i] = w.qf[i % S::kQkSteps];
#else
    if (i < kNumPv) frag[i] = w.v_frag(v_lds, i);
    else frag[i] = w.k_frag(k_lds, i - kNumPv);
#endif
  };
  auto mfma = [&](int i) {
    if (i < kNumPv) w.pv_mfma(p_prev, i, frag[i]);
    else w.qk_mfma(s_next, i - kNumPv, frag[i]);
  };
  auto score = [&](int e) -> float { return s_cur[e >> 4][e & 15]; };

#pragma unroll
  for (int i = 0; i < kAhead && i < kNum; ++i) fetch(i);

  // ---- row maximum under the first MFMAs ------------------------------------------------------
  float mx[4] = {score(0), score(1), score(2), score(3)};
#pragma unroll
  for (int i = 0; i < kMaxSlots; ++i) {
    if (i < kNum) {
      if (i + kAhead < kNum) fetch(i + kAhead);
      mfma(i);
    }
#pragma unroll
    for (int e = 4 + 7 * i; e < 4 + 7 * (i + 1) && e < 32; ++e) mx[e & 3] = fmaxf(mx[e & 3], score(e));
  }
  float row_max = fmaxf(fmaxf(mx[0], mx[1]), fmaxf(mx[2], mx[3]));
  row_max = max_with_partner(row_max);
  const float alpha = w.update_reference(row_max);
  const float mc = w.m_ref * w.c2;

  // ---- exponentials, sums and bf16 conversion under the remaining MFMAs ------------------------
  constexpr int kRest = kNum > kMaxSlots ? kNum - kMaxSlots : 0;
  // 32 scores over kRest slots; with no MFMAs left (pipeline drain) everything is emitted at once
  constexpr int kPerSlot = kRest > 0 ? (32 + 2 + kRest - 1) / kRest : 34;
  float p[32];
  float ps[4] = {0.f, 0.f, 0.f, 0.f};
  auto micro = [&](int t) {  // t = 0..33: exponentiate score t, retire score t-2
#ifdef CA_EXP_NOSOFTMAX
    if (t < 32) p[t] = score(t);
#else
    if (t < 32) p[t] = __builtin_amdgcn_exp2f(__builtin_fmaf(score(t), w.c2, -mc));
#endif
    const int r = t - 2;
    if (r >= 0) {
      ps[r & 3] += p[r];
      if (r & 1) {
        p_cur[r >> 4][(r >> 3) & 1][(r & 7) - 1] = (__bf16)p[r - 1];
        p_cur[r >> 4][(r >> 3) & 1][r & 7] = (__bf16)p[r];
      }
    }
  };
  if constexpr (kRest > 0) {
#pragma unroll
    for (int i = kMaxSlots; i < kNum; ++i) {
      if (i + kAhead < kNum) fetch(i + kAhead);
      mfma(i);
#pragma unroll
      for (int t = (i - kMaxSlots) * kPerSlot; t < (i - kMaxSlots + 1) * kPerSlot && t < 34; ++t) micro(t);
    }
  } else {
#pragma unroll
    for (int t = 0; t < 34; ++t) micro(t);
  }
  w.l_run = w.l_run * alpha + ((ps[0] + ps[1]) + (ps[2] + ps[3]));
  // The probabilities are first needed by the next step; without a use here the backend sinks the
  // exponentials down to that use, i.e. out of the shadow of this step's MFMAs.
  asm volatile("" : "+v"(p_cur[0][0]), "+v"(p_cur[0][1]), "+v"(p_cur[1][0]), "+v"(p_cur[1][1]));
  return alpha;
}

#ifdef CA_PROFILE
// Development aid: per-workgroup cycle totals of the loop phases (wave 0), read back by a debug hook.
static __device__ unsigned long long g_profile[8 * 65536];
#define PROF_NOW() __builtin_readcyclecounter()
#else
#define PROF_NOW() 0ull
#endif

// Per kept tile the kernel reads one packed word, tile id | padding class << 24, prefetched three
// tiles ahead into scalar registers so that no dependent scalar load sits between two steps.
constexpr int kMetaClassShift = 24;
constexpr int32_t kMetaTileMask = (1 << kMetaClassShift) - 1;

template <int B, int D>
__global__ __attribute__((amdgpu_flat_work_group_size(B * 2, B * 2), amdgpu_waves_per_eu(2, 2)))
void attn_bf16_kernel(AttnArgs a) {
  using S = Shape<B, D>;
  constexpr int kUnits = S::kUnits;
  extern __shared__ __attribute__((aligned(1024))) char lds[];  // K slot 0, K slot 1, V slot 0, V slot 1

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);

  // Workgroup ids are dealt round-robin to the 8 XCDs, each with an L2 of its own.  Remap them so
  // that the workgroups resident on one XCD at a time are `chunk` consecutive entries of the launch
  // order (same head, neighbouring query tiles, equal list lengths): they walk nearly the same key
  // tiles at nearly the same time, so one of them pulls a tile into that L2 and the others hit.
  const int64_t rows = (int64_t)a.num_heads * a.n;
  int64_t linear = blockIdx.x;
  {
    const int64_t span = 8 * (int64_t)a.xcd_chunk, total = rows * a.batch;
    if (linear < total / span * span) {
      const int64_t xcd = linear & 7, seq = linear >> 3;
      linear = (seq / a.xcd_chunk) * span + xcd * a.xcd_chunk + seq % a.xcd_chunk;
    }
  }
  const int64_t item = linear % rows;
  const int64_t batch = linear / rows;
  const int64_t row = a.order ? (int64_t)a.order[item] : item;
  const int64_t head = row / a.n, q_tile = row - head * a.n;
  const int64_t plane = (batch * a.num_heads + head) * a.n * (int64_t)S::kTileBytes;
  const char* Kp = static_cast<const char*>(a.k) + plane;
  const char* Vp = static_cast<const char*>(a.v) + plane;

  // kept tiles of this row: a slice of the packed CSR, or the shared 0..n-1 list of the dense walk
  const int64_t begin = a.row_ptr ? a.row_ptr[row] : 0;
  const int n = (int)(a.row_ptr ? a.row_ptr[row + 1] - begin : a.n);
  const auto meta = CONST_PTR(int32_t, a.col_meta + begin);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class

  Wave<S> w;
  w.init(lane, wave, a.scale);

  // Q fragment: B operand of S^T, lane (qi, g) holds d = 16*step + 8*g .. +7 of its query.
  const int64_t q_row = q_tile * B + wave * 32 + w.qi;
  {
    const char* Qp = static_cast<const char*>(a.q) + plane + q_row * S::kRowBytes + w.g * 16;
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) w.qf[s] = *reinterpret_cast<const bf16x8*>(Qp + s * 32);
    // Touch the fragments so that the compiler waits for these loads here, before the loop: inside
    // the loop the vector-memory counter must belong to the tile copies alone.
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) asm volatile("" : "+v"(w.qf[s]));
  }

  const UnitLoader<S, false> k_loader(wave, lane);
  const UnitLoader<S, true> v_loader(wave, lane);
  const uint32_t lds_base = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds;
  // LDS slots: the K rows of unit u sit in K slot u&1, its V rows in V slot u&1.
  auto k_slot = [&](int u) -> uint32_t { return lds_base + (uint32_t)(u & 1) * S::kUnitBytes; };
  auto v_slot = [&](int u) -> uint32_t { return lds_base + (uint32_t)(2 + (u & 1)) * S::kUnitBytes; };

  // Window of packed words for tiles jj .. jj+3 of the row (0 past the end).
  int jj = 0;
  int32_t w0 = n > 0 ? meta[0] : 0, w1 = n > 1 ? meta[1] : 0, w2 = n > 2 ? meta[2] : 0, w3 = n > 3 ? meta[3] : 0;
  auto advance = [&]() {
    ++jj;
    w0 = w1; w1 = w2; w2 = w3;
    w3 = jj + 3 < n ? meta[jj + 3] : 0;
  };
  // Packed word of the tile that holds unit u, for u / kUnits in jj .. jj+2.
  auto word_of = [&](int u) -> int32_t {
    const int d = u / kUnits - jj;
    return d == 0 ? w0 : (d == 1 ? w1 : w2);
  };
  auto unit_offset = [&](int u) -> int64_t {
    // wave-uniform by construction; said explicitly so that the address stays in scalar registers
#ifdef CA_EXP_SAMETILE
    const uint32_t tile = (uint32_t)__builtin_amdgcn_readfirstlane(word_of(u) & 3);
#else
    const uint32_t tile = (uint32_t)__builtin_amdgcn_readfirstlane(word_of(u) & kMetaTileMask);
#endif
    const uint32_t half = (uint32_t)__builtin_amdgcn_readfirstlane(u % kUnits);
    static_assert((S::kTileBytes & (S::kTileBytes - 1)) == 0, "tile size is a power of two");
    return (int64_t)(((uint64_t)tile << __builtin_ctz(S::kTileBytes)) + half * (uint32_t)S::kUnitBytes);
  };
#ifdef CA_EXP_HALFLOAD
  auto load_k = [&](int u) { if (((u / kUnits) & 1) == 0) k_loader.issue(Kp + unit_offset(u), k_slot(u), wave); };
  auto load_v = [&](int u) { if (((u / kUnits) & 1) == 0) v_loader.issue(Vp + unit_offset(u), v_slot(u), wave); };
#else
  auto load_k = [&](int u) { k_loader.issue(Kp + unit_offset(u), k_slot(u), wave); };
  auto load_v = [&](int u) { v_loader.issue(Vp + unit_offset(u), v_slot(u), wave); };
#endif
  auto mask_if_padded = [&](floatx16 (&s)[2], int u) {
    const int cls = word_of(u) >> kMetaClassShift;
    if (cls != 0) {
      const int idx = cls * 4 + 2 * (u % kUnits);
      w.mask_padding(s, class_mask[idx], class_mask[idx + 1]);
    }
  };
  const int U = n * kUnits;  // units of this row
  // Before step u: every copy issued before the previous step has landed for every wave, and every
  // wave is done with K slot u&1 (unit u, read by the previous step) and V slot u&1 (unit u-2);
  // then K(u+2) and V(u) are put in flight, to be used by step u+1.
  unsigned long long prof[6] = {0, 0, 0, 0, 0, 0};
  unsigned long long prof_t = PROF_NOW();
  auto prof_mark = [&](int slot) {
#ifdef CA_PROFILE
    const unsigned long long now = PROF_NOW();
    prof[slot] += now - prof_t;
    prof_t = now;
#endif
  };
  auto before_step = [&](int u) {
    prof_mark(4);
    if (u > 0 && u % kUnits == 0) advance();   // now jj == u / kUnits
    WAIT_VMCNT0();
    prof_mark(0);
    BARRIER();
    prof_mark(1);
    if (u + 2 < U) load_k(u + 2);
    load_v(u);
    prof_mark(2);
  };

  floatx16 s_a[2], s_b[2];
  bf16x8 p_a[2][2], p_b[2][2];

  if (n > 0) {
    load_k(0);
    if (U > 1) load_k(1);
    WAIT_VMCNT0();
    BARRIER();
    w.qk_all(s_a, k_slot(0));
    mask_if_padded(s_a, 0);

    // step 0 (even state: scores in s_a, probabilities go to p_a)
    before_step(0);
    if (U == 1) {
      const float alpha = pipeline_step<S, false, false>(w, s_a, s_b, p_b, p_a, 0, 0);
      w.rescale_if_needed(alpha);
    } else {
      const float alpha = pipeline_step<S, false, true>(w, s_a, s_b, p_b, p_a, k_slot(1), 0);
      w.rescale_if_needed(alpha);
      mask_if_padded(s_b, 1);
      int u = 1;
      for (;;) {
        // odd state: scores in s_b, previous probabilities in p_a
        if (u == U - 1) {
#pragma unroll
          for (int kb = 0; kb < 2; ++kb) {
            s_a[kb] = s_b[kb];
            p_b[kb][0] = p_a[kb][0];
            p_b[kb][1] = p_a[kb][1];
          }
          break;
        }
        before_step(u);
        {
          const float alpha1 = pipeline_step<S, true, true>(w, s_b, s_a, p_a, p_b, k_slot(u + 1), v_slot(u - 1));
          prof_mark(3);
          w.rescale_if_needed(alpha1);
          mask_if_padded(s_a, u + 1);
        }
        ++u;
        // even state: scores in s_a, previous probabilities in p_b
        if (u == U - 1) break;
        before_step(u);
        {
          const float alpha2 = pipeline_step<S, true, true>(w, s_a, s_b, p_b, p_a, k_slot(u + 1), v_slot(u - 1));
          prof_mark(3);
          w.rescale_if_needed(alpha2);
          mask_if_padded(s_b, u + 1);
        }
        ++u;
      }
      // last step, even state, u = U-1 >= 1
      before_step(u);
      const float alpha3 = pipeline_step<S, true, false>(w, s_a, s_b, p_b, p_a, 0, v_slot(u - 1));
      w.rescale_if_needed(alpha3);
    }
    // drain: O += V(U-1)^T P(U-1)^T
    WAIT_VMCNT0();
    BARRIER();
    w.pv_all(p_a, v_slot(U - 1));
  }

#ifdef CA_PROFILE
  prof_mark(5);
  if (threadIdx.x == 0 && blockIdx.x < 65536) {
    for (int i = 0; i < 6; ++i) g_profile[blockIdx.x * 8 + i] = prof[i];
    g_profile[blockIdx.x * 8 + 6] = (unsigned long long)n;
  }
#endif
  // ---- epilogue: O = O^T / l, padding queries and empty rows give zeros ------------------------
  const float l_tot = sum_with_partner(w.l_run);
  // slots 32*wave .. +31 of the query tile are this wave's queries
  const uint32_t q_valid = class_mask[CONST_PTR(int32_t, a.tile_class)[q_tile] * 4 + wave];
  const bool q_real = (q_valid >> w.qi) & 1u;
  const float inv = (q_real && l_tot > 0.f) ? 1.0f / l_tot : 0.f;
  char* Op = static_cast<char*>(a.out) + plane + q_row * S::kRowBytes;
#pragma unroll
  for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(w.acc_o[db][4 * r4 + e] * inv);
      const int d0 = db * 32 + 8 * r4 + 4 * w.g;
      *reinterpret_cast<bf16x4*>(Op + d0 * 2) = o4;
    }
}

template <int B, int D>
hipError_t launch(const AttnArgs& a, hipStream_t stream) {
  using S = Shape<B, D>;
  static hipError_t attr = hipFuncSetAttribute(reinterpret_cast<const void*>(&attn_bf16_kernel<B, D>),
                                               hipFuncAttributeMaxDynamicSharedMemorySize, S::kLdsBytes);
  if (attr != hipSuccess) return attr;
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  hipLaunchKernelGGL((attn_bf16_kernel<B, D>), dim3((unsigned)items), dim3(B * 2), S::kLdsBytes, stream, a);
  return hipGetLastError();
}

}  // namespace

#ifdef CA_PROFILE
extern "C" int compact_attn_debug_read_profile(unsigned long long* host, size_t count) {
  return (int)hipMemcpyFromSymbol(host, HIP_SYMBOL(g_profile), count * sizeof(unsigned long long));
}
#endif

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  if (items == 0) return hipSuccess;
  if (items > 0x7fffffff) return hipErrorInvalidValue;
  if (a.B == 128 && a.D == 128) return launch<128, 128>(a, stream);
  if (a.B == 128 && a.D == 64) return launch<128, 64>(a, stream);
  if (a.B == 64 && a.D == 128) return launch<64, 128>(a, stream);
  if (a.B == 64 && a.D == 64) return launch<64, 64>(a, stream);
  return hipErrorInvalidValue;
}

}  // namespace ca
