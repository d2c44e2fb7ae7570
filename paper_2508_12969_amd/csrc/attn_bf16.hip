// Block-sparse attention forward on bf16 MFMA for gfx950 (Appendix D of the paper: a block loop
// with online softmax that visits only the kept key tiles of each query tile).
//
// Work decomposition.  One workgroup owns one (batch, head, query tile) row of the layout and
// walks that row's kept key tiles.  A wave owns 32 query tokens; the workgroup has B/32 waves.
// Two workgroups share a CU (LDS: one K and one V tile each), and their phases drift apart, so
// that one workgroup's waits (tile copies, barriers) and softmax are covered by the other's
// matrix products.
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
// per lane, no VGPR staging).  K rows are read back as 16-byte row fragments (A operand of
// S^T).  V stays row-major [key][d] in LDS and is read with ds_read_b64_tr_b16, which hands each
// lane four consecutive keys of one d column, i.e. the A operand of O^T.  Both tiles are stored
// with an XOR swizzle of the 16-byte chunk index, applied on the global side of the copy (the LDS
// side of global_load_lds is lane-contiguous), so that both read patterns spread over all banks
// (measured: no LDS bank conflicts).
//
// Pipeline.  One K buffer and one V buffer per workgroup: K(j+1) is fetched while the softmax and
// the PV product of tile j run, V(j+1) while the next QK^T runs.
//
// Rescaling.  The reference value m of the exponent only moves when the row maximum exceeds it by
// more than 2^kLazyLog2 (probabilities then stay below that factor, far inside fp32 and bf16
// range); the accumulator rescale O *= alpha is then a rarely taken wave-uniform branch.  The
// result is still the exact softmax: numerator and denominator share the same reference.
#include "attn_bf16_common.h"

namespace ca {
namespace {

// kNat: q, k, v and out are in natural token order ([batch, heads, N_real, D]); the gather of the
// tiles and the scatter of the output happen in the copies of this kernel instead of in separate
// permutation passes.
template <int B, int D, bool kNat>
__global__ __attribute__((amdgpu_flat_work_group_size(B * 2, B * 2), amdgpu_waves_per_eu(2, 2)))
void attn_bf16_kernel(AttnArgs a) {
  using S = Shape<B, D>;
  __shared__ __attribute__((aligned(1024))) char lds_k[S::kTileBytes];
  __shared__ __attribute__((aligned(1024))) char lds_v[S::kTileBytes];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int qi = lane & 31;  // query column owned by this lane inside the wave's 32 queries
  const int g = lane >> 5;   // lane group: which half of every 8-key / 8-d pair this lane holds

  const int64_t rows = (int64_t)a.num_heads * a.n;
  // Workgroup ids are dealt round-robin to the 8 XCDs, each with an L2 of its own.  They are
  // remapped so that the workgroups resident on one XCD at a time are kXcdChunk consecutive entries
  // of the launch order (same head, neighbouring query tiles, equal list lengths) instead of every
  // eighth entry: their key-tile lists overlap, so more of the K/V tile copies hit that L2.
  int64_t linear = blockIdx.x;
  {
    const int64_t span = 8 * (int64_t)kXcdChunk, total = rows * a.batch;
    if (linear < total / span * span) {
      const int64_t xcd = linear & 7, seq = linear >> 3;
      linear = (seq / kXcdChunk) * span + xcd * kXcdChunk + seq % kXcdChunk;
    }
  }
  const int64_t item = linear % rows;
  const int64_t batch = linear / rows;
  const int64_t row = a.order ? a.order[item] : item;
  const int64_t head = row / a.n, q_tile = row - head * a.n;
  const int64_t plane = (batch * a.num_heads + head) * (kNat ? a.N_real * (int64_t)S::kRowBytes : a.n * (int64_t)S::kTileBytes);
  const char* Kp = static_cast<const char*>(a.k) + plane;
  const char* Vp = static_cast<const char*>(a.v) + plane;
  // Natural order: a KiB block of a tile (kRowsPerLoad consecutive slots, inside one run of tw
  // tokens) is contiguous there too, at row tile_origin[tile] + (dt*H + dy)*W + dx of the plane; a
  // text tile is contiguous as a whole.  row_in_tile[i] is that offset for the i-th block this wave copies.
  const auto tile_origin = CONST_PTR(int32_t, a.tile_origin);
  int32_t row_in_tile[kNat ? S::kLoadsPerThread : 1];
  if constexpr (kNat) {
#pragma unroll
    for (int i = 0; i < S::kLoadsPerThread; ++i) {
      const int slot0 = (wave * S::kLoadsPerThread + i) * S::kRowsPerLoad;
      const int dx = slot0 % a.tw, run = slot0 / a.tw, dy = run % a.th, dt = run / a.th;
      row_in_tile[i] = (dt * a.H + dy) * a.W + dx;
    }
  }
  // copy of one tile: tile order = one contiguous block; natural order = one base per KiB block
  auto issue_tile = [&](const auto& loader, const char* base, int tile, int32_t origin, uint32_t lds_addr) {
    if constexpr (!kNat) {
      loader.issue(base + (int64_t)tile * S::kTileBytes, lds_addr, wave);
    } else {
      const bool text = tile >= a.n_vid;
      const char* sb[S::kLoadsPerThread];
      bool inside = true;
#pragma unroll
      for (int i = 0; i < S::kLoadsPerThread; ++i) {
        const int32_t row = origin + (text ? (wave * S::kLoadsPerThread + i) * S::kRowsPerLoad : row_in_tile[i]);
        inside = inside && row + S::kRowsPerLoad <= a.N_real;
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
          const int32_t first = min(row, (int32_t)a.N_real - 1);
          loader.issue_clamped(base + (int64_t)first * S::kRowBytes, (int32_t)a.N_real - 1 - first, i, lds_addr, wave, lane);
        }
      }
    }
  };

  const int64_t begin = a.row_ptr ? a.row_ptr[row] : 0;
  const int count = (int)(a.row_ptr ? a.row_ptr[row + 1] - begin : a.n);
  // one packed word per kept tile: tile id | padding class << 24 (a slice of the packed CSR, or the
  // shared 0..n-1 list of the dense walk)
  const auto meta = CONST_PTR(int32_t, a.col_meta + begin);
  const auto tile_class = CONST_PTR(int32_t, a.tile_class);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class

  const float c2 = a.scale * kLog2e;
  // A wave whose 32 query slots are all padding (the far half of a tile on a padded grid face)
  // takes part in the tile copies and barriers only.
  const uint32_t q_valid = class_mask[tile_class[q_tile] * 4 + wave];  // slots 32*wave .. +31 are this wave's queries
  const bool wave_active = q_valid != 0;

  // Q fragment: B operand of S^T, lane (qi, g) holds d = 16*step + 8*g .. +7 of its query.
  int64_t q_row = q_tile * B + wave * 32 + qi;
  if constexpr (kNat) {
    const int slot = wave * 32 + qi;
    const int dx = slot % a.tw, run = slot / a.tw, dy = run % a.th, dt = run / a.th;
    const int64_t row = tile_origin[q_tile] + (q_tile >= a.n_vid ? slot : (dt * a.H + dy) * a.W + dx);
    q_row = row < a.N_real ? row : a.N_real - 1;  // a padding slot reads some real row; its result is not stored
  }
  bf16x8 qf[S::kQkSteps];
  {
    const char* Qp = static_cast<const char*>(a.q) + plane + q_row * S::kRowBytes + g * 16;
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(Qp + s * 32);
    // Touch the fragments so that the compiler waits for these loads here, before the loop: inside
    // the loop the vector-memory counter must belong to the tile copies alone.
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) asm volatile("" : "+v"(qf[s]));
  }

  floatx16 acc_o[S::kDBlocks];
#pragma unroll
  for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
  // Exponent reference of this lane's query (raw score units): the first tile's row maximum,
  // afterwards a lagging running maximum.  neg_m holds -m_run in all 16 registers and is the C operand of the
  // first contraction step, so the score accumulator comes out as (score - reference).
  float m_run = 0.f;
  floatx16 neg_m;
#pragma unroll
  for (int r = 0; r < 16; ++r) neg_m[r] = 0.f;
  float l_run = 0.f;              // this lane's share of the running sum (partner lane holds the rest)

  // Per-lane LDS read offsets.
  // K: row (32*kb + qi), logical chunk 2*step + g.
  const int k_lane_row_off = qi * S::kRowBytes;
  const int k_lane_swz = k_swizzle<D>(qi);  // 32*kb does not change the swizzle
  // V: transposing read; lane covers key row 4*g + (lane%16)/4 (+ 32*kb + 16*t + 8*half) and the
  // 8-byte half-chunk that holds d = 32*db + 16*((lane/16)%2) + 4*(lane%4) .. +3.
  const int v_lane_row = 4 * g + ((lane & 15) >> 2);
  const int v_lane_swz = v_swizzle<D>(v_lane_row);  // multiples of 8 rows keep it (D=128); see below for D=64
  const int v_lane_chunk = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
  const int v_lane_half = (lane & 1) * 8;

  const TileLoader<S, false> k_loader(wave, lane);
  const TileLoader<S, true> v_loader(wave, lane);
  const uint32_t lds_k_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_k;
  const uint32_t lds_v_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_v;

  const float lazy_raw = kLazyLog2 / c2;  // kLazyLog2 in raw score units
  // the packed words are fetched two steps ahead of their use (the tables are readable two words
  // past their end), so that no scalar load is waited for between two steps
  int32_t word = 0, word1 = 0;
  if (count > 0) {
    word = meta[0];
    word1 = meta[1];
    const int32_t origin = kNat ? tile_origin[word & 0xffffff] : 0;
    issue_tile(k_loader, Kp, word & 0xffffff, origin, lds_k_addr);
    issue_tile(v_loader, Vp, word & 0xffffff, origin, lds_v_addr);
  }

  // A wave without real queries only moves tiles: the same copies, waits and barriers as below.
  const int active_count = wave_active ? count : 0;
  for (int j = active_count; j < count; ++j) {
    const int next_tile = (j + 1 < count) ? (meta[j + 1] & 0xffffff) : 0;
    const int32_t next_origin = kNat ? tile_origin[next_tile] : 0;
    WAIT_VMCNT(S::kLoadsPerThread);
    BARRIER();
    BARRIER();
    if (j + 1 < count) issue_tile(k_loader, Kp, next_tile, next_origin, lds_k_addr);
    if (j + 1 < count) WAIT_VMCNT(S::kLoadsPerThread);
    else WAIT_VMCNT(0);
    BARRIER();
    BARRIER();
    if (j + 1 < count) issue_tile(v_loader, Vp, next_tile, next_origin, lds_v_addr);
  }

  for (int j = 0; j < active_count; ++j) {
    const int32_t word2 = meta[j + 2];
    const int next_tile = word1 & 0xffffff;
    const int32_t next_origin = kNat ? tile_origin[next_tile] : 0;  // requested a phase ahead of the copy that uses it
    const int cls = (word >> 24) & 0x7f;
    // keys B/2 .. B-1 of this tile are padding only: the products of the upper key blocks are skipped
    const bool upper_keys = word >= 0;

    // ---- S^T = K Q^T ----------------------------------------------------------------------
    WAIT_VMCNT(S::kLoadsPerThread);  // K(j) landed (V(j) may still be in flight)
    BARRIER();
    floatx16 acc_s[S::kKeyBlocks];
    constexpr int kLowerBlocks = S::kKeyBlocks / 2;
    {
#pragma unroll
      for (int s = 0; s < S::kQkSteps; ++s) {
#pragma unroll
        for (int kb = 0; kb < kLowerBlocks; ++kb) {
          const int off = kb * 32 * S::kRowBytes + k_lane_row_off + (((2 * s + g) ^ k_lane_swz) << 4);
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(lds_k + off);
          acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? neg_m : acc_s[kb], 0, 0, 0);
        }
      }
      if (upper_keys) {
#pragma unroll
        for (int s = 0; s < S::kQkSteps; ++s) {
#pragma unroll
          for (int kb = kLowerBlocks; kb < S::kKeyBlocks; ++kb) {
            const int off = kb * 32 * S::kRowBytes + k_lane_row_off + (((2 * s + g) ^ k_lane_swz) << 4);
            const bf16x8 kf = *reinterpret_cast<const bf16x8*>(lds_k + off);
            acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? neg_m : acc_s[kb], 0, 0, 0);
          }
        }
      } else {
#pragma unroll
        for (int kb = kLowerBlocks; kb < S::kKeyBlocks; ++kb)
#pragma unroll
          for (int r = 0; r < 16; ++r) acc_s[kb][r] = kMinusInf;
      }
    }
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading K(j)
    if (j + 1 < count) issue_tile(k_loader, Kp, next_tile, next_origin, lds_k_addr);

    bf16x8 pf[S::kKeyBlocks][2];
    {
      // ---- padding keys never take part ---------------------------------------------------------
      // Only tiles on a padded face of the grid have invalid slots (wave-uniform test).  The valid
      // bits of a 32-key block are one scalar word; the select mask of each score register is built
      // on the scalar unit (lanes 0-31 hold key 8*(r/4) + r%4 of the block, lanes 32-63 that key + 4)
      // and applied with one v_cndmask per register.
      if (cls != 0) {
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

      // ---- online softmax (one query per lane) ---------------------------------------------------
      // acc_s holds score - reference in raw units.  The reference is set to the row maximum on the
      // first tile and afterwards moves only for rows whose maximum exceeds it by more than
      // 2^kLazyLog2; that is a wave-uniform, rarely taken branch, and the common path is exp2 alone.
      float mx = acc_s[0][0];
#pragma unroll
      for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[kb][r]);
      mx = max_with_partner(mx);
      {
        const uint64_t over = __builtin_amdgcn_ballot_w64(mx > lazy_raw);
        if (j == 0 || __builtin_amdgcn_readfirstlane((uint32_t)over | (uint32_t)(over >> 32)) != 0) {
          float delta = (j == 0 || mx > lazy_raw) ? mx : 0.f;
          if (delta == kMinusInf) delta = 0.f;  // a row that has seen no real key yet keeps its reference
          const float alpha = j == 0 ? 1.0f : __builtin_amdgcn_exp2f(-delta * c2);
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
      // probabilities, rounded to bf16 (the B operand of the second product); the row sum adds up the
      // rounded values, two per v_dot2, so numerator and denominator see the same numbers
      {
        bf16x2 ones;
        ones[0] = (__bf16)1.0f;
        ones[1] = (__bf16)1.0f;
#pragma unroll
        for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
          for (int t = 0; t < 2; ++t)
          {
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
    }

    // ---- O^T += V^T P^T ------------------------------------------------------------------------
    if (j + 1 < count) WAIT_VMCNT(S::kLoadsPerThread);  // V(j) landed (K(j+1) may be in flight)
    else WAIT_VMCNT(0);
    BARRIER();
    {
#pragma unroll
      for (int kb = 0; kb < kLowerBlocks; ++kb) {
#pragma unroll
        for (int t = 0; t < 2; ++t) {
#pragma unroll
          for (int db = 0; db < S::kDBlocks; ++db) {
            const int chunk = (db * 4 + v_lane_chunk) ^ v_lane_swz;
            const int base = (kb * 32 + t * 16 + v_lane_row) * S::kRowBytes + chunk * 16 + v_lane_half;
            const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (shortx4 __attribute__((address_space(3)))*)LDS_PTR(lds_v + base));
            const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                (shortx4 __attribute__((address_space(3)))*)LDS_PTR(lds_v + base + 8 * S::kRowBytes));
            bf16x8 vf;
            vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][t], acc_o[db], 0, 0, 0);
          }
        }
      }
      if (upper_keys) {
#pragma unroll
        for (int kb = kLowerBlocks; kb < S::kKeyBlocks; ++kb) {
#pragma unroll
          for (int t = 0; t < 2; ++t) {
#pragma unroll
            for (int db = 0; db < S::kDBlocks; ++db) {
              const int chunk = (db * 4 + v_lane_chunk) ^ v_lane_swz;
              const int base = (kb * 32 + t * 16 + v_lane_row) * S::kRowBytes + chunk * 16 + v_lane_half;
              const shortx4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (shortx4 __attribute__((address_space(3)))*)LDS_PTR(lds_v + base));
              const shortx4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16(
                  (shortx4 __attribute__((address_space(3)))*)LDS_PTR(lds_v + base + 8 * S::kRowBytes));
              bf16x8 vf;
              vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
              acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][t], acc_o[db], 0, 0, 0);
            }
          }
        }
      }
    }
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading V(j)
    if (j + 1 < count) issue_tile(v_loader, Vp, next_tile, next_origin, lds_v_addr);
    word = word1;
    word1 = word2;
  }

  // ---- epilogue: O = O^T / l, padding queries and empty rows give zeros ------------------------
  const float l_tot = sum_with_partner(l_run);
  const bool q_real = (q_valid >> qi) & 1u;
  const float inv = (q_real && l_tot > 0.f) ? 1.0f / l_tot : 0.f;
  char* Op = static_cast<char*>(a.out) + plane + q_row * S::kRowBytes;
  if (kNat && !q_real) return;  // natural order has no row for a padding slot
#pragma unroll
  for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
    for (int r4 = 0; r4 < 4; ++r4) {
      bf16x4 o4;
#pragma unroll
      for (int e = 0; e < 4; ++e) o4[e] = (__bf16)(acc_o[db][4 * r4 + e] * inv);
      const int d0 = db * 32 + 8 * r4 + 4 * g;
      *reinterpret_cast<bf16x4*>(Op + d0 * 2) = o4;
    }
}

template <int B, int D>
hipError_t launch(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  if (a.natural) {
    if (a.tw % Shape<B, D>::kRowsPerLoad != 0) return hipErrorInvalidValue;  // a KiB block must stay inside one run
    hipLaunchKernelGGL((attn_bf16_kernel<B, D, true>), dim3((unsigned)items), dim3(B * 2), 0, stream, a);
  } else {
    hipLaunchKernelGGL((attn_bf16_kernel<B, D, false>), dim3((unsigned)items), dim3(B * 2), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_heads * a.n;
  if (items == 0) return hipSuccess;
  if (items > 0x7fffffff) return hipErrorInvalidValue;
  if (a.B == 128 && a.D == 128) return launch<128, 128>(a, stream);
  if (a.B == 128 && a.D == 64) return launch<128, 64>(a, stream);
  if (a.B == 64 && a.D == 128) return launch_attn_bf16_pair(a, stream);  // two query tiles per workgroup
  if (a.B == 64 && a.D == 64) return launch<64, 64>(a, stream);
  return hipErrorInvalidValue;
}

}  // namespace ca
