// Block-sparse attention forward for 64-token tiles, head dim 128, on bf16 MFMA (Appendix D of the
// paper: block loop with online softmax over the kept key tiles), two query tiles per workgroup.
//
// A 64-token tile gives a K/V copy only half the matrix work of a 128-token tile, and the copies
// were what limited the one-tile-per-workgroup kernel at this tile size (a third of its time).
// Here a workgroup owns the two neighbouring query tiles 2p and 2p+1 of one head: waves 0-1 work
// for the first, waves 2-3 for the second, and both share one K and one V buffer.  The kept lists
// of neighbours overlap almost completely (shifted windows, shared arms of a cross, every tile of
// a global head), so the workgroup walks the union of the two lists, merged on the host into one
// list of words (tile id, padding class, one membership bit per query tile), and copies each key
// tile once for both.  A wave sits out the products of a tile its own query tile does not keep
// (wave-uniform branch) but takes part in the copies and barriers.  The walk words are fetched two
// steps ahead of their use, so that the scalar loads never stand between two steps.  Everything
// inside a tile step is as in attn_bf16.hip.
#include "attn_bf16_common.h"

namespace ca {
namespace {

struct PairShape {  // B = 64, D = 128, four waves
  static constexpr int B = 64, D = 128;
  static constexpr int kThreads = 256;
  static constexpr int kKeyBlocks = 2, kQkSteps = 8, kDBlocks = 4;
  static constexpr int kRowBytes = 256, kChunksPerRow = 16;
  static constexpr int kTileBytes = 64 * 256;
  static constexpr int kLoadsPerThread = kTileBytes / (kThreads * 16);  // 4
  static constexpr int kRowsPerLoad = 4;
};

// kNat: q, k, v, out in natural token order, gathered and scattered here (see attn_bf16.hip)
template <bool kNat>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void attn_bf16_pair_kernel(AttnArgs a) {
  using S = PairShape;
  constexpr int D = S::D;
  __shared__ __attribute__((aligned(1024))) char lds_k[S::kTileBytes];
  __shared__ __attribute__((aligned(1024))) char lds_v[S::kTileBytes];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int member = wave >> 1;  // which query tile of the pair this wave works for
  const int block = wave & 1;    // which 32 queries of that tile
  const int qi = lane & 31;      // query column owned by this lane inside the wave's 32 queries
  const int g = lane >> 5;       // lane group: which half of every 8-key / 8-d pair this lane holds

  const int64_t pairs = a.num_pairs;
  // XCD-aware launch order as in attn_bf16.hip; an XCD holds 64 of these workgroups at a time
  constexpr int kChunk = 64;
  int64_t linear = blockIdx.x;
  {
    const int64_t span = 8 * (int64_t)kChunk, total = pairs * a.batch;
    if (linear < total / span * span) {
      const int64_t xcd = linear & 7, seq = linear >> 3;
      linear = (seq / kChunk) * span + xcd * kChunk + seq % kChunk;
    }
  }
  const int64_t item = linear % pairs;
  const int64_t batch = linear / pairs;
  const auto pair_rows = CONST_PTR(int32_t, a.pair_rows);
  const int64_t row_a = pair_rows[2 * item], row_b = pair_rows[2 * item + 1];
  const bool has_b = row_b >= 0;
  const int64_t head = row_a / a.n;
  const int64_t tile_a = row_a - head * a.n, tile_b = has_b ? row_b - head * a.n : tile_a;
  const int64_t q_tile = member ? tile_b : tile_a;
  const int64_t plane = (batch * a.num_heads + head) * (kNat ? a.N_real * (int64_t)S::kRowBytes : a.n * (int64_t)S::kTileBytes);
  const char* Kp = static_cast<const char*>(a.k) + plane;
  const char* Vp = static_cast<const char*>(a.v) + plane;
  const auto tile_origin = CONST_PTR(int32_t, a.tile_origin);
  int32_t row_in_tile[kNat ? S::kLoadsPerThread : 1];  // natural order: row offset of each KiB block this wave copies
  if constexpr (kNat) {
#pragma unroll
    for (int i = 0; i < S::kLoadsPerThread; ++i) {
      const int slot0 = (wave * S::kLoadsPerThread + i) * S::kRowsPerLoad;
      const int dx = slot0 % a.tw, run = slot0 / a.tw, dy = run % a.th, dt = run / a.th;
      row_in_tile[i] = (dt * a.H + dy) * a.W + dx;
    }
  }
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
#pragma unroll
        for (int i = 0; i < S::kLoadsPerThread; ++i) {
          const int32_t row = origin + (text ? (wave * S::kLoadsPerThread + i) * S::kRowsPerLoad : row_in_tile[i]);
          const int32_t first = min(row, (int32_t)a.N_real - 1);
          loader.issue_clamped(base + (int64_t)first * S::kRowBytes, (int32_t)a.N_real - 1 - first, i, lds_addr, wave, lane);
        }
      }
    }
  };

  // the pair's walk: one word per tile of the union of the two rows, ascending tile ids:
  // tile id | padding class << 24 | bit 30: kept by the first query tile | bit 31: by the second
  const int64_t begin = a.pair_walk_ptr ? a.pair_walk_ptr[item] : 0;
  const int count = (int)(a.pair_walk_ptr ? a.pair_walk_ptr[item + 1] - begin : a.n);
  const auto walk = CONST_PTR(int32_t, a.pair_walk + begin);
  const auto tile_class = CONST_PTR(int32_t, a.tile_class);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class

  const float c2 = a.scale * kLog2e;
  const uint32_t q_valid = class_mask[tile_class[q_tile] * 4 + block];
  // a wave without a query tile (odd tile count) or without real queries only moves tiles
  const bool wave_active = q_valid != 0 && (member == 0 || has_b);

  // Q fragment: B operand of S^T, lane (qi, g) holds d = 16*step + 8*g .. +7 of its query.
  int64_t q_row = q_tile * S::B + block * 32 + qi;
  if constexpr (kNat) {
    const int slot = block * 32 + qi;
    const int dx = slot % a.tw, run = slot / a.tw, dy = run % a.th, dt = run / a.th;
    const int64_t row = tile_origin[q_tile] + (q_tile >= a.n_vid ? slot : (dt * a.H + dy) * a.W + dx);
    q_row = row < a.N_real ? row : a.N_real - 1;
  }
  bf16x8 qf[S::kQkSteps];
  {
    const char* Qp = static_cast<const char*>(a.q) + plane + q_row * S::kRowBytes + g * 16;
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) qf[s] = *reinterpret_cast<const bf16x8*>(Qp + s * 32);
    // wait for these loads here: inside the loop the vector-memory counter belongs to the tile copies
#pragma unroll
    for (int s = 0; s < S::kQkSteps; ++s) asm volatile("" : "+v"(qf[s]));
  }

  floatx16 acc_o[S::kDBlocks];
#pragma unroll
  for (int db = 0; db < S::kDBlocks; ++db)
#pragma unroll
    for (int r = 0; r < 16; ++r) acc_o[db][r] = 0.f;
  // exponent reference (raw units) and -reference as the C operand of the first contraction step
  float m_run = 0.f, l_run = 0.f;
  floatx16 neg_m;
#pragma unroll
  for (int r = 0; r < 16; ++r) neg_m[r] = 0.f;
  bool seen = false;  // this wave has processed a tile of its own list (wave-uniform)

  const int k_lane_row_off = qi * S::kRowBytes;
  const int k_lane_swz = k_swizzle<D>(qi);
  const int v_lane_row = 4 * g + ((lane & 15) >> 2);
  const int v_lane_swz = v_swizzle<D>(v_lane_row);
  const int v_lane_chunk = ((lane >> 4) & 1) * 2 + ((lane & 3) >> 1);
  const int v_lane_half = (lane & 1) * 8;
  const TileLoader<S, false> k_loader(wave, lane);
  const TileLoader<S, true> v_loader(wave, lane);
  const uint32_t lds_k_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_k;
  const uint32_t lds_v_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_v;
  const float lazy_raw = kLazyLog2 / c2;

  // ---- the walk, with its words two steps ahead (the table is readable two words past its end) --
  int32_t word = walk[0], word1 = walk[1];
  if (count > 0) {
    const int32_t origin = kNat ? tile_origin[word & 0xffffff] : 0;
    issue_tile(k_loader, Kp, word & 0xffffff, origin, lds_k_addr);
    issue_tile(v_loader, Vp, word & 0xffffff, origin, lds_v_addr);
  }

  for (int j = 0; j < count; ++j) {
    const int32_t word2 = walk[j + 2];
    const int next_tile = word1 & 0xffffff;
    const int32_t next_origin = kNat ? tile_origin[next_tile] : 0;
    const bool more = j + 1 < count;
    const bool mine = wave_active && ((word >> (30 + member)) & 1);
    const int cls = (word >> 24) & 0x3f;

    // ---- S^T = K Q^T ----------------------------------------------------------------------
    WAIT_VMCNT(S::kLoadsPerThread);  // K landed (V may still be in flight)
    BARRIER();
    floatx16 acc_s[S::kKeyBlocks];
    if (mine) {
#pragma unroll
      for (int s = 0; s < S::kQkSteps; ++s) {
#pragma unroll
        for (int kb = 0; kb < S::kKeyBlocks; ++kb) {
          const int off = kb * 32 * S::kRowBytes + k_lane_row_off + (((2 * s + g) ^ k_lane_swz) << 4);
          const bf16x8 kf = *reinterpret_cast<const bf16x8*>(lds_k + off);
          acc_s[kb] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(kf, qf[s], s == 0 ? neg_m : acc_s[kb], 0, 0, 0);
        }
      }
    }
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading K
    if (more) issue_tile(k_loader, Kp, next_tile, next_origin, lds_k_addr);

    bf16x8 pf[S::kKeyBlocks][2];
    if (mine) {
      // ---- padding keys never take part (see attn_bf16.hip) ----
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
      // ---- online softmax with a lazy exponent reference (see attn_bf16.hip) ----
      float mx = acc_s[0][0];
#pragma unroll
      for (int kb = 0; kb < S::kKeyBlocks; ++kb)
#pragma unroll
        for (int r = 0; r < 16; ++r) mx = fmaxf(mx, acc_s[kb][r]);
      mx = max_with_partner(mx);
      const uint64_t over = __builtin_amdgcn_ballot_w64(mx > lazy_raw);
      if (!seen || __builtin_amdgcn_readfirstlane((uint32_t)over | (uint32_t)(over >> 32)) != 0) {
        float delta = (!seen || mx > lazy_raw) ? mx : 0.f;
        if (delta == kMinusInf) delta = 0.f;
        const float alpha = !seen ? 1.0f : __builtin_amdgcn_exp2f(-delta * c2);
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
      seen = true;
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

    // ---- O^T += V^T P^T ------------------------------------------------------------------------
    if (more) WAIT_VMCNT(S::kLoadsPerThread);  // V landed (the next K may be in flight)
    else WAIT_VMCNT(0);
    BARRIER();
    if (mine) {
#pragma unroll
      for (int kb = 0; kb < S::kKeyBlocks; ++kb) {
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
            const bf16x8 vf = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
            acc_o[db] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(vf, pf[kb][t], acc_o[db], 0, 0, 0);
          }
        }
      }
    }
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading V
    if (more) issue_tile(v_loader, Vp, next_tile, next_origin, lds_v_addr);
    word = word1;
    word1 = word2;
  }

  // ---- epilogue: O = O^T / l, padding queries and empty rows give zeros ------------------------
  if (member && !has_b) return;
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

}  // namespace

hipError_t launch_attn_bf16_pair(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_pairs;
  if (items == 0) return hipSuccess;
  if (items > 0x7fffffff || a.B != 64 || a.D != 128 || !a.pair_rows) return hipErrorInvalidValue;
  if (a.natural) {
    if (a.tw % PairShape::kRowsPerLoad != 0) return hipErrorInvalidValue;  // a KiB block must stay inside one run
    hipLaunchKernelGGL(attn_bf16_pair_kernel<true>, dim3((unsigned)items), dim3(256), 0, stream, a);
  } else {
    hipLaunchKernelGGL(attn_bf16_pair_kernel<false>, dim3((unsigned)items), dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace ca
