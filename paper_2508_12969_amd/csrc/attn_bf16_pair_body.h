// Block-sparse attention forward on bf16 MFMA, head dim 128 (Appendix D of the paper: block loop with
// online softmax over the kept key tiles), two query tiles per workgroup.
//
// 64-token tiles.  A 64-token tile gives a K/V copy only half the matrix work of a 128-token tile,
// and the copies were what limited the one-tile-per-workgroup kernel at this tile size (a third of
// its time).  Here a workgroup owns two neighbouring query tiles of one head: waves 0-1 work for the
// first, waves 2-3 for the second, and both share one K and one V buffer.
// 128-token tiles.  A query tile on a padded face of the grid holds tokens for one to three waves;
// the host packs the waves of such tiles, neighbours along w, four to a workgroup (at most two
// tiles per workgroup), so that no wave idles while the workgroup pays for copies and barriers.
// Which wave works for which tile and from which query slot on is one word per workgroup
// (pair_desc, see layout.h).
//
// The kept lists of neighbours overlap almost completely (shifted windows, shared arms of a cross,
// every tile of a global head), so the workgroup walks the union of the two lists, merged on the
// host into one list of words (tile id, padding class, one membership bit per query tile), and
// copies each key tile once for both.  A wave sits out the products of a tile its own query tile
// does not keep (wave-uniform branch) but takes part in the copies and barriers.  The walk words
// are fetched two steps ahead of their use, so that the scalar loads never stand between two
// steps.  The tile step itself is QueryWave in attn_bf16_common.h, shared with attn_bf16.hip.
#pragma once

#include "attn_bf16_common.h"

namespace ca {
namespace {

template <int B>
using PairShape = Shape<B, 128, 4>;  // four waves that share the tile copies

// The work of one workgroup: entry `item` of the pair tables, batch entry `batch`; lds_k, lds_v: one
// tile each.  kNat: q, k, v, out in natural token order, gathered and scattered here (see attn_bf16.hip).
template <int B, bool kNat>
__device__ __forceinline__ void attn_pair_body(const AttnArgs& a, int64_t item, int64_t batch, char* lds_k, char* lds_v) {
  using S = PairShape<B>;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const auto pair_rows = CONST_PTR(int32_t, a.pair_rows);
  const int64_t row_a = pair_rows[2 * item], row_b = pair_rows[2 * item + 1];
  const bool has_b = row_b >= 0;
  // this wave's share of the workgroup: which of the two query tiles, from which query slot on, or none
  const uint32_t desc = (uint32_t)CONST_PTR(int32_t, a.pair_desc)[item];
  const int member = (desc >> wave) & 1u;
  const bool wave_used = (desc >> (4 + wave)) & 1u;
  const int first_slot = (int)((desc >> (8 + 4 * wave)) & 0xFu) * 32;
  const int64_t head = row_a / a.n;
  const int64_t tile_a = row_a - head * a.n, tile_b = has_b ? row_b - head * a.n : tile_a;
  const int64_t q_tile = member ? tile_b : tile_a;
  const int64_t plane = (batch * a.num_heads + head) * (kNat ? a.N_real * (int64_t)S::kRowBytes : a.n * (int64_t)S::kTileBytes);
  const char* Kp = static_cast<const char*>(a.k) + plane;
  const char* Vp = static_cast<const char*>(a.v) + plane;
  const auto tile_origin = CONST_PTR(int32_t, a.tile_origin);
  const TileSource<S, kNat> src(a, wave, lane);

  // the pair's walk: one word per tile of the union of the two rows, ascending tile ids:
  // tile id | padding class << 24 | bit 30: kept by the first query tile | bit 31: by the second
  const int64_t begin = a.pair_walk_ptr ? a.pair_walk_ptr[item] : 0;
  const int count = (int)(a.pair_walk_ptr ? a.pair_walk_ptr[item + 1] - begin : a.n);
  const auto walk = CONST_PTR(int32_t, a.pair_walk + begin);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class

  QueryWave<S> w(lane, a.scale);
  const QuerySlot qs = query_slot<S::B>(a, q_tile, first_slot, w.qi);
  // a wave without a share, without a query tile (odd tile count) or without real queries only moves tiles
  const bool wave_active = wave_used && qs.wave_active && (member == 0 || has_b);
  const int64_t q_row = kNat ? src.query_row(a, q_tile, qs.slot) : q_tile * S::B + qs.slot;
  w.load_q(static_cast<const char*>(a.q) + plane + q_row * S::kRowBytes);
  bool seen = false;  // this wave has processed a tile of its own list (wave-uniform)

  const TileLoader<S, false> k_loader(wave, lane);
  const TileLoader<S, true> v_loader(wave, lane);
  const uint32_t lds_k_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_k;
  const uint32_t lds_v_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_v;
  const LdsTile k_tile = (LdsTile)lds_k, v_tile = (LdsTile)lds_v;

  // ---- the walk, with its words two steps ahead (the table is readable two words past its end) --
  int32_t word = walk[0], word1 = walk[1];
  if (count > 0) {
    const int32_t origin = kNat ? tile_origin[word & 0xffffff] : 0;
    src.issue(k_loader, Kp, word & 0xffffff, origin, lds_k_addr);
    src.issue(v_loader, Vp, word & 0xffffff, origin, lds_v_addr);
  }

  for (int j = 0; j < count; ++j) {
    const int32_t word2 = walk[j + 2];
    const int next_tile = word1 & 0xffffff;
    const int32_t next_origin = kNat ? tile_origin[next_tile] : 0;
    const bool more = j + 1 < count;
    const bool mine = wave_active && ((word >> (30 + member)) & 1);
    const int cls = (word >> 24) & 0x3f;  // padding class of the key tile

    if (!mine) {
      // not this wave's tile: the same waits, barriers and copies as below, none of the arithmetic
      WAIT_VMCNT(S::kLoadsPerThread);
      BARRIER();
      BARRIER();
      if (more) src.issue(k_loader, Kp, next_tile, next_origin, lds_k_addr);
      if (more) WAIT_VMCNT(S::kLoadsPerThread);
      else WAIT_VMCNT(0);
      BARRIER();
      BARRIER();
      if (more) src.issue(v_loader, Vp, next_tile, next_origin, lds_v_addr);
    } else {
      // 128-token key tiles whose upper half holds no token (a padded face along t) cost half the products
      const bool upper_keys = S::B < 128 || !((a.upper_empty_classes >> cls) & 1u);
      // ---- S^T = K Q^T ----------------------------------------------------------------------
      WAIT_VMCNT(S::kLoadsPerThread);  // K landed (V may still be in flight)
      BARRIER();
      floatx16 acc_s[S::kKeyBlocks];
      w.qk_tile(k_tile, acc_s, upper_keys);
      WAIT_LGKMCNT0();
      BARRIER();  // every wave has finished reading K
      if (more) src.issue(k_loader, Kp, next_tile, next_origin, lds_k_addr);

      bf16x8 pf[S::kKeyBlocks][2];
      w.mask_padding_keys(acc_s, cls, class_mask);
      w.softmax(acc_s, !seen, pf);
      seen = true;

      // ---- O^T += V^T P^T ------------------------------------------------------------------------
      if (more) WAIT_VMCNT(S::kLoadsPerThread);  // V landed (the next K may be in flight)
      else WAIT_VMCNT(0);
      BARRIER();
      w.pv_tile(v_tile, pf, upper_keys);
      WAIT_LGKMCNT0();
      BARRIER();  // every wave has finished reading V
      if (more) src.issue(v_loader, Vp, next_tile, next_origin, lds_v_addr);
    }
    word = word1;
    word1 = word2;
  }

  if (!wave_used || (member && !has_b)) return;
  w.store(static_cast<char*>(a.out) + plane + q_row * S::kRowBytes, qs.real, !kNat || qs.real);
  if constexpr (!kNat && S::B > 64) {
    // A packed tile has waves only for the slots that hold tokens; the wave with the tile's last
    // tokens also writes the zero rows of the padding slots that no wave owns (tile-order output).
    const int cls_q = CONST_PTR(int32_t, a.tile_class)[q_tile];
    const auto mask = CONST_PTR(uint32_t, a.class_mask) + cls_q * 4;
    const int valid = __builtin_popcount(mask[0]) + __builtin_popcount(mask[1]) + __builtin_popcount(mask[2]) + __builtin_popcount(mask[3]);
    const int owned = (valid + 31) / 32 * 32;
    if (first_slot + 32 == owned && w.g == 0) {
      char* tile_out = static_cast<char*>(a.out) + plane + q_tile * (int64_t)S::kTileBytes;
      for (int s = owned + w.qi; s < S::B; s += 32) {
        uint4* row = reinterpret_cast<uint4*>(tile_out + (int64_t)a.class_perm[cls_q * 128 + s] * S::kRowBytes);
#pragma unroll
        for (int c = 0; c < S::kRowBytes / 16; ++c) row[c] = uint4{0, 0, 0, 0};
      }
    }
  }
}

}  // namespace
}  // namespace ca
