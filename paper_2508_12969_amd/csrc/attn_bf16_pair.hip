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
// steps ahead of their use, so that the scalar loads never stand between two steps.  The tile step
// itself is QueryWave in attn_bf16_common.h, shared with attn_bf16.hip.
#include "attn_bf16_common.h"

namespace ca {
namespace {

using PairShape = Shape<64, 128, 4>;  // four waves: two per query tile, all four share the tile copies

// kNat: q, k, v, out in natural token order, gathered and scattered here (see attn_bf16.hip)
template <bool kNat>
__global__ __attribute__((amdgpu_flat_work_group_size(256, 256), amdgpu_waves_per_eu(2, 2)))
void attn_bf16_pair_kernel(AttnArgs a) {
  using S = PairShape;
  __shared__ __attribute__((aligned(1024))) char lds_k[S::kTileBytes];
  __shared__ __attribute__((aligned(1024))) char lds_v[S::kTileBytes];

  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int member = wave >> 1;  // which query tile of the pair this wave works for
  const int block = wave & 1;    // which 32 queries of that tile

  const int64_t pairs = a.num_pairs;
  __shared__ int pool_ticket;
  const int64_t linear = launch_entry(a, &pool_ticket);
  if (linear < 0) return;  // a surplus pool workgroup (all of its threads)
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
  const TileSource<S, kNat> src(a, wave, lane);

  // the pair's walk: one word per tile of the union of the two rows, ascending tile ids:
  // tile id | padding class << 24 | bit 30: kept by the first query tile | bit 31: by the second
  const int64_t begin = a.pair_walk_ptr ? a.pair_walk_ptr[item] : 0;
  const int count = (int)(a.pair_walk_ptr ? a.pair_walk_ptr[item + 1] - begin : a.n);
  const auto walk = CONST_PTR(int32_t, a.pair_walk + begin);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class

  QueryWave<S> w(lane, a.scale);
  const QuerySlot qs = query_slot<S::B>(a, q_tile, block * 32, w.qi);
  // a wave without a query tile (odd tile count) or without real queries only moves tiles
  const bool wave_active = qs.wave_active && (member == 0 || has_b);
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

    // ---- S^T = K Q^T ----------------------------------------------------------------------
    WAIT_VMCNT(S::kLoadsPerThread);  // K landed (V may still be in flight)
    BARRIER();
    floatx16 acc_s[S::kKeyBlocks];
    if (mine) w.qk_tile(k_tile, acc_s, true);
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading K
    if (more) src.issue(k_loader, Kp, next_tile, next_origin, lds_k_addr);

    bf16x8 pf[S::kKeyBlocks][2];
    if (mine) {
      w.mask_padding_keys(acc_s, cls, class_mask);
      w.softmax(acc_s, !seen, pf);
      seen = true;
    }

    // ---- O^T += V^T P^T ------------------------------------------------------------------------
    if (more) WAIT_VMCNT(S::kLoadsPerThread);  // V landed (the next K may be in flight)
    else WAIT_VMCNT(0);
    BARRIER();
    if (mine) w.pv_tile(v_tile, pf, true);
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading V
    if (more) src.issue(v_loader, Vp, next_tile, next_origin, lds_v_addr);
    word = word1;
    word1 = word2;
  }

  if (member && !has_b) return;
  w.store(static_cast<char*>(a.out) + plane + q_row * S::kRowBytes, qs.real, !kNat || qs.real);
}

}  // namespace

hipError_t launch_attn_bf16_pair(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.num_pairs;
  if (items == 0) return hipSuccess;
  if (a.B != 64 || a.D != 128 || !a.pair_rows) return hipErrorInvalidValue;
  if (a.static_items + a.pool_wgs > 0x7fffffff || a.static_items + a.pool_items != items) return hipErrorInvalidValue;
  const int64_t grid = a.static_items + a.pool_wgs;
  if (a.natural) {
    if (a.tw % PairShape::kRowsPerLoad != 0) return hipErrorInvalidValue;  // a KiB block must stay inside one run
    hipLaunchKernelGGL(attn_bf16_pair_kernel<true>, dim3((unsigned)grid), dim3(256), 0, stream, a);
  } else {
    hipLaunchKernelGGL(attn_bf16_pair_kernel<false>, dim3((unsigned)grid), dim3(256), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace ca
