// Block-sparse attention forward on bf16 MFMA for gfx950 (Appendix D of the paper: a block loop
// with online softmax that visits only the kept key tiles of each query tile).
//
// Work decomposition.  One workgroup owns one (batch, head, query tile) row of the layout and
// walks that row's kept key tiles.  A wave owns 32 query tokens; the workgroup has B/32 waves.
// Two workgroups share a CU (LDS: one K and one V tile each), and their phases drift apart, so
// that one workgroup's waits (tile copies, barriers) and softmax are covered by the other's
// matrix products.  What a wave does with one key tile (the transposed products, the padding
// mask, the lazy online softmax) is QueryWave in attn_bf16_common.h.
//
// Operand staging.  K and V tiles go from HBM/L2 straight into LDS (global_load_lds, 16 bytes
// per lane, no VGPR staging).  K rows are read back as 16-byte row fragments (A operand of
// S^T).  V stays row-major [key][d] in LDS and is read with a transposing LDS read.  Both tiles are
// stored with an XOR swizzle of the 16-byte chunk index, applied on the global side of the copy (the
// LDS side of global_load_lds is lane-contiguous), so that both read patterns spread over all banks
// (measured: no LDS bank conflicts).
//
// Pipeline.  One K buffer and one V buffer per workgroup: K(j+1) is fetched while the softmax and
// the PV product of tile j run, V(j+1) while the next QK^T runs.
//
// Grids with a padded face (128-token tiles, head dim 128): the launch order then also holds the
// workgroups that serve two packed query tiles (attn_bf16_pair_body.h); an entry below zero is the
// complement of such a workgroup's index, and one launch runs both kinds, longest first.
#include "attn_bf16_pair_body.h"

namespace ca {
namespace {

// kNat: q, k, v and out are in natural token order ([batch, heads, N_real, D]); the gather of the
// tiles and the scatter of the output happen in the copies of this kernel instead of in separate
// permutation passes.
template <int B, int D, bool kNat>
__device__ __forceinline__ void attn_row_body(const AttnArgs& a, int64_t row, int64_t batch, char* lds_k, char* lds_v) {
  using S = Shape<B, D>;
  const int lane = threadIdx.x & 63;
  const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int64_t head = row / a.n, q_tile = row - head * a.n;
  const int64_t plane = (batch * a.num_heads + head) * (kNat ? a.N_real * (int64_t)S::kRowBytes : a.n * (int64_t)S::kTileBytes);
  const char* Kp = static_cast<const char*>(a.k) + plane;
  const char* Vp = static_cast<const char*>(a.v) + plane;
  const auto tile_origin = CONST_PTR(int32_t, a.tile_origin);
  const TileSource<S, kNat> src(a, wave, lane);

  const int64_t begin = a.row_ptr ? a.row_ptr[row] : 0;
  const int count = (int)(a.row_ptr ? a.row_ptr[row + 1] - begin : a.n);
  // one packed word per kept tile: tile id | padding class << 24 (a slice of the packed CSR, or the
  // shared 0..n-1 list of the dense walk)
  const auto meta = CONST_PTR(int32_t, a.col_meta + begin);
  const auto class_mask = CONST_PTR(uint32_t, a.class_mask);  // 4 words per class

  // A wave without a real query (see query_slot) takes part in the tile copies and barriers only.
  QueryWave<S> w(lane, a.scale);
  const QuerySlot qs = query_slot<B>(a, q_tile, wave * 32, w.qi);
  const bool wave_active = qs.wave_active;
  const int64_t q_row = kNat ? src.query_row(a, q_tile, qs.slot) : q_tile * B + qs.slot;
  w.load_q(static_cast<const char*>(a.q) + plane + q_row * S::kRowBytes);

  const TileLoader<S, false> k_loader(wave, lane);
  const TileLoader<S, true> v_loader(wave, lane);
  const uint32_t lds_k_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_k;
  const uint32_t lds_v_addr = (uint32_t)(uintptr_t)(__attribute__((address_space(3))) char*)lds_v;
  const LdsTile k_tile = (LdsTile)lds_k, v_tile = (LdsTile)lds_v;

  // the packed words are fetched two steps ahead of their use (the tables are readable two words
  // past their end), so that no scalar load is waited for between two steps
  int32_t word = 0, word1 = 0;
  if (count > 0) {
    word = meta[0];
    word1 = meta[1];
    const int32_t origin = kNat ? tile_origin[word & 0xffffff] : 0;
    src.issue(k_loader, Kp, word & 0xffffff, origin, lds_k_addr);
    src.issue(v_loader, Vp, word & 0xffffff, origin, lds_v_addr);
  }

  // A wave without real queries only moves tiles: the same copies, waits and barriers as below.
  const int active_count = wave_active ? count : 0;
  for (int j = active_count; j < count; ++j) {
    const int next_tile = (j + 1 < count) ? (meta[j + 1] & 0xffffff) : 0;
    const int32_t next_origin = kNat ? tile_origin[next_tile] : 0;
    WAIT_VMCNT(S::kLoadsPerThread);
    BARRIER();
    BARRIER();
    if (j + 1 < count) src.issue(k_loader, Kp, next_tile, next_origin, lds_k_addr);
    if (j + 1 < count) WAIT_VMCNT(S::kLoadsPerThread);
    else WAIT_VMCNT(0);
    BARRIER();
    BARRIER();
    if (j + 1 < count) src.issue(v_loader, Vp, next_tile, next_origin, lds_v_addr);
  }

  for (int j = 0; j < active_count; ++j) {
    const int32_t word2 = meta[j + 2];
    const int next_tile = word1 & 0xffffff;
    const int32_t next_origin = kNat ? tile_origin[next_tile] : 0;  // requested a phase ahead of the copy that uses it
    const int cls = (word >> 24) & 0x7f;  // padding class of the key tile
    // bit 31: keys B/2 .. B-1 of this tile are padding only, the products of the upper key blocks are skipped
    const bool upper_keys = word >= 0;

    // ---- S^T = K Q^T ----------------------------------------------------------------------
    WAIT_VMCNT(S::kLoadsPerThread);  // K(j) landed (V(j) may still be in flight)
    BARRIER();
    floatx16 acc_s[S::kKeyBlocks];
    w.qk_tile(k_tile, acc_s, upper_keys);
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading K(j)
    if (j + 1 < count) src.issue(k_loader, Kp, next_tile, next_origin, lds_k_addr);

    bf16x8 pf[S::kKeyBlocks][2];
    w.mask_padding_keys(acc_s, cls, class_mask);
    w.softmax(acc_s, j == 0, pf);

    // ---- O^T += V^T P^T ------------------------------------------------------------------------
    if (j + 1 < count) WAIT_VMCNT(S::kLoadsPerThread);  // V(j) landed (K(j+1) may be in flight)
    else WAIT_VMCNT(0);
    BARRIER();
    w.pv_tile(v_tile, pf, upper_keys);
    WAIT_LGKMCNT0();
    BARRIER();  // every wave has finished reading V(j)
    if (j + 1 < count) src.issue(v_loader, Vp, next_tile, next_origin, lds_v_addr);
    word = word1;
    word1 = word2;
  }

  w.store(static_cast<char*>(a.out) + plane + q_row * S::kRowBytes, qs.real, !kNat || qs.real);
}

// kPacked: the launch order may hold workgroups of two packed query tiles (entries below zero)
template <int B, int D, bool kNat, bool kPacked>
__global__ __attribute__((amdgpu_flat_work_group_size(B * 2, B * 2), amdgpu_waves_per_eu(2, 2)))
void attn_bf16_kernel(AttnArgs a) {
  using S = Shape<B, D>;
  __shared__ __attribute__((aligned(1024))) char lds_k[S::kTileBytes];
  __shared__ __attribute__((aligned(1024))) char lds_v[S::kTileBytes];
  __shared__ int pool_ticket;
  const int64_t linear = launch_entry(a, &pool_ticket);
  if (linear < 0) return;  // a surplus pool workgroup (all of its threads)
  const int64_t item = linear % a.entries;
  const int64_t batch = linear / a.entries;
  const int64_t entry = a.order ? a.order[item] : item;
  if constexpr (kPacked) {
    static_assert(B == 128 && D == 128, "packed query tiles exist for 128-token tiles with head dim 128");
    if (entry < 0) {
      attn_pair_body<128, kNat>(a, ~entry, batch, lds_k, lds_v);
      return;
    }
  }
  attn_row_body<B, D, kNat>(a, entry, batch, lds_k, lds_v);
}

template <int B, int D>
hipError_t launch(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = a.static_items + a.pool_wgs;
  if (a.natural) {
    if (a.tw % Shape<B, D>::kRowsPerLoad != 0) return hipErrorInvalidValue;  // a KiB block must stay inside one run
    hipLaunchKernelGGL((attn_bf16_kernel<B, D, true, false>), dim3((unsigned)items), dim3(B * 2), 0, stream, a);
  } else {
    hipLaunchKernelGGL((attn_bf16_kernel<B, D, false, false>), dim3((unsigned)items), dim3(B * 2), 0, stream, a);
  }
  return hipGetLastError();
}

}  // namespace

hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream) {
  const int64_t items = (int64_t)a.batch * a.entries;
  if (items == 0) return hipSuccess;
  if (a.static_items + a.pool_wgs > 0x7fffffff || a.static_items + a.pool_items != items) return hipErrorInvalidValue;
  if (a.B == 128 && a.D == 128) {
    // One instantiation serves grids with and without packed query tiles (without, no entry of the
    // launch order is below zero).  Measured on an unpadded 32 x 48 x 80 grid: 56.9 ms against 57.4 ms
    // for an instantiation without the pair body: the row body happens to come out better in this one.
    if (a.packed && (!a.order || !a.pair_rows || !a.pair_desc)) return hipErrorInvalidValue;
    if (a.natural && a.tw % Shape<128, 128>::kRowsPerLoad != 0) return hipErrorInvalidValue;
    const dim3 grid((unsigned)(a.static_items + a.pool_wgs)), block(256);
    if (a.natural) hipLaunchKernelGGL((attn_bf16_kernel<128, 128, true, true>), grid, block, 0, stream, a);
    else hipLaunchKernelGGL((attn_bf16_kernel<128, 128, false, true>), grid, block, 0, stream, a);
    return hipGetLastError();
  }
  if (a.B == 128 && a.D == 64) return launch<128, 64>(a, stream);
  if (a.B == 64 && a.D == 64) return launch<64, 64>(a, stream);
  return hipErrorInvalidValue;
}

}  // namespace ca
