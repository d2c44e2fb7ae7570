// Launch interfaces of the device kernels.  Each launcher validates nothing: api.cpp has
// already checked shapes, alignment and support before it calls them.
#pragma once

#include <hip/hip_runtime.h>

#include <cstdint>

#include "layout.h"

namespace ca {

struct PermuteArgs {
  const void* src;
  void* dst;
  int32_t T, H, W, tt, th, tw, nH, nW;
  int64_t n_vid, B, N_real, N_pad, N_video;
  int64_t planes;     // batch * num_heads
  int32_t row_bytes;  // head_dim * sizeof(element), a multiple of 16
  int32_t inverse;
};
hipError_t launch_permute(const PermuteArgs& a, hipStream_t stream);

struct AttnArgs {
  const void* q;
  const void* k;
  const void* v;
  void* out;
  const int64_t* row_ptr;      // device; null selects the dense walk: every row uses col_meta[0..n)
  const int32_t* col_meta;     // device; per kept tile: tile id | padding class << 24; readable two words past the end
  const int32_t* order;        // device [entries]; the launch order: row ids; null = identity
  int64_t entries;             // launch-order entries per batch entry (num_heads * n rows, or fewer entries when query tiles are packed)
  int32_t packed;              // 1: `order` also holds workgroups of two packed query tiles, as the complement of their index in the pair tables
  const int32_t* pair_rows;    // device [2*num_pairs]; row ids of the two query tiles of a workgroup (-1: none), paired kernel only
  int64_t num_pairs;
  const int32_t* pair_desc;    // device [num_pairs]; wave assignment of every workgroup of the paired kernel (layout.h)
  uint64_t upper_empty_classes; // bit c: tiles of padding class c hold no token in the upper half of their slots (paired kernel, 128-token tiles)
  const int64_t* pair_walk_ptr; // device [num_pairs + 1]; null selects the dense walk: every pair uses pair_walk[0..n)
  const int32_t* pair_walk;     // device; per walked tile: tile id | padding class << 24 | kPairInFirst | kPairInSecond,
                                // readable two words past the last entry
  const int32_t* tile_class;   // device [n]
  const SlotMask* class_mask;  // device
  const uint8_t* class_perm;   // device [num_classes * 128]; per class: valid slots ascending, then padding slots ascending
  int32_t batch, num_heads;
  int64_t n;                   // tiles
  int32_t B, D;
  float scale;
  // natural-order variant (bf16 kernels): q, k, v, out are [batch, heads, N_real, D] and the kernel gathers / scatters
  int32_t natural;
  const int32_t* tile_origin;  // device [n]; natural-order row of slot 0 of every tile
  int32_t H, W, th, tw;
  int64_t n_vid, N_real;
  // bf16 kernels: workgroup ids below static_items map to launch-order entries through the XCD-aware
  // order; the pool_wgs workgroups after them draw a ticket from *pool_counter and take entry
  // static_items + ticket while that is below static_items + pool_items (the rest have nothing to do)
  int64_t static_items;
  int32_t pool_items, pool_wgs;
  int32_t* pool_counter;       // device; zero before and after every launch
};
// fp32 problems, B <= 128, D in {32, 64, 128}
hipError_t launch_attn_f32(const AttnArgs& a, hipStream_t stream);
// bf16 problems, (B, D) in {64,128} x {64,128}
hipError_t launch_attn_bf16(const AttnArgs& a, hipStream_t stream);
// bf16 problems with D = 128: workgroups that serve two query tiles (B = 64: every pair of neighbours; B = 128: the
// packed tiles of the grid's padded faces)
hipError_t launch_attn_bf16_pair(const AttnArgs& a, hipStream_t stream);

struct MassArgs {
  const void* q;               // [batch, heads, N_pad, D] tile order, bf16
  const void* k;
  float* mass;                 // [batch, heads, n, n]
  float* partial;              // device workspace, partial_rows * n * B * 2 floats: per query and key tile (sum, reference) of the row a workgroup is working on
  int64_t partial_rows;        // blocks of the workspace = most workgroups a launch may have
  int64_t rows_per_launch;     // rows one launch covers (all of them, or a multiple of partial_rows)
  int64_t row_base, row_count; // set by the launcher: the rows of one launch, drawn by ticket
  int32_t* counter;            // device; the ticket counter, zero before and after every launch
  const int32_t* dense_meta;   // device [n + 2]; per key tile: tile id | padding class << 24 | bit 31: upper key blocks empty
  const int32_t* tile_class;   // device [n]
  const SlotMask* class_mask;  // device
  const uint8_t* class_perm;   // device [num_classes * 128]
  int32_t batch, num_heads;
  int64_t n;
  int32_t B, D;
  float scale;
};
// bf16 problems, (B, D) in {64,128} x {64,128}
hipError_t launch_tile_mass(const MassArgs& a, hipStream_t stream);

}  // namespace ca
