// Internal representation of a built layout.  Host tables are filled by layout.cpp (no HIP
// calls); device copies are created by api.cpp and consumed by the kernels.
#pragma once

#include <atomic>
#include <cstdint>
#include <mutex>
#include <vector>

#include "compact_attn.h"

namespace ca {

// Membership bits of a walk word of the paired kernel (bits 30 and 31; the tile id is below bit 24).
constexpr uint32_t kPairInFirst = 1u << 30, kPairInSecond = 1u << 31;

// How the four waves of a workgroup of the paired kernel are assigned (one word per workgroup):
// bit w: wave w works for the second query tile of the pair (else the first); bit 4 + w: wave w has
// queries at all; bits 8 + 4w .. 11 + 4w: the wave's first query slot / 32, counted in the tile's
// token-holding-slots-first order.  The plain pair of two 64-token tiles is kPairPlain: waves 0-1 hold
// slots 0-63 of the first tile, waves 2-3 those of the second.
constexpr uint32_t kPairPlain = 0xCu | 0xF0u | (0x1010u << 8);
constexpr uint32_t pair_desc_wave(int wave, int second, int first_slot32) {
  return ((uint32_t)second << wave) | (1u << (4 + wave)) | ((uint32_t)first_slot32 << (8 + 4 * wave));
}

// Validity of the B token slots of a tile, one bit per slot (B <= 128).
struct SlotMask {
  uint32_t w[4];
};

// How the entries of a launch order (rows or pairs of one batch entry, sorted by descending length)
// are handed out: the first static_entries by workgroup id, the remaining pool_entries by ticket.
struct LaunchSplit {
  int64_t static_entries = 0;
  int32_t pool_entries = 0;
};
constexpr int kPoolSlots = 64;          // pool counters per layout
constexpr int64_t kPoolMinItems = 4096; // smaller launches are dealt statically as a whole
// `work[i]`: cost of launch-order entry i (tile steps); returns the split of one batch entry's launch.
LaunchSplit split_launch(const int64_t* work, int64_t entries);

// Device-resident tables.  All pointers are device memory owned by the layout.
struct DeviceTables {
  int64_t* row_ptr = nullptr;    // [num_heads*n + 1] offsets into col_idx (global over heads)
  int32_t* col_meta = nullptr;   // [nnz] kept key tiles, ascending inside each row: tile id | class << 24
  int32_t* dense_meta = nullptr; // [n] the same packing for the list 0..n-1 (dense walk)
  int32_t* order = nullptr;      // [num_heads*n] launch order of row ids head*n + tile
  int32_t* launch_rows = nullptr; // [num_launch_rows] launch order when query tiles are packed (row ids, and ~i for packed workgroup i); else null: `order`
  int64_t num_launch_rows = 0;
  int32_t* pair_desc = nullptr;  // [num_pairs] wave assignment of every workgroup of the paired kernel
  int32_t* pair_rows = nullptr;  // [2*num_pairs] row ids of the two query tiles a workgroup of the paired kernel owns (-1: none), in launch order
  int64_t num_pairs = 0;
  int64_t* pair_walk_ptr = nullptr;   // [num_pairs + 1]
  int32_t* pair_walk = nullptr;       // packed walk words (tile id | class << 24 | membership bits), two words of padding
  int32_t* dense_pair_walk = nullptr; // [n + 2] the walk 0..n-1 kept by both tiles (dense path)
  int32_t* tile_class = nullptr; // [n] index into class_mask; 0 = every slot holds a token
  SlotMask* class_mask = nullptr; // [num_classes]
  uint8_t* class_perm = nullptr;  // [num_classes * 128] per class: its valid slots ascending, then its padding slots ascending
  int32_t* tile_origin = nullptr; // [n] natural-order row of slot 0 of every tile
  int32_t* pool_counters = nullptr; // [pool_slots] tickets of the dynamically drawn tail of a launch; zero between launches
  int32_t pool_slots = 0;           // concurrent launches on one layout take different counters, round-robin
  float* mass_partial = nullptr;  // workspace of the tile-mass kernel, mass_partial_rows (= workgroups of its launch) * n * B * 2 floats; allocated at its first call
  int64_t mass_partial_rows = 0;
  int32_t* mass_counter = nullptr; // its ticket counter (inside the same allocation)
};

}  // namespace ca

struct ca_layout {
  ca_problem prob{};
  int32_t nT = 0, nH = 0, nW = 0;
  int64_t B = 0, n_vid = 0, n_txt = 0, n = 0, N_real = 0, N_pad = 0;
  float scale = 0.f;

  // host tables
  std::vector<int64_t> row_ptr;             // [num_heads*n + 1], global offsets
  std::vector<int32_t> col_idx;             // [nnz]
  std::vector<std::vector<int64_t>> head_row_ptr;  // per head, relative offsets (C-ABI view)
  std::vector<int32_t> order;               // [num_heads*n]
  std::vector<int32_t> pair_rows;           // [2*num_pairs], empty unless the paired kernel serves (part of) this layout
  std::vector<int32_t> pair_desc;           // [num_pairs] wave assignment (kPairPlain for a plain pair)
  // 128-token tiles, head dim 128: query tiles whose tokens fill fewer than four waves (tiles on a
  // padded face of the grid) are packed several to a workgroup (pair_rows, pair_desc), and
  // `launch_rows` is the launch order of everything, longest first: `order` without the packed
  // rows, and the complement ~i of packed workgroup i.
  bool packed_faces = false;
  std::vector<int32_t> launch_rows;
  std::vector<int64_t> pair_walk_ptr;       // [num_pairs + 1] offsets into pair_walk
  std::vector<int32_t> pair_walk;           // per pair: union of its two rows, tile id | kPairInFirst | kPairInSecond
  std::vector<int32_t> tile_class;          // [n]
  std::vector<ca::SlotMask> class_mask;     // class 0 = all valid

  // A launch deals most of its workgroups to the XCDs statically and
  // leaves the cheapest entries at the end of the launch order to be drawn by whichever XCD gets there
  // first: rows / pairs of the sparse and of the dense walk.
  ca::LaunchSplit split_rows, split_rows_dense, split_pairs, split_pairs_dense;
  mutable std::atomic<uint32_t> launch_seq{0};  // picks the pool counter of a launch

  // device tables, created once
  std::mutex upload_mutex;
  bool uploaded = false;
  int device = -1;
  ca::DeviceTables dev;

  // The tables of the sparse forward as one block of bytes with 256-byte aligned parts, ready to be
  // copied into a fixed device array (compact_attn_forward_static); packed on first use.
  uint64_t serial = 0;                      // unique per layout object, never reused
  std::vector<unsigned char> static_image;
  struct StaticOffsets {
    size_t row_ptr = 0, col_meta = 0, order = 0, pair_rows = 0, pair_walk_ptr = 0, pair_walk = 0, tile_class = 0,
           class_mask = 0, class_perm = 0, pool_counter = 0, pair_desc = 0, launch_rows = 0;
  } static_off;
};

namespace ca {

void set_error(const char* fmt, ...);
void clear_error();
const char* last_error();

// Fills every host table of `L` from L.prob and the head descriptions.  Returns a ca_status.
int build_host_tables(ca_layout& L, const ca_head* heads);
// The same from per-head CSR arrays (validated: extents, ids in range, strictly ascending rows).
int import_host_tables(ca_layout& L, const int64_t* const* row_ptr, const int32_t* const* col_idx);
// Row-wise union of two layouts of the same geometry and head count.
int union_host_tables(ca_layout& L, const ca_layout& a, const ca_layout& b);
// |A and B| / |A or B| over the tile pairs of head `ha` of a and head `hb` of b (1 if both are empty).
double head_similarity(const ca_layout& a, int32_t ha, const ca_layout& b, int32_t hb);
// Window search of one head (search.cpp); mass is host float [n*n], groups_out has num_groups entries.
int search_head_windows(const ca_layout& L, const float* mass, const int32_t* group_max_dt, int32_t num_groups, double tau,
                        double lambda, int32_t pattern, ca_group* groups_out, double* recall_out, double* kept_out);
// Host images of the tables the kernels read, packed from the layout's host tables (no HIP calls).
struct PackedTables {
  std::vector<int32_t> col_meta, dense_meta, pair_walk, dense_pair_walk, tile_origin;
  std::vector<uint8_t> class_perm;
};
// `forward_only` leaves out what only the dense and the natural-order walks read.  Returns a ca_status.
int pack_device_tables(const ca_layout& layout, bool forward_only, PackedTables& t);
// Derived tables (per-head views, launch order, padding classes) once row_ptr / col_idx are set.
void finish_host_tables(ca_layout& L);

}  // namespace ca
