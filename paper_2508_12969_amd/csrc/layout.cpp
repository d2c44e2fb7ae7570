// Host-side layout builder: per-head CSR of kept key tiles, launch order and padding masks.
//
// Keep rule (Sec. 4.1 of the paper, with Eq. 1 / Eq. 2 read in tile units): the tile-frame
// distance |kt-qt| selects a group; inside the group a key tile is kept when it lies in either
// of two query-centred windows, clipped by the tile grid.  Both windows contain the query's own
// column, so on one tile row of one frame the kept columns form a single interval; the builder
// walks frames and tile rows in ascending order and emits those intervals, which yields the
// ascending tile ids directly.  No HIP call is made here.
#include <algorithm>
#include <cstdint>
#include <cstdarg>
#include <cstdio>
#include <cstring>
#include <new>

#include "layout.h"

namespace ca {

static thread_local char g_error[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_error, sizeof(g_error), fmt, ap);
  va_end(ap);
}
void clear_error() { g_error[0] = '\0'; }
const char* last_error() { return g_error; }

namespace {

struct Interval {
  int32_t lo, hi;  // inclusive; empty when lo > hi
};

inline Interval clip(int32_t center, int32_t radius, int32_t len) {
  // radius can be as large as INT32_MAX; widen before adding
  int64_t lo = (int64_t)center - radius, hi = (int64_t)center + radius;
  return {(int32_t)std::max<int64_t>(lo, 0), (int32_t)std::min<int64_t>(hi, len - 1)};
}

// Tiles of one axis a window covers: clipped around the query, or (clamp) moved inward so that it
// keeps its 2*radius+1 tiles (the whole axis if that is shorter).
inline Interval window_range(int32_t center, int32_t radius, int32_t len, bool clamp) {
  if (!clamp) return clip(center, radius, len);
  if (2 * (int64_t)radius + 1 >= len) return {0, len - 1};
  const int32_t c = std::min(std::max(center, radius), len - 1 - radius);
  return {c - radius, c + radius};
}

inline bool present(const ca_window& w) { return w.rh >= 0 && w.rw >= 0; }

// Resolved windows of one head for every tile-frame distance 0..nT-1 (group lookup done once).
struct HeadPlan {
  std::vector<int8_t> has;      // [nT] distance covered by some group
  std::vector<ca_window> a, b;  // [nT]
  bool clamp = false;           // windows keep their size at the border (centre moved inward)
};

int plan_head(const ca_head& h, int32_t head_index, int32_t nT, HeadPlan& plan) {
  if (h.num_groups < 0 || h.num_groups > CA_MAX_GROUPS) {
    set_error("head %d: num_groups=%d outside 0..%d", head_index, h.num_groups, CA_MAX_GROUPS);
    return CA_ERR_INVALID_ARG;
  }
  if (h.num_groups > 0 && h.groups == nullptr) {
    set_error("head %d: groups is null", head_index);
    return CA_ERR_INVALID_ARG;
  }
  int32_t last = -1;
  for (int32_t g = 0; g < h.num_groups; ++g) {
    if (h.groups[g].max_dt <= last) {
      set_error("head %d: max_dt must be non-negative and strictly increasing (group %d has %d after %d)",
                head_index, g, h.groups[g].max_dt, last);
      return CA_ERR_INVALID_ARG;
    }
    last = h.groups[g].max_dt;
  }
  if (h.clamp_centre != 0 && h.clamp_centre != 1) {
    set_error("head %d: clamp_centre must be 0 or 1", head_index);
    return CA_ERR_INVALID_ARG;
  }
  plan.clamp = h.clamp_centre == 1;
  plan.has.assign(nT, 0);
  plan.a.assign(nT, ca_window{-1, -1});
  plan.b.assign(nT, ca_window{-1, -1});
  int32_t g = 0;
  for (int32_t dt = 0; dt < nT; ++dt) {
    while (g < h.num_groups && h.groups[g].max_dt < dt) ++g;
    if (g == h.num_groups) break;
    plan.has[dt] = 1;
    plan.a[dt] = h.groups[g].a;
    plan.b[dt] = h.groups[g].b;
  }
  return CA_OK;
}

// Visits the kept video tiles of query tile (qt,qh,qw) as runs [first_id, first_id+len) in ascending order.
template <class F>
inline void for_each_run(const ca_layout& L, const HeadPlan& plan, int32_t qt, int32_t qh, int32_t qw, F&& emit) {
  for (int32_t kt = 0; kt < L.nT; ++kt) {
    const int32_t dt = kt > qt ? kt - qt : qt - kt;
    if (!plan.has[dt]) continue;
    const ca_window &wa = plan.a[dt], &wb = plan.b[dt];
    const bool pa = present(wa), pb = present(wb);
    if (!pa && !pb) continue;
    Interval ha{0, -1}, hb{0, -1}, ca_{0, -1}, cb{0, -1};
    if (pa) { ha = window_range(qh, wa.rh, L.nH, plan.clamp); ca_ = window_range(qw, wa.rw, L.nW, plan.clamp); }
    if (pb) { hb = window_range(qh, wb.rh, L.nH, plan.clamp); cb = window_range(qw, wb.rw, L.nW, plan.clamp); }
    const int32_t h_lo = pa && pb ? std::min(ha.lo, hb.lo) : (pa ? ha.lo : hb.lo);
    const int32_t h_hi = pa && pb ? std::max(ha.hi, hb.hi) : (pa ? ha.hi : hb.hi);
    for (int32_t kh = h_lo; kh <= h_hi; ++kh) {
      const bool in_a = pa && kh >= ha.lo && kh <= ha.hi;
      const bool in_b = pb && kh >= hb.lo && kh <= hb.hi;
      int32_t lo, hi;
      if (in_a && in_b) { lo = std::min(ca_.lo, cb.lo); hi = std::max(ca_.hi, cb.hi); }
      else if (in_a) { lo = ca_.lo; hi = ca_.hi; }
      else if (in_b) { lo = cb.lo; hi = cb.hi; }
      else continue;  // rows between two disjoint height ranges cannot occur (both contain qh, clamped or not), kept for safety
      const int64_t first = ((int64_t)kt * L.nH + kh) * L.nW + lo;
      emit((int32_t)first, hi - lo + 1);
    }
  }
}

void build_slot_masks(ca_layout& L) {
  // A tile's padding pattern depends only on whether it is the last tile along each axis.
  const ca_problem& p = L.prob;
  const int32_t rem_t = p.T - (L.nT - 1) * p.tt, rem_h = p.H - (L.nH - 1) * p.th, rem_w = p.W - (L.nW - 1) * p.tw;
  L.class_mask.clear();
  SlotMask full{};
  for (int64_t s = 0; s < L.B; ++s) full.w[s >> 5] |= 1u << (s & 31);
  L.class_mask.push_back(full);
  int class_of_edge[8];
  for (int e = 0; e < 8; ++e) {
    const int32_t lim_t = (e & 4) ? rem_t : p.tt, lim_h = (e & 2) ? rem_h : p.th, lim_w = (e & 1) ? rem_w : p.tw;
    if (lim_t == p.tt && lim_h == p.th && lim_w == p.tw) { class_of_edge[e] = 0; continue; }
    SlotMask m{};
    for (int32_t dt = 0; dt < lim_t; ++dt)
      for (int32_t dy = 0; dy < lim_h; ++dy)
        for (int32_t dx = 0; dx < lim_w; ++dx) {
          const int32_t s = (dt * p.th + dy) * p.tw + dx;
          m.w[s >> 5] |= 1u << (s & 31);
        }
    class_of_edge[e] = (int)L.class_mask.size();
    L.class_mask.push_back(m);
  }
  L.tile_class.assign(L.n, 0);
  for (int32_t kt = 0; kt < L.nT; ++kt)
    for (int32_t kh = 0; kh < L.nH; ++kh)
      for (int32_t kw = 0; kw < L.nW; ++kw) {
        const int e = (kt == L.nT - 1 ? 4 : 0) | (kh == L.nH - 1 ? 2 : 0) | (kw == L.nW - 1 ? 1 : 0);
        L.tile_class[((int64_t)kt * L.nH + kh) * L.nW + kw] = class_of_edge[e];
      }
}

void build_order(ca_layout& L) {
  // Descending kept count, ties by ascending row id: a counting sort over counts 0..n.
  const int64_t rows = (int64_t)L.prob.num_heads * L.n;
  std::vector<int64_t> bucket_start(L.n + 2, 0);
  for (int64_t r = 0; r < rows; ++r) {
    const int64_t c = L.row_ptr[r + 1] - L.row_ptr[r];
    ++bucket_start[(L.n - c) + 1];  // bucket 0 holds count n, bucket n holds count 0
  }
  for (int64_t b = 0; b <= L.n; ++b) bucket_start[b + 1] += bucket_start[b];
  L.order.resize(rows);
  for (int64_t r = 0; r < rows; ++r) {
    const int64_t c = L.row_ptr[r + 1] - L.row_ptr[r];
    L.order[bucket_start[L.n - c]++] = (int32_t)r;
  }
}

}  // namespace

// A workgroup of the paired kernel: two rows of one head (b = -1: one), the assignment of its waves,
// and the length of its walk (the union of the two rows).
struct PairGroup {
  int32_t a, b;
  uint32_t desc;
  int64_t walked;
};

static int64_t union_size(const ca_layout& L, int64_t ra, int64_t rb) {
  if (rb < 0) return L.row_ptr[ra + 1] - L.row_ptr[ra];
  int64_t i = L.row_ptr[ra], ie = L.row_ptr[ra + 1], j = L.row_ptr[rb], je = L.row_ptr[rb + 1], m = 0;
  while (i < ie && j < je) {
    const int32_t ti = L.col_idx[i], tj = L.col_idx[j];
    i += ti <= tj;
    j += tj <= ti;
    ++m;
  }
  return m + (ie - i) + (je - j);
}

// Launch order and walk lists of the paired kernel from its workgroups: longest walks first, ties
// in the order built (head, then tile id); pair_rows[2i], pair_rows[2i+1] are row ids head*n + tile.
// The walk of a workgroup is the union of its two rows in ascending tile order, one word per tile:
// tile id | kPairInFirst if the first row keeps the tile | kPairInSecond if the second does.
static void emit_pair_tables(ca_layout& L, std::vector<PairGroup>& groups) {
  std::stable_sort(groups.begin(), groups.end(), [](const PairGroup& x, const PairGroup& y) { return x.walked > y.walked; });
  L.pair_rows.resize(2 * groups.size());
  L.pair_desc.resize(groups.size());
  for (size_t i = 0; i < groups.size(); ++i) {
    L.pair_rows[2 * i] = groups[i].a;
    L.pair_rows[2 * i + 1] = groups[i].b;
    L.pair_desc[i] = (int32_t)groups[i].desc;
  }
  L.pair_walk_ptr.assign(groups.size() + 1, 0);
  for (size_t i = 0; i < groups.size(); ++i) L.pair_walk_ptr[i + 1] = L.pair_walk_ptr[i] + groups[i].walked;
  L.pair_walk.resize((size_t)L.pair_walk_ptr[groups.size()]);
  for (size_t p = 0; p < groups.size(); ++p) {
    const int64_t ra = groups[p].a, rb = groups[p].b;
    int64_t i = L.row_ptr[ra], ie = L.row_ptr[ra + 1];
    int64_t j = rb < 0 ? 0 : L.row_ptr[rb], je = rb < 0 ? 0 : L.row_ptr[rb + 1];
    int64_t o = L.pair_walk_ptr[p];
    while (i < ie || j < je) {
      const int32_t ti = i < ie ? L.col_idx[i] : INT32_MAX, tj = j < je ? L.col_idx[j] : INT32_MAX;
      const int32_t t = ti < tj ? ti : tj;
      L.pair_walk[o++] = (int32_t)((uint32_t)t | (ti == t ? kPairInFirst : 0u) | (tj == t ? kPairInSecond : 0u));
      i += ti == t;
      j += tj == t;
    }
  }
}

// 64-token tiles: every query tile of a head is paired with a neighbour.
static void build_pair_table(ca_layout& L) {
  // Partner of a video tile: its neighbour along one grid axis (coordinates 2i and 2i+1; the last
  // tile of an odd extent stays single).  Which axis costs the fewest walked tiles depends on the
  // head's windows (a neighbour along an axis in which the windows are wide shares almost all of
  // its list), so every head takes the axis with the smallest sum of union sizes.  Text tiles pair
  // up in id order.
  const int64_t n = L.n;
  const int32_t ext[3] = {L.nT, L.nH, L.nW};
  const int64_t stride[3] = {(int64_t)L.nH * L.nW, L.nW, 1};
  auto for_pairs = [&](int axis, auto&& visit) {  // visit(tile_a, tile_b or -1) over the video tiles
    for (int32_t t = 0; t < L.nT; ++t)
      for (int32_t h = 0; h < L.nH; ++h)
        for (int32_t w = 0; w < L.nW; ++w) {
          const int32_t c[3] = {t, h, w};
          if (c[axis] & 1) continue;
          const int64_t id = ((int64_t)t * L.nH + h) * L.nW + w;
          visit(id, c[axis] + 1 < ext[axis] ? id + stride[axis] : (int64_t)-1);
        }
  };
  std::vector<PairGroup> groups;
  for (int32_t head = 0; head < L.prob.num_heads; ++head) {
    const int64_t base = (int64_t)head * n;
    // candidates: the axes with at least two tiles, tried in the order w, h, t; the first of the cheapest wins
    int best_axis = 2;
    int64_t best_cost = -1;
    for (int axis = 2; axis >= 0; --axis) {
      if (ext[axis] < 2) continue;
      int64_t cost = 0;
      for_pairs(axis, [&](int64_t a, int64_t b) { cost += union_size(L, base + a, b < 0 ? -1 : base + b); });
      if (best_cost < 0 || cost < best_cost) best_cost = cost, best_axis = axis;
    }
    constexpr uint32_t kSingle = pair_desc_wave(0, 0, 0) | pair_desc_wave(1, 0, 1);  // a tile without a partner
    for_pairs(best_axis, [&](int64_t a, int64_t b) {
      const int64_t rb = b < 0 ? -1 : base + b;
      groups.push_back({(int32_t)(base + a), (int32_t)rb, rb < 0 ? kSingle : kPairPlain, union_size(L, base + a, rb)});
    });
    for (int64_t a = L.n_vid; a < n; a += 2) {
      const int64_t rb = a + 1 < n ? base + a + 1 : -1;
      groups.push_back({(int32_t)(base + a), (int32_t)rb, rb < 0 ? kSingle : kPairPlain, union_size(L, base + a, rb)});
    }
  }
  emit_pair_tables(L, groups);
}

// 128-token tiles: a query tile on a padded face of the grid holds tokens for one to three waves
// only (its slots are handed to lanes token-holding slots first), and in a workgroup of its own the
// other waves idle while the workgroup still pays for the tile copies and the barriers of every
// step.  Such tiles are packed along w, inside one row of tiles of the grid: their waves fill
// workgroups of four in order, a tile's waves may continue in the next workgroup, and a workgroup
// serves at most two tiles (it walks the union of their rows).  A head is packed only if that is
// cheaper by the measured cost of a tile step with 1, 2, 3 or 4 working waves (65, 73, 88, 100):
// neighbours with narrow windows share too little of their lists.  launch_rows is then the launch
// order of both kinds of workgroup: the rows that keep a workgroup of their own and the packed ones.
static void build_packed_faces(ca_layout& L) {
  const int64_t n = L.n;
  static const int64_t kStepCost[5] = {0, 65, 73, 88, 100};
  std::vector<int32_t> waves(n, 4);
  bool any = false;
  for (int64_t t = 0; t < L.n_vid; ++t) {
    const SlotMask& m = L.class_mask[L.tile_class[t]];
    const int valid = __builtin_popcount(m.w[0]) + __builtin_popcount(m.w[1]) + __builtin_popcount(m.w[2]) + __builtin_popcount(m.w[3]);
    waves[t] = (valid + 31) / 32;
    any = any || waves[t] < 4;
  }
  L.packed_faces = false;
  L.launch_rows.clear();
  if (!any) return;
  std::vector<PairGroup> groups, head_groups;
  std::vector<char> packed((size_t)L.prob.num_heads * n, 0);
  for (int32_t head = 0; head < L.prob.num_heads; ++head) {
    const int64_t base = (int64_t)head * n;
    head_groups.clear();
    int64_t plain_cost = 0;
    for (int32_t kt = 0; kt < L.nT; ++kt)
      for (int32_t kh = 0; kh < L.nH; ++kh) {
        PairGroup cur{-1, -1, 0, 0};
        int used = 0;
        auto flush = [&]() {
          if (used) head_groups.push_back(cur);
          cur = PairGroup{-1, -1, 0, 0};
          used = 0;
        };
        for (int32_t kw = 0; kw < L.nW; ++kw) {
          const int64_t t = ((int64_t)kt * L.nH + kh) * L.nW + kw;
          if (waves[t] >= 4) {
            flush();
            continue;
          }
          plain_cost += (L.row_ptr[base + t + 1] - L.row_ptr[base + t]) * kStepCost[waves[t]];
          for (int first = 0; first < waves[t];) {
            if (used == 4 || (cur.b >= 0 && cur.b != base + t)) flush();
            int second = 0;
            if (cur.a < 0) cur.a = (int32_t)(base + t);
            else if (cur.a != base + t) cur.b = (int32_t)(base + t), second = 1;
            const int take = std::min(waves[t] - first, 4 - used);
            for (int i = 0; i < take; ++i) cur.desc |= pair_desc_wave(used + i, second, first + i);
            used += take;
            first += take;
          }
        }
        flush();
      }
    int64_t packed_cost = 0;
    for (PairGroup& g : head_groups) {
      g.walked = union_size(L, g.a, g.b);
      packed_cost += g.walked * kStepCost[__builtin_popcount((g.desc >> 4) & 0xFu)];
    }
    if (head_groups.empty() || packed_cost >= plain_cost) continue;
    for (const PairGroup& g : head_groups) {
      packed[g.a] = 1;
      if (g.b >= 0) packed[g.b] = 1;
      groups.push_back(g);
    }
  }
  if (groups.empty()) return;
  emit_pair_tables(L, groups);
  L.packed_faces = true;
  // one launch order for both kinds of workgroup, longest first: a row id, or the complement of a
  // packed workgroup's index (ties: the packed workgroup first)
  L.launch_rows.reserve(L.order.size());
  size_t g = 0;
  for (int32_t r : L.order) {
    if (packed[r]) continue;
    const int64_t len = L.row_ptr[r + 1] - L.row_ptr[r];
    while (g < groups.size() && groups[g].walked >= len) L.launch_rows.push_back(~(int32_t)g++);
    L.launch_rows.push_back(r);
  }
  while (g < groups.size()) L.launch_rows.push_back(~(int32_t)g++);
}

// The XCDs of one card do not run at the same speed (measured: up to 5 % apart in finishing time on
// equal shares), and workgroup ids are bound to XCDs, so a launch dealt out by id alone ends when the
// slowest XCD does.  The entries that hold the last kPoolWork of the launch's work (the shortest
// rows: the order is by descending length) are therefore not bound to ids: workgroups past the
// static part draw them by ticket, and an XCD that is ahead draws more.  The static part is a whole
// number of rounds of the XCD-aware order (8 chunks of 64).
LaunchSplit split_launch(const int64_t* work, int64_t entries) {
  constexpr double kPoolWork = 0.06;
  constexpr int64_t kRound = 8 * 64;
  constexpr int64_t kEntryCost = 3;  // fixed cost of an entry in tile steps (launch, first copies, epilogue)
  LaunchSplit sp;
  sp.static_entries = entries;
  if (entries < kPoolMinItems) return sp;
  double total = 0;
  for (int64_t i = 0; i < entries; ++i) total += (double)(work[i] + kEntryCost);
  double tail = 0;
  int64_t s = entries;
  while (s > 0 && tail + (double)(work[s - 1] + kEntryCost) <= kPoolWork * total) tail += (double)(work[--s] + kEntryCost);
  s = (s + kRound - 1) / kRound * kRound;
  if (s < entries && entries - s < ((int64_t)1 << 30)) {
    sp.static_entries = s;
    sp.pool_entries = (int32_t)(entries - s);
  }
  return sp;
}

namespace {
void build_launch_splits(ca_layout& L) {
  const std::vector<int32_t>& launched = L.packed_faces ? L.launch_rows : L.order;
  const int64_t rows = (int64_t)launched.size();
  std::vector<int64_t> work(rows);
  for (int64_t i = 0; i < rows; ++i) {
    const int32_t e = launched[i];
    work[i] = e < 0 ? L.pair_walk_ptr[~e + 1] - L.pair_walk_ptr[~e] : L.row_ptr[e + 1] - L.row_ptr[e];
  }
  L.split_rows = split_launch(work.data(), rows);
  std::fill(work.begin(), work.end(), L.n);
  L.split_rows_dense = split_launch(work.data(), rows);
  const int64_t pairs = (int64_t)L.pair_rows.size() / 2;
  L.split_pairs = L.split_pairs_dense = LaunchSplit{};
  if (pairs && !L.packed_faces) {
    work.resize(pairs);
    for (int64_t i = 0; i < pairs; ++i) work[i] = L.pair_walk_ptr[i + 1] - L.pair_walk_ptr[i];
    L.split_pairs = split_launch(work.data(), pairs);
    std::fill(work.begin(), work.end(), L.n);
    L.split_pairs_dense = split_launch(work.data(), pairs);
  }
}
}  // namespace

void finish_host_tables(ca_layout& L) {
  const int32_t Hd = L.prob.num_heads;
  // per-head relative offsets for the C-ABI view
  L.head_row_ptr.assign(Hd, std::vector<int64_t>());
  for (int32_t h = 0; h < Hd; ++h) {
    L.head_row_ptr[h].resize(L.n + 1);
    const int64_t base = L.row_ptr[(int64_t)h * L.n];
    for (int64_t q = 0; q <= L.n; ++q) L.head_row_ptr[h][q] = L.row_ptr[(int64_t)h * L.n + q] - base;
  }
  build_order(L);
  build_slot_masks(L);
  L.pair_rows.clear();
  L.pair_desc.clear();
  L.pair_walk_ptr.clear();
  L.pair_walk.clear();
  L.packed_faces = false;
  L.launch_rows.clear();
  if (L.prob.dtype == CA_BF16 && L.B == 64 && L.prob.head_dim == 128) build_pair_table(L);
  if (L.prob.dtype == CA_BF16 && L.B == 128 && L.prob.head_dim == 128) build_packed_faces(L);
  build_launch_splits(L);
}

int import_host_tables(ca_layout& L, const int64_t* const* row_ptr, const int32_t* const* col_idx) {
  const int32_t Hd = L.prob.num_heads;
  for (int32_t h = 0; h < Hd; ++h) {
    if (!row_ptr[h] || (!col_idx[h] && row_ptr[h][L.n] != 0)) {
      set_error("head %d: null CSR array", h);
      return CA_ERR_INVALID_ARG;
    }
    if (row_ptr[h][0] != 0) {
      set_error("head %d: row_ptr[0] must be 0", h);
      return CA_ERR_INVALID_ARG;
    }
    for (int64_t q = 0; q < L.n; ++q) {
      const int64_t b = row_ptr[h][q], e = row_ptr[h][q + 1];
      if (e < b || e - b > L.n) {
        set_error("head %d: row %lld has an invalid extent", h, (long long)q);
        return CA_ERR_INVALID_ARG;
      }
      for (int64_t i = b; i < e; ++i) {
        const int32_t c = col_idx[h][i];
        if (c < 0 || c >= L.n || (i > b && c <= col_idx[h][i - 1])) {
          set_error("head %d: row %lld must list tile ids in [0, n) in strictly ascending order", h, (long long)q);
          return CA_ERR_INVALID_ARG;
        }
      }
    }
  }
  try {
    const int64_t rows = (int64_t)Hd * L.n;
    L.row_ptr.assign(rows + 1, 0);
    int64_t total = 0;
    for (int32_t h = 0; h < Hd; ++h) {
      for (int64_t q = 0; q < L.n; ++q) L.row_ptr[(int64_t)h * L.n + q] = total + row_ptr[h][q];
      total += row_ptr[h][L.n];
    }
    L.row_ptr[rows] = total;
    L.col_idx.resize(total);
    for (int32_t h = 0; h < Hd; ++h) {
      const int64_t cnt = row_ptr[h][L.n];
      if (cnt) std::memcpy(L.col_idx.data() + L.row_ptr[(int64_t)h * L.n], col_idx[h], cnt * sizeof(int32_t));
    }
    finish_host_tables(L);
  } catch (const std::bad_alloc&) {
    set_error("out of host memory while importing the layout");
    return CA_ERR_ALLOC;
  }
  return CA_OK;
}

int union_host_tables(ca_layout& L, const ca_layout& a, const ca_layout& b) {
  try {
    const int64_t rows = (int64_t)L.prob.num_heads * L.n;
    L.row_ptr.assign(rows + 1, 0);
    L.col_idx.clear();
    L.col_idx.reserve(std::max(a.col_idx.size(), b.col_idx.size()));
    for (int64_t r = 0; r < rows; ++r) {
      const int32_t *pa = a.col_idx.data() + a.row_ptr[r], *ea = a.col_idx.data() + a.row_ptr[r + 1];
      const int32_t *pb = b.col_idx.data() + b.row_ptr[r], *eb = b.col_idx.data() + b.row_ptr[r + 1];
      while (pa < ea || pb < eb) {  // merge of two ascending lists without duplicates
        if (pb == eb || (pa < ea && *pa < *pb)) L.col_idx.push_back(*pa++);
        else if (pa == ea || *pb < *pa) L.col_idx.push_back(*pb++);
        else { L.col_idx.push_back(*pa++); ++pb; }
      }
      L.row_ptr[r + 1] = (int64_t)L.col_idx.size();
    }
    finish_host_tables(L);
  } catch (const std::bad_alloc&) {
    set_error("out of host memory while merging the layouts");
    return CA_ERR_ALLOC;
  }
  return CA_OK;
}

double head_similarity(const ca_layout& a, int32_t ha, const ca_layout& b, int32_t hb) {
  int64_t both = 0, either = 0;
  for (int64_t q = 0; q < a.n; ++q) {
    const int64_t ra = (int64_t)ha * a.n + q, rb = (int64_t)hb * b.n + q;
    const int32_t *pa = a.col_idx.data() + a.row_ptr[ra], *ea = a.col_idx.data() + a.row_ptr[ra + 1];
    const int32_t *pb = b.col_idx.data() + b.row_ptr[rb], *eb = b.col_idx.data() + b.row_ptr[rb + 1];
    while (pa < ea && pb < eb) {
      if (*pa < *pb) ++pa;
      else if (*pb < *pa) ++pb;
      else { ++both; ++pa; ++pb; }
    }
    either += (a.row_ptr[ra + 1] - a.row_ptr[ra]) + (b.row_ptr[rb + 1] - b.row_ptr[rb]);
  }
  either -= both;
  return either == 0 ? 1.0 : (double)both / (double)either;
}

int build_host_tables(ca_layout& L, const ca_head* heads) {
  const ca_problem& p = L.prob;
  const int32_t Hd = p.num_heads;
  std::vector<HeadPlan> plans(Hd);
  for (int32_t h = 0; h < Hd; ++h) {
    const int st = plan_head(heads[h], h, L.nT, plans[h]);
    if (st != CA_OK) return st;
  }
  try {
    const int64_t rows = (int64_t)Hd * L.n;
    L.row_ptr.assign(rows + 1, 0);
    // pass 1: row lengths
    for (int32_t h = 0; h < Hd; ++h)
      for (int64_t q = 0; q < L.n; ++q) {
        int64_t cnt;
        if (q >= L.n_vid) {
          cnt = L.n;  // text query tile keeps everything
        } else {
          const int32_t qw = (int32_t)(q % L.nW), qh = (int32_t)((q / L.nW) % L.nH), qt = (int32_t)(q / ((int64_t)L.nW * L.nH));
          cnt = L.n_txt;
          for_each_run(L, plans[h], qt, qh, qw, [&](int32_t, int32_t len) { cnt += len; });
        }
        L.row_ptr[(int64_t)h * L.n + q + 1] = cnt;
      }
    for (int64_t r = 0; r < rows; ++r) L.row_ptr[r + 1] += L.row_ptr[r];
    // pass 2: column ids
    L.col_idx.resize(L.row_ptr[rows]);
    for (int32_t h = 0; h < Hd; ++h)
      for (int64_t q = 0; q < L.n; ++q) {
        int32_t* dst = L.col_idx.data() + L.row_ptr[(int64_t)h * L.n + q];
        if (q >= L.n_vid) {
          for (int64_t k = 0; k < L.n; ++k) *dst++ = (int32_t)k;
          continue;
        }
        const int32_t qw = (int32_t)(q % L.nW), qh = (int32_t)((q / L.nW) % L.nH), qt = (int32_t)(q / ((int64_t)L.nW * L.nH));
        for_each_run(L, plans[h], qt, qh, qw, [&](int32_t first, int32_t len) {
          for (int32_t i = 0; i < len; ++i) *dst++ = first + i;
        });
        for (int64_t k = L.n_vid; k < L.n; ++k) *dst++ = (int32_t)k;
      }
    finish_host_tables(L);
  } catch (const std::bad_alloc&) {
    set_error("out of host memory while building the layout");
    return CA_ERR_ALLOC;
  }
  return CA_OK;
}

// The kernels read one packed word per kept tile: tile id | padding class << 24, and bit 31 set
// when the upper half of the tile's slots is padding only (such a tile costs half the products).
// `forward_only` leaves out what only the dense and the natural-order walks read.
int pack_device_tables(const ca_layout& layout, bool forward_only, PackedTables& t) {
  const ca_layout* L = &layout;
  if (L->n >= (int64_t)1 << 24 || L->class_mask.size() > 127) {
    set_error("layout too large for the device tables (%lld tiles, %zu padding classes)", (long long)L->n,
              L->class_mask.size());
    return CA_ERR_UNSUPPORTED;
  }
  try {
    std::vector<uint32_t> class_word(L->class_mask.size());
    const int words = (int)((L->B + 31) / 32);
    for (size_t c = 0; c < class_word.size(); ++c) {
      bool upper_empty = words >= 2;
      for (int w = words / 2; w < words; ++w) upper_empty = upper_empty && L->class_mask[c].w[w] == 0;
      class_word[c] = ((uint32_t)c << 24) | (upper_empty ? 0x80000000u : 0u);
    }
    // Query slots of a tile in the order the bf16 kernels hand them to lanes: the slots that hold a
    // token first, so that the queries of a padded tile fill as few 32-query waves as possible.
    t.class_perm.assign(L->class_mask.size() * 128, 0);
    for (size_t c = 0; c < L->class_mask.size(); ++c) {
      int at = 0;
      for (int pass = 0; pass < 2; ++pass)
        for (int slot = 0; slot < (int)L->B && slot < 128; ++slot) {
          const bool valid = (L->class_mask[c].w[slot >> 5] >> (slot & 31)) & 1u;
          if (valid == (pass == 0)) t.class_perm[c * 128 + at++] = (uint8_t)slot;
        }
    }
    // two words of padding: the kernels fetch these tables two entries ahead of the one in use
    t.col_meta.assign(L->col_idx.size() + 2, 0);
    for (size_t i = 0; i < L->col_idx.size(); ++i)
      t.col_meta[i] = (int32_t)((uint32_t)L->col_idx[i] | class_word[L->tile_class[L->col_idx[i]]]);
    if (!forward_only) {
      t.dense_meta.assign(L->n + 2, 0);
      for (int64_t i = 0; i < L->n; ++i) t.dense_meta[i] = (int32_t)((uint32_t)i | class_word[L->tile_class[i]]);
      // natural-order row of slot 0 of every tile (kernels that gather tiles from natural order)
      const ca_problem& pr = L->prob;
      const int64_t n_video = (int64_t)pr.T * pr.H * pr.W;
      if (L->N_real < ((int64_t)1 << 31)) {
        t.tile_origin.resize(L->n);
        for (int64_t i = 0; i < L->n; ++i) {
          if (i >= L->n_vid) {
            t.tile_origin[i] = (int32_t)(n_video + (i - L->n_vid) * L->B);
          } else {
            const int64_t kw = i % L->nW, kh = (i / L->nW) % L->nH, kt = i / ((int64_t)L->nW * L->nH);
            t.tile_origin[i] = (int32_t)(((kt * pr.tt) * pr.H + kh * pr.th) * pr.W + kw * pr.tw);
          }
        }
      }
    }
    if (!L->pair_rows.empty()) {
      // walk words of the paired kernel carry the class in bits 24-29, below the two membership bits
      if (L->class_mask.size() > 63) {
        set_error("layout has too many padding classes for the paired kernel (%zu)", L->class_mask.size());
        return CA_ERR_UNSUPPORTED;
      }
      t.pair_walk.assign(L->pair_walk.size() + 2, 0);
      for (size_t i = 0; i < L->pair_walk.size(); ++i) {
        const uint32_t w = (uint32_t)L->pair_walk[i];
        t.pair_walk[i] = (int32_t)(w | ((uint32_t)L->tile_class[w & 0xffffffu] << 24));
      }
      if (!forward_only) {
        t.dense_pair_walk.assign(L->n + 2, 0);
        for (int64_t i = 0; i < L->n; ++i)
          t.dense_pair_walk[i] =
              (int32_t)((uint32_t)i | ((uint32_t)L->tile_class[i] << 24) | ca::kPairInFirst | ca::kPairInSecond);
      }
    }
  } catch (const std::bad_alloc&) {
    set_error("out of host memory while packing the device tables");
    return CA_ERR_ALLOC;
  }
  return CA_OK;
}


}  // namespace ca
