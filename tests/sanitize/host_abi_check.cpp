// Host-side exercise of the C ABI for a build with AddressSanitizer and UndefinedBehaviorSanitizer
// (host code only; no kernel is launched and no GPU is needed).  It walks the pointer-heavy host
// paths: the layout builder, CSR import with malformed input, union, similarity, query-tile pairs,
// the window search, and the packing of the device tables including the two padding words the
// kernels are allowed to read past the end of every list.  Any sanitizer report aborts the run;
// a wrong result prints a message and exits with status 1.
#include <cstdint>
#include <cstdio>
#include <cstdlib>
#include <random>
#include <vector>

#include "compact_attn.h"
#include "kernels.h"
#include "layout.h"

// The kernels are not part of this build: the launchers only have to exist for the link.
namespace ca {
hipError_t launch_permute(const PermuteArgs&, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_attn_f32(const AttnArgs&, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_attn_bf16(const AttnArgs&, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_attn_bf16_pair(const AttnArgs&, hipStream_t) { return hipErrorInvalidValue; }
hipError_t launch_tile_mass(const MassArgs&, hipStream_t) { return hipErrorInvalidValue; }
}  // namespace ca

namespace {

int failures = 0;
#define CHECK(cond)                                                        \
  do {                                                                     \
    if (!(cond)) {                                                         \
      std::printf("FAILED %s:%d: %s\n", __FILE__, __LINE__, #cond);        \
      ++failures;                                                          \
    }                                                                      \
  } while (0)

struct Heads {
  std::vector<std::vector<ca_group>> groups;
  std::vector<ca_head> heads;
};

Heads random_heads(std::mt19937& rng, int num_heads, int nT, int nH, int nW) {
  Heads h;
  h.groups.resize(num_heads);
  for (int i = 0; i < num_heads; ++i) {
    const int count = (int)(rng() % 4);
    int dt = -1;
    for (int g = 0; g < count; ++g) {
      dt += 1 + (int)(rng() % 2);
      if (dt >= nT + 1) break;
      ca_group grp{};
      grp.max_dt = dt;
      grp.a = ca_window{(int)(rng() % (nH + 2)) - 1, (int)(rng() % (nW + 2)) - 1};
      grp.b = ca_window{(int)(rng() % (nH + 2)) - 1, (int)(rng() % (nW + 2)) - 1};
      h.groups[i].push_back(grp);
    }
    h.heads.push_back(ca_head{(int32_t)h.groups[i].size(), (int32_t)(rng() % 2), h.groups[i].data()});
  }
  return h;
}

// Reads every element of the packed tables, the padding words included, and checks the fields.
void check_packing(const ca_layout* L) {
  for (int forward_only = 0; forward_only < 2; ++forward_only) {
    ca::PackedTables t;
    CHECK(ca::pack_device_tables(*L, forward_only != 0, t) == CA_OK);
    CHECK(t.col_meta.size() == L->col_idx.size() + 2);
    int64_t sum = 0;
    for (size_t i = 0; i < t.col_meta.size(); ++i) sum += t.col_meta[i];
    for (size_t i = 0; i < L->col_idx.size(); ++i) {
      const uint32_t w = (uint32_t)t.col_meta[i];
      CHECK((int32_t)(w & 0xffffffu) == L->col_idx[i]);
      CHECK(((w >> 24) & 0x7fu) == (uint32_t)L->tile_class[L->col_idx[i]]);
    }
    CHECK(t.col_meta[L->col_idx.size()] == 0 && t.col_meta[L->col_idx.size() + 1] == 0);
    CHECK(t.class_perm.size() == L->class_mask.size() * 128);
    for (size_t c = 0; c < L->class_mask.size(); ++c) {
      std::vector<int> seen(128, 0);
      for (int i = 0; i < (int)L->B && i < 128; ++i) seen[t.class_perm[c * 128 + i]]++;
      for (int i = 0; i < (int)L->B && i < 128; ++i) CHECK(seen[i] == 1);
    }
    if (!forward_only) {
      CHECK(t.dense_meta.size() == (size_t)L->n + 2);
      for (size_t i = 0; i < t.dense_meta.size(); ++i) sum += t.dense_meta[i];
      for (size_t i = 0; i < t.tile_origin.size(); ++i) CHECK(t.tile_origin[i] >= 0 && t.tile_origin[i] < L->N_real);
    }
    if (!L->pair_rows.empty()) {
      CHECK(t.pair_walk.size() == L->pair_walk.size() + 2);
      for (size_t i = 0; i < t.pair_walk.size(); ++i) sum += t.pair_walk[i];
      if (!forward_only) {
        CHECK(t.dense_pair_walk.size() == (size_t)L->n + 2);
        for (size_t i = 0; i < t.dense_pair_walk.size(); ++i) sum += t.dense_pair_walk[i];
      }
    }
    if (sum == 0x7fffffffffffffffLL) std::printf("unlikely\n");  // keeps the reads alive
  }
}

// The split of a launch into a statically dealt part and a dynamically drawn tail: the static part
// is whole rounds of 512 entries, the two parts cover the launch order exactly, and the tail holds the
// cheapest entries, at most about 6 % of the work plus the rounding to a round.
void check_split(const ca::LaunchSplit& sp, const std::vector<int64_t>& work) {
  const int64_t entries = (int64_t)work.size();
  CHECK(sp.static_entries >= 0 && sp.pool_entries >= 0);
  CHECK(sp.static_entries + sp.pool_entries == entries);
  if (entries < ca::kPoolMinItems) CHECK(sp.pool_entries == 0);
  if (sp.pool_entries > 0) {
    CHECK(sp.static_entries % 512 == 0);
    double total = 0, tail = 0;
    for (int64_t i = 0; i < entries; ++i) total += (double)(work[i] + 3);
    for (int64_t i = sp.static_entries; i < entries; ++i) tail += (double)(work[i] + 3);
    CHECK(tail <= 0.06 * total + 1e-9);
  }
}

void check_layout_splits(const ca_layout* L) {
  const std::vector<int32_t>& launched = L->packed_faces ? L->launch_rows : L->order;
  const int64_t rows = (int64_t)launched.size();
  std::vector<int64_t> work(rows);
  for (int64_t i = 0; i < rows; ++i) {
    const int32_t e = launched[i];  // a row, or the complement of a packed workgroup's index
    work[i] = e < 0 ? L->pair_walk_ptr[~e + 1] - L->pair_walk_ptr[~e] : L->row_ptr[e + 1] - L->row_ptr[e];
  }
  for (int64_t i = 1; i < rows; ++i) CHECK(work[i] <= work[i - 1]);  // the launch order is by descending length
  check_split(L->split_rows, work);
  check_split(L->split_rows_dense, std::vector<int64_t>(rows, L->n));
  const int64_t pairs = (int64_t)L->pair_rows.size() / 2;
  if (pairs && !L->packed_faces) {
    work.assign(pairs, 0);
    for (int64_t i = 0; i < pairs; ++i) work[i] = L->pair_walk_ptr[i + 1] - L->pair_walk_ptr[i];
    check_split(L->split_pairs, work);
    check_split(L->split_pairs_dense, std::vector<int64_t>(pairs, L->n));
  } else {
    CHECK(L->split_pairs.pool_entries == 0 && L->split_pairs_dense.pool_entries == 0);
  }
}

// Who computes which queries: every 32-query wave slot of every row that holds a token belongs to
// exactly one wave, either of the row's own workgroup (launch_rows: all four) or of a workgroup of
// two query tiles (pair_desc); walks are unions of the two rows with the right membership bits.
void check_wave_assignment(const ca_layout* L) {
  const int64_t rows = (int64_t)L->prob.num_heads * L->n;
  const int64_t pairs = (int64_t)L->pair_rows.size() / 2;
  CHECK(L->pair_desc.size() == (size_t)pairs);
  if (!pairs) {
    CHECK(!L->packed_faces && L->launch_rows.empty());
    return;
  }
  const int slots = (int)((L->B + 31) / 32);
  std::vector<int> owners((size_t)rows * 4, 0);
  if (L->packed_faces) {
    // launch_rows: `order` without the packed rows, in the same order, and every packed workgroup once
    std::vector<char> own(rows, 0);
    std::vector<int32_t> kept_rows;
    std::vector<int> seen_group(pairs, 0);
    for (int32_t e : L->launch_rows) {
      if (e >= 0) kept_rows.push_back(e);
      else if (~e < pairs) seen_group[~e]++;
      else CHECK(false);
    }
    for (int64_t g = 0; g < pairs; ++g) CHECK(seen_group[g] == 1);
    size_t at = 0;
    for (int32_t r : L->order)
      if (at < kept_rows.size() && kept_rows[at] == r) own[r] = 1, ++at;
    CHECK(at == kept_rows.size());
    for (int64_t r = 0; r < rows; ++r)
      if (own[r]) for (int w = 0; w < slots; ++w) owners[r * 4 + w]++;
  }
  for (int64_t p = 0; p < pairs; ++p) {
    const int32_t a = L->pair_rows[2 * p], b = L->pair_rows[2 * p + 1];
    const uint32_t desc = (uint32_t)L->pair_desc[p];
    CHECK(a >= 0 && a < rows && b < rows && a != b);
    if (b >= 0) CHECK(a / L->n == b / L->n);
    for (int w = 0; w < 4; ++w) {
      if (!((desc >> (4 + w)) & 1u)) continue;
      const int second = (desc >> w) & 1u, first = (desc >> (8 + 4 * w)) & 0xFu;
      CHECK(first < 4);
      if (second) CHECK(b >= 0);
      const int64_t r = second ? b : a;
      if (r >= 0 && first < 4) owners[r * 4 + first]++;
    }
    if (p > 0) CHECK(L->pair_walk_ptr[p + 1] - L->pair_walk_ptr[p] <= L->pair_walk_ptr[p] - L->pair_walk_ptr[p - 1]);
    // the walk: ascending tile ids, each kept by at least one of the two rows, bits as the rows say
    std::vector<char> in_a(L->n, 0), in_b(L->n, 0);
    for (int64_t i = L->row_ptr[a]; i < L->row_ptr[a + 1]; ++i) in_a[L->col_idx[i]] = 1;
    if (b >= 0) for (int64_t i = L->row_ptr[b]; i < L->row_ptr[b + 1]; ++i) in_b[L->col_idx[i]] = 1;
    int64_t members = 0;
    int32_t last = -1;
    for (int64_t i = L->pair_walk_ptr[p]; i < L->pair_walk_ptr[p + 1]; ++i) {
      const uint32_t word = (uint32_t)L->pair_walk[i];
      const int32_t t = (int32_t)(word & 0xffffffu);
      CHECK(t > last && t < L->n);
      last = t;
      CHECK(((word >> 30) & 1u) == (uint32_t)in_a[t] && (word >> 31) == (uint32_t)in_b[t]);
      CHECK(in_a[t] || in_b[t]);
      members += in_a[t] + in_b[t];
    }
    CHECK(members == (L->row_ptr[a + 1] - L->row_ptr[a]) + (b >= 0 ? L->row_ptr[b + 1] - L->row_ptr[b] : 0));
  }
  for (int64_t r = 0; r < rows; ++r) {
    const ca::SlotMask& m = L->class_mask[L->tile_class[r % L->n]];
    const int valid = __builtin_popcount(m.w[0]) + __builtin_popcount(m.w[1]) + __builtin_popcount(m.w[2]) + __builtin_popcount(m.w[3]);
    for (int w = 0; w < 4; ++w) {
      const bool holds_tokens = w * 32 < valid;
      if (holds_tokens) CHECK(owners[r * 4 + w] == 1);
      else CHECK(owners[r * 4 + w] <= 1);
    }
  }
}

void check_split_function() {
  std::mt19937 rng(7);
  for (int rep = 0; rep < 40; ++rep) {
    const int64_t entries = rep < 4 ? (int64_t)(rep * 1365) : 4096 + (int64_t)(rng() % 40000);
    std::vector<int64_t> work(entries);
    int64_t v = 1 + (int64_t)(rng() % 2000);
    for (int64_t i = 0; i < entries; ++i) {
      work[i] = v;
      if (v > 0 && rng() % 8 == 0) v -= (int64_t)(rng() % 3);
      if (v < 0) v = 0;
    }
    if (rep % 5 == 4) work.assign(entries, rep % 2 ? 0 : 1000);  // all entries alike
    check_split(ca::split_launch(work.data(), entries), work);
  }
}

void check_layout_views(const ca_layout* L, const ca_problem& p) {
  int64_t n = 0, B = 0, n_real = 0, n_pad = 0, nnz = 0;
  CHECK(compact_attn_layout_info(L, &n, &B, &n_real, &n_pad, &nnz) == CA_OK);
  CHECK(n_pad == n * B);
  int64_t total = 0;
  for (int h = 0; h < p.num_heads; ++h) {
    const int64_t* rp = nullptr;
    const int32_t* ci = nullptr;
    CHECK(compact_attn_layout_csr(L, h, &rp, &ci) == CA_OK);
    CHECK(rp[0] == 0);
    for (int64_t q = 0; q < n; ++q) {
      CHECK(rp[q + 1] >= rp[q]);
      for (int64_t i = rp[q]; i < rp[q + 1]; ++i) {
        CHECK(ci[i] >= 0 && ci[i] < n);
        if (i > rp[q]) CHECK(ci[i] > ci[i - 1]);
      }
    }
    total += rp[n];
  }
  CHECK(total == nnz);
  const int32_t* order = nullptr;
  CHECK(compact_attn_layout_order(L, &order) == CA_OK);
  std::vector<char> hit((size_t)p.num_heads * n, 0);
  for (int64_t i = 0; i < (int64_t)p.num_heads * n; ++i) {
    CHECK(order[i] >= 0 && order[i] < p.num_heads * n);
    hit[order[i]] = 1;
  }
  for (char c : hit) CHECK(c == 1);
  const int32_t* pairs = nullptr;
  int64_t num_pairs = 0;
  const int64_t* walk_ptr = nullptr;
  const int32_t* walk = nullptr;
  CHECK(compact_attn_layout_pairs(L, &pairs, &num_pairs, &walk_ptr, &walk) == CA_OK);
  for (int64_t i = 0; i < num_pairs; ++i) {
    CHECK(pairs[2 * i] >= 0 && pairs[2 * i + 1] >= -1);
    for (int64_t j = walk_ptr[i]; j < walk_ptr[i + 1]; ++j) CHECK((walk[j] & 0xffffff) < n);
  }
}

void run_case(std::mt19937& rng, ca_problem p) {
  const int nT = (p.T + p.tt - 1) / p.tt, nH = (p.H + p.th - 1) / p.th, nW = (p.W + p.tw - 1) / p.tw;
  Heads h = random_heads(rng, p.num_heads, nT, nH, nW);
  ca_layout* L = nullptr;
  CHECK(compact_attn_build_layout(&p, h.heads.data(), &L) == CA_OK);
  if (!L) return;
  check_layout_views(L, p);
  check_packing(L);
  check_layout_splits(L);
  check_wave_assignment(L);

  // round trip through the CSR import, then union with a second random layout and similarity
  int64_t n = 0;
  compact_attn_layout_info(L, &n, nullptr, nullptr, nullptr, nullptr);
  std::vector<const int64_t*> rps(p.num_heads);
  std::vector<const int32_t*> cis(p.num_heads);
  for (int i = 0; i < p.num_heads; ++i) compact_attn_layout_csr(L, i, &rps[i], &cis[i]);
  ca_layout* copy = nullptr;
  CHECK(compact_attn_layout_from_csr(&p, rps.data(), cis.data(), &copy) == CA_OK);
  Heads h2 = random_heads(rng, p.num_heads, nT, nH, nW);
  ca_layout* other = nullptr;
  CHECK(compact_attn_build_layout(&p, h2.heads.data(), &other) == CA_OK);
  ca_layout* merged = nullptr;
  CHECK(compact_attn_layout_union(copy, other, &merged) == CA_OK);
  if (merged) {
    check_layout_views(merged, p);
    check_packing(merged);
    check_layout_splits(merged);
    check_wave_assignment(merged);
    double sim = -1;
    CHECK(compact_attn_layout_similarity(merged, 0, merged, 0, &sim) == CA_OK && sim == 1.0);
    CHECK(compact_attn_layout_similarity(L, 0, other, p.num_heads - 1, &sim) == CA_OK && sim >= 0.0 && sim <= 1.0);
  }

  // malformed CSR: a row that descends, an id out of range, a row_ptr that does not start at 0
  if (rps[0][n] >= 2) {
    std::vector<int32_t> bad(cis[0], cis[0] + rps[0][n]);
    int64_t q = 0;
    while (q < n && rps[0][q + 1] - rps[0][q] < 2) ++q;
    if (q < n) {
      std::swap(bad[rps[0][q]], bad[rps[0][q] + 1]);
      std::vector<const int32_t*> cis_bad = cis;
      cis_bad[0] = bad.data();
      ca_layout* none = nullptr;
      CHECK(compact_attn_layout_from_csr(&p, rps.data(), cis_bad.data(), &none) == CA_ERR_INVALID_ARG && none == nullptr);
      bad[rps[0][q]] = (int32_t)n;  // out of range
      CHECK(compact_attn_layout_from_csr(&p, rps.data(), cis_bad.data(), &none) == CA_ERR_INVALID_ARG);
    }
    std::vector<int64_t> rp_bad(rps[0], rps[0] + n + 1);
    rp_bad[0] = 1;
    std::vector<const int64_t*> rps_bad = rps;
    rps_bad[0] = rp_bad.data();
    ca_layout* none = nullptr;
    CHECK(compact_attn_layout_from_csr(&p, rps_bad.data(), cis.data(), &none) == CA_ERR_INVALID_ARG);
    rp_bad[0] = 0;
    rp_bad[n] += 5;  // extent past the array
    rp_bad[n / 2] = rp_bad[n] + 1;
    CHECK(compact_attn_layout_from_csr(&p, rps_bad.data(), cis.data(), &none) == CA_ERR_INVALID_ARG);
  }

  // window search on a random non-negative mass, every pattern
  std::vector<float> mass((size_t)n * n);
  std::uniform_real_distribution<float> u(0.f, 1.f);
  for (float& x : mass) x = u(rng) * u(rng);
  std::vector<int32_t> bounds;
  for (int dt = 0; dt < nT && (int)bounds.size() < CA_MAX_GROUPS; dt += 1 + (int)(rng() % 2)) bounds.push_back(dt);
  std::vector<ca_group> found(bounds.size());
  for (int pattern = 0; pattern < 3; ++pattern) {
    double recall = -1, kept = -1;
    CHECK(compact_attn_search_head(L, mass.data(), bounds.data(), (int32_t)bounds.size(), 0.8, 0.9, pattern, found.data(), &recall,
                                   &kept) == CA_OK);
    CHECK(recall >= 0.0 && recall <= 1.0 + 1e-12 && kept >= 0.0 && kept <= 1.0);  // pairs beyond the last group may start it below tau
    ca_head hd{(int32_t)found.size(), 0, found.data()};
    std::vector<ca_head> same(p.num_heads, hd);
    ca_layout* from_search = nullptr;
    CHECK(compact_attn_build_layout(&p, same.data(), &from_search) == CA_OK);
    compact_attn_free_layout(from_search);
  }
  mass[0] = -1.f;
  CHECK(compact_attn_search_head(L, mass.data(), bounds.data(), (int32_t)bounds.size(), 0.8, 0.9, 2, found.data(), nullptr,
                                 nullptr) == CA_ERR_INVALID_ARG);

  // compute entry points: everything the host can refuse is refused before any device call
  const uintptr_t base = 1u << 20;
  CHECK(compact_attn_forward((void*)(base + 1), (void*)base, (void*)base, L, (void*)(base * 4), nullptr) != CA_OK);
  CHECK(compact_attn_forward((void*)base, (void*)base, (void*)base, L, (void*)base, nullptr) != CA_OK);
  CHECK(compact_attn_permute((void*)base, (void*)base, L, 0, nullptr) == CA_ERR_INVALID_ARG);
  CHECK(compact_attn_permute((void*)base, (void*)(base * 64), L, 7, nullptr) == CA_ERR_INVALID_ARG);

  compact_attn_free_layout(merged);
  compact_attn_free_layout(other);
  compact_attn_free_layout(copy);
  compact_attn_free_layout(L);
}

}  // namespace

int main() {
  std::mt19937 rng(2508);
  const ca_problem cases[] = {
      //  T   H   W  tt th tw text batch heads D  dtype    scale
      {4, 8, 8, 1, 4, 4, 0, 1, 2, 64, CA_F32, 0.f},
      {5, 13, 20, 2, 8, 8, 128, 1, 3, 128, CA_BF16, 0.f},    // padded T and H, one text tile
      {3, 13, 20, 1, 8, 8, 64, 2, 4, 128, CA_BF16, 0.05f},   // 64-token tiles, head dim 128: query-tile pairs
      {3, 9, 17, 1, 8, 8, 0, 1, 2, 64, CA_BF16, 0.f},        // padded H and W
      {7, 5, 3, 2, 2, 4, 16, 1, 5, 32, CA_F32, 0.f},         // odd everything
      {1, 1, 1, 1, 1, 1, 0, 1, 1, 8, CA_BF16, 0.f},          // a single token
      {9, 33, 35, 2, 8, 8, 256, 1, 6, 128, CA_BF16, 0.f},
      {8, 64, 64, 1, 8, 8, 0, 1, 8, 64, CA_BF16, 0.f},       // 4096 rows: the tail of the launch is drawn dynamically
      {6, 64, 64, 1, 8, 8, 64, 1, 24, 128, CA_BF16, 0.f},    // the same for query-tile pairs
  };
  for (const ca_problem& p : cases)
    for (int rep = 0; rep < 3; ++rep) run_case(rng, p);
  check_split_function();

  // malformed problems and heads
  ca_layout* L = nullptr;
  ca_problem bad = cases[0];
  bad.n_text = 5;
  ca_head none{0, 0, nullptr};
  std::vector<ca_head> two(2, none);
  CHECK(compact_attn_build_layout(&bad, two.data(), &L) == CA_ERR_INVALID_ARG && L == nullptr);
  ca_group unordered[2] = {{2, {0, 0}, {-1, -1}}, {1, {0, 0}, {-1, -1}}};
  two[0] = ca_head{2, 0, unordered};
  CHECK(compact_attn_build_layout(&cases[0], two.data(), &L) == CA_ERR_INVALID_ARG);
  two[0] = ca_head{CA_MAX_GROUPS + 1, 0, unordered};
  CHECK(compact_attn_build_layout(&cases[0], two.data(), &L) == CA_ERR_INVALID_ARG);
  CHECK(compact_attn_build_layout(nullptr, two.data(), &L) == CA_ERR_INVALID_ARG);
  compact_attn_free_layout(nullptr);

  if (failures) {
    std::printf("%d check(s) failed\n", failures);
    return 1;
  }
  std::printf("host ABI checks passed under the sanitizers\n");
  return 0;
}
