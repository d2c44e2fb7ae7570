// Mask search by boundary contraction (Sec. 4.2 of the paper), host side.
//
// Input is one head's attention mass per tile pair (compact_attn_tile_mass) and the frame-distance
// boundaries of the groups; output is one pair of windows per group.  The paper gives the frame
// (start from full coverage, tighten window boundaries where the recall lost per unit of cost
// saved is lowest, per frame group, two thresholds tau and lambda) and leaves the moves open;
// the reading taken here:
//   - Only video-to-video tile pairs take part; recall and cost are fractions of the head's
//     video-to-video mass and tile pairs, so a step's ratio (delta recall / delta cost) is the
//     attention density of what it removes relative to uniform attention.
//   - On folded offsets (|dh|, |dw|) a group keeps a box (h2, w1) minus a notch at its far corner
//     (cells with |dh| > h1 and |dw| > w2): exactly the union of a wide window (h1, w1) and a tall
//     window (h2, w2), the dual windows of Eq. 2.
//   - Moves: lower the box, narrow the box, open the notch at the corner cell, deepen it, widen it,
//     or drop the group.  A move must remove at least one tile pair, keep recall >= tau and have a
//     ratio <= lambda.  Every live group proposes its cheapest such move, the cheapest proposal
//     overall is applied, a group without a proposal is finished.  The groups shrink independently
//     (each on its own table, with its own region) but share the head's one recall budget tau, so
//     their proposals compete in a single greedy order.
//   - A negative or non-finite mass entry is an error; a mass that sums to zero leaves no recall to
//     rank moves by, so no move is admissible and full coverage is returned.
//   - Pattern families (the columns of Table 3): dual windows as above; frame groups with one
//     window each (no notch moves); a cubic window, i.e. one spatial window shared by all kept
//     groups plus a temporal radius (lower / narrow it in every kept group at once, or drop the
//     outermost kept group).
#include <cmath>
#include <cstdint>
#include <vector>

#include "layout.h"

namespace ca {
namespace {

struct Region {  // box (h2, w1) with the cells i > h1 && j > w2 removed
  int h1, h2, w1, w2;
  bool dropped;
  bool has(int i, int j) const { return !dropped && i <= h2 && j <= w1 && !(i > h1 && j > w2); }
};

enum Move { kLowerBox, kNarrowBox, kOpenNotch, kDeepenNotch, kWidenNotch, kDropGroup, kNumMoves };

bool apply(const Region& r, int move, Region* out) {
  Region n = r;
  switch (move) {
    case kLowerBox:
      if (n.h2 == 0) return false;
      n.h2 -= 1;
      if (n.h1 > n.h2) n.h1 = n.h2;
      break;
    case kNarrowBox:
      if (n.w1 == 0) return false;
      n.w1 -= 1;
      if (n.w2 > n.w1) n.w2 = n.w1;
      break;
    case kOpenNotch:
      if (!(n.h1 == n.h2 && n.w2 == n.w1 && n.h2 > 0 && n.w1 > 0)) return false;
      n.h1 -= 1;
      n.w2 -= 1;
      break;
    case kDeepenNotch:
      if (n.h1 == 0) return false;
      n.h1 -= 1;
      break;
    case kWidenNotch:
      if (n.w2 == 0) return false;
      n.w2 -= 1;
      break;
    default:
      n.dropped = true;
      break;
  }
  *out = n;
  return true;
}

struct Proposal {
  bool valid = false;
  double ratio = 0, d_recall = 0;
  int64_t pairs = 0;
  Region next{};
};

}  // namespace

int search_head_windows(const ca_layout& L, const float* mass, const int32_t* group_max_dt, int32_t num_groups, double tau,
                        double lambda, int32_t pattern, ca_group* groups_out, double* recall_out, double* kept_out) {
  const int nT = L.nT, nH = L.nH, nW = L.nW;
  const int64_t n = L.n, n_vid = L.n_vid;
  const int G = num_groups;
  // mass and pair count per (group, |dh|, |dw|), accumulated in ascending (query, key) order
  std::vector<double> R((size_t)G * nH * nW, 0.0);
  std::vector<int64_t> C((size_t)G * nH * nW, 0);
  double lost_mass = 0.0;
  int64_t lost_pairs = 0;
  std::vector<int> group_of_dt(nT, G);
  for (int dt = 0; dt < nT; ++dt)
    for (int g = 0; g < G; ++g)
      if (dt <= group_max_dt[g]) {
        group_of_dt[dt] = g;
        break;
      }
  for (int64_t q = 0; q < n_vid; ++q) {
    const int qw = (int)(q % nW), qh = (int)((q / nW) % nH), qt = (int)(q / ((int64_t)nW * nH));
    const float* row = mass + q * n;
    int64_t k = 0;
    for (int kt = 0; kt < nT; ++kt) {
      const int g = group_of_dt[kt > qt ? kt - qt : qt - kt];
      for (int kh = 0; kh < nH; ++kh) {
        const int i = kh > qh ? kh - qh : qh - kh;
        for (int kw = 0; kw < nW; ++kw, ++k) {
          const int j = kw > qw ? kw - qw : qw - kw;
          if (!(row[k] >= 0.0f) || std::isinf(row[k])) {
            set_error("attention mass of tile pair (%lld, %lld) is negative or not finite", (long long)q, (long long)k);
            return CA_ERR_INVALID_ARG;
          }
          if (g == G) {
            lost_mass += (double)row[k];
            ++lost_pairs;
          } else {
            const size_t cell = ((size_t)g * nH + i) * nW + j;
            R[cell] += (double)row[k];
            C[cell] += 1;
          }
        }
      }
    }
  }
  double kept_mass = 0.0;
  int64_t kept_pairs = 0;
  for (size_t c = 0; c < R.size(); ++c) {
    kept_mass += R[c];
    kept_pairs += C[c];
  }
  // kept_mass adds the cells in array order (group, |dh|, |dw| ascending)
  const double total_mass = kept_mass + lost_mass;
  const int64_t total_pairs = kept_pairs + lost_pairs;
  if (!(total_mass > 0)) {  // nothing to rank the moves by: keep everything
    for (int g = 0; g < G; ++g) groups_out[g] = ca_group{group_max_dt[g], ca_window{nH - 1, nW - 1}, ca_window{-1, -1}};
    if (recall_out) *recall_out = 1.0;
    if (kept_out) *kept_out = total_pairs > 0 ? (double)kept_pairs / (double)total_pairs : 1.0;
    return CA_OK;
  }
  double recall = kept_mass / total_mass;

  if (pattern == CA_PATTERN_CUBIC) {
    int h = nH - 1, w = nW - 1, k = G;
    while (k > 0) {
      // the three joint moves in the order lower, narrow, drop outermost; cells visited in ascending (g, i, j)
      bool have = false;
      double best_ratio = 0, best_d_recall = 0;
      int64_t best_pairs = 0;
      int best_move = -1;
      for (int move = 0; move < 3; ++move) {
        if ((move == 0 && h == 0) || (move == 1 && w == 0)) continue;
        int64_t pairs = 0;
        double d_mass = 0.0;
        const int g0 = move == 2 ? k - 1 : 0;
        for (int g = g0; g < k; ++g)
          for (int i = (move == 0 ? h : 0); i <= h; ++i)
            for (int j = (move == 1 ? w : 0); j <= w; ++j) {
              const size_t cell = ((size_t)g * nH + i) * nW + j;
              pairs += C[cell];
              d_mass += R[cell];
            }
        if (pairs == 0) continue;
        const double d_recall = d_mass / total_mass;
        const double ratio = d_recall / ((double)pairs / (double)total_pairs);
        if (ratio > lambda || recall - d_recall < tau) continue;
        if (!have || ratio < best_ratio) have = true, best_ratio = ratio, best_d_recall = d_recall, best_pairs = pairs, best_move = move;
      }
      if (!have) break;
      if (best_move == 0) --h;
      else if (best_move == 1) --w;
      else --k;
      recall -= best_d_recall;
      kept_pairs -= best_pairs;
    }
    for (int g = 0; g < G; ++g) {
      ca_group out{};
      out.max_dt = group_max_dt[g];
      out.a = g < k ? ca_window{h, w} : ca_window{-1, -1};
      out.b = ca_window{-1, -1};
      groups_out[g] = out;
    }
    if (recall_out) *recall_out = recall;
    if (kept_out) *kept_out = total_pairs > 0 ? (double)kept_pairs / (double)total_pairs : 1.0;
    return CA_OK;
  }
  const bool notch_moves = pattern == CA_PATTERN_DUAL;

  std::vector<Region> regions(G, Region{nH - 1, nH - 1, nW - 1, nW - 1, false});
  std::vector<char> live(G, 1);
  auto propose = [&](int g) {
    Proposal best;
    const Region& now = regions[g];
    if (now.dropped) return best;
    for (int move = 0; move < kNumMoves; ++move) {
      Region nxt;
      if (!notch_moves && (move == kOpenNotch || move == kDeepenNotch || move == kWidenNotch)) continue;
      if (!apply(now, move, &nxt)) continue;
      int64_t pairs = 0;
      double d_mass = 0.0;
      for (int i = 0; i <= now.h2; ++i)        // removed cells are added in ascending (i, j)
        for (int j = 0; j <= now.w1; ++j)
          if (now.has(i, j) && !nxt.has(i, j)) {
            const size_t cell = ((size_t)g * nH + i) * nW + j;
            pairs += C[cell];
            d_mass += R[cell];
          }
      if (pairs == 0) continue;
      const double d_recall = d_mass / total_mass;
      const double d_cost = (double)pairs / (double)total_pairs;
      const double ratio = d_recall / d_cost;
      if (ratio > lambda || recall - d_recall < tau) continue;
      if (!best.valid || ratio < best.ratio) {
        best.valid = true;
        best.ratio = ratio;
        best.d_recall = d_recall;
        best.pairs = pairs;
        best.next = nxt;
      }
    }
    return best;
  };
  for (;;) {
    int chosen = -1;
    Proposal choice;
    for (int g = 0; g < G; ++g) {
      if (!live[g]) continue;
      const Proposal p = propose(g);
      if (!p.valid) {
        live[g] = 0;
        continue;
      }
      if (chosen < 0 || p.ratio < choice.ratio) {
        chosen = g;
        choice = p;
      }
    }
    if (chosen < 0) break;
    regions[chosen] = choice.next;
    recall -= choice.d_recall;
    kept_pairs -= choice.pairs;
  }
  for (int g = 0; g < G; ++g) {
    const Region& r = regions[g];
    ca_group out{};
    out.max_dt = group_max_dt[g];
    if (r.dropped) {
      out.a = ca_window{-1, -1};
      out.b = ca_window{-1, -1};
    } else if (r.h1 == r.h2 || r.w1 == r.w2) {  // no notch left: one window is enough
      out.a = ca_window{r.h2, r.w1};
      out.b = ca_window{-1, -1};
    } else {
      out.a = ca_window{r.h1, r.w1};
      out.b = ca_window{r.h2, r.w2};
    }
    groups_out[g] = out;
  }
  if (recall_out) *recall_out = recall;
  if (kept_out) *kept_out = total_pairs > 0 ? (double)kept_pairs / (double)total_pairs : 1.0;
  return CA_OK;
}

}  // namespace ca
