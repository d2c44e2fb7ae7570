"""Attention mass per tile pair and the recall of a tile mask (oracle side; test infrastructure).

Sec. 4.2 searches masks by the recall they retain: the share of the full attention's
probability mass that falls on kept tile pairs.  The quantity behind it has a plain definition,
written out here in fp64 on natural-order tokens with no padding:

    P            = softmax_rows(scale * Q K^T)            over all real tokens of one head
    mass[a, b]   = sum_{i in tile a} sum_{j in tile b} P[i, j]
    recall(mask) = sum_{a,b: mask[a,b]} mass[a, b] / N_real

Every row of P sums to 1, so row a of `mass` sums to the number of real tokens of tile a and the
full mask has recall 1.
"""
import numpy as np

from .attention import default_scale, softmax_rows
from .geometry import Geometry


def tile_mass(geom: Geometry, q, k, scale=None):
    """q, k: [N_real, D] of one head, natural order -> fp64 [n, n]."""
    token_tile, _ = geom.token_tile_and_slot()
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    if scale is None:
        scale = default_scale(q.shape[-1])
    p = softmax_rows(scale * (q @ k.T))
    onehot = np.zeros((geom.N_real, geom.n), dtype=np.float64)
    onehot[np.arange(geom.N_real), token_tile] = 1.0
    return onehot.T @ p @ onehot


def mask_recall(mass, mask):
    """Share of the attention mass that a boolean tile mask [n, n] keeps."""
    mass = np.asarray(mass, dtype=np.float64)
    return float(mass[np.asarray(mask, dtype=bool)].sum() / mass.sum())


# ---------------------------------------------------------------------------------------------
# Mask search by boundary contraction (Sec. 4.2).
#
# The paper fixes the frame of the search and leaves its moves open: start from full coverage,
# tighten window boundaries step by step, always where the recall lost per unit of cost saved is
# lowest, independently per frame group, and stop on two thresholds: recall must stay >= tau, and a
# step whose (delta recall / delta cost) exceeds lambda is not taken.  The reading implemented here
# (and, separately, in the library):
#
#   * Only video-to-video tile pairs are searched (text tiles are always kept).  Recall and cost are
#     fractions of the head's video-to-video mass and of its n_vid^2 tile pairs, so the ratio of a
#     step is the attention density of what it removes relative to uniform attention (ratio 1).
#   * Inside a frame group the kept region is described on folded offsets (|dh|, |dw|) as a box
#     (h2, w1) with a notch cut from its far corner: cells with |dh| > h1 and |dw| > w2 are dropped.
#     That is exactly the union of the wide window (h1, w1) and the tall window (h2, w2) of Eq. 2.
#   * Moves of a group: A lower the box (h2-1), C narrow the box (w1-1), N0 open the notch at the
#     corner cell, N1 deepen the notch (h1-1), N2 widen the notch (w2-1), Z drop the whole group.
#     A move is a candidate when it removes at least one tile pair.
#   * A move is admissible when it keeps recall >= tau and its ratio is <= lambda.  One global greedy
#     loop: every live group proposes its cheapest admissible move (lowest ratio, ties by the order
#     A, C, N0, N1, N2, Z); a group without one is finished; the cheapest proposal overall (ties:
#     lowest group) is applied; the search ends when no group is live.
#   * "Independently across frame groups" (Sec. 4.2) is read as: every group owns its region and its
#     moves and shrinks on its own table of masses, but the recall floor tau is one budget of the
#     whole head (the paper states a single tau per search), so the groups' proposals compete in one
#     greedy order and a cheap step of one group can use up the recall a dearer step of another would
#     have needed.
#   * A mass with a negative or non-finite entry is an error.  A mass that sums to zero has no
#     recall to preserve or to lose: no move is admissible and full coverage is returned.
#   * Pattern families (the three columns of Table 3), each a restriction of the one before:
#       "dual"          everything above: per group a pair of windows;
#       "frame_groups"  per group ONE window: moves A, C and Z only;
#       "cubic"         one spatial window shared by all kept groups and a temporal radius, the
#                       sliding-tile cube the table starts from: a single region and the moves A and
#                       C applied to every kept group at once, Z dropping the outermost kept group.
# ---------------------------------------------------------------------------------------------

def fold_group_tables(geom: Geometry, mass, group_max_dt):
    """Per group g: R[g, i, j] mass and C[g, i, j] number of video tile pairs at folded offsets
    i = |dh|, j = |dw|, frame distance in (max_dt[g-1], max_dt[g]]; pairs beyond the last group are
    returned separately as (lost_mass, lost_pairs).  Accumulated in ascending (query, key) order."""
    nT, nH, nW, n_vid = geom.nT, geom.nH, geom.nW, geom.n_vid
    G = len(group_max_dt)
    R = np.zeros((G, nH, nW), dtype=np.float64)
    C = np.zeros((G, nH, nW), dtype=np.int64)
    lost_mass, lost_pairs = 0.0, 0
    t, h, w = np.unravel_index(np.arange(n_vid), (nT, nH, nW))
    bounds = np.asarray(group_max_dt)
    for q in range(n_vid):
        dt = np.abs(t - t[q])
        grp = np.searchsorted(bounds, dt, side="left")          # first group with dt <= max_dt
        i, j = np.abs(h - h[q]), np.abs(w - w[q])
        row = np.asarray(mass[q, :n_vid], dtype=np.float64)
        inside = grp < G
        np.add.at(R, (grp[inside], i[inside], j[inside]), row[inside])
        np.add.at(C, (grp[inside], i[inside], j[inside]), 1)
        for kk in np.nonzero(~inside)[0]:
            lost_mass += row[kk]
        lost_pairs += int((~inside).sum())
    return R, C, lost_mass, lost_pairs


class _Region:
    """Box (h2, w1) with a notch: cells (i, j) with i > h1 and j > w2 removed.  dropped = nothing kept."""

    def __init__(self, nH, nW):
        self.h1 = self.h2 = nH - 1
        self.w1 = self.w2 = nW - 1
        self.dropped = False

    def cells(self):
        if self.dropped:
            return set()
        return {(i, j) for i in range(self.h2 + 1) for j in range(self.w1 + 1) if not (i > self.h1 and j > self.w2)}

    def after(self, move):
        r = _Region(1, 1)
        r.h1, r.h2, r.w1, r.w2, r.dropped = self.h1, self.h2, self.w1, self.w2, self.dropped
        if move == "A":
            if r.h2 == 0:
                return None
            r.h2 -= 1
            r.h1 = min(r.h1, r.h2)
        elif move == "C":
            if r.w1 == 0:
                return None
            r.w1 -= 1
            r.w2 = min(r.w2, r.w1)
        elif move == "N0":
            if not (r.h1 == r.h2 and r.w2 == r.w1 and r.h2 > 0 and r.w1 > 0):
                return None
            r.h1 -= 1
            r.w2 -= 1
        elif move == "N1":
            if r.h1 == 0:
                return None
            r.h1 -= 1
        elif move == "N2":
            if r.w2 == 0:
                return None
            r.w2 -= 1
        elif move == "Z":
            r.dropped = True
        return r


MOVES = ("A", "C", "N0", "N1", "N2", "Z")
PATTERNS = ("cubic", "frame_groups", "dual")


def _search_cubic(geom, R, C, lost_mass, lost_pairs, group_max_dt, tau, lam):
    """One window (h, w) for the groups 0 .. k-1, the rest dropped; greedy over three joint moves."""
    total_mass = R.sum() + lost_mass
    total_pairs = int(C.sum()) + lost_pairs
    G = len(group_max_dt)
    h, w, k = geom.nH - 1, geom.nW - 1, G
    recall = float(R.sum() / total_mass) if total_mass > 0 else 1.0
    kept_pairs = int(C.sum())
    while k > 0:
        candidates = []
        if h > 0:
            candidates.append(((h - 1, w, k), [(g, h, j) for g in range(k) for j in range(w + 1)]))
        if w > 0:
            candidates.append(((h, w - 1, k), [(g, i, w) for g in range(k) for i in range(h + 1)]))
        candidates.append(((h, w, k - 1), [(k - 1, i, j) for i in range(h + 1) for j in range(w + 1)]))
        best = None
        for state, gone in candidates:
            pairs = sum(int(C[c]) for c in gone)
            if pairs == 0:
                continue
            d_mass = 0.0
            for c in sorted(gone):
                d_mass += R[c]
            d_recall = d_mass / total_mass if total_mass > 0 else 0.0
            ratio = d_recall / (pairs / total_pairs)
            if ratio > lam or recall - d_recall < tau:
                continue
            if best is None or ratio < best[0]:
                best = (ratio, state, d_recall, pairs)
        if best is None:
            break
        _, (h, w, k), d_recall, pairs = best
        recall -= d_recall
        kept_pairs -= pairs
    groups = [(int(group_max_dt[g]), (h, w) if g < k else (-1, -1), (-1, -1)) for g in range(G)]
    return groups, recall, kept_pairs / total_pairs


def search_head(geom: Geometry, mass, group_max_dt, tau, lam, pattern="dual"):
    """Returns (groups, recall, kept_pair_fraction): groups as [(max_dt, (rh, rw), (rh, rw)), ...] in the
    head format of oracle.layout, recall and kept fraction over video-to-video tile pairs."""
    if pattern not in PATTERNS:
        raise ValueError(f"pattern must be one of {PATTERNS}")
    video = np.asarray(mass, dtype=np.float64)[:geom.n_vid, :geom.n_vid]
    if not np.all(np.isfinite(video)) or np.any(video < 0):
        raise ValueError("attention mass must be finite and non-negative")
    R, C, lost_mass, lost_pairs = fold_group_tables(geom, mass, group_max_dt)
    if not (R.sum() + lost_mass > 0):          # nothing to rank the moves by: keep everything
        full = [(int(d), (geom.nH - 1, geom.nW - 1), (-1, -1)) for d in group_max_dt]
        total = int(C.sum()) + lost_pairs
        return full, 1.0, (int(C.sum()) / total if total else 1.0)
    if pattern == "cubic":
        return _search_cubic(geom, R, C, lost_mass, lost_pairs, group_max_dt, tau, lam)
    moves = MOVES if pattern == "dual" else ("A", "C", "Z")
    total_mass = R.sum() + lost_mass
    total_pairs = int(C.sum()) + lost_pairs
    G = len(group_max_dt)
    regions = [_Region(geom.nH, geom.nW) for _ in range(G)]
    live = [True] * G
    recall = float(R.sum() / total_mass) if total_mass > 0 else 1.0
    kept_pairs = int(C.sum())

    def proposal(g):
        best = None
        now = regions[g].cells()
        if regions[g].dropped:
            return None
        for move in moves:
            nxt = regions[g].after(move)
            if nxt is None:
                continue
            gone = now - nxt.cells()
            pairs = sum(int(C[g, i, j]) for (i, j) in gone)
            if pairs == 0:
                continue
            d_mass = 0.0
            for (i, j) in sorted(gone):
                d_mass += R[g, i, j]
            d_recall = d_mass / total_mass if total_mass > 0 else 0.0
            d_cost = pairs / total_pairs
            ratio = d_recall / d_cost
            if ratio > lam or recall - d_recall < tau:
                continue
            if best is None or ratio < best[0]:
                best = (ratio, move, nxt, d_recall, pairs)
        return best

    while True:
        choice = None
        for g in range(G):
            if not live[g]:
                continue
            p = proposal(g)
            if p is None:
                live[g] = False
                continue
            if choice is None or p[0] < choice[1][0]:
                choice = (g, p)
        if choice is None:
            break
        g, (ratio, move, nxt, d_recall, pairs) = choice
        regions[g] = nxt
        recall -= d_recall
        kept_pairs -= pairs

    groups = []
    for g in range(G):
        r = regions[g]
        if r.dropped:
            groups.append((int(group_max_dt[g]), (-1, -1), (-1, -1)))
        elif r.h1 == r.h2 or r.w1 == r.w2:      # no notch left: one window is enough
            groups.append((int(group_max_dt[g]), (r.h2, r.w1), (-1, -1)))
        else:
            groups.append((int(group_max_dt[g]), (r.h1, r.w1), (r.h2, r.w2)))
    return groups, recall, kept_pairs / total_pairs
