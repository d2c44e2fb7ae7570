"""Tile-level keep rule and sparse layout (oracle side; test infrastructure).

What is computed (Sec. 4.1).  Each head owns a list of frame-distance groups.
A group is `(max_dt, window_a, window_b)`; a window is `(rh, rw)`, radii in
tiles along the height and width axes, and is absent when a radius is
negative.  For a query tile (qt, qh, qw) and a key tile (kt, kh, kw):

  * dt = |kt - qt| selects the first group with dt <= max_dt (groups have
    strictly increasing max_dt).  No such group: the key tile is dropped.
  * the key tile is kept iff it lies in window a or in window b, a window
    being the query-centred box |kh - qh| <= rh and |kw - qw| <= rw
    (Eq. 1 is one such box; Eq. 2 is the union of two; a box at least as
    large as the tile grid is the global pattern of Sec. 3.2).  Boxes are
    clipped by the grid, never re-centred.
  * text tiles are kept by every query tile, and a text query tile keeps
    every tile.

Readings taken where the paper is silent: radii in tile units, absolute
distance between tile-frame indices, ascending tile ids inside a row.

Variant (not in the paper's equations; the sliding-tile scheme it builds on
does this): a `ClampedHead` keeps every window at its full 2r+1 tiles near a
border by moving the window's centre inward, to min(max(q, r), L-1-r) on an
axis of L tiles; a window of 2r+1 >= L tiles covers the whole axis.

Three independent formulations live here so that they can be checked against
each other: `keep_pair` (the rule on one pair), `kept_tiles` (enumeration of
the two clipped boxes per key frame) and `row_count_closed_form`.  `keep_mask`
evaluates the pair rule on coordinate arrays of all tile pairs of a head at
once, for full-size grids where a loop over pairs would take hours; it is
pinned to the other three.
"""
import numpy as np

from .geometry import Geometry


def window_present(win):
    return win[0] >= 0 and win[1] >= 0


class ClampedHead(tuple):
    """A head (tuple of groups) whose windows are moved inward at the border instead of clipped."""


def is_clamped(head):
    return isinstance(head, ClampedHead)


def in_window(q, k, radius, length, clamped):
    """Is position k inside the window of a query at position q on an axis of `length` tiles?"""
    if not clamped:
        return abs(k - q) <= radius
    if 2 * radius + 1 >= length:
        return True
    return abs(k - min(max(q, radius), length - 1 - radius)) <= radius


def check_head(head):
    """Validate one head's group list; returns it as a tuple of plain tuples."""
    out = []
    last = -1
    for grp in head:
        max_dt, a, b = grp
        if max_dt <= last:
            raise ValueError("max_dt must be non-negative and strictly increasing")
        last = max_dt
        out.append((int(max_dt), (int(a[0]), int(a[1])), (int(b[0]), int(b[1]))))
    return ClampedHead(out) if is_clamped(head) else tuple(out)


def group_of(head, dt):
    """First group whose max_dt covers the tile-frame distance dt, or None."""
    for grp in head:
        if dt <= grp[0]:
            return grp
    return None


def keep_pair(geom: Geometry, head, q_tile, k_tile):
    """The keep rule evaluated on a single (query tile, key tile) pair."""
    if q_tile >= geom.n_vid or k_tile >= geom.n_vid:
        return True  # text rows keep everything; text columns are always kept
    qt, qh, qw = geom.tile_coords(q_tile)
    kt, kh, kw = geom.tile_coords(k_tile)
    grp = group_of(head, abs(kt - qt))
    if grp is None:
        return False
    c = is_clamped(head)
    for win in (grp[1], grp[2]):
        if not window_present(win):
            continue
        if in_window(qh, kh, win[0], geom.nH, c) and in_window(qw, kw, win[1], geom.nW, c):
            return True
    return False


def keep_mask_bruteforce(geom: Geometry, heads):
    """bool[num_heads, n, n] from the pair rule; a triple loop, tiny grids only."""
    mask = np.zeros((len(heads), geom.n, geom.n), dtype=bool)
    for h, head in enumerate(heads):
        head = check_head(head)
        for q in range(geom.n):
            for k in range(geom.n):
                mask[h, q, k] = keep_pair(geom, head, q, k)
    return mask


def keep_mask(geom: Geometry, head):
    """bool[n, n] of one head: mask[q, k] = the pair rule of Sec. 4.1 for query tile q and key tile k,
    evaluated on arrays of tile coordinates (every pair at once instead of one pair per call)."""
    clamped = is_clamped(head)
    head = check_head(head)
    n, nv = geom.n, geom.n_vid
    ids = np.arange(nv)
    w = ids % geom.nW
    h = (ids // geom.nW) % geom.nH
    t = ids // (geom.nW * geom.nH)

    def axis_inside(pos, radius, length):
        q, k = pos[:, None], pos[None, :]
        if not clamped:
            return np.abs(k - q) <= radius
        if 2 * radius + 1 >= length:
            return np.ones((nv, nv), dtype=bool)
        centre = np.minimum(np.maximum(q, radius), length - 1 - radius)
        return np.abs(k - centre) <= radius

    dt = np.abs(t[None, :] - t[:, None])
    video = np.zeros((nv, nv), dtype=bool)
    decided = np.zeros((nv, nv), dtype=bool)          # pairs whose frame distance an earlier group covers
    for max_dt, win_a, win_b in head:
        mine = (dt <= max_dt) & ~decided
        decided |= dt <= max_dt
        inside = np.zeros((nv, nv), dtype=bool)
        for win in (win_a, win_b):
            if window_present(win):
                inside |= axis_inside(h, win[0], geom.nH) & axis_inside(w, win[1], geom.nW)
        video |= mine & inside
    mask = np.ones((n, n), dtype=bool)                 # text rows keep everything, text columns are always kept
    mask[:nv, :nv] = video
    return mask


def _clipped_box(center, radius, length):
    """Inclusive index range of |i - center| <= radius inside [0, length)."""
    return max(center - radius, 0), min(center + radius, length - 1)


def _moved_box(center, radius, length):
    """Inclusive index range of a window of 2*radius+1 tiles that contains `center` and stays inside
    [0, length): pushed right from a negative start, pushed left from an overhanging end."""
    if 2 * radius + 1 >= length:
        return 0, length - 1
    lo, hi = center - radius, center + radius
    if lo < 0:
        lo, hi = 0, 2 * radius
    if hi > length - 1:
        lo, hi = length - 1 - 2 * radius, length - 1
    return lo, hi


def kept_tiles(geom: Geometry, head, q_tile):
    """Ascending int32 array of key tiles kept by `q_tile` under `head`.

    Second formulation: for each key tile-frame, list the tiles of the two
    clipped boxes and take their union.
    """
    if q_tile >= geom.n_vid:
        return np.arange(geom.n, dtype=np.int32)
    head = check_head(head)
    qt, qh, qw = geom.tile_coords(q_tile)
    kept = []
    for kt in range(geom.nT):
        grp = group_of(head, abs(kt - qt))
        if grp is None:
            continue
        frame = set()
        for win in (grp[1], grp[2]):
            if not window_present(win):
                continue
            box = _moved_box if is_clamped(head) else _clipped_box
            h0, h1 = box(qh, win[0], geom.nH)
            w0, w1 = box(qw, win[1], geom.nW)
            for kh in range(h0, h1 + 1):
                for kw in range(w0, w1 + 1):
                    frame.add(geom.tile_id(kt, kh, kw))
        kept.extend(sorted(frame))
    kept.extend(range(geom.n_vid, geom.n))
    return np.asarray(kept, dtype=np.int32)


def build_csr(geom: Geometry, heads):
    """Per head: (row_ptr int64[n+1], col_idx int32[nnz]) with ascending columns."""
    out = []
    for head in heads:
        rows = [kept_tiles(geom, head, q) for q in range(geom.n)]
        row_ptr = np.zeros(geom.n + 1, dtype=np.int64)
        row_ptr[1:] = np.cumsum([len(r) for r in rows])
        col_idx = np.concatenate(rows).astype(np.int32) if rows else np.zeros(0, np.int32)
        out.append((row_ptr, col_idx))
    return out


def _range_1d(q, radius, length, clamped):
    """(lo, hi) of a window on one axis: clipped around q, or of full size 2r+1 moved inward."""
    if clamped:
        size = min(2 * radius + 1, length)
        lo = min(max(q - radius, 0), length - size)
        return lo, lo + size - 1
    return max(q - radius, 0), min(q + radius, length - 1)


def _overlap(r1, r2):
    return max(0, min(r1[1], r2[1]) - max(r1[0], r2[0]) + 1)


def row_count_closed_form(geom: Geometry, head, q_tile):
    """Number of kept key tiles of a row by inclusion-exclusion on the two boxes: |A| + |B| - |A and B|,
    every box a product of two index ranges (written without the helper the enumeration uses)."""
    if q_tile >= geom.n_vid:
        return geom.n
    head = check_head(head)
    c = is_clamped(head)
    qt, qh, qw = geom.tile_coords(q_tile)
    total = geom.n_txt
    for kt in range(geom.nT):
        grp = group_of(head, abs(kt - qt))
        if grp is None:
            continue
        boxes = [(_range_1d(qh, w[0], geom.nH, c), _range_1d(qw, w[1], geom.nW, c)) for w in (grp[1], grp[2]) if window_present(w)]
        for hr, wr in boxes:
            total += _overlap(hr, hr) * _overlap(wr, wr)
        if len(boxes) == 2:
            total -= _overlap(boxes[0][0], boxes[1][0]) * _overlap(boxes[0][1], boxes[1][1])
    return total


def row_counts(geom: Geometry, heads):
    """int64[num_heads, n] of closed-form row counts."""
    out = np.zeros((len(heads), geom.n), dtype=np.int64)
    for h, head in enumerate(heads):
        for q in range(geom.n):
            out[h, q] = row_count_closed_form(geom, head, q)
    return out


def work_order(counts):
    """Order in which (head, query tile) rows are handed to the device.

    Rows with the most kept tiles go first so that long rows do not land at
    the tail of the launch; ties keep ascending (head, tile) order.  `counts`
    is int[num_heads, n]; the result is int32[num_heads * n] of flat row ids
    head * n + tile.  (Not in the paper: a scheduling choice of this build.)
    """
    flat = np.asarray(counts).reshape(-1)
    return np.argsort(-flat, kind="stable").astype(np.int32)


def sparsity(geom: Geometry, heads):
    """Fraction of dropped tile pairs over num_heads * n^2 (padded grid, text included)."""
    kept = int(row_counts(geom, heads).sum())
    return 1.0 - kept / (len(heads) * geom.n * geom.n)


def mask_similarity(mask_a, mask_b):
    """Sim(M_A, M_B) of Eq. 3: |A and B| / |A or B| for two binary masks."""
    a = np.asarray(mask_a, dtype=bool)
    b = np.asarray(mask_b, dtype=bool)
    union = np.logical_or(a, b).sum()
    return 1.0 if union == 0 else float(np.logical_and(a, b).sum()) / float(union)


def csr_of_mask(mask):
    """(row_ptr int64[n+1], col_idx int32[nnz]) of one head's boolean tile mask [n, n], columns ascending."""
    mask = np.asarray(mask, dtype=bool)
    counts = mask.sum(axis=1)
    row_ptr = np.zeros(mask.shape[0] + 1, dtype=np.int64)
    row_ptr[1:] = np.cumsum(counts)
    col_idx = np.nonzero(mask)[1].astype(np.int32)
    return row_ptr, col_idx


def mask_of_csr(n, row_ptr, col_idx):
    """Boolean [n, n] mask of one head's CSR."""
    mask = np.zeros((n, n), dtype=bool)
    for q in range(n):
        mask[q, col_idx[row_ptr[q]:row_ptr[q + 1]]] = True
    return mask


def union_masks(mask_a, mask_b):
    """Merge of two configurations (Sec. 4.2: configurations found for different prompts are
    merged by union, so that every region either of them needs is retained)."""
    return np.logical_or(np.asarray(mask_a, dtype=bool), np.asarray(mask_b, dtype=bool))



def pair_table(geom: Geometry, masks):
    """Pairs of query tiles that share a workgroup, in launch order (a scheduling choice of this
    build, not in the paper; the attention result does not depend on it).

    `masks` is bool[num_heads, n, n].  In every head each video tile with an even coordinate along
    one grid axis is paired with its neighbour at that coordinate + 1 (no partner at the end of an
    odd extent); the axis is the one whose pairs have the smallest total union of kept key tiles,
    among the axes with at least two tiles, tried in the order w, h, t with the first minimum
    winning (w, all single, if no axis has two tiles).  Text tiles pair up in id order.  The pairs
    of all heads are sorted by descending union size, ties keeping the order (head, first tile).
    Returns int32[num_pairs, 2] of row ids head * n + tile, -1 for a missing partner.
    """
    masks = np.asarray(masks, dtype=bool)
    n = geom.n
    extents = {"w": geom.nW, "h": geom.nH, "t": geom.nT}

    def video_pairs(axis):
        out = []
        for t in range(geom.nT):
            for h in range(geom.nH):
                for w in range(geom.nW):
                    c = {"t": t, "h": h, "w": w}
                    if c[axis] % 2:
                        continue
                    first = (t * geom.nH + h) * geom.nW + w
                    c[axis] += 1
                    second = (c["t"] * geom.nH + c["h"]) * geom.nW + c["w"] if c[axis] < extents[axis] else -1
                    out.append((first, second))
        return out

    def walked(mask, pair):
        a, b = pair
        return int(mask[a].sum()) if b < 0 else int(np.logical_or(mask[a], mask[b]).sum())

    entries = []
    for hd in range(masks.shape[0]):
        candidates = [ax for ax in ("w", "h", "t") if extents[ax] >= 2] or ["w"]
        costs = [sum(walked(masks[hd], p) for p in video_pairs(ax)) for ax in candidates]
        axis = candidates[int(np.argmin(costs))]
        pairs = video_pairs(axis)
        for a in range(geom.n_vid, n, 2):
            pairs.append((a, a + 1 if a + 1 < n else -1))
        for a, b in pairs:
            entries.append((walked(masks[hd], (a, b)), hd * n + a, -1 if b < 0 else hd * n + b))
    order = sorted(range(len(entries)), key=lambda i: -entries[i][0])  # sorted() is stable
    return np.array([[entries[i][1], entries[i][2]] for i in order], dtype=np.int32).reshape(-1, 2)


def pair_walks(masks, pairs):
    """For every pair of `pair_table`: the key tiles either of its rows keeps, ascending, with who
    keeps them.  Returns (walk_ptr int64[num_pairs + 1], tiles int32, in_first bool, in_second bool)."""
    masks = np.asarray(masks, dtype=bool)
    n = masks.shape[1]
    flat = masks.reshape(-1, n)
    ptr, tiles, first, second = [0], [], [], []
    for a, b in np.asarray(pairs):
        ra = flat[a]
        rb = flat[b] if b >= 0 else np.zeros(n, dtype=bool)
        ids = np.nonzero(ra | rb)[0]
        tiles.append(ids)
        first.append(ra[ids])
        second.append(rb[ids])
        ptr.append(ptr[-1] + len(ids))
    cat = lambda parts, dt: np.concatenate(parts).astype(dt) if parts else np.zeros(0, dtype=dt)
    return np.asarray(ptr, dtype=np.int64), cat(tiles, np.int32), cat(first, bool), cat(second, bool)
