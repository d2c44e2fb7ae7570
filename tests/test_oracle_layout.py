"""Pins for the oracle's keep rule, CSR builder, row counts and work order.

None of these touch the HIP library.  Each test checks the oracle against
something it does not itself define: hand-worked tile sets, the pair rule by
brute force, inclusion-exclusion counts, special cases with known answers.
"""
import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

from oracle.geometry import Geometry
from oracle import layout as L
from workloads import get_workload

ABSENT = (-1, -1)


def _geom(wl):
    return Geometry(wl.T, wl.H, wl.W, *wl.tile, wl.n_text)


def test_hand_worked_3x3_single_frame():
    # one frame, 3x3 tiles (ids row-major):  0 1 2 / 3 4 5 / 6 7 8
    g = Geometry(1, 3, 3, 1, 1, 1)
    local1 = [(0, (1, 1), ABSENT)]
    assert L.kept_tiles(g, local1, 4).tolist() == [0, 1, 2, 3, 4, 5, 6, 7, 8]
    assert L.kept_tiles(g, local1, 0).tolist() == [0, 1, 3, 4]          # clipped, not re-centred
    assert L.kept_tiles(g, local1, 5).tolist() == [1, 2, 4, 5, 7, 8]
    cross0 = [(0, (0, 2), (2, 0))]                                      # full row + full column
    assert L.kept_tiles(g, cross0, 4).tolist() == [1, 3, 4, 5, 7]
    assert L.kept_tiles(g, cross0, 0).tolist() == [0, 1, 2, 3, 6]
    assert L.kept_tiles(g, cross0, 8).tolist() == [2, 5, 6, 7, 8]
    wide_only = [(0, (0, 1), ABSENT)]                                   # rh=0, rw=1: same row, +-1 column
    assert L.kept_tiles(g, wide_only, 4).tolist() == [3, 4, 5]          # an rh/rw swap would give [1,4,7]


def test_hand_worked_frame_groups():
    # 4 frames of 1x2 tiles: ids 2*t + w
    g = Geometry(4, 1, 2, 1, 1, 1)
    head = [(0, (0, 1), ABSENT), (2, (0, 0), ABSENT)]   # same frame: both tiles; |dt| in 1..2: own column; dt 3: dropped
    assert L.kept_tiles(g, head, 0).tolist() == [0, 1, 2, 4]
    assert L.kept_tiles(g, head, 3).tolist() == [1, 2, 3, 5, 7]
    assert L.kept_tiles(g, head, 7).tolist() == [3, 5, 6, 7]
    # a group with both windows absent expresses "skip nearby frames"
    far = [(0, (0, 0), ABSENT), (1, ABSENT, ABSENT), (3, (0, 1), ABSENT)]
    assert L.kept_tiles(g, far, 0).tolist() == [0, 4, 5, 6, 7]


def test_text_tiles_always_kept_and_text_rows_dense():
    g = Geometry(2, 2, 2, 1, 2, 2, n_text=8)            # 2 video tiles of 4 tokens + 2 text tiles
    head = [(0, (0, 0), ABSENT)]
    assert g.n == 4 and g.n_vid == 2
    assert L.kept_tiles(g, head, 0).tolist() == [0, 2, 3]
    assert L.kept_tiles(g, head, 1).tolist() == [1, 2, 3]
    assert L.kept_tiles(g, head, 2).tolist() == [0, 1, 2, 3]
    assert L.kept_tiles(g, head, 3).tolist() == [0, 1, 2, 3]


def test_config1_printed_rows_and_nnz():
    wl = get_workload("cfg1")
    g = _geom(wl)
    assert (g.nT, g.nH, g.nW, g.B, g.n) == (4, 2, 2, 16, 16)
    assert L.kept_tiles(g, wl.heads[0], 0).tolist() == list(range(8))
    assert L.kept_tiles(g, wl.heads[1], 0).tolist() == [0, 1, 2, 4, 5, 6, 8, 9, 10, 12, 13, 14]
    assert L.kept_tiles(g, wl.heads[1], 5).tolist() == [0, 1, 3, 4, 5, 7, 8, 9, 11, 12, 13, 15]
    csr = L.build_csr(g, wl.heads)
    assert [int(rp[-1]) for rp, _ in csr] == [160, 192]
    assert abs(L.sparsity(g, wl.heads) - 0.3125) < 1e-12


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_small_configs_bruteforce_equals_builder(name):
    wl = get_workload(name)
    g = _geom(wl)
    mask = L.keep_mask_bruteforce(g, wl.heads)
    csr = L.build_csr(g, wl.heads)
    counts = L.row_counts(g, wl.heads)
    for h, (row_ptr, col_idx) in enumerate(csr):
        assert int(row_ptr[-1]) == wl.expected_nnz[h]
        for q in range(g.n):
            cols = col_idx[row_ptr[q]:row_ptr[q + 1]]
            assert np.array_equal(cols, np.nonzero(mask[h, q])[0])
            assert counts[h, q] == len(cols)


@pytest.mark.parametrize("name", ["cfg3", "cfg4-S50", "cfg4-S65", "cfg4-S80", "cfg5"])
def test_large_configs_closed_form_nnz_matches_table(name):
    wl = get_workload(name)
    g = _geom(wl)
    counts = L.row_counts(g, wl.heads)
    assert tuple(int(c) for c in counts.sum(axis=1)) == wl.expected_nnz
    # a few rows enumerated in full, against the pair rule
    rng = np.random.default_rng(7)
    for h in rng.choice(wl.num_heads, 3, replace=False):
        for q in list(rng.choice(g.n, 3, replace=False)) + [0, g.n - 1]:
            cols = L.kept_tiles(g, wl.heads[h], int(q))
            assert len(cols) == counts[h, q]
            brute = [k for k in range(g.n) if L.keep_pair(g, L.check_head(wl.heads[h]), int(q), k)]
            assert cols.tolist() == brute


def test_padded_shapes_of_configs():
    shapes = {"cfg2": (128, 8192), "cfg3": (1260, 80640), "cfg4-S65": (1022, 130816), "cfg5": (1920, 245760)}
    for name, (n, n_pad) in shapes.items():
        g = _geom(get_workload(name))
        assert (g.n, g.N_pad) == (n, n_pad)


def test_full_window_keeps_everything_and_identity_keeps_self():
    g = Geometry(3, 5, 7, 1, 2, 3, n_text=0)
    full = [(g.nT - 1, (g.nH - 1, g.nW - 1), ABSENT)]
    ident = [(0, (0, 0), ABSENT)]
    for q in range(g.n):
        assert L.kept_tiles(g, full, q).tolist() == list(range(g.n))
        assert L.kept_tiles(g, ident, q).tolist() == [q]
    assert L.sparsity(g, [full]) == 0.0


def test_invalid_heads_rejected():
    with pytest.raises(ValueError):
        L.check_head([(2, (0, 0), ABSENT), (2, (1, 1), ABSENT)])
    with pytest.raises(ValueError):
        L.check_head([(3, (0, 0), ABSENT), (1, (1, 1), ABSENT)])
    with pytest.raises(ValueError):
        L.check_head([(-1, (0, 0), ABSENT)])


_win = st.tuples(st.integers(-1, 4), st.integers(-1, 4))


@st.composite
def _cases(draw):
    tt, th, tw = draw(st.integers(1, 2)), draw(st.integers(1, 3)), draw(st.integers(1, 3))
    T, H, W = draw(st.integers(1, 5)), draw(st.integers(1, 7)), draw(st.integers(1, 7))
    n_txt = draw(st.integers(0, 2))
    g = Geometry(T, H, W, tt, th, tw, n_text=n_txt * tt * th * tw)
    n_groups = draw(st.integers(0, 3))
    dts = sorted(draw(st.sets(st.integers(0, 5), min_size=n_groups, max_size=n_groups)))
    head = [(dt, draw(_win), draw(_win)) for dt in dts]
    return g, head


@settings(max_examples=120, deadline=None)
@given(_cases())
def test_three_formulations_agree(case):
    g, head = case
    mask = L.keep_mask_bruteforce(g, [head])[0]
    for q in range(g.n):
        cols = L.kept_tiles(g, head, q)
        assert np.array_equal(cols, np.nonzero(mask[q])[0])
        assert L.row_count_closed_form(g, head, q) == len(cols)
        assert np.all(np.diff(cols) > 0)


@settings(max_examples=120, deadline=None)
@given(_cases())
def test_three_formulations_agree_with_clamped_centres(case):
    g, head = case
    head = L.ClampedHead(head)
    mask = L.keep_mask_bruteforce(g, [head])[0]
    clipped = L.keep_mask_bruteforce(g, [list(head)])[0]
    assert np.all(mask >= clipped)                     # moving a window inward never loses a clipped tile
    for q in range(g.n):
        cols = L.kept_tiles(g, head, q)
        assert np.array_equal(cols, np.nonzero(mask[q])[0])
        assert L.row_count_closed_form(g, head, q) == len(cols)


def test_clamped_centres_hand_worked():
    # one frame, one tile row, six tile columns; radius 1 along w
    g = Geometry(1, 1, 6, 1, 1, 1, 0)
    clipped = [(0, (0, 1), ABSENT)]
    assert [L.kept_tiles(g, clipped, q).tolist() for q in range(6)] == [[0, 1], [0, 1, 2], [1, 2, 3], [2, 3, 4], [3, 4, 5], [4, 5]]
    clamped = L.ClampedHead(clipped)
    assert [L.kept_tiles(g, clamped, q).tolist() for q in range(6)] == [[0, 1, 2], [0, 1, 2], [1, 2, 3], [2, 3, 4], [3, 4, 5], [3, 4, 5]]
    # radius 3 needs 7 columns: longer than the axis, the window covers it from every query
    wide = L.ClampedHead([(0, (0, 3), ABSENT)])
    assert all(L.kept_tiles(g, wide, q).tolist() == list(range(6)) for q in range(6))
    # a window that fits has its full size in every row: (2*1+1) * (2*2+1) tiles per kept frame
    g = Geometry(3, 5, 7, 1, 1, 1, 0)
    head = L.ClampedHead([(1, (1, 2), ABSENT)])
    frames = lambda q: 2 if g.tile_coords(q)[0] in (0, g.nT - 1) else 3
    assert all(L.row_count_closed_form(g, head, q) == 15 * frames(q) for q in range(g.n))
    # two windows of one group get different centres near a border and still both contain the query
    head = L.ClampedHead([(0, (0, 2), (1, 0))])
    assert L.kept_tiles(g, head, 0).tolist() == [0, 1, 2, 3, 4, 7, 14]


def test_work_order_is_descending_count_with_stable_ties():
    rng = np.random.default_rng(3)
    counts = rng.integers(0, 6, size=(5, 37))
    order = L.work_order(counts)
    flat = counts.reshape(-1)
    ref = np.lexsort((np.arange(flat.size), -flat))
    assert np.array_equal(order, ref)
    assert np.all(np.diff(flat[order]) <= 0)
    assert sorted(order.tolist()) == list(range(flat.size))


def test_mask_similarity_closed_forms():
    a = np.zeros((4, 4), bool)
    b = np.zeros((4, 4), bool)
    a[:2] = True
    b[1:3] = True
    assert L.mask_similarity(a, a) == 1.0
    assert L.mask_similarity(a, ~a) == 0.0
    assert L.mask_similarity(a, b) == pytest.approx(4 / 12)


def test_mask_csr_conversions_and_union():
    g = Geometry(2, 6, 6, 1, 2, 2, 4)
    heads = [[(1, (1, 0), (0, 1))], [(0, (2, 2), (-1, -1))]]
    masks = L.keep_mask_bruteforce(g, heads)
    csr = L.build_csr(g, heads)
    for h in range(2):
        rp, ci = L.csr_of_mask(masks[h])
        assert np.array_equal(rp, csr[h][0]) and np.array_equal(ci, csr[h][1])
        assert np.array_equal(L.mask_of_csr(g.n, rp, ci), masks[h])
    u = L.union_masks(masks[0], masks[1])
    assert u.sum() == masks[0].sum() + masks[1].sum() - (masks[0] & masks[1]).sum()
    assert np.all(u >= masks[0]) and np.all(u >= masks[1])
    assert L.mask_similarity(masks[0], u) == masks[0].sum() / u.sum()


def _axis_cost_by_reshape(g, mask, axis):
    """Total union size of the video pairs along one tile-grid axis, computed on the reshaped mask."""
    n_vid = g.n_vid
    m = mask[:n_vid].reshape(g.nT, g.nH, g.nW, -1)
    m = np.moveaxis(m, axis, 0)
    even, odd = m[0::2], m[1::2]
    cost = int(np.logical_or(even[:odd.shape[0]], odd).sum())
    if even.shape[0] > odd.shape[0]:
        cost += int(even[-1].sum())
    return cost


def test_pair_table_hand_worked():
    # 2 x 2 tile grid in one frame.  Head 0 keeps a query's own tile row (both columns): tiles 0 and 1
    # have the same list, so pairing along w walks 2 tiles per pair and pairing along h walks 4.
    # Head 1 keeps the own column (both rows): the other way round.
    g = Geometry(1, 16, 16, 1, 8, 8, 0)
    masks = L.keep_mask_bruteforce(g, [[(0, (0, 1), (-1, -1))], [(0, (1, 0), (-1, -1))]])
    assert L.pair_table(g, masks).tolist() == [[0, 1], [2, 3], [4, 6], [5, 7]]
    # 1 x 3 grid plus three text tiles: the odd column and the odd text tile stay single; the text
    # rows keep all 6 tiles, the video rows their own tile and the text: unions 6, 6, 5 (tiles 0|1), 4
    g = Geometry(1, 8, 24, 1, 8, 8, 192)
    masks = L.keep_mask_bruteforce(g, [[(0, (0, 0), (-1, -1))]])
    assert L.pair_table(g, masks).tolist() == [[3, 4], [5, -1], [0, 1], [2, -1]]
    ptr, tiles, first, second = L.pair_walks(masks, L.pair_table(g, masks))
    assert ptr.tolist() == [0, 6, 12, 17, 21]
    assert tiles[12:17].tolist() == [0, 1, 3, 4, 5] and first[12:17].tolist() == [True, False, True, True, True]
    assert second[12:17].tolist() == [False, True, True, True, True]
    assert tiles[17:].tolist() == [2, 3, 4, 5] and first[17:].all() and not second[17:].any()
    # a single tile: nothing to pair with
    g = Geometry(1, 8, 8, 1, 8, 8, 0)
    assert L.pair_table(g, np.ones((1, 1, 1), bool)).tolist() == [[0, -1]]


def test_pair_table_invariants_on_random_masks():
    rng = np.random.default_rng(5)
    for (T, H, W, tile, n_text) in [(3, 16, 24, (1, 8, 8), 64), (4, 8, 8, (2, 4, 8), 0), (5, 12, 4, (4, 4, 4), 128)]:
        g = Geometry(T, H, W, *tile, n_text)
        masks = rng.random((3, g.n, g.n)) < 0.3
        # make the heads prefer different axes: head 0 gets lists that only depend on (h, w), head 1 on (t, w)
        t_of = np.arange(g.n_vid) // (g.nH * g.nW)
        hw_of = np.arange(g.n_vid) % (g.nH * g.nW)
        masks[0, :g.n_vid] = masks[0, hw_of]
        masks[1, :g.n_vid] = masks[1, (t_of * g.nH * g.nW + hw_of % g.nW)]
        pairs = L.pair_table(g, masks)
        rows = pairs[pairs >= 0]
        assert sorted(rows.tolist()) == list(range(3 * g.n))            # every row exactly once
        walked = []
        for a, b in pairs:
            hd, ta = divmod(int(a), g.n)
            if b >= 0:
                assert b // g.n == hd and b > a
            walked.append(int((masks[hd, ta] | masks[hd, b % g.n]).sum()) if b >= 0 else int(masks[hd, ta].sum()))
        assert np.all(np.diff(walked) <= 0)                             # longest unions first
        for hd in range(3):
            mine = pairs[(pairs[:, 0] // g.n) == hd]
            video = mine[mine[:, 0] % g.n < g.n_vid]
            strides = set(int(b - a) for a, b in video if b >= 0)
            assert len(strides) <= 1                                    # one axis per head
            cost = sum(w for w, (a, _) in zip(walked, pairs) if a // g.n == hd and a % g.n < g.n_vid)
            by_axis = [_axis_cost_by_reshape(g, masks[hd], ax) for ax in range(3)
                       if (g.nT, g.nH, g.nW)[ax] >= 2]
            assert cost == min(by_axis)                                 # and it is the cheapest one
        # head 0's lists do not depend on t, so neighbours along t share their list and that axis wins;
        # head 1's do not depend on h
        first = {hd: pairs[(pairs[:, 0] // g.n == hd) & (pairs[:, 1] >= 0) & (pairs[:, 0] % g.n < g.n_vid)][0] for hd in (0, 1)}
        assert int(first[0][1] - first[0][0]) == g.nH * g.nW
        if g.nH >= 2:
            assert int(first[1][1] - first[1][0]) == g.nW


# ---------------------------------------------------------------- keep_mask (all pairs of a head at once)

def test_keep_mask_hand_worked_rows():
    g = Geometry(1, 3, 3, 1, 1, 1)
    m = L.keep_mask(g, [(0, (0, 2), (2, 0))])                           # full row + full column
    assert np.nonzero(m[4])[0].tolist() == [1, 3, 4, 5, 7]
    assert np.nonzero(m[0])[0].tolist() == [0, 1, 2, 3, 6]
    m = L.keep_mask(g, [(0, (0, 1), ABSENT)])                           # rh=0, rw=1: an rh/rw swap gives [1,4,7]
    assert np.nonzero(m[4])[0].tolist() == [3, 4, 5]
    g = Geometry(4, 1, 2, 1, 1, 1)
    far = [(0, (0, 0), ABSENT), (1, ABSENT, ABSENT), (3, (0, 1), ABSENT)]   # the first covering group decides
    assert np.nonzero(L.keep_mask(g, far)[0])[0].tolist() == [0, 4, 5, 6, 7]
    g = Geometry(2, 2, 2, 1, 2, 2, n_text=8)
    m = L.keep_mask(g, [(0, (0, 0), ABSENT)])
    assert m.astype(int).tolist() == [[1, 0, 1, 1], [0, 1, 1, 1], [1, 1, 1, 1], [1, 1, 1, 1]]


@settings(max_examples=40, deadline=None)
@given(st.data())
def test_keep_mask_equals_pair_rule_on_random_heads(data):
    T, H, W = (data.draw(st.integers(1, 4)), data.draw(st.integers(1, 9)), data.draw(st.integers(1, 9)))
    tt, th, tw = (data.draw(st.integers(1, 2)), data.draw(st.integers(1, 3)), data.draw(st.integers(1, 3)))
    g = Geometry(T, H, W, tt, th, tw, n_text=data.draw(st.integers(0, 2)) * tt * th * tw)
    win = st.tuples(st.integers(-1, 4), st.integers(-1, 4))
    bounds = sorted(data.draw(st.sets(st.integers(0, 4), min_size=0, max_size=3)))
    head = [(b, data.draw(win), data.draw(win)) for b in bounds]
    if data.draw(st.booleans()):
        head = L.ClampedHead(head)
    assert np.array_equal(L.keep_mask(g, head), L.keep_mask_bruteforce(g, [head])[0])


@pytest.mark.parametrize("name", ["cfg2", "cfg3", "cfg4-S50", "cfg4-S65", "cfg4-S80", "cfg5"])
def test_keep_mask_reproduces_tabulated_counts_and_sampled_rows(name):
    wl = get_workload(name)
    g = _geom(wl)
    rng = np.random.default_rng(7)
    for h in range(wl.num_heads):
        m = L.keep_mask(g, wl.heads[h])
        assert int(m.sum()) == wl.expected_nnz[h]
        for q in rng.choice(g.n, 3, replace=False).tolist() + [0, g.n_vid - 1, g.n - 1]:
            assert np.array_equal(np.nonzero(m[q])[0], L.kept_tiles(g, wl.heads[h], q))
            assert int(m[q].sum()) == L.row_count_closed_form(g, wl.heads[h], q)
