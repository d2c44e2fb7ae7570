"""Pins for the oracle's tile mass and recall: closed forms and brute force."""
import numpy as np
import pytest

from oracle.geometry import Geometry
from oracle import attention as A
from oracle import layout as L
from oracle import search as S

ABSENT = (-1, -1)


def _tokens_per_tile(g):
    tok_tile, _ = g.token_tile_and_slot()
    return np.bincount(tok_tile, minlength=g.n)


def test_rows_sum_to_tile_population_and_full_mask_has_recall_one():
    g = Geometry(3, 5, 7, 1, 4, 4, 16)          # padded H and W, one text tile
    rng = np.random.default_rng(0)
    q, k = rng.standard_normal((2, g.N_real, 8))
    m = S.tile_mass(g, q, k)
    assert m.shape == (g.n, g.n) and np.all(m >= 0)
    assert np.allclose(m.sum(axis=1), _tokens_per_tile(g), atol=1e-10)
    assert abs(S.mask_recall(m, np.ones((g.n, g.n), bool)) - 1.0) < 1e-12
    assert S.mask_recall(m, np.zeros((g.n, g.n), bool)) == 0.0


def test_zero_queries_spread_mass_by_population():
    """Q = 0 makes every row of P uniform: mass[a, b] = |a| * |b| / N_real."""
    g = Geometry(2, 6, 5, 1, 4, 4, 0)
    rng = np.random.default_rng(1)
    k = rng.standard_normal((g.N_real, 8))
    m = S.tile_mass(g, np.zeros_like(k), k)
    pop = _tokens_per_tile(g)
    assert np.allclose(m, np.outer(pop, pop) / g.N_real, atol=1e-12)


def test_brute_force_on_a_tiny_grid_and_transposition_sensitivity():
    g = Geometry(1, 4, 4, 1, 2, 2, 0)
    rng = np.random.default_rng(2)
    q, k = rng.standard_normal((2, g.N_real, 4))
    tok_tile, _ = g.token_tile_and_slot()
    scale = 4 ** -0.5
    want = np.zeros((g.n, g.n))
    for i in range(g.N_real):
        s = [scale * float(np.dot(q[i], k[j])) for j in range(g.N_real)]
        mx = max(s)
        e = [np.exp(x - mx) for x in s]
        z = sum(e)
        for j in range(g.N_real):
            want[tok_tile[i], tok_tile[j]] += e[j] / z
    got = S.tile_mass(g, q, k)
    assert np.allclose(got, want, atol=1e-13)
    assert not np.allclose(got, got.T, atol=1e-3)           # a transposed operand would show


def test_recall_of_a_layout_equals_the_kept_probability():
    """Recall from the mass matrix equals the kept probability summed token by token."""
    g = Geometry(2, 6, 6, 1, 2, 2, 4)
    heads = [[(1, (1, 0), (0, 1))]]
    rng = np.random.default_rng(3)
    q, k = 1.5 * rng.standard_normal((2, g.N_real, 8))
    mask = L.keep_mask_bruteforce(g, heads)[0]
    m = S.tile_mass(g, q, k)
    tok_tile, _ = g.token_tile_and_slot()
    p = A.softmax_rows(8 ** -0.5 * (q @ k.T))
    kept = mask[tok_tile][:, tok_tile]
    assert abs(S.mask_recall(m, mask) - p[kept].sum() / g.N_real) < 1e-12


# ---------------------------------------------------------------- mask search (Sec. 4.2)

def _unit_tiles(nT, nH, nW):
    return Geometry(nT, nH, nW, 1, 1, 1, 0)             # one token per tile: masses are easy to write down


def _coords(g):
    return np.unravel_index(np.arange(g.n), (g.nT, g.nH, g.nW))


def test_search_recovers_a_local_window_and_drops_far_frames():
    g = _unit_tiles(4, 6, 8)
    t, h, w = _coords(g)
    keep = (np.abs(t[:, None] - t) <= 1) & (np.abs(h[:, None] - h) <= 1) & (np.abs(w[:, None] - w) <= 2)
    mass = keep / keep.sum(axis=1, keepdims=True)
    groups, recall, kept = S.search_head(g, mass, [0, 1, 3], 1.0 - 1e-12, 0.5)
    assert groups == [(0, (1, 2), ABSENT), (1, (1, 2), ABSENT), (3, ABSENT, ABSENT)]
    assert abs(recall - 1.0) < 1e-12
    assert kept == keep.sum() / g.n ** 2


def test_search_recovers_a_cross_as_two_windows():
    g = _unit_tiles(2, 6, 8)
    t, h, w = _coords(g)
    keep = (h[:, None] == h) | (w[:, None] == w)
    mass = keep / keep.sum(axis=1, keepdims=True)
    groups, recall, kept = S.search_head(g, mass, [1], 1.0 - 1e-12, 0.5)
    assert groups == [(1, (0, 7), (5, 0))]
    assert abs(recall - 1.0) < 1e-12 and kept == keep.sum() / g.n ** 2


def test_uniform_attention_is_left_alone_and_thresholds_bind():
    g = _unit_tiles(3, 4, 5)
    mass = np.full((g.n, g.n), 1.0 / g.n)
    groups, recall, kept = S.search_head(g, mass, [0, 2], 0.5, 0.9)      # every move has ratio 1 > lambda
    assert groups == [(0, (3, 4), ABSENT), (2, (3, 4), ABSENT)] and recall == 1.0 and kept == 1.0
    groups, recall, kept = S.search_head(g, mass, [0, 2], 0.75, 2.0)     # now only tau stops it
    assert 0.75 <= recall < 1.0 and abs(recall - kept) < 1e-12           # uniform: recall == kept share


def test_reported_recall_equals_the_recall_of_the_built_mask():
    """The search's own bookkeeping (folded offsets, clipped windows, frame groups) against the
    layout rule: build the mask from the groups it returns and measure its recall directly."""
    g = Geometry(5, 9, 7, 1, 2, 2, 0)                   # 5 x 5 x 4 tiles
    rng = np.random.default_rng(4)
    q, k = rng.standard_normal((2, g.N_real, 8))
    q *= 3.0
    k += 0.8 * np.repeat(rng.standard_normal((g.N_real // 7 + 1, 8)), 7, axis=0)[:g.N_real]
    mass = S.tile_mass(g, q, k)
    for tau, lam in ((0.9, 0.5), (0.6, 1.5), (0.99, 0.2)):
        groups, recall, kept = S.search_head(g, mass, [0, 1, 4], tau, lam)
        mask = L.keep_mask_bruteforce(g, [groups])[0]
        assert abs(S.mask_recall(mass, mask) - recall) < 1e-12
        assert abs(mask.sum() / g.n ** 2 - kept) < 1e-12
        assert recall >= tau
        assert all(a[0] <= b[0] and a[1] >= b[1] for _, a, b in groups if b != ABSENT)   # wide / tall roles


# ---------------------------------------------------------------- pattern families (the columns of Table 3)

def test_pattern_families_closed_forms():
    """A head whose exact support is known: a cross whose arms shrink with the frame distance.
    dual finds the support itself; one window per group needs the bounding box of each group's
    cross; a cube needs the bounding box of the widest group in every kept frame."""
    g = _unit_tiles(4, 6, 8)
    t, h, w = _coords(g)
    dt, dh, dw = np.abs(t[:, None] - t), np.abs(h[:, None] - h), np.abs(w[:, None] - w)
    near = (dt == 0) & (((dh == 0) & (dw <= 4)) | ((dw == 0) & (dh <= 3)))
    mid = (dt == 1) & (((dh == 0) & (dw <= 2)) | ((dw == 0) & (dh <= 1)))
    keep = near | mid
    mass = keep / keep.sum(axis=1, keepdims=True)
    bounds, tau, lam = [0, 1, 3], 1.0 - 1e-12, 0.5
    dual, r2, k2 = S.search_head(g, mass, bounds, tau, lam, "dual")
    assert dual == [(0, (0, 4), (3, 0)), (1, (0, 2), (1, 0)), (3, ABSENT, ABSENT)]
    fg, r1, k1 = S.search_head(g, mass, bounds, tau, lam, "frame_groups")
    assert fg == [(0, (3, 4), ABSENT), (1, (1, 2), ABSENT), (3, ABSENT, ABSENT)]
    cube, r0, k0 = S.search_head(g, mass, bounds, tau, lam, "cubic")
    assert cube == [(0, (3, 4), ABSENT), (1, (3, 4), ABSENT), (3, ABSENT, ABSENT)]
    assert abs(r0 - 1) < 1e-12 and abs(r1 - 1) < 1e-12 and abs(r2 - 1) < 1e-12
    assert k2 < k1 < k0 < 1.0                                            # each family strictly sparser here
    for groups, kept in ((dual, k2), (fg, k1), (cube, k0)):
        assert L.keep_mask_bruteforce(g, [groups])[0].sum() / g.n ** 2 == kept
    assert k2 == keep.sum() / g.n ** 2


def test_pattern_families_on_random_mass_report_their_own_mask():
    g = Geometry(5, 9, 7, 1, 2, 2, 0)
    rng = np.random.default_rng(6)
    q, k = rng.standard_normal((2, g.N_real, 8))
    q *= 3.0
    k += 0.8 * np.repeat(rng.standard_normal((g.N_real // 7 + 1, 8)), 7, axis=0)[:g.N_real]
    mass = S.tile_mass(g, q, k)
    for pattern in S.PATTERNS:
        for tau, lam in ((0.9, 0.5), (0.6, 1.5)):
            groups, recall, kept = S.search_head(g, mass, [0, 1, 2, 4], tau, lam, pattern)
            mask = L.keep_mask_bruteforce(g, [groups])[0]
            assert abs(S.mask_recall(mass, mask) - recall) < 1e-12 and abs(mask.sum() / g.n ** 2 - kept) < 1e-12
            assert recall >= tau
            if pattern != "dual":
                assert all(b == ABSENT for _, _, b in groups)
            if pattern == "cubic":
                live = [a for _, a, _ in groups if a != ABSENT]
                assert len(set(live)) <= 1                                # one window
                flags = [a != ABSENT for _, a, _ in groups]
                assert flags == sorted(flags, reverse=True)               # kept groups are the innermost ones
    with pytest.raises(ValueError):
        S.search_head(g, mass, [0], 0.9, 0.5, "spiral")


# ---------------------------------------------------------------- the paper's thresholds, worked by hand

def two_density_mass(g):
    """One frame of 6 x 6 unit tiles.  A tile pair at folded offset (|dh|, |dw|) lies in the core
    (max <= 1), in ring 1 (max == 2) or in ring 2 (max >= 3).  Pair counts per offset are
    (6-|dh|)(6-|dw|) times 2 per non-zero offset: core 36+60+60+100 = 256, ring 1 48+80+64+48+80 = 320,
    ring 2 the remaining 720 of 36^2 = 1296.  With 0.03 per ring-1 pair, 0.005 per ring-2 pair and
    (1296 - 320*0.03 - 720*0.005) / 256 = 5.0109375 per core pair the mean mass per pair is exactly 1,
    so a step's (delta recall / delta cost) is the mean mass per pair of what it removes: 0.005 for
    ring-2 cells, 0.03 for ring-1 cells, at least (0.03*64 + 0.005*96) / 160 = 0.015 for any row or
    column segment that contains a ring-1 cell (the least is cell (2,2) with the ring-2 cells behind
    it), and above 1 for anything that touches the core."""
    t, h, w = np.unravel_index(np.arange(g.n), (g.nT, g.nH, g.nW))
    far = np.maximum(np.abs(h[:, None] - h), np.abs(w[:, None] - w))
    mass = np.where(far <= 1, 5.0109375, np.where(far == 2, 0.03, 0.005))
    assert abs(mass.sum() - 1296.0) < 1e-9
    return mass


@pytest.mark.parametrize("pattern", ["frame_groups", "dual"])
def test_thresholds_of_the_paper_on_a_two_density_mass(pattern):
    """tau = 0.9 with lambda = 0.011 and 0.04 (the operating points of Table 3 and Sec. 6.2): the ring
    at 0.5 % of uniform density is cut at both, the ring at 3 % only at lambda = 0.04, the core never;
    recall stays at 256*5.0109375/1296 = 0.9898 or above, so tau does not bind."""
    g = _unit_tiles(1, 6, 6)
    mass = two_density_mass(g)
    groups, recall, kept = S.search_head(g, mass, [0], 0.9, 0.011, pattern)
    assert groups == [(0, (2, 2), ABSENT)]
    assert abs(recall - (1296 - 720 * 0.005) / 1296) < 1e-12 and kept == (256 + 320) / 1296
    groups, recall, kept = S.search_head(g, mass, [0], 0.9, 0.04, pattern)
    assert groups == [(0, (1, 1), ABSENT)]
    assert abs(recall - 256 * 5.0109375 / 1296) < 1e-12 and kept == 256 / 1296
    groups, recall, kept = S.search_head(g, mass, [0], 0.9, 0.004, pattern)     # below both rings: nothing is cut
    assert groups == [(0, (5, 5), ABSENT)] and recall == 1.0 and kept == 1.0


def competing_groups_mass():
    """Two frames of 1 x 2 unit tiles, groups at frame distance 0 and 1, total mass 100.  Per group and
    folded offset |dw| there are 4 tile pairs; masses per cell: group 0: 60 at |dw|=0, 6 at |dw|=1;
    group 1: 29 at |dw|=0, 5 at |dw|=1.  Narrowing group 0 loses recall 0.06 for cost 4/16 (ratio
    0.24); narrowing group 1 loses 0.05 (ratio 0.20).  With tau = 0.9 only one of them fits."""
    g = _unit_tiles(2, 1, 2)
    t, h, w = np.unravel_index(np.arange(g.n), (g.nT, g.nH, g.nW))
    dt, dw = np.abs(t[:, None] - t), np.abs(w[:, None] - w)
    mass = np.where(dt == 0, np.where(dw == 0, 15.0, 1.5), np.where(dw == 0, 7.25, 1.25))
    assert mass.sum() == 100.0
    return g, mass


@pytest.mark.parametrize("pattern", ["frame_groups", "dual"])
def test_groups_compete_for_one_recall_budget(pattern):
    """The cheaper step (group 1, ratio 0.20) is taken first and leaves recall 0.95; the step of group 0
    would then go to 0.89 < tau and is refused.  A search with a recall budget per group, or one that
    took steps in group order, would narrow group 0 instead or as well."""
    g, mass = competing_groups_mass()
    groups, recall, kept = S.search_head(g, mass, [0, 1], 0.9, 0.3, pattern)
    assert groups == [(0, (0, 1), ABSENT), (1, (0, 0), ABSENT)]
    assert abs(recall - 0.95) < 1e-12 and kept == 12 / 16
    groups, recall, _ = S.search_head(g, mass, [0, 1], 0.85, 0.3, pattern)       # room for both
    assert groups == [(0, (0, 0), ABSENT), (1, (0, 0), ABSENT)] and abs(recall - 0.89) < 1e-12
    groups, recall, _ = S.search_head(g, mass, [0, 1], 0.9, 0.21, pattern)       # lambda refuses group 0's step anyway
    assert groups == [(0, (0, 1), ABSENT), (1, (0, 0), ABSENT)]


def test_degenerate_masses():
    g = _unit_tiles(2, 3, 3)
    for pattern in S.PATTERNS:
        groups, recall, kept = S.search_head(g, np.zeros((g.n, g.n)), [0, 1], 0.9, 0.5, pattern)
        assert groups == [(0, (2, 2), ABSENT), (1, (2, 2), ABSENT)] and recall == 1.0 and kept == 1.0
    bad = np.ones((g.n, g.n))
    for value in (np.nan, np.inf, -1.0):
        bad[3, 4] = value
        with pytest.raises(ValueError):
            S.search_head(g, bad, [0, 1], 0.9, 0.5)
