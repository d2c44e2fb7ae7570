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
