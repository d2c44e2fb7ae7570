"""The C-ABI library without a GPU: it loads, exports what the header declares, and its
host-side layout builder agrees bit for bit with the oracle."""
import ctypes
import os
import re

import numpy as np
import pytest
from hypothesis import given, settings, strategies as st

import paper_2508_12969_amd as ca
from paper_2508_12969_amd import binding
from oracle.geometry import Geometry
from oracle import layout as OL
from workloads import get_workload, WORKLOAD_NAMES

from helpers import build_layout, geometry_of

ABSENT = (-1, -1)


def test_library_exports_every_declared_symbol(repo_root):
    header = open(os.path.join(repo_root, "include", "compact_attn.h")).read()
    declared = set(re.findall(r"\b(compact_attn_\w+)\s*\(", header))
    assert declared == set(binding.EXPORTED)
    lib = ca.load_library()
    for name in declared:
        assert hasattr(lib, name), name
    assert ca.compact_attn_last_error() == ""


@pytest.mark.parametrize("name", ["cfg1", "cfg2"])
def test_small_config_csr_bit_exact(name):
    wl = get_workload(name)
    g = geometry_of(wl)
    lay = build_layout(ca, wl)
    info = ca.compact_attn_layout_info(lay)
    assert (info["n_tiles"], info["tokens_per_tile"], info["n_tokens_real"], info["n_tokens_padded"]) == (
        g.n, g.B, g.N_real, g.N_pad)
    want = OL.build_csr(g, wl.heads)
    for h in range(wl.num_heads):
        row_ptr, col_idx = ca.compact_attn_layout_csr(lay, h)
        assert row_ptr.dtype == np.int64 and col_idx.dtype == np.int32
        assert np.array_equal(row_ptr, want[h][0])
        assert np.array_equal(col_idx, want[h][1])
    assert info["nnz_total"] == sum(int(w[0][-1]) for w in want)
    assert np.array_equal(ca.compact_attn_layout_order(lay), OL.work_order(OL.row_counts(g, wl.heads)))


@pytest.mark.parametrize("name", [n for n in WORKLOAD_NAMES if n not in ("cfg1", "cfg2")])
def test_large_config_counts_order_and_sampled_rows(name):
    wl = get_workload(name)
    g = geometry_of(wl)
    lay = build_layout(ca, wl)
    counts = OL.row_counts(g, wl.heads)                       # closed form, every row
    rng = np.random.default_rng(11)
    full_heads = set(int(h) for h in rng.choice(wl.num_heads, 2, replace=False))
    for h in range(wl.num_heads):
        row_ptr, col_idx = ca.compact_attn_layout_csr(lay, h)
        assert np.array_equal(np.diff(row_ptr), counts[h])
        assert int(row_ptr[-1]) == wl.expected_nnz[h]
        rows = range(g.n) if h in full_heads else [int(x) for x in rng.choice(g.n, 6, replace=False)] + [0, g.n - 1]
        if h in full_heads:
            rows = [int(x) for x in rng.choice(g.n, 60, replace=False)] + [0, g.n_vid - 1, g.n - 1]
        for q in rows:
            assert np.array_equal(col_idx[row_ptr[q]:row_ptr[q + 1]], OL.kept_tiles(g, wl.heads[h], q)), (h, q)
    assert np.array_equal(ca.compact_attn_layout_order(lay), OL.work_order(counts))
    assert ca.compact_attn_layout_info(lay)["nnz_total"] == int(counts.sum())


_win = st.tuples(st.integers(-1, 4), st.integers(-1, 4))


@st.composite
def _cases(draw):
    tt, th, tw = draw(st.integers(1, 2)), draw(st.integers(1, 3)), draw(st.integers(1, 3))
    T, H, W = draw(st.integers(1, 5)), draw(st.integers(1, 7)), draw(st.integers(1, 7))
    n_txt = draw(st.integers(0, 2))
    heads = []
    for _ in range(draw(st.integers(1, 3))):
        k = draw(st.integers(0, 3))
        dts = sorted(draw(st.sets(st.integers(0, 6), min_size=k, max_size=k)))
        heads.append([(dt, draw(_win), draw(_win)) for dt in dts])
    return (T, H, W, (tt, th, tw), n_txt * tt * th * tw, heads)


@settings(max_examples=150, deadline=None)
@given(_cases())
def test_random_small_layouts_bit_exact(case):
    T, H, W, tile, n_text, heads = case
    g = Geometry(T, H, W, *tile, n_text)
    lay = ca.compact_attn_build_layout(T, H, W, tile, n_text, 1, len(heads), 8, "f32", heads)
    want = OL.build_csr(g, heads)
    for h in range(len(heads)):
        row_ptr, col_idx = ca.compact_attn_layout_csr(lay, h)
        assert np.array_equal(row_ptr, want[h][0]) and np.array_equal(col_idx, want[h][1])
    assert np.array_equal(ca.compact_attn_layout_order(lay), OL.work_order(OL.row_counts(g, heads)))
    lay.free()
    # the same heads with windows that keep their size at the border (flag per head: first on, rest off)
    flags = [h == 0 for h in range(len(heads))]
    lay = ca.compact_attn_build_layout(T, H, W, tile, n_text, 1, len(heads), 8, "f32", heads, clamp_centre=flags)
    moved = [OL.ClampedHead(head) if f else head for head, f in zip(heads, flags)]
    want = OL.build_csr(g, moved)
    for h in range(len(heads)):
        row_ptr, col_idx = ca.compact_attn_layout_csr(lay, h)
        assert np.array_equal(row_ptr, want[h][0]) and np.array_equal(col_idx, want[h][1])
    lay.free()


def test_huge_radius_and_many_groups():
    heads = [[(i, (2 ** 31 - 1, 0), (0, 2 ** 31 - 1)) for i in range(8)]]
    g = Geometry(9, 5, 6, 1, 1, 1)
    lay = ca.compact_attn_build_layout(9, 5, 6, (1, 1, 1), 0, 1, 1, 8, "f32", heads)
    want = OL.build_csr(g, heads)
    row_ptr, col_idx = ca.compact_attn_layout_csr(lay, 0)
    assert np.array_equal(row_ptr, want[0][0]) and np.array_equal(col_idx, want[0][1])


def _expect_error(status, **kw):
    args = dict(T=2, H=4, W=4, tile=(1, 2, 2), n_text=0, batch=1, num_heads=1, head_dim=8, dtype="f32",
                heads=[[(0, (0, 0), ABSENT)]])
    args.update(kw)
    with pytest.raises(ca.CompactAttnError) as e:
        ca.compact_attn_build_layout(**args)
    assert e.value.status == status
    assert ca.compact_attn_last_error() != ""


def test_invalid_arguments_are_rejected_on_the_host():
    _expect_error(binding.CA_ERR_INVALID_ARG, T=0)
    _expect_error(binding.CA_ERR_INVALID_ARG, tile=(1, 0, 2))
    _expect_error(binding.CA_ERR_INVALID_ARG, n_text=3)
    _expect_error(binding.CA_ERR_INVALID_ARG, head_dim=3)                                   # 12-byte rows
    _expect_error(binding.CA_ERR_INVALID_ARG, heads=[[(1, (0, 0), ABSENT), (1, (1, 1), ABSENT)]])
    _expect_error(binding.CA_ERR_INVALID_ARG, heads=[[(-1, (0, 0), ABSENT)]])
    _expect_error(binding.CA_ERR_INVALID_ARG, heads=[[(i, (0, 0), ABSENT) for i in range(9)]])
    _expect_error(binding.CA_ERR_INVALID_ARG, scale=float("nan"))
    _expect_error(binding.CA_ERR_INVALID_ARG, clamp_centre=2)
    lib = ca.load_library()
    assert lib.compact_attn_build_layout(None, None, None) == binding.CA_ERR_INVALID_ARG
    assert lib.compact_attn_layout_info(None, None, None, None, None, None) == binding.CA_ERR_INVALID_ARG
    assert lib.compact_attn_forward(None, None, None, None, None, None) == binding.CA_ERR_INVALID_ARG
    assert lib.compact_attn_permute(None, None, None, 0, None) == binding.CA_ERR_INVALID_ARG
    lib.compact_attn_free_layout(None)
    # a good call clears the message
    ca.compact_attn_build_layout(2, 4, 4, (1, 2, 2), 0, 1, 1, 8, "f32", [[(0, (0, 0), ABSENT)]])
    assert ca.compact_attn_last_error() == ""


def test_unsupported_shapes_rejected_before_any_device_work():
    # bf16 tile of 16 tokens: valid layout, no kernel for it
    lay = ca.compact_attn_build_layout(2, 4, 4, (1, 4, 4), 0, 1, 1, 64, "bf16", [[(0, (0, 0), ABSENT)]])
    buf = (ctypes.c_char * 64)()
    addr = (ctypes.addressof(buf) + 15) & ~15
    lib = ca.load_library()
    st_ = lib.compact_attn_forward(addr, addr + 16, addr + 32, lay.handle, addr + 48 - 16 * 3 + 48, None)
    assert st_ == binding.CA_ERR_UNSUPPORTED
    assert "bf16" in ca.compact_attn_last_error()
    assert lib.compact_attn_forward(addr + 1, addr + 16, addr + 32, lay.handle, addr, None) == binding.CA_ERR_INVALID_ARG


def test_overlapping_buffers_rejected_on_the_host():
    """Byte ranges of the whole tensors are compared, not base pointers: an output that starts inside
    an input is refused before anything is enqueued (the addresses below are never dereferenced)."""
    lay = ca.compact_attn_build_layout(2, 8, 8, (1, 8, 8), 0, 1, 2, 64, "bf16", [[(0, (0, 0), ABSENT)]] * 2)
    lib = ca.load_library()
    size = 2 * lay.n_tokens_padded * 64 * 2                   # bytes of one tile-ordered tensor
    base = 1 << 30
    q, k, v = base, base + size, base + 2 * size
    for fn in (lib.compact_attn_forward, lib.compact_attn_dense, lib.compact_attn_forward_static):
        for out in (q, q + 16, k + size - 16, v - 16, v + size - 16):
            assert fn(q, k, v, lay.handle, out, None) == binding.CA_ERR_INVALID_ARG
            assert "overlap" in ca.compact_attn_last_error()
    nat = 2 * lay.n_tokens_real * 64 * 2
    assert lib.compact_attn_forward_natural(q, k, v, lay.handle, q + nat - 16, None) == binding.CA_ERR_INVALID_ARG
    assert lib.compact_attn_permute(q, q + 16, lay.handle, 0, None) == binding.CA_ERR_INVALID_ARG
    assert lib.compact_attn_permute(q, q + size - 16, lay.handle, 1, None) == binding.CA_ERR_INVALID_ARG
    mass_bytes = 2 * lay.n_tiles * lay.n_tiles * 4
    assert lib.compact_attn_tile_mass(q, k, lay.handle, k - mass_bytes + 4, None) == binding.CA_ERR_INVALID_ARG
    assert "overlap" in ca.compact_attn_last_error()
    assert lib.compact_attn_tile_mass(q, k, lay.handle, base - mass_bytes - 2, None) == binding.CA_ERR_INVALID_ARG
    assert "aligned" in ca.compact_attn_last_error()


# ---------------------------------------------------------------- import, union, similarity

def _random_masks(rng, num_heads, n, density):
    m = rng.random((num_heads, n, n)) < density
    m[:, :, 0] |= ~m.any(axis=2)            # no empty rows in this helper
    return m


def test_layout_from_csr_roundtrip_and_order():
    rng = np.random.default_rng(11)
    T, H, W, tile, n_text, Hd = 3, 9, 10, (1, 4, 4), 16, 3
    g = Geometry(T, H, W, *tile, n_text)
    masks = _random_masks(rng, Hd, g.n, 0.3)
    masks[1, 5] = False                       # an empty row is a legal mask
    csr = [OL.csr_of_mask(masks[h]) for h in range(Hd)]
    lay = ca.compact_attn_layout_from_csr(T, H, W, tile, n_text, 1, Hd, 8, "f32", csr)
    assert lay.n_tiles == g.n and lay.nnz_total == int(masks.sum())
    for h in range(Hd):
        rp, ci = ca.compact_attn_layout_csr(lay, h)
        assert np.array_equal(rp, csr[h][0]) and np.array_equal(ci, csr[h][1])
        assert np.array_equal(OL.mask_of_csr(g.n, rp, ci), masks[h])
    assert np.array_equal(ca.compact_attn_layout_order(lay), OL.work_order(masks.sum(axis=2)))
    # importing what the builder produced gives the builder's layout back
    wl = get_workload("cfg2")
    built = build_layout(ca, wl)
    again = ca.compact_attn_layout_from_csr(wl.T, wl.H, wl.W, wl.tile, wl.n_text, wl.batch, wl.num_heads, wl.head_dim,
                                            wl.dtype, [ca.compact_attn_layout_csr(built, h) for h in range(wl.num_heads)])
    for h in range(wl.num_heads):
        a, b = ca.compact_attn_layout_csr(built, h), ca.compact_attn_layout_csr(again, h)
        assert np.array_equal(a[0], b[0]) and np.array_equal(a[1], b[1])
    assert np.array_equal(ca.compact_attn_layout_order(built), ca.compact_attn_layout_order(again))


def test_layout_from_csr_rejects_malformed_input():
    args = (1, 8, 8, (1, 4, 4), 0, 1, 1, 8, "f32")       # n = 4
    ok = (np.array([0, 1, 2, 3, 4]), np.array([0, 1, 2, 3]))
    ca.compact_attn_layout_from_csr(*args, [ok]).free()
    bad = [
        (np.array([1, 1, 2, 3, 4]), np.array([0, 1, 2, 3])),      # row_ptr[0] != 0
        (np.array([0, 2, 1, 3, 4]), np.array([0, 1, 2, 3])),      # decreasing offsets
        (np.array([0, 2, 2, 3, 4]), np.array([1, 0, 2, 3])),      # unsorted row
        (np.array([0, 2, 2, 3, 4]), np.array([1, 1, 2, 3])),      # duplicate
        (np.array([0, 1, 2, 3, 4]), np.array([0, 1, 2, 4])),      # id out of range
        (np.array([0, 1, 2, 3, 4]), np.array([0, -1, 2, 3])),     # negative id
    ]
    for csr in bad:
        with pytest.raises(ca.CompactAttnError) as e:
            ca.compact_attn_layout_from_csr(*args, [csr])
        assert e.value.status == binding.CA_ERR_INVALID_ARG


def test_union_and_similarity_match_the_mask_algebra():
    """Union of configurations (Sec. 4.2) and Sim of Eq. 3 against the oracle's boolean masks."""
    T, H, W, tile, n_text = 4, 12, 12, (1, 4, 4), 16
    g = Geometry(T, H, W, *tile, n_text)
    heads_a = [[(1, (1, 1), ABSENT)], [(3, (0, 2), (2, 0))], []]
    heads_b = [[(0, (2, 2), ABSENT), (3, (0, 0), ABSENT)], [(3, (0, 2), (2, 0))], [(3, (2, 2), ABSENT)]]
    la = ca.compact_attn_build_layout(T, H, W, tile, n_text, 1, 3, 8, "f32", heads_a)
    lb = ca.compact_attn_build_layout(T, H, W, tile, n_text, 1, 3, 8, "f32", heads_b)
    ma, mb = OL.keep_mask_bruteforce(g, heads_a), OL.keep_mask_bruteforce(g, heads_b)
    lu = ca.compact_attn_layout_union(la, lb)
    for h in range(3):
        rp, ci = ca.compact_attn_layout_csr(lu, h)
        assert np.array_equal(OL.mask_of_csr(g.n, rp, ci), OL.union_masks(ma[h], mb[h]))
        for h2 in range(3):
            assert ca.compact_attn_layout_similarity(la, h, lb, h2) == pytest.approx(OL.mask_similarity(ma[h], mb[h2]), abs=1e-15)
    assert np.array_equal(ca.compact_attn_layout_order(lu), OL.work_order(OL.union_masks(ma, mb).sum(axis=2)))
    # closed forms: a mask against itself, against its union, disjoint masks
    assert ca.compact_attn_layout_similarity(la, 1, lb, 1) == 1.0
    assert ca.compact_attn_layout_similarity(la, 0, lu, 0) == pytest.approx(ma[0].sum() / (ma[0] | mb[0]).sum())
    n = g.n
    eye = [OL.csr_of_mask(np.eye(n, dtype=bool))]
    off = [OL.csr_of_mask(np.roll(np.eye(n, dtype=bool), 1, axis=1))]
    le = ca.compact_attn_layout_from_csr(T, H, W, tile, n_text, 1, 1, 8, "f32", eye)
    lo = ca.compact_attn_layout_from_csr(T, H, W, tile, n_text, 1, 1, 8, "f32", off)
    assert ca.compact_attn_layout_similarity(le, 0, lo, 0) == 0.0
    with pytest.raises(ca.CompactAttnError):
        ca.compact_attn_layout_union(la, le)             # different head counts


# ---------------------------------------------------------------- window search (host part of Sec. 4.2)

def test_search_head_matches_the_oracle_search():
    from oracle import search as OS
    rng = np.random.default_rng(8)
    cases = [
        (Geometry(5, 9, 7, 1, 2, 2, 0), [0, 1, 4]),
        (Geometry(4, 12, 12, 1, 4, 4, 16), [1, 3]),          # one text tile: takes no part
        (Geometry(6, 8, 8, 2, 4, 4, 0), [0, 2]),             # tt = 2; frame distances beyond 2 are dropped
    ]
    for g, dts in cases:
        q, k = rng.standard_normal((2, g.N_real, 8))
        q *= 3.0
        k += 0.8 * np.repeat(rng.standard_normal((g.N_real // 5 + 1, 8)), 5, axis=0)[:g.N_real]
        mass = OS.tile_mass(g, q, k).astype(np.float32)
        lay = ca.compact_attn_build_layout(g.T, g.H, g.W, (g.tt, g.th, g.tw), g.n_text, 1, 1, 8, "f32", [[]])
        for tau, lam, pattern in [(t, l, p) for (t, l) in ((0.95, 0.3), (0.8, 0.8), (0.5, 3.0), (1.0, 0.0))
                                  for p in ("dual", "frame_groups", "cubic")]:
            want, want_recall, want_kept = OS.search_head(g, mass, dts, tau, lam, pattern)
            got, recall, kept = ca.compact_attn_search_head(lay, mass, dts, tau, lam, pattern)
            assert got == want, (g, dts, tau, lam, pattern)
            assert recall == pytest.approx(want_recall, abs=1e-12) and kept == pytest.approx(want_kept, abs=1e-15)
            # and the recall it reports is the recall of the mask the builder makes from its answer
            built = ca.compact_attn_build_layout(g.T, g.H, g.W, (g.tt, g.th, g.tw), g.n_text, 1, 1, 8, "f32", [got])
            rp, ci = ca.compact_attn_layout_csr(built, 0)
            mask = OL.mask_of_csr(g.n, rp, ci)[:g.n_vid, :g.n_vid]
            m64 = mass.astype(np.float64)[:g.n_vid, :g.n_vid]
            assert m64[mask].sum() / m64.sum() == pytest.approx(recall, abs=1e-9)
            assert recall >= tau - 1e-12
        lay.free()


def test_search_head_closed_forms_and_errors():
    g = Geometry(4, 6, 8, 1, 1, 1, 0)
    t, h, w = np.unravel_index(np.arange(g.n), (g.nT, g.nH, g.nW))
    lay = ca.compact_attn_build_layout(4, 6, 8, (1, 1, 1), 0, 1, 1, 8, "f32", [[]])
    local = (np.abs(t[:, None] - t) <= 1) & (np.abs(h[:, None] - h) <= 1) & (np.abs(w[:, None] - w) <= 2)
    groups, recall, kept = ca.compact_attn_search_head(lay, local / local.sum(axis=1, keepdims=True), [0, 1, 3], 1.0 - 1e-6, 0.5)
    assert groups == [(0, (1, 2), ABSENT), (1, (1, 2), ABSENT), (3, ABSENT, ABSENT)]
    assert kept == pytest.approx(local.sum() / g.n ** 2)
    cross = (h[:, None] == h) | (w[:, None] == w)
    groups, recall, kept = ca.compact_attn_search_head(lay, cross / cross.sum(axis=1, keepdims=True), [3], 1.0 - 1e-6, 0.5)
    assert groups == [(3, (0, 7), (5, 0))] and recall == pytest.approx(1.0, abs=1e-6)
    uniform = np.full((g.n, g.n), 1.0 / g.n)
    groups, recall, kept = ca.compact_attn_search_head(lay, uniform, [3], 0.5, 0.9)
    assert groups == [(3, (5, 7), ABSENT)] and kept == 1.0
    # the same cross under the narrower families: one window must cover both arms (everything), a cube too
    for pattern in ("frame_groups", "cubic"):
        groups, recall, kept = ca.compact_attn_search_head(lay, cross / cross.sum(axis=1, keepdims=True), [3], 1.0 - 1e-6,
                                                           0.5, pattern)
        assert groups == [(3, (5, 7), ABSENT)] and kept == 1.0
    # the local head: per-group windows find it exactly; the cube has one window for the frames it keeps
    for pattern in ("frame_groups", "cubic"):
        groups, _, kept = ca.compact_attn_search_head(lay, local / local.sum(axis=1, keepdims=True), [0, 1, 3], 1.0 - 1e-6,
                                                      0.5, pattern)
        assert groups == [(0, (1, 2), ABSENT), (1, (1, 2), ABSENT), (3, ABSENT, ABSENT)]
    with pytest.raises(ca.CompactAttnError):
        binding.load_library()  # the raw call: a pattern value outside the enum
        dts = (ctypes.c_int32 * 1)(3)
        out = (binding.ca_group * 1)()
        m = np.ascontiguousarray(uniform, dtype=np.float32)
        binding._check(binding.load_library().compact_attn_search_head(
            lay.handle, m.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), dts, 1, 0.9, 0.5, 7, out, None, None))
    for bad in (dict(group_max_dt=[2, 1]), dict(group_max_dt=[-1]), dict(tau=1.5), dict(lam=-1.0), dict(group_max_dt=[])):
        kw = dict(group_max_dt=[3], tau=0.9, lam=0.5)
        kw.update(bad)
        with pytest.raises(ca.CompactAttnError):
            ca.compact_attn_search_head(lay, uniform, kw["group_max_dt"], kw["tau"], kw["lam"])


# ---------------------------------------------------------------- query-tile pairs (work ordering of the paired kernel)

@st.composite
def _pair_cases(draw):
    tile = draw(st.sampled_from([(1, 8, 8), (2, 4, 8), (4, 4, 4), (1, 4, 16)]))
    nT, nH, nW = draw(st.integers(1, 4)), draw(st.integers(1, 4)), draw(st.integers(1, 5))
    T = nT * tile[0] - draw(st.integers(0, tile[0] - 1))
    H = nH * tile[1] - draw(st.integers(0, tile[1] - 1))
    W = nW * tile[2] - draw(st.integers(0, tile[2] - 1))
    n_text = 64 * draw(st.integers(0, 3))
    win = st.tuples(st.integers(-1, 3), st.integers(-1, 3))
    heads = []
    for _ in range(draw(st.integers(1, 3))):
        k = draw(st.integers(0, 3))
        dts = sorted(draw(st.sets(st.integers(0, 4), min_size=k, max_size=k)))
        heads.append([(dt, draw(win), draw(win)) for dt in dts])
    return T, H, W, tile, n_text, heads


def test_search_head_hand_worked_thresholds_and_degenerate_masses():
    """The library on the hand-worked cases of test_oracle_search.py (the expected windows follow from
    the arithmetic written there, not from the oracle): the paper's thresholds on a two-density mass,
    two groups competing for one recall budget, and masses that cannot be searched."""
    from test_oracle_search import competing_groups_mass, two_density_mass
    lay = ca.compact_attn_build_layout(1, 6, 6, (1, 1, 1), 0, 1, 1, 64, "bf16", [[]])
    mass = two_density_mass(Geometry(1, 6, 6, 1, 1, 1, 0))
    for pattern in ("frame_groups", "dual"):
        groups, recall, kept = ca.compact_attn_search_head(lay, mass, [0], 0.9, 0.011, pattern)
        assert groups == [(0, (2, 2), ABSENT)] and kept == (256 + 320) / 1296
        groups, recall, kept = ca.compact_attn_search_head(lay, mass, [0], 0.9, 0.04, pattern)
        assert groups == [(0, (1, 1), ABSENT)] and kept == 256 / 1296
        assert abs(recall - np.float32(5.0109375) * 256 / np.float32(mass).astype(np.float64).sum()) < 1e-9
    g, mass = competing_groups_mass()
    lay2 = ca.compact_attn_build_layout(2, 1, 2, (1, 1, 1), 0, 1, 1, 64, "bf16", [[]])
    for pattern in ("frame_groups", "dual"):
        groups, recall, kept = ca.compact_attn_search_head(lay2, mass, [0, 1], 0.9, 0.3, pattern)
        assert groups == [(0, (0, 1), ABSENT), (1, (0, 0), ABSENT)] and abs(recall - 0.95) < 1e-12 and kept == 0.75
    for pattern in ("cubic", "frame_groups", "dual"):
        groups, recall, kept = ca.compact_attn_search_head(lay2, np.zeros((4, 4)), [0, 1], 0.9, 0.5, pattern)
        assert groups == [(0, (0, 1), ABSENT), (1, (0, 1), ABSENT)] and recall == 1.0 and kept == 1.0
    for value in (np.nan, np.inf, -1.0):
        bad = np.ones((4, 4), np.float32)
        bad[1, 2] = value
        with pytest.raises(ca.CompactAttnError) as e:
            ca.compact_attn_search_head(lay2, bad, [0, 1], 0.9, 0.5)
        assert e.value.status == binding.CA_ERR_INVALID_ARG and "mass" in str(e.value)


@settings(max_examples=60, deadline=None)
@given(_pair_cases())
def test_pair_table_bit_exact(case):
    T, H, W, tile, n_text, heads = case
    g = Geometry(T, H, W, *tile, n_text)
    lay = ca.compact_attn_build_layout(T, H, W, tile, n_text, 1, len(heads), 128, "bf16", heads)
    masks = np.stack([OL.mask_of_csr(g.n, *csr) for csr in OL.build_csr(g, heads)])
    _check_pairs(lay, g, masks)
    lay.free()


def _check_pairs(lay, g, masks):
    pairs, walk_ptr, walk = ca.compact_attn_layout_pairs(lay)
    want = OL.pair_table(g, masks)
    assert np.array_equal(pairs, want)
    want_ptr, tiles, first, second = OL.pair_walks(masks, want)
    assert np.array_equal(walk_ptr, want_ptr)
    words = walk.view(np.uint32)
    assert np.array_equal(words & 0xFFFFFF, tiles)
    assert np.array_equal((words >> 30) & 1, first) and np.array_equal(words >> 31, second)
    assert not np.any(words & 0x3F000000)


def _check_wave_assignment(lay, g, masks):
    """Every 32-query wave slot of every row that holds a token belongs to exactly one wave of one
    workgroup: the row's own (launch_rows, four waves) or a workgroup of two packed query tiles."""
    pairs, walk_ptr, walk = ca.compact_attn_layout_pairs(lay)
    desc, launch = ca.compact_attn_layout_packing(lay)
    Hd, n = masks.shape[0], g.n
    valid = np.bincount(g.token_slots() // g.B, minlength=n)
    owners = np.zeros((Hd * n, 4), dtype=int)
    rows_kept = launch[launch >= 0]
    for r in rows_kept:
        owners[r, :] += 1
    groups_seen = np.sort(~launch[launch < 0])
    assert np.array_equal(groups_seen, np.arange(len(pairs)))
    order = ca.compact_attn_layout_order(lay)
    assert np.array_equal(rows_kept, order[np.isin(order, rows_kept)])        # same relative order as the full launch order
    counts = masks.reshape(Hd * n, n).sum(axis=1)
    lengths = np.array([counts[e] if e >= 0 else walk_ptr[~e + 1] - walk_ptr[~e] for e in launch])
    assert np.all(np.diff(lengths) <= 0)                                      # longest first
    words = walk.view(np.uint32)
    for i, (a, b) in enumerate(pairs):
        assert a >= 0 and a != b and (b < 0 or a // n == b // n)
        d = int(desc[i])
        for w in range(4):
            if not (d >> (4 + w)) & 1:
                continue
            second, first = (d >> w) & 1, (d >> (8 + 4 * w)) & 0xF
            assert first < 4 and (not second or b >= 0)
            owners[b if second else a, first] += 1
        seg = words[walk_ptr[i]:walk_ptr[i + 1]]
        ma = masks.reshape(Hd * n, n)[a]
        mb = masks.reshape(Hd * n, n)[b] if b >= 0 else np.zeros(n, dtype=bool)
        assert np.array_equal(seg & 0xFFFFFF, np.flatnonzero(ma | mb))
        assert np.array_equal((seg >> 30) & 1, ma[ma | mb]) and np.array_equal(seg >> 31, mb[ma | mb])
    for r in range(Hd * n):
        need = -(-int(valid[r % n]) // 32)
        assert np.all(owners[r, :need] == 1) and np.all(owners[r, need:] <= 1), (r, owners[r], need)


def test_packed_face_tiles_hand_worked():
    """128-token tiles (2x8x8) on a 3 x 13 x 16 grid: 2 x 2 x 2 tiles.  Tiles 0, 1 are full; 2, 3 (last
    tile row: 5 of 8 rows) hold 80 tokens = three waves; 4..7 (last tile frame: 1 of 2 frames) hold 64
    or 40 tokens = two waves.  With a head that keeps every tile, packing along w gives, in the order
    built: [tile 2: waves 0-2 | tile 3: wave 3], [tile 3: its other two waves], [4 | 5], [6 | 7]; all
    walks have the same length, so these four come first in the launch order, then rows 0 and 1."""
    T, H, W, tile = 3, 13, 16, (2, 8, 8)
    g = Geometry(T, H, W, *tile, 0)
    heads = [[(9, (9, 9), ABSENT)]]
    lay = ca.compact_attn_build_layout(T, H, W, tile, 0, 1, 1, 128, "bf16", heads)
    pairs, walk_ptr, walk = ca.compact_attn_layout_pairs(lay)
    desc, launch = ca.compact_attn_layout_packing(lay)
    assert pairs.tolist() == [[2, 3], [3, -1], [4, 5], [6, 7]]
    wave = lambda w, second, first: (second << w) | (1 << (4 + w)) | (first << (8 + 4 * w))
    assert desc.tolist() == [wave(0, 0, 0) | wave(1, 0, 1) | wave(2, 0, 2) | wave(3, 1, 0),
                             wave(0, 0, 1) | wave(1, 0, 2),
                             wave(0, 0, 0) | wave(1, 0, 1) | wave(2, 1, 0) | wave(3, 1, 1),
                             wave(0, 0, 0) | wave(1, 0, 1) | wave(2, 1, 0) | wave(3, 1, 1)]
    assert launch.tolist() == [~0, ~1, ~2, ~3, 0, 1]
    assert np.array_equal(walk_ptr, np.arange(5) * 8)
    masks = np.stack([OL.mask_of_csr(g.n, *csr) for csr in OL.build_csr(g, heads)])
    _check_wave_assignment(lay, g, masks)
    lay.free()
    # a head whose windows are one tile wide shares nothing between neighbours along w: not packed
    lay = ca.compact_attn_build_layout(T, H, W, tile, 0, 1, 1, 128, "bf16", [[(9, (9, 0), ABSENT)]])
    assert ca.compact_attn_layout_pairs(lay)[0].shape == (0, 2)
    desc, launch = ca.compact_attn_layout_packing(lay)
    assert len(desc) == 0 and np.array_equal(launch, ca.compact_attn_layout_order(lay))
    lay.free()


@settings(max_examples=40, deadline=None)
@given(st.integers(1, 7), st.integers(3, 40), st.integers(3, 40), st.sampled_from([(2, 8, 8), (1, 8, 16), (4, 4, 8)]),
       st.integers(0, 2), st.lists(st.tuples(st.integers(0, 3), _win, _win), min_size=1, max_size=3), st.integers(0, 10 ** 6))
def test_packed_face_tiles_cover_every_query_once(T, H, W, tile, n_txt, groups, seed):
    rng = np.random.default_rng(seed)
    heads = [sorted({dt: (dt, a, b) for dt, a, b in groups}.values()), [(9, (9, 9), ABSENT)],
             [(int(rng.integers(0, 3)), (int(rng.integers(0, 3)), 9), ABSENT)]]
    g = Geometry(T, H, W, *tile, n_txt * 128)
    lay = ca.compact_attn_build_layout(T, H, W, tile, n_txt * 128, 1, len(heads), 128, "bf16", heads)
    masks = np.stack([OL.mask_of_csr(g.n, *csr) for csr in OL.build_csr(g, heads)])
    _check_wave_assignment(lay, g, masks)
    lay.free()


def test_pair_table_of_config3_heads_and_absent_elsewhere():
    wl = get_workload("cfg3")
    g = geometry_of(wl)
    picked = [0, 7, 19, 33]
    heads = [wl.heads[h] for h in picked]
    lay = ca.compact_attn_build_layout(wl.T, wl.H, wl.W, wl.tile, wl.n_text, 1, len(heads), wl.head_dim, wl.dtype, heads)
    masks = np.stack([OL.mask_of_csr(g.n, *csr) for csr in OL.build_csr(g, heads)])
    _check_pairs(lay, g, masks)
    lay.free()
    # layouts served by the one-tile-per-workgroup kernels carry no pair table
    for name in ("cfg1", "cfg2"):
        lay = build_layout(ca, get_workload(name))
        assert ca.compact_attn_layout_pairs(lay)[0].shape == (0, 2)
        lay.free()
