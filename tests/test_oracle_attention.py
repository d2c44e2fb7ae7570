"""Pins for the oracle's masked attention.

The oracle is checked against: a token-by-token pure-Python evaluation of the
definition, scipy's softmax on the dense special case, per-tile dense
attention on the block-diagonal special case, closed forms (Q = 0, two-key
logistic), and invariances the definition implies.
"""
import math

import numpy as np
import pytest
import scipy.special

from oracle.geometry import Geometry
from oracle import attention as A
from oracle import layout as L

ABSENT = (-1, -1)


def _rand_qkv(g, heads, D, seed=0):
    rng = np.random.default_rng(seed)
    return tuple(rng.standard_normal((heads, g.N_real, D)) for _ in range(3))


def _python_reference(g, heads, q, k, v, scale):
    """Definition evaluated scalar by scalar with math.exp; no numpy arithmetic."""
    tok_tile, _ = g.token_tile_and_slot()
    Hd, N, D = q.shape
    out = [[[0.0] * D for _ in range(N)] for _ in range(Hd)]
    for h in range(Hd):
        head = L.check_head(heads[h])
        for i in range(N):
            keys = [j for j in range(N) if L.keep_pair(g, head, int(tok_tile[i]), int(tok_tile[j]))]
            s = [scale * sum(float(q[h, i, c]) * float(k[h, j, c]) for c in range(D)) for j in keys]
            m = max(s)
            e = [math.exp(x - m) for x in s]
            z = sum(e)
            for c in range(D):
                out[h][i][c] = sum(e[a] * float(v[h, j, c]) for a, j in enumerate(keys)) / z
    return np.array(out)


def test_against_scalar_python_evaluation():
    g = Geometry(3, 3, 4, 1, 2, 2, n_text=4)           # padded rows, text tile
    heads = [[(0, (0, 1), (1, 0)), (1, (0, 0), ABSENT)], [(2, (1, 1), ABSENT)]]
    q, k, v = _rand_qkv(g, 2, 5, seed=1)
    got = A.masked_attention(g, heads, q, k, v)
    ref = _python_reference(g, heads, q, k, v, 5 ** -0.5)
    assert np.max(np.abs(got - ref)) < 1e-13


def test_full_mask_equals_library_dense_softmax():
    g = Geometry(2, 5, 6, 1, 2, 4, n_text=8)
    full = [[(g.nT - 1, (g.nH - 1, g.nW - 1), ABSENT)]] * 3
    q, k, v = _rand_qkv(g, 3, 16, seed=2)
    got = A.masked_attention(g, full, q, k, v)
    scores = np.einsum("hid,hjd->hij", q, k) / math.sqrt(16)
    ref = np.einsum("hij,hjd->hid", scipy.special.softmax(scores, axis=-1), v)
    assert np.max(np.abs(got - ref)) < 1e-13
    assert np.max(np.abs(A.dense_attention(q, k, v) - ref)) < 1e-13


def test_value_and_key_roles_are_not_swapped():
    # D_v != D_qk makes any q/k/v mix-up a shape or value error
    g = Geometry(1, 2, 4, 1, 2, 2)
    rng = np.random.default_rng(3)
    q = rng.standard_normal((1, 8, 4))
    k = rng.standard_normal((1, 8, 4))
    v = rng.standard_normal((1, 8, 7))
    full = [[(0, (0, 1), ABSENT)]]
    got = A.masked_attention(g, full, q, k, v)
    ref = scipy.special.softmax(q[0] @ k[0].T / 2.0, axis=-1) @ v[0]
    assert got.shape == (1, 8, 7) and np.max(np.abs(got[0] - ref)) < 1e-13


def test_probabilities_sum_to_one_and_cover_exactly_allowed_keys():
    g = Geometry(3, 5, 5, 1, 2, 2)
    head = [(1, (0, 2), (2, 0))]
    q, k, v = _rand_qkv(g, 1, 8, seed=4)
    tok_tile, _ = g.token_tile_and_slot()
    for q_tile in range(g.n):
        idx, o, J, p = A.attention_tile(g, head, q_tile, q[0], k[0], v[0], return_probs=True)
        assert np.max(np.abs(p.sum(axis=1) - 1.0)) < 1e-12
        allowed = np.isin(tok_tile, L.kept_tiles(g, head, q_tile))
        assert np.array_equal(J, np.nonzero(allowed)[0])
        assert np.all(tok_tile[idx] == q_tile)


def test_self_only_layout_is_per_tile_dense_attention():
    g = Geometry(2, 4, 6, 1, 2, 3)
    ident = [[(0, (0, 0), ABSENT)]]
    q, k, v = _rand_qkv(g, 1, 8, seed=5)
    got = A.masked_attention(g, ident, q, k, v)[0]
    tok_tile, _ = g.token_tile_and_slot()
    for tile in range(g.n):
        idx = np.nonzero(tok_tile == tile)[0]
        ref = scipy.special.softmax(q[0, idx] @ k[0, idx].T / math.sqrt(8), axis=-1) @ v[0, idx]
        assert np.max(np.abs(got[idx] - ref)) < 1e-13


def test_zero_query_gives_mean_of_allowed_values_and_tile_indicator_probe():
    g = Geometry(3, 5, 6, 1, 2, 2, n_text=4)          # padded rows: tiles hold 4 or 2 real tokens
    head = [(0, (1, 1), ABSENT), (1, (0, 0), ABSENT)]
    tok_tile, _ = g.token_tile_and_slot()
    D = g.n                                            # one indicator channel per tile
    q = np.zeros((1, g.N_real, D))
    k = np.random.default_rng(6).standard_normal((1, g.N_real, D))
    v = np.zeros((1, g.N_real, D))
    v[0, np.arange(g.N_real), tok_tile] = 1.0
    got = A.masked_attention(g, [head], q, k, v)[0]
    real_per_tile = np.bincount(tok_tile, minlength=g.n).astype(float)
    for i in range(g.N_real):
        kept = L.kept_tiles(g, head, int(tok_tile[i]))
        want = np.zeros(D)
        want[kept] = real_per_tile[kept] / real_per_tile[kept].sum()
        assert np.max(np.abs(got[i] - want)) < 1e-14


def test_two_key_logistic_closed_form_pins_the_scale():
    g = Geometry(1, 1, 2, 1, 1, 1)
    full = [[(0, (0, 1), ABSENT)]]
    D = 4
    q = np.array([[[1.0, 2.0, 0.0, -1.0], [0.0, 0.0, 0.0, 0.0]]])
    k = np.array([[[0.5, 0.25, 3.0, 1.0], [1.0, -1.0, 2.0, 0.0]]])
    v = np.array([[[1.0, 0, 0, 0], [0, 1.0, 0, 0]]])
    got = A.masked_attention(g, full, q, k, v)
    s0 = (0.5 + 0.5 - 1.0) / 2.0      # <q0,k0> / sqrt(4)
    s1 = (1.0 - 2.0) / 2.0
    p0 = 1.0 / (1.0 + math.exp(s1 - s0))
    assert got[0, 0, 0] == pytest.approx(p0, abs=1e-15)
    assert got[0, 0, 1] == pytest.approx(1 - p0, abs=1e-15)
    assert got[0, 1, :2].tolist() == [0.5, 0.5]
    # explicit scale overrides the default
    got2 = A.masked_attention(g, full, q, k, v, scale=1.0)
    assert got2[0, 0, 0] == pytest.approx(1.0 / (1.0 + math.exp(-1.0 - 0.0)), abs=1e-15)


def test_shift_and_key_order_invariance():
    g = Geometry(2, 4, 4, 1, 2, 2)
    head = [(1, (0, 1), (1, 0))]
    q, k, v = _rand_qkv(g, 1, 8, seed=8)
    base = A.masked_attention(g, [head], q, k, v)
    # adding a per-query constant to all scores (k -> k + c along a q-orthogonal trick is awkward;
    # use: q scaled by 0 on an extra channel where k carries a constant) leaves softmax unchanged
    q2 = np.concatenate([q, np.ones_like(q[..., :1])], axis=-1) * math.sqrt(9 / 8)
    k2 = np.concatenate([k, np.full_like(k[..., :1], 37.0)], axis=-1)
    shifted = A.masked_attention(g, [head], q2, k2, v)
    assert np.max(np.abs(shifted - base)) < 1e-11
    # large scores do not overflow (max subtraction)
    big = A.masked_attention(g, [head], q * 300, k, v)
    assert np.all(np.isfinite(big))


def test_row_without_keys_yields_zeros():
    g = Geometry(2, 2, 2, 1, 2, 2)
    head = [(0, ABSENT, ABSENT)]
    q, k, v = _rand_qkv(g, 1, 4, seed=9)
    assert np.all(A.masked_attention(g, [head], q, k, v) == 0)


def test_tile_mask_attention_agrees_with_the_head_rule_and_with_dense():
    """The mask-driven form of the definition: on a head-described layout it must equal
    masked_attention, on the all-ones mask the textbook dense softmax, on the identity mask
    per-tile attention."""
    g = Geometry(3, 6, 7, 1, 4, 4, 16)
    heads = [[(1, (0, 1), (1, 0))], [(2, (1, 1), ABSENT)]]
    rng = np.random.default_rng(3)
    q, k, v = (rng.standard_normal((2, g.N_real, 8)) for _ in range(3))
    masks = L.keep_mask_bruteforce(g, heads)
    assert np.allclose(A.tile_mask_attention(g, masks, q, k, v), A.masked_attention(g, heads, q, k, v), atol=1e-13)
    ones = np.ones((2, g.n, g.n), dtype=bool)
    assert np.allclose(A.tile_mask_attention(g, ones, q, k, v), A.dense_attention(q, k, v), atol=1e-13)
    eye = np.broadcast_to(np.eye(g.n, dtype=bool), (2, g.n, g.n))
    got = A.tile_mask_attention(g, eye, q, k, v)
    tok_tile, _ = g.token_tile_and_slot()
    for t in (0, g.n // 2, g.n - 1):
        idx = np.nonzero(tok_tile == t)[0]
        assert np.allclose(got[:, idx], A.dense_attention(q[:, idx], k[:, idx], v[:, idx]), atol=1e-13)
