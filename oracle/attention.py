"""Exact softmax attention restricted to kept tiles (oracle side; test infrastructure).

Appendix D describes the computation as FlashAttention's block loop with an
online softmax that visits only kept blocks.  That loop is an exact
re-association of the definition below, so the oracle is the definition
itself, in fp64, on natural-order tokens with no padding:

    for head h and real query token i in tile ti:
        J   = { real key tokens j : keep(h, ti, tile(j)) }
        s_j = scale * <q_i, k_j>                       j in J
        p_j = exp(s_j - max_J s) / sum_J exp(s_j - max_J s)
        o_i = sum_J p_j v_j                            (zeros if J is empty)

`keep` is the pair rule of `oracle.layout.keep_pair`; scale defaults to
head_dim ** -0.5 (the paper does not state it).
"""
import numpy as np

from .geometry import Geometry
from .layout import check_head, keep_pair


def default_scale(head_dim):
    return float(head_dim) ** -0.5


def softmax_rows(s):
    """Row softmax of a 2-D fp64 array by the max-subtracted definition."""
    m = s.max(axis=1, keepdims=True)
    e = np.exp(s - m)
    return e / e.sum(axis=1, keepdims=True)


def attention_tile(geom: Geometry, head, q_tile, q, k, v, scale=None, token_tile=None, return_probs=False):
    """Outputs of the real query tokens of one query tile, one head.

    q, k, v: [N_real, D] natural order (any float dtype; widened to fp64).
    Returns (idx, o): natural-order indices of the tile's real tokens and
    their outputs fp64[len(idx), D]; with return_probs also (J, p).
    """
    head = check_head(head)
    if token_tile is None:
        token_tile, _ = geom.token_tile_and_slot()
    D = q.shape[-1]
    if scale is None:
        scale = default_scale(D)
    idx = np.nonzero(token_tile == q_tile)[0]
    tile_kept = np.array([keep_pair(geom, head, q_tile, kt) for kt in range(geom.n)], dtype=bool)
    J = np.nonzero(tile_kept[token_tile])[0]
    qi = np.asarray(q[idx], dtype=np.float64)
    if len(J) == 0 or len(idx) == 0:
        o = np.zeros((len(idx), v.shape[-1]), dtype=np.float64)
        return (idx, o, J, np.zeros((len(idx), 0))) if return_probs else (idx, o)
    kj = np.asarray(k[J], dtype=np.float64)
    vj = np.asarray(v[J], dtype=np.float64)
    s = scale * (qi @ kj.T)
    p = softmax_rows(s)
    o = p @ vj
    return (idx, o, J, p) if return_probs else (idx, o)


def tile_mask_attention(geom: Geometry, masks, q, k, v, scale=None):
    """The same definition with the kept set given directly as boolean tile masks.

    masks: bool [num_heads, n, n], masks[h, qt, kt] = query tile qt of head h keeps key tile kt
    (any block mask, e.g. an imported or merged layout).  q, k, v: [num_heads, N_real, D].
    """
    token_tile, _ = geom.token_tile_and_slot()
    masks = np.asarray(masks, dtype=bool)
    D = q.shape[-1]
    if scale is None:
        scale = default_scale(D)
    out = np.zeros(q.shape[:-1] + (v.shape[-1],), dtype=np.float64)
    for h in range(masks.shape[0]):
        for q_tile in range(geom.n):
            idx = np.nonzero(token_tile == q_tile)[0]
            J = np.nonzero(masks[h, q_tile][token_tile])[0]
            if len(J) == 0 or len(idx) == 0:
                continue
            s = scale * (np.asarray(q[h][idx], dtype=np.float64) @ np.asarray(k[h][J], dtype=np.float64).T)
            out[h, idx] = softmax_rows(s) @ np.asarray(v[h][J], dtype=np.float64)
    return out


def masked_attention(geom: Geometry, heads, q, k, v, scale=None):
    """q, k, v: [num_heads, N_real, D] natural order -> fp64 [num_heads, N_real, D]."""
    token_tile, _ = geom.token_tile_and_slot()
    out = np.zeros(q.shape[:-1] + (v.shape[-1],), dtype=np.float64)
    for h, head in enumerate(heads):
        for q_tile in range(geom.n):
            idx, o = attention_tile(geom, head, q_tile, q[h], k[h], v[h], scale, token_tile)
            out[h, idx] = o
    return out


def dense_attention(q, k, v, scale=None):
    """Textbook softmax(scale * Q K^T) V per head, fp64; q, k, v: [num_heads, N, D]."""
    q = np.asarray(q, dtype=np.float64)
    k = np.asarray(k, dtype=np.float64)
    v = np.asarray(v, dtype=np.float64)
    if scale is None:
        scale = default_scale(q.shape[-1])
    out = np.empty(q.shape[:-1] + (v.shape[-1],), dtype=np.float64)
    for h in range(q.shape[0]):
        out[h] = softmax_rows(scale * (q[h] @ k[h].T)) @ v[h]
    return out
