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
