"""Tile-order flattening of the token sequence (oracle side; test infrastructure).

Sec. 3.1 / Appendix D: instead of flattening (f, h, w) row-major, tokens are
grouped so that every run of B consecutive positions is one space-time tile.
Padded positions (grid not a tile multiple) hold zeros; the inverse drops
them.  Pure data movement: results are exact.

`Geometry.token_slots()` gives, for every real token in natural order, its
position tile * B + slot in the padded tile order; it is checked against the
loop form `Geometry.token_tile_and_slot()` by the tests.
"""
import numpy as np

from .geometry import Geometry


def permute(geom: Geometry, x):
    """natural order [..., N_real, D] -> tile order, padded [..., N_pad, D]."""
    x = np.asarray(x)
    if x.shape[-2] != geom.N_real:
        raise ValueError("token axis must have N_real entries")
    out = np.zeros(x.shape[:-2] + (geom.N_pad, x.shape[-1]), dtype=x.dtype)
    out[..., geom.token_slots(), :] = x
    return out


def unpermute(geom: Geometry, y):
    """tile order, padded [..., N_pad, D] -> natural order [..., N_real, D]."""
    y = np.asarray(y)
    if y.shape[-2] != geom.N_pad:
        raise ValueError("token axis must have N_pad entries")
    return y[..., geom.token_slots(), :]


def slot_valid(geom: Geometry):
    """bool[N_pad]: which padded tile-order positions hold a real token."""
    valid = np.zeros(geom.N_pad, dtype=bool)
    valid[geom.token_slots()] = True
    return valid
