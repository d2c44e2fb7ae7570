"""Pins for the oracle's tile-order flattening."""
import numpy as np
from hypothesis import given, settings, strategies as st

from oracle.geometry import Geometry
from oracle import permute as P


def test_hand_worked_order():
    # 1 frame, 2 rows x 4 columns, tiles of 2x2: natural ids
    #   0 1 | 2 3
    #   4 5 | 6 7
    g = Geometry(1, 2, 4, 1, 2, 2)
    x = np.arange(8, dtype=np.float32)[:, None]
    assert P.permute(g, x)[:, 0].tolist() == [0, 1, 4, 5, 2, 3, 6, 7]


def test_hand_worked_padding_and_time():
    # 3 frames of 1x2 tokens, tile 2x1x2: frame pairs (0,1) and (2,pad); ids 2*t + x
    g = Geometry(3, 1, 2, 2, 1, 2)
    x = (np.arange(6, dtype=np.float32) + 1)[:, None]
    assert P.permute(g, x)[:, 0].tolist() == [1, 2, 3, 4, 5, 6, 0, 0]
    assert P.slot_valid(g).tolist() == [True] * 6 + [False] * 2
    # with tt=2 and a padded row, valid slots are not a prefix of the tile
    g2 = Geometry(2, 1, 1, 2, 2, 1)     # slots (dt, dy): (0,0) (0,1)pad (1,0) (1,1)pad
    assert P.slot_valid(g2).tolist() == [True, False, True, False]


def test_text_tokens_follow_video_tiles():
    g = Geometry(1, 2, 2, 1, 2, 2, n_text=8)
    x = np.arange(12, dtype=np.float32)[:, None]
    assert P.permute(g, x)[:, 0].tolist() == list(range(12))


@st.composite
def _geoms(draw):
    tt, th, tw = draw(st.integers(1, 3)), draw(st.integers(1, 4)), draw(st.integers(1, 4))
    return Geometry(draw(st.integers(1, 6)), draw(st.integers(1, 9)), draw(st.integers(1, 9)), tt, th, tw,
                    n_text=draw(st.integers(0, 2)) * tt * th * tw)


@settings(max_examples=80, deadline=None)
@given(_geoms())
def test_bijection_roundtrip_and_loop_form(g):
    slots = g.token_slots()
    tile, slot = g.token_tile_and_slot()
    assert np.array_equal(slots, tile * g.B + slot)
    assert len(np.unique(slots)) == g.N_real and slots.min() >= 0 and slots.max() < g.N_pad
    rng = np.random.default_rng(0)
    x = rng.standard_normal((2, g.N_real, 3)).astype(np.float32)
    y = P.permute(g, x)
    assert y.shape == (2, g.N_pad, 3)
    assert np.array_equal(P.unpermute(g, y), x)
    assert np.all(y[:, ~P.slot_valid(g)] == 0)
    # every tile holds tokens of one tile box only
    for i in range(g.N_video):
        t, r = divmod(i, g.H * g.W)
        yy, xx = divmod(r, g.W)
        assert tile[i] == g.tile_id(t // g.tt, yy // g.th, xx // g.tw)
