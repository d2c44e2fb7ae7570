"""Token grid and space-time tile arithmetic (oracle side; test infrastructure).

A video latent is a grid of T x H x W tokens (frames, rows, columns).  A
space-time tile is a box of tt x th x tw neighbouring tokens (Sec. 4.1: a
cluster of tokens adjacent in space and time); it is the unit of masking.
Grids that are not a multiple of the tile shape are padded on the high side
of each axis; padded positions hold no token.  `n_text` prompt tokens, a
multiple of the tile size, follow the video tokens and form tiles of their
own after the video tiles.

Orders (the paper fixes neither; any choice gives the same attention result):
natural order is row-major (t, y, x), text last; tile ids are row-major over
the tile grid; positions inside a tile are row-major (t, y, x).
"""
from dataclasses import dataclass

import numpy as np


def ceil_div(a, b):
    return -(-a // b)


@dataclass(frozen=True)
class Geometry:
    T: int
    H: int
    W: int
    tt: int
    th: int
    tw: int
    n_text: int = 0

    def __post_init__(self):
        for name in ("T", "H", "W", "tt", "th", "tw"):
            if getattr(self, name) <= 0:
                raise ValueError(f"{name} must be positive")
        if self.n_text < 0 or self.n_text % self.B != 0:
            raise ValueError("n_text must be a non-negative multiple of the tile size")

    @property
    def B(self):
        """tokens per tile"""
        return self.tt * self.th * self.tw

    @property
    def nT(self):
        return ceil_div(self.T, self.tt)

    @property
    def nH(self):
        return ceil_div(self.H, self.th)

    @property
    def nW(self):
        return ceil_div(self.W, self.tw)

    @property
    def n_vid(self):
        """number of video tiles"""
        return self.nT * self.nH * self.nW

    @property
    def n_txt(self):
        """number of text tiles"""
        return self.n_text // self.B

    @property
    def n(self):
        """number of tiles"""
        return self.n_vid + self.n_txt

    @property
    def N_video(self):
        return self.T * self.H * self.W

    @property
    def N_real(self):
        """tokens that exist (natural order length)"""
        return self.N_video + self.n_text

    @property
    def N_pad(self):
        """tile-ordered, padded length"""
        return self.n * self.B

    def tile_coords(self, tile):
        """(kt, kh, kw) of a video tile id."""
        if not 0 <= tile < self.n_vid:
            raise ValueError("not a video tile")
        kw = tile % self.nW
        kh = (tile // self.nW) % self.nH
        kt = tile // (self.nW * self.nH)
        return kt, kh, kw

    def tile_id(self, kt, kh, kw):
        return (kt * self.nH + kh) * self.nW + kw

    def token_tile_and_slot(self):
        """For every real token in natural order: (tile id, position in tile).

        Written as explicit loops over the grid so that it can be read against
        the definition; vectorised users should call `token_slots()`.
        """
        tile = np.empty(self.N_real, dtype=np.int64)
        slot = np.empty(self.N_real, dtype=np.int64)
        i = 0
        for t in range(self.T):
            for y in range(self.H):
                for x in range(self.W):
                    tile[i] = self.tile_id(t // self.tt, y // self.th, x // self.tw)
                    slot[i] = ((t % self.tt) * self.th + (y % self.th)) * self.tw + (x % self.tw)
                    i += 1
        for j in range(self.n_text):
            tile[i] = self.n_vid + j // self.B
            slot[i] = j % self.B
            i += 1
        return tile, slot

    def token_slots(self):
        """Padded tile-order index (tile * B + slot) of every real token, natural order."""
        t, y, x = np.meshgrid(np.arange(self.T), np.arange(self.H), np.arange(self.W), indexing="ij")
        tile = ((t // self.tt) * self.nH + (y // self.th)) * self.nW + (x // self.tw)
        slot = ((t % self.tt) * self.th + (y % self.th)) * self.tw + (x % self.tw)
        vid = (tile * self.B + slot).reshape(-1).astype(np.int64)
        txt = self.n_vid * self.B + np.arange(self.n_text, dtype=np.int64)
        return np.concatenate([vid, txt])
