"""The oracle's layout rule against hand-worked examples stored as text (derivations in the file)."""
import os

import numpy as np
import pytest

from oracle import layout as L
from oracle.geometry import Geometry

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "layout_worked_examples.txt")


def _cases():
    out = []
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, grid, tile, n_text, heads, nnz, sparsity = [f.strip() for f in line.split("|")]
        hs = []
        for h in heads.split(";"):
            groups = []
            for grp in h.split(","):
                dt, rha, rwa, rhb, rwb = [int(x) for x in grp.strip().split(":")]
                groups.append((dt, (rha, rwa), (rhb, rwb)))
            hs.append(groups)
        out.append(pytest.param(tuple(int(x) for x in grid.split()), tuple(int(x) for x in tile.split()),
                                int(n_text), hs, [int(x) for x in nnz.split()], float(sparsity), id=name))
    return out


@pytest.mark.parametrize("grid,tile,n_text,heads,nnz,sparsity", _cases())
def test_worked_example(grid, tile, n_text, heads, nnz, sparsity):
    g = Geometry(*grid, *tile, n_text)
    csr = L.build_csr(g, heads)
    assert [int(rp[-1]) for rp, _ in csr] == nnz
    mask = L.keep_mask_bruteforce(g, heads)
    assert [int(m.sum()) for m in mask] == nnz
    assert L.row_counts(g, heads).sum(axis=1).tolist() == nnz
    assert abs(L.sparsity(g, heads) - sparsity) < 1e-12
    for h, (rp, ci) in enumerate(csr):
        for q in range(g.n):
            assert np.array_equal(ci[rp[q]:rp[q + 1]], np.nonzero(mask[h, q])[0])
