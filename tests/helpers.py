"""Shared plumbing for the tests: build the same problem on both sides, move data, compare."""
import numpy as np

from oracle.geometry import Geometry

BF16_MAX_ABS = 2e-2     # bar stated for bf16 outputs
BF16_MEAN_ABS = 2e-3
F32_MAX_ABS = 1e-4      # fp32 path: fp32 accumulation over <= 1e5 keys of O(1) values
F32_MEAN_ABS = 1e-5


def geometry_of(wl):
    return Geometry(wl.T, wl.H, wl.W, *wl.tile, wl.n_text)


def build_layout(ca, wl, scale=0.0):
    return ca.compact_attn_build_layout(wl.T, wl.H, wl.W, wl.tile, wl.n_text, wl.batch, wl.num_heads, wl.head_dim,
                                        wl.dtype, wl.heads, scale)


def make_workload(name, T, H, W, tile, n_text, num_heads, head_dim, dtype, heads, cfg=9):
    from workloads.configs import Workload
    return Workload(name, cfg, T, H, W, tuple(tile), n_text, num_heads, head_dim, dtype, tuple(heads), None)


def gpu_attention(ca, wl, layout, q, k, v, dense=False):
    """natural-order device tensors -> natural-order output, every step on the library's kernels."""
    qp = ca.compact_attn_permute(q, layout)
    kp = ca.compact_attn_permute(k, layout)
    vp = ca.compact_attn_permute(v, layout)
    fn = ca.compact_attn_dense if dense else ca.compact_attn_forward
    op = fn(qp, kp, vp, layout)
    return ca.compact_attn_permute(op, layout, inverse=True), op


def to_f64(t):
    return t.detach().to("cpu").double().numpy()


def compare(got, want, max_abs, mean_abs, what=""):
    got = np.asarray(got, dtype=np.float64)
    want = np.asarray(want, dtype=np.float64)
    assert got.shape == want.shape, (got.shape, want.shape)
    assert np.all(np.isfinite(got)), f"{what}: non-finite output"
    err = np.abs(got - want)
    assert err.max() <= max_abs, f"{what}: max abs err {err.max():.3e} > {max_abs}"
    assert err.mean() <= mean_abs, f"{what}: mean abs err {err.mean():.3e} > {mean_abs}"
    return err.max(), err.mean()


def tolerances(dtype):
    return (BF16_MAX_ABS, BF16_MEAN_ABS) if dtype == "bf16" else (F32_MAX_ABS, F32_MEAN_ABS)


def sample_query_tiles(geom, counts_head, rng, extra=4):
    """Stratified query tiles of one head: fewest / most kept, edges, text, a few random."""
    n = geom.n
    picks = {int(np.argmin(counts_head)), int(np.argmax(counts_head)), 0, geom.n_vid - 1}
    picks.add(geom.tile_id(geom.nT - 1, geom.nH - 1, 0))       # T-edge and H-edge tile
    picks.add(geom.tile_id(geom.nT // 2, geom.nH - 1, geom.nW // 2))
    picks.add(geom.tile_id(geom.nT // 2, geom.nH // 2, geom.nW // 2))
    if geom.n_txt:
        picks.add(n - 1)
    picks.update(int(x) for x in rng.choice(n, extra, replace=False))
    return sorted(picks)
