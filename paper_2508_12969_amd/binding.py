"""ctypes binding of libcompact_attn.so: argument marshalling only.

Every function has the name of the C entry point it calls (see
include/compact_attn.h).  Tensors are torch tensors used purely as device
buffers; their data pointers and the current torch stream are handed to the
library.  There is no fallback: if the shared library is missing or a call
fails, an exception is raised.
"""
import ctypes
import os

import numpy as np

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "libcompact_attn.so")

CA_OK = 0
CA_ERR_INVALID_ARG = -1
CA_ERR_UNSUPPORTED = -2
CA_ERR_ALLOC = -3
CA_ERR_HIP = -4
CA_F32 = 0
CA_BF16 = 1
CA_MAX_GROUPS = 8

EXPORTED = (
    "compact_attn_build_layout",
    "compact_attn_layout_from_csr",
    "compact_attn_layout_union",
    "compact_attn_layout_similarity",
    "compact_attn_layout_info",
    "compact_attn_layout_csr",
    "compact_attn_layout_order",
    "compact_attn_layout_pairs",
    "compact_attn_layout_packing",
    "compact_attn_layout_upload",
    "compact_attn_free_layout",
    "compact_attn_permute",
    "compact_attn_forward",
    "compact_attn_forward_static",
    "compact_attn_forward_natural",
    "compact_attn_dense",
    "compact_attn_tile_mass",
    "compact_attn_search_head",
    "compact_attn_last_error",
)


class ca_window(ctypes.Structure):
    _fields_ = [("rh", ctypes.c_int32), ("rw", ctypes.c_int32)]


class ca_group(ctypes.Structure):
    _fields_ = [("max_dt", ctypes.c_int32), ("a", ca_window), ("b", ca_window)]


class ca_head(ctypes.Structure):
    _fields_ = [("num_groups", ctypes.c_int32), ("clamp_centre", ctypes.c_int32), ("groups", ctypes.POINTER(ca_group))]


class ca_problem(ctypes.Structure):
    _fields_ = [
        ("T", ctypes.c_int32), ("H", ctypes.c_int32), ("W", ctypes.c_int32),
        ("tt", ctypes.c_int32), ("th", ctypes.c_int32), ("tw", ctypes.c_int32),
        ("n_text", ctypes.c_int32),
        ("batch", ctypes.c_int32), ("num_heads", ctypes.c_int32), ("head_dim", ctypes.c_int32),
        ("dtype", ctypes.c_int32),
        ("scale", ctypes.c_float),
    ]


class CompactAttnError(RuntimeError):
    def __init__(self, status, message):
        super().__init__(f"compact_attn status {status}: {message}")
        self.status = status


_lib = None


def library_path():
    return _LIB_PATH


def load_library():
    """Load libcompact_attn.so (built in-tree by paper_2508_12969_amd.build). No fallback."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise RuntimeError(
            f"{_LIB_PATH} is missing: build it with `python -m paper_2508_12969_amd.build` "
            "(there is no CPU or PyTorch fallback)"
        )
    lib = ctypes.CDLL(_LIB_PATH)
    vp, i32, i64p = ctypes.c_void_p, ctypes.c_int32, ctypes.POINTER(ctypes.c_int64)
    lib.compact_attn_build_layout.argtypes = [ctypes.POINTER(ca_problem), ctypes.POINTER(ca_head), ctypes.POINTER(vp)]
    lib.compact_attn_layout_from_csr.argtypes = [ctypes.POINTER(ca_problem), ctypes.POINTER(i64p),
                                                 ctypes.POINTER(ctypes.POINTER(ctypes.c_int32)), ctypes.POINTER(vp)]
    lib.compact_attn_layout_union.argtypes = [vp, vp, ctypes.POINTER(vp)]
    lib.compact_attn_layout_similarity.argtypes = [vp, i32, vp, i32, ctypes.POINTER(ctypes.c_double)]
    lib.compact_attn_layout_info.argtypes = [vp, i64p, i64p, i64p, i64p, i64p]
    lib.compact_attn_layout_csr.argtypes = [vp, i32, ctypes.POINTER(i64p), ctypes.POINTER(ctypes.POINTER(ctypes.c_int32))]
    lib.compact_attn_layout_order.argtypes = [vp, ctypes.POINTER(ctypes.POINTER(ctypes.c_int32))]
    lib.compact_attn_layout_pairs.argtypes = [vp, ctypes.POINTER(ctypes.POINTER(ctypes.c_int32)), i64p, ctypes.POINTER(i64p),
                                              ctypes.POINTER(ctypes.POINTER(ctypes.c_int32))]
    lib.compact_attn_layout_packing.argtypes = [vp, ctypes.POINTER(ctypes.POINTER(ctypes.c_int32)),
                                                ctypes.POINTER(ctypes.POINTER(ctypes.c_int32)), i64p]
    lib.compact_attn_layout_upload.argtypes = [vp]
    lib.compact_attn_free_layout.argtypes = [vp]
    lib.compact_attn_free_layout.restype = None
    lib.compact_attn_permute.argtypes = [vp, vp, vp, i32, vp]
    lib.compact_attn_forward.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.compact_attn_forward_natural.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.compact_attn_forward_static.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.compact_attn_dense.argtypes = [vp, vp, vp, vp, vp, vp]
    lib.compact_attn_tile_mass.argtypes = [vp, vp, vp, vp, vp]
    lib.compact_attn_search_head.argtypes = [vp, ctypes.POINTER(ctypes.c_float), ctypes.POINTER(i32), i32, ctypes.c_double,
                                             ctypes.c_double, i32, ctypes.POINTER(ca_group), ctypes.POINTER(ctypes.c_double),
                                             ctypes.POINTER(ctypes.c_double)]
    lib.compact_attn_last_error.argtypes = []
    lib.compact_attn_last_error.restype = ctypes.c_char_p
    for name in EXPORTED:
        if name not in ("compact_attn_free_layout", "compact_attn_last_error"):
            getattr(lib, name).restype = ctypes.c_int
    _lib = lib
    return lib


def compact_attn_last_error():
    return load_library().compact_attn_last_error().decode()


def _check(status):
    if status != CA_OK:
        raise CompactAttnError(status, compact_attn_last_error())


class Layout:
    """Owner of a ca_layout*; keeps the problem description for shape checks."""

    def __init__(self, handle, problem):
        self.handle = handle
        self.problem = problem
        n, B, n_real, n_pad, nnz = (ctypes.c_int64() for _ in range(5))
        _check(load_library().compact_attn_layout_info(handle, n, B, n_real, n_pad, nnz))
        self.n_tiles, self.tokens_per_tile = n.value, B.value
        self.n_tokens_real, self.n_tokens_padded, self.nnz_total = n_real.value, n_pad.value, nnz.value

    def free(self):
        if self.handle is not None:
            load_library().compact_attn_free_layout(self.handle)
            self.handle = None

    def __del__(self):
        try:
            self.free()
        except Exception:
            pass

    def shape(self, padded):
        p = self.problem
        return (p.batch, p.num_heads, self.n_tokens_padded if padded else self.n_tokens_real, p.head_dim)


def compact_attn_build_layout(T, H, W, tile, n_text, batch, num_heads, head_dim, dtype, heads, scale=0.0, clamp_centre=False):
    """heads: per head a list of (max_dt, (rh, rw), (rh, rw)); dtype "f32" or "bf16".
    clamp_centre: one flag for all heads or one per head: windows keep their size at the border."""
    lib = load_library()
    if len(heads) != num_heads:
        raise ValueError("one head description per head is required")
    prob = ca_problem(T, H, W, tile[0], tile[1], tile[2], n_text, batch, num_heads, head_dim,
                      {"f32": CA_F32, "bf16": CA_BF16}[dtype], scale)
    keep = []
    c_heads = (ca_head * num_heads)()
    for i, groups in enumerate(heads):
        arr = (ca_group * max(len(groups), 1))()
        for j, (max_dt, a, b) in enumerate(groups):
            arr[j] = ca_group(max_dt, ca_window(*a), ca_window(*b))
        keep.append(arr)
        c_heads[i].num_groups = len(groups)
        c_heads[i].clamp_centre = int(clamp_centre[i] if isinstance(clamp_centre, (list, tuple)) else clamp_centre)
        c_heads[i].groups = ctypes.cast(arr, ctypes.POINTER(ca_group))
    handle = ctypes.c_void_p()
    _check(lib.compact_attn_build_layout(ctypes.byref(prob), c_heads, ctypes.byref(handle)))
    return Layout(handle, prob)


def compact_attn_layout_from_csr(T, H, W, tile, n_text, batch, num_heads, head_dim, dtype, csr, scale=0.0):
    """csr: per head (row_ptr int64[n+1], col_idx int32[nnz]); an arbitrary tile mask, taken as given."""
    lib = load_library()
    if len(csr) != num_heads:
        raise ValueError("one CSR per head is required")
    prob = ca_problem(T, H, W, tile[0], tile[1], tile[2], n_text, batch, num_heads, head_dim,
                      {"f32": CA_F32, "bf16": CA_BF16}[dtype], scale)
    rps = [np.ascontiguousarray(rp, dtype=np.int64) for rp, _ in csr]
    cis = [np.ascontiguousarray(ci, dtype=np.int32) for _, ci in csr]
    rp_arr = (ctypes.POINTER(ctypes.c_int64) * num_heads)(*[a.ctypes.data_as(ctypes.POINTER(ctypes.c_int64)) for a in rps])
    ci_arr = (ctypes.POINTER(ctypes.c_int32) * num_heads)(*[a.ctypes.data_as(ctypes.POINTER(ctypes.c_int32)) for a in cis])
    handle = ctypes.c_void_p()
    _check(lib.compact_attn_layout_from_csr(ctypes.byref(prob), rp_arr, ci_arr, ctypes.byref(handle)))
    return Layout(handle, prob)


def compact_attn_layout_union(a, b):
    handle = ctypes.c_void_p()
    _check(load_library().compact_attn_layout_union(a.handle, b.handle, ctypes.byref(handle)))
    return Layout(handle, a.problem)


def compact_attn_layout_similarity(a, head_a, b, head_b):
    sim = ctypes.c_double()
    _check(load_library().compact_attn_layout_similarity(a.handle, head_a, b.handle, head_b, ctypes.byref(sim)))
    return sim.value


def compact_attn_layout_info(layout):
    return dict(n_tiles=layout.n_tiles, tokens_per_tile=layout.tokens_per_tile, n_tokens_real=layout.n_tokens_real,
                n_tokens_padded=layout.n_tokens_padded, nnz_total=layout.nnz_total)


def compact_attn_layout_csr(layout, head):
    """(row_ptr int64[n+1], col_idx int32[nnz_head]) copied out of the layout."""
    rp = ctypes.POINTER(ctypes.c_int64)()
    ci = ctypes.POINTER(ctypes.c_int32)()
    _check(load_library().compact_attn_layout_csr(layout.handle, head, ctypes.byref(rp), ctypes.byref(ci)))
    row_ptr = np.ctypeslib.as_array(rp, shape=(layout.n_tiles + 1,)).copy()
    nnz = int(row_ptr[-1])
    col_idx = np.ctypeslib.as_array(ci, shape=(nnz,)).copy() if nnz else np.zeros(0, np.int32)
    return row_ptr, col_idx


def compact_attn_layout_order(layout):
    o = ctypes.POINTER(ctypes.c_int32)()
    _check(load_library().compact_attn_layout_order(layout.handle, ctypes.byref(o)))
    return np.ctypeslib.as_array(o, shape=(layout.problem.num_heads * layout.n_tiles,)).copy()


def compact_attn_layout_pairs(layout):
    """(pairs int32 [num_pairs, 2] of row ids, second -1 for a single, in launch order;
    walk_ptr int64 [num_pairs + 1]; walk int32 words: tile id | 1 << 30 (first keeps it) | 1 << 31 (second)).
    All empty if the layout is not served by the paired kernel."""
    p = ctypes.POINTER(ctypes.c_int32)()
    wp = ctypes.POINTER(ctypes.c_int64)()
    w = ctypes.POINTER(ctypes.c_int32)()
    count = ctypes.c_int64(0)
    _check(load_library().compact_attn_layout_pairs(layout.handle, ctypes.byref(p), ctypes.byref(count), ctypes.byref(wp),
                                                    ctypes.byref(w)))
    if count.value == 0:
        return np.zeros((0, 2), dtype=np.int32), np.zeros(1, dtype=np.int64), np.zeros(0, dtype=np.int32)
    pairs = np.ctypeslib.as_array(p, shape=(count.value, 2)).copy()
    walk_ptr = np.ctypeslib.as_array(wp, shape=(count.value + 1,)).copy()
    total = int(walk_ptr[-1])
    walk = np.ctypeslib.as_array(w, shape=(total,)).copy() if total else np.zeros(0, dtype=np.int32)
    return pairs, walk_ptr, walk


def compact_attn_layout_packing(layout):
    """(desc uint32 [num_pairs]: wave assignment of every two-tile workgroup; launch_rows int32: launch order of the
    one-row-per-workgroup kernel: row ids, and ~i for two-tile workgroup i run by the same launch)."""
    d = ctypes.POINTER(ctypes.c_int32)()
    r = ctypes.POINTER(ctypes.c_int32)()
    count = ctypes.c_int64(0)
    _check(load_library().compact_attn_layout_packing(layout.handle, ctypes.byref(d), ctypes.byref(r), ctypes.byref(count)))
    num_pairs = compact_attn_layout_pairs(layout)[0].shape[0]
    desc = np.ctypeslib.as_array(d, shape=(num_pairs,)).copy().view(np.uint32) if num_pairs else np.zeros(0, dtype=np.uint32)
    rows = np.ctypeslib.as_array(r, shape=(count.value,)).copy() if count.value else np.zeros(0, dtype=np.int32)
    return desc, rows


def compact_attn_layout_upload(layout):
    _check(load_library().compact_attn_layout_upload(layout.handle))


def compact_attn_free_layout(layout):
    layout.free()


def _torch_dtype(layout):
    import torch
    return torch.bfloat16 if layout.problem.dtype == CA_BF16 else torch.float32


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _check_tensor(t, layout, padded, name):
    if not t.is_cuda:
        raise ValueError(f"{name} must be a device tensor")
    if not t.is_contiguous():
        raise ValueError(f"{name} must be contiguous")
    if t.dtype != _torch_dtype(layout):
        raise ValueError(f"{name} has dtype {t.dtype}, layout expects {_torch_dtype(layout)}")
    if tuple(t.shape) != layout.shape(padded):
        raise ValueError(f"{name} has shape {tuple(t.shape)}, expected {layout.shape(padded)}")


def compact_attn_permute(src, layout, inverse=False, out=None, stream=None):
    """natural order -> tile order (inverse=False) or back (inverse=True)."""
    import torch
    _check_tensor(src, layout, padded=bool(inverse), name="src")
    if out is None:
        out = torch.empty(layout.shape(padded=not inverse), dtype=src.dtype, device=src.device)
    _check_tensor(out, layout, padded=not inverse, name="out")
    _check(load_library().compact_attn_permute(ctypes.c_void_p(src.data_ptr()), ctypes.c_void_p(out.data_ptr()),
                                               layout.handle, int(bool(inverse)), _stream_ptr(stream)))
    return out


def _attention(fn, q, k, v, layout, out, stream, padded=True):
    import torch
    for name, t in (("q", q), ("k", k), ("v", v)):
        _check_tensor(t, layout, padded, name)
    if out is None:
        out = torch.empty_like(q)
    _check_tensor(out, layout, padded, "out")
    _check(fn(ctypes.c_void_p(q.data_ptr()), ctypes.c_void_p(k.data_ptr()), ctypes.c_void_p(v.data_ptr()),
              layout.handle, ctypes.c_void_p(out.data_ptr()), _stream_ptr(stream)))
    return out


def compact_attn_forward(q, k, v, layout, out=None, stream=None):
    """Sparse attention over tile-ordered, padded q/k/v [batch, heads, N_pad, D]."""
    return _attention(load_library().compact_attn_forward, q, k, v, layout, out, stream)


def compact_attn_forward_static(q, k, v, layout, out=None, stream=None):
    """compact_attn_forward with the layout tables in the library's fixed device array (no allocation
    inside the call; pass `out`, or the binding allocates it before the call)."""
    return _attention(load_library().compact_attn_forward_static, q, k, v, layout, out, stream)


def compact_attn_forward_natural(q, k, v, layout, out=None, stream=None):
    """Sparse attention over natural-order q/k/v [batch, heads, N_real, D]; the result is in natural order too."""
    return _attention(load_library().compact_attn_forward_natural, q, k, v, layout, out, stream, padded=False)


def compact_attn_tile_mass(q, k, layout, out=None, stream=None):
    """q, k: tile-ordered padded device tensors -> float32 [batch, heads, n, n] attention mass per tile pair."""
    import torch
    _check_tensor(q, layout, True, "q")
    _check_tensor(k, layout, True, "k")
    p = layout.problem
    shape = (p.batch, p.num_heads, layout.n_tiles, layout.n_tiles)
    if out is None:
        out = torch.empty(shape, dtype=torch.float32, device=q.device)
    elif tuple(out.shape) != shape or out.dtype != torch.float32 or not out.is_contiguous() or out.device != q.device:
        raise ValueError(f"out must be a contiguous float32 tensor of shape {shape} on {q.device}")
    _check(load_library().compact_attn_tile_mass(q.data_ptr(), k.data_ptr(), layout.handle, out.data_ptr(), _stream_ptr(stream)))
    return out


CA_PATTERNS = {"cubic": 0, "frame_groups": 1, "dual": 2}


def compact_attn_search_head(layout, mass, group_max_dt, tau, lam, pattern="dual"):
    """mass: host float32 [n, n] of one head -> (groups in the head format, recall, kept pair fraction)."""
    if pattern not in CA_PATTERNS:
        raise ValueError(f"pattern must be one of {tuple(CA_PATTERNS)}")
    mass = np.ascontiguousarray(mass, dtype=np.float32)
    if mass.shape != (layout.n_tiles, layout.n_tiles):
        raise ValueError(f"mass must have shape {(layout.n_tiles, layout.n_tiles)}")
    G = len(group_max_dt)
    dts = (ctypes.c_int32 * max(G, 1))(*group_max_dt)
    groups = (ca_group * max(G, 1))()
    recall, kept = ctypes.c_double(), ctypes.c_double()
    _check(load_library().compact_attn_search_head(layout.handle, mass.ctypes.data_as(ctypes.POINTER(ctypes.c_float)), dts, G,
                                                   float(tau), float(lam), CA_PATTERNS[pattern], groups, ctypes.byref(recall),
                                                   ctypes.byref(kept)))
    out = [(g.max_dt, (g.a.rh, g.a.rw), (g.b.rh, g.b.rw)) for g in groups[:G]]
    return out, recall.value, kept.value


def compact_attn_dense(q, k, v, layout, out=None, stream=None):
    """Same kernel with every query tile keeping all tiles."""
    return _attention(load_library().compact_attn_dense, q, k, v, layout, out, stream)
