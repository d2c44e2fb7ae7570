"""compact_attn_forward_static: the sparse forward whose layout tables live in a fixed device array
inside the library (for callers that cannot allocate).  Same kernels as compact_attn_forward, so the
outputs must be equal bit for bit; checked on calls in a row that replace the array's contents with
a larger, then a smaller layout, and on the size limit."""
import ctypes

import pytest
import torch

import paper_2508_12969_amd as ca
from workloads import get_workload, make_qkv

from helpers import build_layout, make_workload

pytestmark = pytest.mark.gpu
ABSENT = (-1, -1)
DEV = "cuda:0"


def _inputs(wl, lay):
    q, k, v = make_qkv(wl, DEV)
    return tuple(ca.compact_attn_permute(t, lay) for t in (q, k, v))


def _raw_static(lay, qp, kp, vp, out):
    """The C symbol itself, with plain pointers (no binding helper in between)."""
    lib = ca.load_library()
    st = lib.compact_attn_forward_static(ctypes.c_void_p(qp.data_ptr()), ctypes.c_void_p(kp.data_ptr()),
                                         ctypes.c_void_p(vp.data_ptr()), lay.handle, ctypes.c_void_p(out.data_ptr()),
                                         ctypes.c_void_p(torch.cuda.current_stream().cuda_stream))
    return st, lib.compact_attn_last_error().decode()


def test_static_forward_two_calls_in_a_row_second_smaller():
    print("static forward: cfg2, then a smaller padded grid, then cfg2 again", flush=True)
    big = get_workload("cfg2")                                          # B=64 D=64, 109 248 kept pairs
    heads = [[(0, (1, 1), ABSENT), (1, (0, 0), ABSENT)], [(2, (0, 2), (1, 0))], []]
    small = make_workload("static-small", 5, 13, 20, (2, 8, 8), 128, len(heads), 128, "bf16", heads)
    paired = make_workload("static-pair", 3, 13, 20, (1, 8, 8), 64, len(heads), 128, "bf16", heads)   # paired kernel
    cases = []
    for wl in (big, small, paired):
        lay = build_layout(ca, wl)
        qp, kp, vp = _inputs(wl, lay)
        want = ca.compact_attn_forward(qp, kp, vp, lay)                 # the existing entry point
        cases.append((wl, lay, qp, kp, vp, want))
    torch.cuda.synchronize()
    for wl, lay, qp, kp, vp, want in cases + cases[:1]:                 # big, small, paired, big again
        out = torch.full_like(qp, float("nan"))
        st, msg = _raw_static(lay, qp, kp, vp, out)
        assert st == 0, msg
        torch.cuda.synchronize()
        assert torch.equal(out, want), wl.name
        out2 = torch.full_like(qp, float("nan"))                        # same layout again: tables already in place
        st, msg = _raw_static(lay, qp, kp, vp, out2)
        assert st == 0, msg
        torch.cuda.synchronize()
        assert torch.equal(out2, want), wl.name


def test_static_forward_rejects_a_layout_beyond_the_array():
    print("static forward: size limit", flush=True)
    wl = get_workload("cfg4-S80")                                       # 5.3 M kept pairs: 21 MB of tile words
    lay = build_layout(ca, wl)
    x = torch.zeros(lay.shape(True), dtype=torch.bfloat16, device=DEV)
    out = torch.full_like(x, 1.0)
    st, msg = _raw_static(lay, x, x.clone(), x.clone(), out)
    assert st == -2 and "static device array holds" in msg, (st, msg)
    torch.cuda.synchronize()
    assert torch.all(out == 1.0)                                        # nothing was enqueued


def test_static_forward_fp32_problem():
    print("static forward: fp32 kernel", flush=True)
    wl = get_workload("cfg1")
    lay = build_layout(ca, wl)
    qp, kp, vp = _inputs(wl, lay)
    want = ca.compact_attn_forward(qp, kp, vp, lay)
    got = ca.compact_attn_forward_static(qp, kp, vp, lay)
    torch.cuda.synchronize()
    assert torch.equal(got, want)


def test_static_forward_in_a_captured_graph_and_upload_refused_under_capture():
    """After one call with a layout outside a capture, compact_attn_forward_static enqueues kernels only and
    can be captured; replays reproduce the eager result.  compact_attn_forward with a layout whose tables
    are not on the device yet refuses to allocate under capture and names the call to make first."""
    print("static forward: graph capture", flush=True)
    heads = [[(0, (1, 1), ABSENT), (1, (0, 0), ABSENT)], [(2, (0, 2), (1, 0))]]
    wl = make_workload("static-graph", 5, 13, 20, (2, 8, 8), 128, len(heads), 128, "bf16", heads)
    lay = build_layout(ca, wl)
    qp, kp, vp = _inputs(wl, lay)
    want = ca.compact_attn_forward(qp, kp, vp, lay)
    out = torch.zeros_like(qp)
    ca.compact_attn_forward_static(qp, kp, vp, lay, out=out)          # stages the tables
    torch.cuda.synchronize()
    assert torch.equal(out, want)
    fresh = build_layout(ca, wl)                                        # never uploaded
    other = torch.zeros_like(qp)
    graph = torch.cuda.CUDAGraph()
    refused = None
    with torch.cuda.graph(graph):
        ca.compact_attn_forward_static(qp, kp, vp, lay, out=out)
        try:
            ca.compact_attn_forward(qp, kp, vp, fresh, out=other)
        except ca.CompactAttnError as exc:
            refused = exc
    assert refused is not None and refused.status == -1 and "compact_attn_layout_upload" in str(refused)
    for rep in range(3):
        out.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(out, want), f"replay {rep}"
        _ = (qp.float() * 1.0001).sum().item()                          # eager work between replays
