#!/usr/bin/env python3
"""Benchmark of the Compact Attention hot path on one MI355X.

A step is one pass of the whole path over one batch of synthetic, HBM-resident
inputs: tile-order permutation of Q, K and V, the block-sparse attention
forward, and the inverse permutation of the output.  The layout (CSR of kept
tiles) is built once before timing, as the method precomputes it offline.

Prints one JSON line: whole-step throughput in effective TFLOP/s (FLOPs of the
kept tile pairs / step time) with the attention kernel's own time, its
fraction of the bf16 MFMA roofline, the speed-up over the same kernel with the
full mask, and the fp64 oracle timed on the host cores for context.
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

PEAK_BF16_TFLOPS = 2500.0   # MI355X dense bf16 MFMA

# HBM bytes of one forward launch, from rocprofv3 FETCH_SIZE / WRITE_SIZE counter runs of this
# script scaled by a 1 GiB device copy in the same run.  A counter run is a separate profiler pass,
# so the figure is a recorded measurement, not one taken live: it is printed with the summary file
# it comes from, and as null for a workload without a committed counter run.
RECORDED_TRAFFIC = {
    "cfg4-S65": {"bytes": 113.8e9, "source": "profiles/attn_bf16_kernel_cfg4-S65_pmc.md"},
    "cfg3": {"bytes": 60.3e9, "source": "profiles/attn_bf16_pair_kernel_cfg3.md"},
}
OTHER_CONFIGS = ("cfg4-S50", "cfg4-S80", "cfg3", "cfg5")


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=20)
    ap.add_argument("--warmup", type=int, default=5)
    ap.add_argument("--workload", default="cfg4-S65")
    ap.add_argument("--dense-calls", type=int, default=3, help="timed calls of the dense kernel (0 = skip)")
    ap.add_argument("--cpu-seconds", type=float, default=15.0, help="budget of the oracle leg (0 = skip)")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also launch one plain 1 GiB device copy (torch) so that a rocprofv3 --pmc run of this "
                         "command holds a kernel of known traffic to scale FETCH_SIZE / WRITE_SIZE by")
    ap.add_argument("--mass-calls", type=int, default=2, help="timed calls of the tile-mass kernel (0 = skip)")
    ap.add_argument("--natural-calls", type=int, default=3,
                    help="timed calls of compact_attn_forward_natural, the forward with the gather / scatter fused in "
                         "(0 = skip)")
    ap.add_argument("--pattern-report", action="store_true",
                    help="also search masks under the three pattern families of Table 3 on structured synthetic heads "
                         "and report the sparsity each family reaches")
    ap.add_argument("--context-calls", type=int, default=3,
                    help="timed calls of the forward on all-zero inputs and of a plain device copy (0 = skip)")
    ap.add_argument("--other-calls", type=int, default=5,
                    help="timed sparse forward calls on each of the other configurations (cfg4 at 50 %% and 80 %% "
                         "sparsity, cfg3, cfg5), each with the dense kernel at the same shape beside it (0 = skip)")
    return ap.parse_args()


def executed_fraction(ca, lay, wl):
    """Share of the nominal matrix products the kernel really issues.  The queries of a padded tile
    are packed into as few 32-query waves as possible and the remaining waves skip their products;
    on the key side the upper half of a tile's key blocks is skipped when it holds padding only."""
    import numpy as np
    tt, th, tw = wl.tile
    B = tt * th * tw
    nT, nH, nW = -(-wl.T // tt), -(-wl.H // th), -(-wl.W // tw)
    n_vid = nT * nH * nW
    if B < 64:
        return 1.0
    a, b, c = np.meshgrid(np.arange(tt), np.arange(th), np.arange(tw), indexing="ij")
    a, b, c = a.ravel(), b.ravel(), c.ravel()                      # slot -> offsets inside a tile
    tf, hf, wf = np.unravel_index(np.arange(n_vid), (nT, nH, nW))
    valid = ((tf[:, None] * tt + a[None] < wl.T) & (hf[:, None] * th + b[None] < wl.H)
             & (wf[:, None] * tw + c[None] < wl.W))                # [n_vid, B]
    valid = np.concatenate([valid, np.ones((lay.n_tiles - n_vid, B), bool)])
    blocks = valid.reshape(lay.n_tiles, B // 32, 32).any(axis=2)    # [n, B/32]
    q_waves = np.ceil(valid.sum(axis=1) / 32) / (B // 32)           # active query waves of a tile
    k_share = np.where(blocks[:, B // 64:].any(axis=1), 1.0, 0.5)   # upper key half skipped when empty
    done = 0.0
    for h in range(wl.num_heads):
        row_ptr, col_idx = ca.compact_attn_layout_csr(lay, h)
        per_row = np.add.reduceat(k_share[col_idx], row_ptr[:-1]) if len(col_idx) else np.zeros(lay.n_tiles)
        per_row[np.diff(row_ptr) == 0] = 0.0
        done += float((per_row * q_waves).sum())
    return done / lay.nnz_total


def cpu_baseline(wl, q, k, v, budget_s):
    """The oracle, as it stands, on a bounded sample of query tiles of the same workload."""
    import numpy as np
    from oracle import attention as OA
    from oracle import layout as OL
    from oracle.geometry import Geometry
    geom = Geometry(wl.T, wl.H, wl.W, *wl.tile, wl.n_text)

    try:
        from threadpoolctl import threadpool_info
        threads = max([p.get("num_threads", 1) for p in threadpool_info()] or [os.cpu_count() or 1])
    except Exception:
        threads = os.cpu_count() or 1
    rng = np.random.default_rng(2508)
    tok_tile, _ = geom.token_tile_and_slot()
    pairs = 0
    tiles = 0
    heads_used = set()
    t0 = time.perf_counter()
    cache = {}
    while time.perf_counter() - t0 < budget_s:
        h = int(rng.integers(wl.num_heads))
        if h not in cache:
            cache.clear()
            cache[h] = tuple(t[0, h].cpu().double().numpy() for t in (q, k, v))
        q_tile = int(rng.integers(geom.n))
        OA.attention_tile(geom, wl.heads[h], q_tile, *cache[h], token_tile=tok_tile)
        pairs += OL.row_count_closed_form(geom, wl.heads[h], q_tile)
        tiles += 1
        heads_used.add(h)
    dt = time.perf_counter() - t0
    flops = pairs * 4.0 * geom.B * geom.B * wl.head_dim
    return {
        "value": flops / dt / 1e12, "unit": "TFLOP/s", "cores": int(threads), "kind": "oracle",
        "sample": f"{tiles} random (head, query tile) rows of {wl.name} ({pairs} tile pairs) in {dt:.1f} s, "
                  "fp64 numpy incl. host copies; FLOPs counted as for the GPU (4*B^2*D per kept tile pair)",
    }


# Head kinds of Sec. 3.2 as gains of the positional code per axis (t, y, x); see workloads/inputs.py
PATTERN_HEADS = (("local", (2.5, 2.5, 2.5)), ("cross, fading with frame distance", (1.0, 3.0, 3.0)),
                 ("global", (0.0, 0.0, 0.0)), ("own frame", (3.0, 1.0, 1.0)), ("cross, time-invariant", (0.0, 2.5, 2.5)))


def pattern_report(ca, dev, tau=0.9, lam=0.6):
    """Sparsity reached by the window search under each pattern family (the structure of Table 3: a
    cubic window, + one window per frame group, + dual windows) on synthetic heads with the same
    thresholds.  The numbers describe the synthetic heads, not a trained model."""
    import torch
    from workloads.configs import Workload
    from workloads.inputs import make_qkv
    heads = [[]] * len(PATTERN_HEADS)
    wl = Workload("patterns", 9, 12, 48, 80, (2, 8, 8), 0, len(heads), 128, "bf16", tuple(heads), None)
    lay = ca.compact_attn_build_layout(wl.T, wl.H, wl.W, wl.tile, wl.n_text, wl.batch, wl.num_heads, wl.head_dim,
                                       wl.dtype, wl.heads, 0.0)
    q, k, _ = make_qkv(wl, dev, axis_gain=[g for _, g in PATTERN_HEADS])
    mass = ca.compact_attn_tile_mass(ca.compact_attn_permute(q, lay), ca.compact_attn_permute(k, lay), lay)
    torch.cuda.synchronize()
    mass = mass[0].cpu().numpy()
    nT = -(-wl.T // wl.tile[0])
    bounds = list(range(nT))                      # one group per tile-frame distance
    out = {"tau": tau, "lambda": lam, "grid_tiles": [nT, -(-wl.H // wl.tile[1]), -(-wl.W // wl.tile[2])], "heads": {}}
    totals = {p: 0.0 for p in ("cubic", "frame_groups", "dual")}
    for h, (kind, _) in enumerate(PATTERN_HEADS):
        row = {}
        for pattern in totals:
            _, recall, kept = ca.compact_attn_search_head(lay, mass[h], bounds, tau, lam, pattern)
            row[pattern] = {"sparsity": 1.0 - kept, "recall": recall}
            totals[pattern] += (1.0 - kept) / len(PATTERN_HEADS)
        out["heads"][kind] = row
    out["overall_sparsity"] = totals
    lay.free()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        print("bench.py: this build runs on one GPU only (the path has no collective); use --gpus 1", file=sys.stderr)
        sys.exit(2)
    import torch

    import paper_2508_12969_amd as ca
    from workloads import get_workload, make_qkv

    torch.cuda.set_device(0)
    dev = "cuda:0"
    wl = get_workload(args.workload)

    def layout_of(w):
        return ca.compact_attn_build_layout(w.T, w.H, w.W, w.tile, w.n_text, w.batch, w.num_heads, w.head_dim, w.dtype, w.heads)

    t0 = time.perf_counter()
    lay = layout_of(wl)
    ca.compact_attn_layout_upload(lay)
    layout_build_s = time.perf_counter() - t0
    q, k, v = make_qkv(wl, dev)
    shape_p = lay.shape(True)
    qp, kp, vp, op = (torch.empty(shape_p, dtype=q.dtype, device=dev) for _ in range(4))
    out = torch.empty_like(q)

    ev = lambda: torch.cuda.Event(enable_timing=True)

    def median_ms(fn, calls):
        fn()
        torch.cuda.synchronize()
        ts = []
        for _ in range(calls):
            a, b = ev(), ev()
            a.record()
            fn()
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        return sorted(ts)[len(ts) // 2]

    n_ev = args.steps
    e_fwd = [(ev(), ev()) for _ in range(n_ev)]
    e_perm = [(ev(), ev()) for _ in range(n_ev)]

    def step(i=None):
        if i is not None:
            e_perm[i][0].record()
        ca.compact_attn_permute(q, lay, out=qp)
        ca.compact_attn_permute(k, lay, out=kp)
        ca.compact_attn_permute(v, lay, out=vp)
        if i is not None:
            e_perm[i][1].record()
            e_fwd[i][0].record()
        ca.compact_attn_forward(qp, kp, vp, lay, out=op)
        if i is not None:
            e_fwd[i][1].record()
        ca.compact_attn_permute(op, lay, inverse=True, out=out)

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(i)
    torch.cuda.synchronize()
    ms_per_step = (time.perf_counter() - t0) * 1e3 / args.steps
    fwd_ms = sorted(a.elapsed_time(b) for a, b in e_fwd)
    perm_ms = sorted(a.elapsed_time(b) for a, b in e_perm)
    fwd_avg = sum(fwd_ms) / len(fwd_ms)
    fwd_med = fwd_ms[len(fwd_ms) // 2]
    perm3_avg = sum(perm_ms) / len(perm_ms)

    B, D, n = lay.tokens_per_tile, wl.head_dim, lay.n_tiles
    flops = lay.nnz_total * wl.batch * 4.0 * B * B * D
    dense_flops = wl.num_heads * wl.batch * n * n * 4.0 * B * B * D
    kept = lay.nnz_total / (wl.num_heads * n * n)
    executed = executed_fraction(ca, lay, wl)
    esz = 2 if wl.dtype == "bf16" else 4
    perm_bytes = 3 * wl.batch * wl.num_heads * (lay.n_tokens_real + lay.n_tokens_padded) * D * esz

    dense_ms = None
    if args.dense_calls > 0:
        ca.compact_attn_dense(qp, kp, vp, lay, out=op)
        torch.cuda.synchronize()
        ts = []
        for _ in range(args.dense_calls):
            a, b = ev(), ev()
            a.record()
            ca.compact_attn_dense(qp, kp, vp, lay, out=op)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        dense_ms = sorted(ts)[len(ts) // 2]

    # What the chip's power management does to this kernel: the same launch on all-zero q, k, v (no
    # operand bit ever toggles in the matrix pipes) and a plain device-to-device copy of one tensor,
    # the practical ceiling the permutation is measured against.
    context = {}
    if args.context_calls > 0:
        zq, zk, zv = (torch.zeros_like(qp) for _ in range(3))
        context["attn_ms_all_zero_inputs"] = median_ms(lambda: ca.compact_attn_forward(zq, zk, zv, lay, out=op), args.context_calls)
        context["attn_frac_all_zero_inputs"] = flops / context["attn_ms_all_zero_inputs"] / 1e9 / PEAK_BF16_TFLOPS
        del zq, zk, zv
        scratch = torch.empty_like(qp)
        copy_ms = median_ms(lambda: scratch.copy_(qp), args.context_calls)
        context["device_copy_gbps"] = 2 * qp.numel() * esz / copy_ms / 1e6
        del scratch
        ca.compact_attn_forward(qp, kp, vp, lay, out=op)

    mass = None
    if args.mass_calls > 0 and wl.dtype == "bf16":
        # offline step of the method (Sec. 4.2): attention mass per tile pair, one QK^T product per
        # pair (half the FLOPs of a dense attention pass)
        m_out = ca.compact_attn_tile_mass(qp, kp, lay)
        torch.cuda.synchronize()
        ts = []
        for _ in range(args.mass_calls):
            a, b = ev(), ev()
            a.record()
            ca.compact_attn_tile_mass(qp, kp, lay, out=m_out)
            b.record()
            torch.cuda.synchronize()
            ts.append(a.elapsed_time(b))
        mass_ms = sorted(ts)[len(ts) // 2]
        mass_flops = dense_flops / 2
        mass = {"ms": mass_ms, "tflops": mass_flops / mass_ms / 1e9,
                "pct_bf16_mfma_peak": 100.0 * mass_flops / mass_ms / 1e9 / PEAK_BF16_TFLOPS,
                "row_sum_error": float((m_out[0].sum(dim=2).sum(dim=1) - lay.n_tokens_real).abs().max())}
        del m_out

    fused = None
    if args.natural_calls > 0 and wl.dtype == "bf16":
        # the same whole path in one launch: tiles gathered from natural order inside the kernel
        try:
            o2 = ca.compact_attn_forward_natural(q, k, v, lay)
            torch.cuda.synchronize()
            ts = []
            for _ in range(args.natural_calls):
                a, b = ev(), ev()
                a.record()
                ca.compact_attn_forward_natural(q, k, v, lay, out=o2)
                b.record()
                torch.cuda.synchronize()
                ts.append(a.elapsed_time(b))
            nat_ms = sorted(ts)[len(ts) // 2]
            fused = {"ms_per_step": nat_ms, "tflops": flops / nat_ms / 1e9, "speedup_vs_permuted_path": ms_per_step / nat_ms,
                     "same_bits_as_permuted_path": bool(torch.equal(o2, out))}
            del o2
        except ca.CompactAttnError as exc:
            fused = {"unsupported": str(exc)}

    # The other configurations: the forward and the dense kernel alone, on tile-ordered tensors.
    others = {}
    if args.other_calls > 0:
        del out
        for name in OTHER_CONFIGS:
            w2 = get_workload(name)
            l2 = layout_of(w2)
            ca.compact_attn_layout_upload(l2)
            if w2.cfg != wl.cfg:
                del qp, kp, vp, op
                torch.cuda.empty_cache()
                q2, k2, v2 = make_qkv(w2, dev)
                qp, kp, vp = (ca.compact_attn_permute(t, l2) for t in (q2, k2, v2))
                op = torch.empty_like(qp)
                del q2, k2, v2
            B2, D2, n2 = l2.tokens_per_tile, w2.head_dim, l2.n_tiles
            ms = median_ms(lambda: ca.compact_attn_forward(qp, kp, vp, l2, out=op), args.other_calls)
            same_shape = w2.cfg == wl.cfg and dense_ms is not None
            d_ms = dense_ms if same_shape else median_ms(lambda: ca.compact_attn_dense(qp, kp, vp, l2, out=op), 1)
            f2 = l2.nnz_total * w2.batch * 4.0 * B2 * B2 * D2
            kept2 = l2.nnz_total / (w2.num_heads * n2 * n2)
            ex2 = executed_fraction(ca, l2, w2)
            others[name] = {"ms": ms, "tflops": f2 / ms / 1e9, "frac_bf16_mfma_peak": f2 / ms / 1e9 / PEAK_BF16_TFLOPS,
                            "frac_executed": ex2 * f2 / ms / 1e9 / PEAK_BF16_TFLOPS,
                            "kernel": "attn_bf16_pair_kernel" if (B2, D2) == (64, 128) else "attn_bf16_kernel",
                            "kept_tile_fraction": kept2, "ideal_speedup": 1.0 / kept2,
                            "dense_ms": d_ms, "dense_tflops": w2.num_heads * w2.batch * n2 * n2 * 4.0 * B2 * B2 * D2 / d_ms / 1e9,
                            "speedup_vs_dense": d_ms / ms}
            l2.free()

    if args.calibrate_copy:
        src = torch.empty(1 << 28, dtype=torch.float32, device=dev).normal_()
        dst = torch.empty_like(src)
        dst.copy_(src)            # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del src, dst

    cpu = cpu_baseline(wl, q, k, v, args.cpu_seconds) if args.cpu_seconds > 0 else None

    rec = {
        "metric": "sparse attention hot path, effective TFLOP/s on kept tiles (permute q,k,v + sparse forward + inverse permute)",
        "value": flops / ms_per_step / 1e9,
        "unit": "TFLOP/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
        "ms_per_step": ms_per_step,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": wl.dtype, "data": "synthetic",
        "config": {"workload": f"{wl.name}: T={wl.T} H={wl.H} W={wl.W} +{wl.n_text} text, tile {wl.tile}, "
                               f"{wl.num_heads} heads, D={D}, batch {wl.batch}",
                   "n_tiles": n, "tokens_padded": lay.n_tokens_padded, "kept_tile_fraction": kept,
                   "layout_build_s": layout_build_s},
        "attn": {"ms_per_call_avg": fwd_avg, "ms_per_call_median": fwd_med, "tflops": flops / fwd_avg / 1e9,
                 "pct_bf16_mfma_peak": 100.0 * flops / fwd_avg / 1e9 / PEAK_BF16_TFLOPS,
                 "executed_product_fraction": executed, "tflops_executed": executed * flops / fwd_avg / 1e9,
                 "dense_ms": dense_ms, "dense_tflops": (dense_flops / dense_ms / 1e9) if dense_ms else None,
                 "speedup_vs_dense": (dense_ms / fwd_med) if dense_ms else None, "ideal_speedup": 1.0 / kept},
        "permute": {"ms_q_k_v": perm3_avg, "gbps": perm_bytes / perm3_avg / 1e6, "pct_hbm_peak": perm_bytes / perm3_avg / 1e6 / 8000 * 100},
        "roofline": {"bound": "mfma", "kernel": "attn_bf16_pair_kernel" if (B, D) == (64, 128) else "attn_bf16_kernel", "achieved": flops / fwd_avg / 1e9,
                     "peak": PEAK_BF16_TFLOPS, "unit": "TFLOP/s", "frac": flops / fwd_avg / 1e9 / PEAK_BF16_TFLOPS,
                     "frac_executed": executed * flops / fwd_avg / 1e9 / PEAK_BF16_TFLOPS,
                     "traffic": RECORDED_TRAFFIC.get(wl.name, {}).get("bytes"),
                     "traffic_source": RECORDED_TRAFFIC.get(wl.name, {}).get("source"),
                     "algorithmic_flops_per_launch": flops,
                     "algorithmic_bytes_per_launch": 4 * wl.batch * wl.num_heads * lay.n_tokens_padded * D * esz},
        "context": context or None,
        "tile_mass": mass,
        "fused_gather_scatter": fused,
        "cpu_baseline": cpu,
    }
    if others:
        rec["other_configs"] = others
    if args.pattern_report:
        rec["patterns"] = pattern_report(ca, dev)
    print(json.dumps(rec))


if __name__ == "__main__":
    main()
