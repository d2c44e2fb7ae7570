"""Seeded Q/K/V values: a smooth 3-D positional code plus unit Gaussian noise.

For a video token (t, y, x) and channel c: axis a = c mod 3 (0: t, 1: y,
2: x), m = (c div 3) div 2, u = coordinate_a / length_a, and
pos[c] = sin(pi (m+1) u) when (c div 3) is even, cos(pi (m+1) u) otherwise.
Text tokens have pos = 0.  Q, K, V = 0.5 pos + N(0, 1) noise from three
independent streams (seed, seed+1, seed+2), then rounded to the working
dtype.  Tensors are natural order [batch, heads, N_real, D].

`axis_gain` (optional, one (gt, gy, gx) triple per head) multiplies the positional code of Q and
K on the channels of each axis: it shapes how fast a head's attention falls off along time, height
and width (large on all axes: a local head; large on y and x with a small offset-free background:
the arms of a cross; zero: a global head with no structure), standing in for the head kinds of
Sec. 3.2.  V keeps the plain code.

Values are drawn with torch on whichever device is asked for; the two sides
of a parity test always read the same rounded tensor, so nothing depends on
the generator being reproducible across devices.
"""
import math

import torch


def position_code(T, H, W, n_text, head_dim, device="cpu"):
    """fp32 [T*H*W + n_text, head_dim]"""
    c = torch.arange(head_dim, device=device)
    axis = c % 3
    pair = c // 3
    m = (pair // 2 + 1).to(torch.float32)
    is_sin = (pair % 2) == 0
    t, y, x = torch.meshgrid(
        torch.arange(T, device=device), torch.arange(H, device=device), torch.arange(W, device=device), indexing="ij"
    )
    u = torch.stack([t.reshape(-1) / T, y.reshape(-1) / H, x.reshape(-1) / W], dim=1).to(torch.float32)  # [N, 3]
    arg = math.pi * u[:, axis] * m[None, :]
    pos = torch.where(is_sin[None, :], torch.sin(arg), torch.cos(arg))
    if n_text:
        pos = torch.cat([pos, torch.zeros(n_text, head_dim, device=device)], dim=0)
    return pos


def make_qkv(wl, device="cpu", q_gain=1.0, axis_gain=None):
    """(q, k, v) natural order [batch, heads, N_real, D] in the workload's dtype."""
    dtype = {"f32": torch.float32, "bf16": torch.bfloat16}[wl.dtype]
    pos = 0.5 * position_code(wl.T, wl.H, wl.W, wl.n_text, wl.head_dim, device)
    channel_axis = torch.arange(wl.head_dim, device=device) % 3
    n_real = pos.shape[0]
    out = []
    for stream in range(3):
        gen = torch.Generator(device=device)
        gen.manual_seed(wl.seed + stream)
        x = torch.empty(wl.batch, wl.num_heads, n_real, wl.head_dim, dtype=dtype, device=device)
        for b in range(wl.batch):
            for h in range(wl.num_heads):
                noise = torch.randn(n_real, wl.head_dim, generator=gen, device=device, dtype=torch.float32)
                if axis_gain is not None and stream < 2:
                    gain = torch.tensor([float(x) for x in axis_gain[h]], device=device, dtype=torch.float32)
                    val = pos * gain[channel_axis][None, :] + noise
                else:
                    val = pos + noise
                if stream == 0 and q_gain != 1.0:
                    val = val * q_gain
                x[b, h] = val.to(dtype)
        out.append(x)
    return tuple(out)
