"""The synthetic input recipe: spot values of the positional code, determinism, dtypes."""
import math

import torch

from workloads import get_workload, make_qkv, position_code, WORKLOAD_NAMES


def test_position_code_spot_values():
    pos = position_code(4, 8, 8, 2, 12)
    assert pos.shape == (4 * 8 * 8 + 2, 12)
    i = (3 * 8 + 2) * 8 + 5                     # token (t=3, y=2, x=5)
    u = (3 / 4, 2 / 8, 5 / 8)
    assert pos[i, 0].item() == torch.sin(torch.tensor(math.pi * u[0])).item()           # c=0: axis t, sin, m=0
    assert abs(pos[i, 4].item() - math.cos(math.pi * u[1])) < 1e-6                      # c=4: axis y, cos, m=0
    assert abs(pos[i, 8].item() - math.sin(2 * math.pi * u[2])) < 1e-6                  # c=8: axis x, sin, m=1
    assert abs(pos[i, 11].item() - math.cos(2 * math.pi * u[2])) < 1e-6                 # c=11: axis x, cos, m=1
    assert torch.all(pos[-2:] == 0)


def test_qkv_deterministic_and_shaped():
    wl = get_workload("cfg1")
    a = make_qkv(wl)
    b = make_qkv(wl)
    for x, y in zip(a, b):
        assert x.dtype == torch.float32 and x.shape == (1, 2, 256, 64)
        assert torch.equal(x, y)
    assert not torch.equal(a[0], a[1])
    q = a[0].double()
    assert abs(q.std().item() - (1 + 0.25 * 0.5) ** 0.5) < 0.05


def test_all_workloads_construct():
    for name in WORKLOAD_NAMES:
        wl = get_workload(name)
        assert len(wl.heads) == wl.num_heads == len(wl.expected_nnz)
