"""Seeded synthetic workloads shared by the tests, the smoke check and the benchmark.

Holds only input recipes (grid shapes, per-head window parameters, Q/K/V
values); none of the method's arithmetic lives here.  Neither the oracle nor
the HIP library imports this package: callers pass its plain values to both.
"""
from .configs import Workload, get_workload, WORKLOAD_NAMES  # noqa: F401
from .inputs import make_qkv, position_code  # noqa: F401
