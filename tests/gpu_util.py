"""The GPU tests' helpers live in workloads/device.py (bench.py and the smoke check use them too)."""
from workloads.device import *  # noqa: F401,F403
