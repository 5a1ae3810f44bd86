"""CPU oracle of the RT-Lynx hot path (test infrastructure, not a product path).

Only tests, the smoke check and the benchmark's cpu_baseline leg import this package.
"""
from .oracle import *  # noqa: F401,F403
