"""L3 oracle: test infrastructure, not the product.

Only tests, the smoke check and the benchmark's cpu_baseline leg import this.
"""
from .binding import *  # noqa: F401,F403
