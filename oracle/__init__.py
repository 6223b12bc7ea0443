"""CPU oracle (test infrastructure).  See ssnet_oracle.c for what it computes.

Only tests, the smoke check and the benchmark's CPU-baseline leg may import
this package; the GPU library and its Python binding never do.
"""
from .ssnet_oracle import *  # noqa: F401,F403
