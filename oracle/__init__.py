"""fp64 CPU oracle for the ring-step attention path (test infrastructure only).

Nothing in the product path (the HIP library or its Python binding) may import
this package; only tests, the smoke check and the benchmark's cpu_baseline leg do.
"""
from .ring_attention_oracle import *  # noqa: F401,F403
