"""CPU oracle for PEVLM parallel-encoding attention.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this package; the
GPU library and its Python binding never do, and share no code with it.
"""
from .pevlm_oracle import (  # noqa: F401
    Layout,
    build,
    check_layout,
    positions,
    mask_row,
    mask_matrix,
    visible,
    rope,
    rope_mrope,
    attn,
    forward,
    threads,
)
