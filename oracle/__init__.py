"""CPU oracle for the direct-convolution forward pass.

TEST INFRASTRUCTURE ONLY: imported by tests, the smoke check and the benchmark's
cpu_baseline leg.  The product package never imports this.
"""
from .conv_ref import (  # noqa: F401
    build,
    conv_dgrad,
    conv_forward,
    conv_forward_points,
    conv_forward_reordered,
    conv_wgrad,
    out_dim,
    threads,
    tolerance,
)
from .tail_ref import apply_tail, conv_forward_fused  # noqa: F401,E402
