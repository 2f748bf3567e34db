"""CPU oracle of the low-precision forward pass.

TEST INFRASTRUCTURE ONLY: imported by tests/, the smoke check and the
benchmark's cpu_baseline leg.  It shares nothing with the GPU library and the
GPU library never imports it.
"""
from .lp_oracle import (  # noqa: F401
    ROUND_AWAY,
    ROUND_EVEN,
    act,
    act_stochastic,
    build,
    conv,
    conv_sampled,
    fc,
    maxpool2x2,
    num_threads,
    quantize,
    quantize_stochastic,
    range_acc,
    range_float,
)
