"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests.

This package holds input generation only: random draws, the planted structure of
the workloads (outlier key channels, dominant tokens) and shape bookkeeping.  It
contains none of the method's arithmetic (no quantizer, no scoring, no softmax)
and imports neither the oracle nor the HIP binding.
"""
from .workloads import (  # noqa: F401
    LLAMA31_8B,
    HeadShape,
    LayerInputs,
    make_layer,
    ragged_lengths,
    static_channels,
)
