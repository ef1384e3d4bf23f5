"""CPU oracle of the stride-1 forward convolution (test infrastructure only).

Nothing in the product package imports this; it is called by the tests, the
smoke check and the benchmark's CPU-baseline leg.
"""
from .conv_ref import (conv_ref, conv_ref_points, conv_ref_counted, conv_bias_relu_ref, within_tolerance,  # noqa: F401
                       build)
