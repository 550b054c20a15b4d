"""Input preparation for the attention tests: fp32 projections -> integer tensors and their scales.

The attention layer's parity tests start from quantised Q, K, V so that the CPU oracle and the GPU
path see the very same integers.  The quantisation itself (Section 5.3, first step: symmetric, one
scale per tensor) is the oracle's; this module only calls it, so that no arithmetic of the method
lives in the shared input generators.  (The GPU's own quantiser is tested against the same oracle
function in test_gpu_quantize.py.)
"""
import numpy as np

import oracle


def quantize_inputs_int8(x: np.ndarray):
    """(int8 codes, fp32 scale) with s = max|x| / 127."""
    return oracle.quantize_per_tensor(x, 8)


def quantize_inputs_int4(x: np.ndarray):
    """(bytes holding two 4-bit codes each along the last axis, fp32 scale) with s = max|x| / 7."""
    q, s = oracle.quantize_per_tensor(x, 4)
    return oracle.pack_int4(q), s
