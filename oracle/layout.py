"""CPU oracle for the layout conversion of convolution inputs -- TEST INFRASTRUCTURE, NOT THE PRODUCT.

Sec. 5.2 lists NHWC (mini-batch, height, width, channels) among the layouts the implementation
uses for the inputs and outputs of convolution layers; the statistics of Sec. 4 are defined on
(sample, channel, position) and do not depend on how the tensor is stored.  The conversion is a
pure permutation: element (n, c, y, x) of the result is element (n, y, x, c) of the input.
Only the tests may import this module; it imports nothing from the GPU package.
"""
from __future__ import annotations

import numpy as np


def nhwc_to_nchw(x) -> np.ndarray:
    """[N, H, W, C] -> [N, C, H, W], element by element (any dtype, bits unchanged)."""
    x = np.asarray(x)
    assert x.ndim == 4
    N, H, W, C = x.shape
    out = np.empty((N, C, H, W), dtype=x.dtype)
    for c in range(C):
        out[:, c, :, :] = x[:, :, :, c]
    return out
