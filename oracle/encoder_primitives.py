"""The three encoder subroutines of Alg. 1 that fix the sign conventions.

TEST INFRASTRUCTURE.  Used only to pin the decoder's conventions: that code 0
maps to a group's minimum, code 2^b - 1 to its maximum, and that the
round-trip error is at most half a step.  Not an encoder.
"""
import numpy as np


def fit_quantizer(v, bits):
    """Alg. 1 fit_quantizer on one group: s = (max - min) / (2^b - 1), z = -min / s."""
    v = np.asarray(v, dtype=np.float64)
    s = (v.max() - v.min()) / (2 ** bits - 1)
    z = -v.min() / s
    return s, z


def quantize(v, s, z):
    """Alg. 1 quantize: floor(v / s + z + 0.5)."""
    return np.floor(np.asarray(v, dtype=np.float64) / s + z + 0.5)
