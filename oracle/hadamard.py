"""TEST INFRASTRUCTURE: the quantized Hadamard transform of the SSD output (Section 4.2, "Offline Hadamard matrix
fusion" and "Efficient 4-bit/8-bit Mamba blocks"): y_bar^H = (1/s_y) H_n y, rounded to 8 bits with Eq. 1, the input of
the output projection whose weight carries the matching H_n offline.

H_n is the Sylvester-Hadamard matrix of order n = 2^k (entries +-1, H_n H_n^T = n I, no normalisation: the factor
belongs to the scale).  The code is an integer decided by floating point, so the transform is evaluated in the GPU
kernel's precision (fp32) as the radix-2 butterfly network with the strides in ascending order, which fixes every
rounding: stage h = 1, 2, 4, ..., n/2 replaces each pair (v[i], v[i + h]) with i & h == 0 by (v[i] + v[i + h],
v[i] - v[i + h]).  Nothing here is shared with the HIP path.
"""
from __future__ import annotations

import numpy as np

F = np.float32


def fwht_f32(x) -> np.ndarray:
    """H_n x along the last axis in float32: butterfly stages with strides 1, 2, 4, ..., n/2 in this order, every
    addition and subtraction rounded to float32 on its own."""
    v = np.array(x, dtype=F)
    n = v.shape[-1]
    assert n >= 1 and n & (n - 1) == 0, "the order must be a power of two"
    h = 1
    while h < n:
        w = v.reshape(v.shape[:-1] + (n // (2 * h), 2, h))
        a = w[..., 0, :] + w[..., 1, :]
        b = w[..., 0, :] - w[..., 1, :]
        v = np.stack([a, b], axis=-2).reshape(v.shape)
        h *= 2
    return v


def hadamard_quantize(y, s_y: float) -> np.ndarray:
    """int8 codes of (1/s_y) H_n y for fp16 (or exactly representable) inputs y [..., n]: the transform in float32
    (fwht_f32), then Eq. 1 with the reciprocal scale: code = clamp(rint(v * (1/s_y)), -128, 127), the reciprocal and
    the product rounded to float32, ties to even."""
    v = fwht_f32(np.asarray(y, np.float16).astype(F))
    inv = F(1.0) / F(s_y)
    return np.clip(np.rint(v * inv), -128, 127).astype(np.int8)
