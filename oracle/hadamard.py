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


def paley_hadamard(m: int) -> np.ndarray:
    """The Hadamard matrix of order m = q + 1 by Paley's first construction, q a prime with q = 3 (mod 4): with chi the
    quadratic character mod q (chi(0) = 0, +1 on the non-zero squares, -1 elsewhere) and Q[i, j] = chi(i - j), the
    matrix S = [[0, 1^T], [-1, Q]] is skew-symmetric and H = I + S has entries +-1 with H H^T = m I.  Orders 12 (q = 11)
    and 20 (q = 19) complete the powers of two to the widths 3 * 2^k and 5 * 2^k of the Mamba blocks."""
    q = m - 1
    assert q % 4 == 3 and all(q % d for d in range(2, int(q ** 0.5) + 1)), "m - 1 must be a prime = 3 mod 4"
    squares = {(v * v) % q for v in range(1, q)}
    chi = lambda v: 0 if v % q == 0 else (1 if v % q in squares else -1)
    S = np.zeros((m, m), np.int64)
    S[0, 1:] = 1
    S[1:, 0] = -1
    for i in range(q):
        for j in range(q):
            S[1 + i, 1 + j] = chi(i - j)
    return np.eye(m, dtype=np.int64) + S


def mixed_order(n: int):
    """(m, 2^k) with n = m * 2^k: m = 1 for a power of two, else m = 12 or 20 (n = 3 * 2^(k+2) or 5 * 2^(k+2))."""
    if n & (n - 1) == 0:
        return 1, n
    for m in (12, 20):
        if n % m == 0 and (n // m) & (n // m - 1) == 0:
            return m, n // m
    raise ValueError("the order must be 2^k, 12 * 2^k or 20 * 2^k")


def hadamard_f32(x) -> np.ndarray:
    """H_n x along the last axis in float32 for n = m * 2^k, H_n = H_m (x) H_{2^k} (Kronecker product, the Paley factor
    on the slow index): element a * 2^k + j of the result is sum_a' H_m[a, a'] (H_{2^k} x_a')[j], where x_a' is block a'
    of 2^k consecutive values.  Evaluation order: the butterfly network of `fwht_f32` inside every block, then the sum
    over the blocks a' = 0, 1, ..., m-1 accumulated in this order, every addition rounded to float32 on its own."""
    v = np.array(x, dtype=F)
    n = v.shape[-1]
    m, p = mixed_order(n)
    if m == 1:
        return fwht_f32(v)
    t = fwht_f32(v.reshape(v.shape[:-1] + (m, p)))                  # [..., a', j]
    H = paley_hadamard(m)
    out = np.empty_like(t)
    for a in range(m):
        acc = t[..., 0, :] * F(H[a, 0])
        for b in range(1, m):
            acc = (acc + t[..., b, :] * F(H[a, b])).astype(F)
        out[..., a, :] = acc
    return out.reshape(v.shape)


def hadamard_quantize(y, s_y: float) -> np.ndarray:
    """int8 codes of (1/s_y) H_n y for fp16 (or exactly representable) inputs y [..., n], n = 2^k, 12 * 2^k or 20 * 2^k:
    the transform in float32 (hadamard_f32), then Eq. 1 with the reciprocal scale: code = clamp(rint(v * (1/s_y)), -128, 127), the reciprocal and
    the product rounded to float32, ties to even."""
    v = hadamard_f32(np.asarray(y, np.float16).astype(F))
    inv = F(1.0) / F(s_y)
    return np.clip(np.rint(v * inv), -128, 127).astype(np.int8)
