"""TEST INFRASTRUCTURE: the two optional 8-bit side inputs of the SSD kernel (Section 5.2 lists x, the step size, B,
C and z as its 8-bit loads): the step size from its quantized pre-activation, and the output gate.

    Delta = softplus(s_dt * dt_code + dt_bias[h])        Section 3.2 (Delta_t = softplus(F_Delta(x_t)), with the bias)
    y'    = y * SiLU(s_z * z_code)                       Section 3.2 (the optional residual branch z, applied to the
                                                         SSM output y = C h + D x before the output projection)

Both are plain definitions in float64; nothing here is shared with the HIP path.
"""
from __future__ import annotations

import numpy as np


def dt_from_codes(dt_codes, dt_scale: float, dt_bias=None) -> np.ndarray:
    """Delta [..., H] = log(1 + exp(v)), v = dt_scale * code + bias[h] (Eq. 1 inverse, then softplus), in float64.
    Written as max(v, 0) + log1p(exp(-|v|)), the same function without overflow."""
    v = np.asarray(dt_codes, np.float64) * float(dt_scale)
    if dt_bias is not None:
        v = v + np.asarray(dt_bias, np.float64)
    return np.maximum(v, 0.0) + np.log1p(np.exp(-np.abs(v)))


def silu_gate(y, z_codes, z_scale: float) -> np.ndarray:
    """y * SiLU(z) with z = z_scale * code (inverse of Eq. 1) and SiLU(z) = z / (1 + exp(-z)), in float64."""
    z = np.asarray(z_codes, np.float64) * float(z_scale)
    with np.errstate(over="ignore"):
        return np.asarray(y, np.float64) * (z / (1.0 + np.exp(-z)))
