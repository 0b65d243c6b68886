"""Pins of oracle/gate.py (step size from its quantized pre-activation, output gate) against library routines of a
different formulation, closed forms and limits.  No GPU."""
import numpy as np
from scipy.special import expit

import oracle


def test_softplus_step_size():
    H = 256
    codes = np.arange(-128, 128, dtype=np.int8)[None, :].repeat(3, 0)          # [3, H], one code value per head
    bias = np.linspace(-6, 2, H)
    got = oracle.dt_from_codes(codes, 0.05, bias)
    v = codes.astype(np.float64) * 0.05 + bias
    assert got.shape == (3, H)
    assert np.allclose(got, np.logaddexp(0.0, v), rtol=1e-14, atol=0)          # numpy's own softplus formulation
    assert np.allclose(np.expm1(got), np.exp(v), rtol=1e-12)                   # inverse: exp(Delta) - 1 = exp(v)
    assert np.all(got > 0)
    nob = oracle.dt_from_codes(codes[0], 0.05)                                 # absent bias is zero
    assert np.all(np.diff(nob) > 0)                                            # increasing in the code
    # limits: v -> -inf gives exp(v), v -> +inf gives v; softplus(0) = log 2
    assert np.isclose(oracle.dt_from_codes(np.array([-100], np.int8), 1.0)[0], np.exp(-100.0), rtol=1e-12)
    assert oracle.dt_from_codes(np.array([100], np.int8), 1.0)[0] == 100.0
    assert oracle.dt_from_codes(np.zeros(4, np.int8), 1.0)[0] == np.log(2.0)
    # the bias belongs to the head (last) axis
    b = np.array([0.0, 1.0, -1.0])
    two = oracle.dt_from_codes(np.zeros((2, 5, 3), np.int8), 0.3, b)
    assert two.shape == (2, 5, 3) and np.allclose(two[1, 4], np.logaddexp(0, b))
    # scale applies to the code, not to the bias
    assert np.isclose(oracle.dt_from_codes(np.array([10], np.int8), 0.2, np.array([1.0]))[0], np.logaddexp(0, 3.0))


def test_silu_gate():
    z = np.arange(-128, 128, dtype=np.int8)
    y = np.linspace(-3, 5, 256)
    s = 0.07
    got = oracle.silu_gate(y, z, s)
    zf = z.astype(np.float64) * s
    assert np.allclose(got, y * zf * expit(zf), rtol=1e-13, atol=1e-300)       # library sigmoid, other formulation
    # SiLU(z) - SiLU(-z) = z;  SiLU(0) = 0;  SiLU(z) -> z for large z, -> 0 from below for very negative z
    k = np.arange(1, 128, dtype=np.int8)
    one = np.ones(127)
    assert np.allclose(oracle.silu_gate(one, k, s) - oracle.silu_gate(one, -k, s), k * s, rtol=1e-13)
    assert oracle.silu_gate(np.array([7.0]), np.array([0], np.int8), 3.0)[0] == 0.0
    assert np.isclose(oracle.silu_gate(np.array([2.0]), np.array([100], np.int8), 1.0)[0], 200.0, rtol=1e-12)
    tiny = oracle.silu_gate(np.array([2.0]), np.array([-100], np.int8), 1.0)[0]
    assert -1e-40 < tiny < 0
    assert oracle.silu_gate(np.array([2.0]), np.array([-128], np.int8), 10.0)[0] == 0.0   # exp overflows to inf: z/inf
    # linear in y, elementwise in z
    assert np.allclose(oracle.silu_gate(3 * y, z, s), 3 * got)
    # the minimum of SiLU: -0.2784645 at z = -1.2784645 (scale 1e-2 per code around it)
    zz = np.arange(-128, 0, dtype=np.int8)
    vals = oracle.silu_gate(np.ones(128), zz, 0.01)
    assert np.isclose(vals.min(), -0.2784645, atol=1e-6) and zz[vals.argmin()] == -128   # still decreasing at -1.28
    vals2 = oracle.silu_gate(np.ones(128), zz, 0.02)
    assert np.isclose(vals2.min(), -0.2784645, atol=1e-4) and zz[vals2.argmin()] == -64  # -1.28 on this grid
