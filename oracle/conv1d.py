"""TEST INFRASTRUCTURE: the W8A8 causal convolution in front of the scan (Section 4.2, "Efficient 4-bit/8-bit Mamba
blocks": a W8A8 causal convolution kernel; its channels are reordered offline so that it emits x, B and C in the
sorted order the SSD kernel consumes).

The block convolves the concatenated channels [x | B | C] of every sequence causally over time with one short filter
per channel (depthwise, d_conv = 4 taps), adds a bias, applies SiLU, and the results are the scan's x, B and C.  In
the W8A8 setting the input is int8 codes with one static scale s_in, the filter is int8 codes with one static scale
s_w, and the outputs are quantized with Eq. 1 to the scan's 8-bit operands: x with the sort-and-cluster cell scales,
B and C with their per-state-group scales (Section 4.1).

    acc[t, c]  = sum_{k=0..3} w_code[c, k] * in_code[t - 3 + k, c]        exact in integers; in_code[t < 0] comes from
                                                                           the carried conv state (zeros at the start)
    v          = (s_in s_w) * acc + bias[c]
    out[t, c]  = Eq. 1 (SiLU(v) / s_out[c]),   SiLU(v) = v / (1 + exp(-v))

`conv1d_silu_f64` is that definition in float64 without the final rounding.  The code is an integer decided by
floating point, so `ref_conv1d_q8` takes the decision in the GPU kernel's precision (fp32) as a fixed sequence of
separately rounded operations, written out in its docstring; the exponential is `exp_f32` of the cached-state oracle.
Nothing here is shared with the HIP path.
"""
from __future__ import annotations

import numpy as np

from .state_q8 import exp_f32

F = np.float32
D_CONV = 4


def _window_sums(in_codes, w_codes, conv_state):
    """acc [b,L,C] int64 and the padded input [b, 3+L, C]: plain sliding sums, tap k multiplies the input 3-k steps
    back, so tap 3 is the current token."""
    x = np.asarray(in_codes)
    w = np.asarray(w_codes)
    assert x.dtype == np.int8 and w.dtype == np.int8
    b, L, C = x.shape
    assert w.shape == (C, D_CONV)
    if conv_state is None:
        st = np.zeros((b, D_CONV - 1, C), np.int8)
    else:
        st = np.asarray(conv_state)
        assert st.dtype == np.int8 and st.shape == (b, D_CONV - 1, C)
    pad = np.concatenate([st, x], axis=1).astype(np.int64)          # pad[:, j] is token j - 3
    acc = np.zeros((b, L, C), np.int64)
    for k in range(D_CONV):
        acc += w[:, k].astype(np.int64)[None, None, :] * pad[:, k:k + L, :]
    return acc, pad


def conv1d_silu_f64(in_codes, w_codes, in_w_scale: float, bias=None, conv_state=None) -> np.ndarray:
    """SiLU((s_in s_w) acc + bias) [b,L,C] in float64: the real-valued activations the quantized outputs stand for."""
    acc, _ = _window_sums(in_codes, w_codes, conv_state)
    v = acc.astype(np.float64) * float(in_w_scale)
    if bias is not None:
        v = v + np.asarray(bias, np.float64)[None, None, :]
    with np.errstate(over="ignore"):
        return v / (1.0 + np.exp(-v))


def ref_conv1d_q8(in_codes, w_codes, in_w_scale, bias, out_scales, conv_state=None):
    """int8 codes [b,L,C] of the convolution's activated output, and the conv state to carry on (the last 3 input
    tokens, [b,3,C] int8).  out_scales [C] float32 is the Eq. 1 scale of every output channel.

    Per element, float32, every line one rounding (acc is an exact integer):
        v    = float(acc) * s_cw          then  v = v + bias[c]            s_cw = the float32 product s_in s_w
        e    = exp_f32(-|v|)                                               in (0, 1]; 0 once -|v| log2(e) < -125
        den  = 1 + e
        num  = v            if v >= 0     else  v * e                      SiLU(v) = v / (1 + e^-v) = v e^v / (1 + e^v)
        a    = num / den                                                   IEEE division
        r    = a * (1 / s_out[c])                                          the reciprocal is one IEEE division
        code = clamp(rint(r), -128, 127)                                   Eq. 1, ties to even
    """
    acc, pad = _window_sums(in_codes, w_codes, conv_state)
    C = acc.shape[-1]
    s_cw = F(in_w_scale)
    v = acc.astype(F) * s_cw
    if bias is not None:
        v = v + np.asarray(bias, F)[None, None, :]
    e = exp_f32(-np.abs(v))
    den = F(1.0) + e
    num = np.where(v >= 0, v, v * e).astype(F)
    a = (num / den).astype(F)
    inv = (F(1.0) / np.asarray(out_scales, F)).astype(F)
    assert inv.shape == (C,)
    r = a * inv[None, None, :]
    codes = np.clip(np.rint(r), -128, 127).astype(np.int8)
    new_state = pad[:, -(D_CONV - 1):, :].astype(np.int8)
    return codes, new_state


def output_scales(sc, nheads: int, headdim: int, ngroups: int, d_state: int) -> np.ndarray:
    """Eq. 1 scale of every output channel [H*P + 2*G*N] of the convolution in the order [x | B | C]: the cell scale
    of (head, channel position) for x (Section 4.1, sort-and-cluster), the group's scale for B and C (per-state-group
    quantization)."""
    from .ssd import x_scale_table
    xs = x_scale_table(sc, nheads, headdim, ngroups).reshape(-1)
    return np.concatenate([xs, np.repeat(np.asarray(sc.B_scales), d_state),
                           np.repeat(np.asarray(sc.C_scales), d_state)]).astype(F)
