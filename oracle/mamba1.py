"""TEST INFRASTRUCTURE: the 8-bit Mamba1 selective scan (Section 3.2, Eq. 2 with the Mamba1 parameterisation: B_t, C_t
and Delta_t vary with the input, A is a trained [channels, states] matrix; the framework's 8-bit selective-scan
kernel of Section 4.2).

For every sequence b, channel d and state n, on de-quantized operands (inverse of Eq. 1):

    h_t[d,n] = exp(Delta_t[d] A[d,n]) h_{t-1}[d,n] + Delta_t[d] B_t[n] x_t[d]        (A-dot = exp(Delta A), B-dot = Delta B)
    y_t[d]   = sum_n C_t[n] h_t[d,n] + D[d] x_t[d]

x = s_x(d) * x_code with one scale per channel range (the sort-and-cluster scales of Section 4.1 for a block without
heads: channels sorted by their calibrated maximum and clustered into ranges), B = s_B * B_code and C = s_C * C_code
with one scale each (Mamba1 has a single state group).  Tensors are channel-major, time last, the layout of the
Mamba1 block: x, Delta, y [b, D, L]; B, C [b, N, L].  Plain sequential float64; nothing here is shared with the HIP
path.
"""
from __future__ import annotations

import numpy as np


def channel_scales(x_scales, chan_cluster_end, nchannels: int) -> np.ndarray:
    """[D] float64: the scale of every sorted channel position; range j covers positions
    chan_cluster_end[j-1] .. chan_cluster_end[j]-1 (plain lookups)."""
    ends = np.asarray(chan_cluster_end, np.int64)
    xs = np.asarray(x_scales, np.float64)
    out = np.empty(nchannels, np.float64)
    for d in range(nchannels):
        j = 0
        while j < len(ends) - 1 and d >= ends[j]:
            j += 1
        out[d] = xs[j]
    return out


def ref_mamba1_scan(x_scale_per_channel, B_scale: float, C_scale: float, xq, Bq, Cq, dt, A, D=None, init_state=None):
    """Sequential scan in float64.  xq [b,D,L] int8, Bq/Cq [b,N,L] int8, dt [b,D,L], A [D,N], D [D] or None,
    init_state [b,D,N] or None.  Returns (y [b,D,L], final_state [b,D,N])."""
    xq = np.asarray(xq); Bq = np.asarray(Bq); Cq = np.asarray(Cq)
    assert xq.dtype == np.int8 and Bq.dtype == np.int8 and Cq.dtype == np.int8
    b, Dn, L = xq.shape
    N = Bq.shape[1]
    assert Bq.shape == (b, N, L) and Cq.shape == (b, N, L)
    dt = np.asarray(dt, np.float64); A = np.asarray(A, np.float64)
    assert dt.shape == (b, Dn, L) and A.shape == (Dn, N)
    x = xq.astype(np.float64) * np.asarray(x_scale_per_channel, np.float64)[None, :, None]
    B = Bq.astype(np.float64) * float(B_scale)
    Cm = Cq.astype(np.float64) * float(C_scale)
    h = np.zeros((b, Dn, N)) if init_state is None else np.array(init_state, np.float64)
    assert h.shape == (b, Dn, N)
    y = np.empty((b, Dn, L))
    for t in range(L):
        decay = np.exp(dt[:, :, t, None] * A[None])                                # [b,D,N]
        h = decay * h + (dt[:, :, t] * x[:, :, t])[:, :, None] * B[:, None, :, t]
        y[:, :, t] = np.einsum("bdn,bn->bd", h, Cm[:, :, t])
    if D is not None:
        y = y + np.asarray(D, np.float64)[None, :, None] * x
    return y, h
