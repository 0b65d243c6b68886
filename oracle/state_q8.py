"""TEST INFRASTRUCTURE: the decode step on an 8-bit cached state (Appendix E, "Quantizing cached SSM states").

The cached state of every (sequence, head) is held as int8 codes; the scale of code (h, p, n) is shared by the
(head cluster, channel range) cell of (h, p), the same m x n cells as the input x, and differs per state n, i.e.
d_state x m x n scales per state group.  One generation step de-quantizes the state (inverse of Eq. 1), applies
Eq. 2 once, emits y from the updated state, and re-quantizes the state with Eq. 1 before it is cached again.

The re-quantized code is an integer decided by floating point, so the decision is taken in the precision of the
GPU kernel (fp32) with every operation rounded separately, in the order written in `ref_decode_step_q8`; the
exponential is a fixed sequence of fp32 operations as well (`exp_f32`).  numpy's float32 arithmetic is IEEE
round-to-nearest-even per operation, which is what the steps below rely on.  Nothing here is shared with the HIP
path.
"""
from __future__ import annotations

import math

import numpy as np

from .ssd import Scales

F = np.float32
_LOG2E = F(1.4426950408889634)
# 2^f = sum_i (ln 2)^i / i! f^i, degree 7: truncation error below 5e-9 for |f| <= 1/2
_EXP2_COEF = [F(math.log(2.0) ** i / math.factorial(i)) for i in range(8)]


def exp_f32(z):
    """exp(z) for float32 z as a fixed sequence of float32 operations (each rounded to nearest even):
    t = z * log2(e); k = rint(t); f = t - k; 2^f by Horner's rule with the degree-7 Taylor coefficients of 2^f
    (separate multiply and add); result = 2^f * 2^k (exact scaling).  t < -125 gives 0 (no subnormal results)."""
    z = np.asarray(z, dtype=F)
    t = z * _LOG2E
    k = np.rint(t)
    f = t - k
    p = np.full_like(f, _EXP2_COEF[7])
    for i in range(6, -1, -1):
        p = p * f
        p = p + _EXP2_COEF[i]
    small = t < F(-125.0)
    out = np.ldexp(p, np.where(small, 0, k).astype(np.int32)).astype(F)
    return np.where(small, F(0.0), out)


def cell_index_table(sc: Scales, nheads: int, headdim: int, ngroups: int) -> np.ndarray:
    """[H,P] index of the (group, head cluster, channel range) cell of every (head, channel position): plain
    lookups in the boundary tables of the sort-and-cluster result (Section 4.1), the cells the state scales reuse."""
    hpg = nheads // ngroups
    out = np.empty((nheads, headdim), np.int64)
    for h in range(nheads):
        g, hl = divmod(h, hpg)
        i = 0
        while i < sc.m - 1 and hl >= sc.head_cluster_end[g * sc.m + i]:
            i += 1
        base = (g * sc.m + i) * sc.n
        for p in range(headdim):
            j = 0
            while j < sc.n - 1 and p >= sc.chan_cluster_end[base + j]:
                j += 1
            out[h, p] = base + j
    return out


def state_scales_from_absmax(sc: Scales, absmax: np.ndarray, ngroups: int) -> np.ndarray:
    """Static scales of the cached state from calibrated maxima (absolute-maximum calibration, Appendix C,
    "Quantization setup"): absmax [H,P,N] = max |h| seen per element; scale[cell, n] = (max over the heads and channel positions of the
    cell) / 127 (Eq. 1 with 8 bits), 1.0 for an empty or all-zero cell.  Returns float32 [G*m*n, N]."""
    H, P, N = absmax.shape
    cells = cell_index_table(sc, H, P, ngroups)
    ncell = ngroups * sc.m * sc.n
    mx = np.zeros((ncell, N), F)
    for h in range(H):
        for p in range(P):
            c = cells[h, p]
            mx[c] = np.maximum(mx[c], absmax[h, p].astype(F))
    out = mx / F(127.0)
    out[mx == 0] = F(1.0)
    return out


def quantize_state(sc: Scales, state_scales: np.ndarray, h: np.ndarray, ngroups: int) -> np.ndarray:
    """Eq. 1 on a float32 state [b,H,P,N] with the per-(cell, n) scales: code = clamp(rint(h * (1/s)), -127, 127),
    1/s and the product each rounded to float32, ties to even."""
    b, H, P, N = h.shape
    cells = cell_index_table(sc, H, P, ngroups)
    inv = (F(1.0) / state_scales.astype(F))[cells]        # [H,P,N]
    r = h.astype(F) * inv[None]
    return np.clip(np.rint(r), -127, 127).astype(np.int8)


def ref_decode_step_q8(sc: Scales, state_scales, xq, Bq, Cq, dt, A, D, qstate):
    """One generation step on the int8 cached state qstate [b,H,P,N] (updated in place).  Returns y [b,H,P] float64.

    Per element, float32, every line one rounding:
        xv  = s_x(h,p) * x_code            dtx = dt * xv
        Bv  = s_B[g] * B_code              u   = dtx * Bv              (B-dot x of Eq. 2, B-dot = dt B, Section 3.2)
        sd  = exp_f32(dt * A) * s[cell,n]  d   = sd * state_code        (decay of Eq. 2 times the inverse of Eq. 1:
                                           hn  = d + u                   the decayed scale is shared by the cell)
        r   = hn * (1 / s[cell,n])         code' = clamp(rint(r), -127, 127)   (Eq. 1)
    y[p] = sum_n (s_C[g] C_code[n]) hn + D xv, from the updated state before it is re-quantized; summed here in
    float64 (the output is compared within a tolerance, not bit for bit).
    """
    xq = np.asarray(xq, np.int8); Bq = np.asarray(Bq, np.int8); Cq = np.asarray(Cq, np.int8)
    dt = np.asarray(dt, F); A = np.asarray(A, F)
    b, H, P = xq.shape
    G, N = Bq.shape[1], Bq.shape[2]
    assert qstate.dtype == np.int8 and qstate.shape == (b, H, P, N)
    hpg = H // G
    cells = cell_index_table(sc, H, P, G)
    s = state_scales.astype(F)[cells]                       # [H,P,N]
    inv = (F(1.0) / state_scales.astype(F))[cells]
    sx = sc.x_scales.astype(F)[cells]                       # [H,P]  (x shares the cells)
    gidx = np.arange(H) // hpg
    sB = sc.B_scales.astype(F)[gidx]                        # [H]
    sC = sc.C_scales.astype(F)[gidx]

    xv = sx[None] * xq.astype(F)                            # [b,H,P]
    dtx = dt[:, :, None] * xv
    Bv = sB[None, :, None] * Bq.astype(F)[:, gidx, :]       # [b,H,N]
    u = dtx[:, :, :, None] * Bv[:, :, None, :]              # [b,H,P,N]
    dA = exp_f32(dt * A[None, :])                           # [b,H]
    sd = dA[:, :, None, None] * s[None]                     # [b,H,P,N]
    d = sd * qstate.astype(F)
    hn = d + u
    r = hn * inv[None]
    qstate[...] = np.clip(np.rint(r), -127, 127).astype(np.int8)

    Cv = sC[None, :, None].astype(np.float64) * Cq.astype(np.float64)[:, gidx, :]
    y = np.einsum("bhpn,bhn->bhp", hn.astype(np.float64), Cv)
    if D is not None:
        y = y + np.asarray(D, np.float64)[None, :, None] * xv.astype(np.float64)
    return y
