"""TEST INFRASTRUCTURE: ctypes front of oracle/ssd_ref.c (the fp64 sequential scan, Eq. 2)."""
from __future__ import annotations

import ctypes as C
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "ssd_ref.c")
_LIB = os.path.join(_HERE, "libssd_ref.so")
_lib = None


def build_oracle(force: bool = True) -> str:
    """Compile the C oracle with gcc (strict IEEE arithmetic: no -ffast-math)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=c11",
                               "-Wall", "-Wextra", "-o", _LIB, _SRC, "-lm"])
    return _LIB


class _Shape(C.Structure):
    _fields_ = [(k, C.c_int32) for k in
                ("batch", "seqlen", "nheads", "headdim", "d_state", "ngroups", "m", "n")]


def _load():
    global _lib
    if _lib is None:
        build_oracle(force=False)
        _lib = C.CDLL(_LIB)
        _lib.ssd_ref_prefill.restype = C.c_int
        _lib.ssd_ref_decode_step.restype = C.c_int
    return _lib


@dataclass
class Scales:
    """Sort-and-cluster scale table of x and the per-state-group scales of B and C (Sec. 4.1)."""
    m: int
    n: int
    x_scales: np.ndarray          # [G*m*n] float32
    head_cluster_end: np.ndarray  # [G*m]   int32, exclusive end (head index inside its group)
    chan_cluster_end: np.ndarray  # [G*m*n] int32, exclusive end (sorted channel position)
    B_scales: np.ndarray          # [G] float32
    C_scales: np.ndarray          # [G] float32

    @staticmethod
    def ones(ngroups: int, heads_per_group: int, headdim: int) -> "Scales":
        return Scales(1, 1, np.ones(ngroups, np.float32),
                      np.full(ngroups, heads_per_group, np.int32),
                      np.full(ngroups, headdim, np.int32),
                      np.ones(ngroups, np.float32), np.ones(ngroups, np.float32))


def _p(a, ty):
    return a.ctypes.data_as(C.POINTER(ty)) if a is not None else None


def _c(a, dt):
    return None if a is None else np.ascontiguousarray(a, dtype=dt)


def x_scale_table(sc: Scales, nheads: int, headdim: int, ngroups: int) -> np.ndarray:
    """Expand the m x n table to a [H,P] float32 array (plain lookups, same reading as the C code)."""
    hpg = nheads // ngroups
    out = np.empty((nheads, headdim), np.float32)
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
            out[h, p] = sc.x_scales[base + j]
    return out


def ref_prefill(sc: Scales, xq, Bq, Cq, dt, A, D=None, init_state=None, pairs=None,
                want_y=True, want_state=True, nthreads=0):
    """fp64 sequential scan.  xq [b,L,H,P] int8, Bq/Cq [b,L,G,N] int8, dt [b,L,H], A/D [H].

    Returns (y, final_state, threads).  With pairs=None: y [b,L,H,P], state [b,H,P,N] (float64).
    With pairs = [(b,h), ...]: y [npairs,L,P], state [npairs,P,N].
    """
    lib = _load()
    xq = _c(xq, np.int8); Bq = _c(Bq, np.int8); Cq = _c(Cq, np.int8)
    dt = _c(dt, np.float32); A = _c(A, np.float32); D = _c(D, np.float32)
    b, L, H, P = xq.shape
    G, N = Bq.shape[2], Bq.shape[3]
    assert Bq.shape == (b, L, G, N) and Cq.shape == (b, L, G, N) and dt.shape == (b, L, H)
    assert A.shape == (H,) and H % G == 0
    shp = _Shape(b, L, H, P, N, G, sc.m, sc.n)
    xs = _c(sc.x_scales, np.float32); he = _c(sc.head_cluster_end, np.int32)
    ce = _c(sc.chan_cluster_end, np.int32)
    Bs = _c(sc.B_scales, np.float32); Cs = _c(sc.C_scales, np.float32)
    assert xs.size == G * sc.m * sc.n and he.size == G * sc.m and ce.size == G * sc.m * sc.n
    init = _c(init_state, np.float64)
    if init is not None:
        assert init.shape == (b, H, P, N)
    if pairs is not None:
        pr = np.ascontiguousarray(np.asarray(pairs, np.int32).reshape(-1, 2))
        npairs = pr.shape[0]
    else:
        pr, npairs = None, b * H
    y = np.empty((npairs, L, P), np.float64) if want_y else None
    st = np.empty((npairs, P, N), np.float64) if want_state else None
    used = lib.ssd_ref_prefill(C.byref(shp), _p(xs, C.c_float), _p(he, C.c_int32), _p(ce, C.c_int32),
                               _p(Bs, C.c_float), _p(Cs, C.c_float), _p(xq, C.c_int8), _p(Bq, C.c_int8),
                               _p(Cq, C.c_int8), _p(dt, C.c_float), _p(A, C.c_float), _p(D, C.c_float),
                               _p(init, C.c_double), _p(pr, C.c_int32), C.c_int64(npairs),
                               _p(y, C.c_double), _p(st, C.c_double), C.c_int(nthreads))
    if used < 0:
        raise ValueError("ssd_ref_prefill: bad shape")
    if pairs is None:
        if y is not None:
            y = np.ascontiguousarray(y.reshape(b, H, L, P).transpose(0, 2, 1, 3))
        if st is not None:
            st = st.reshape(b, H, P, N)
    return y, st, used


def ref_decode_step(sc: Scales, xq, Bq, Cq, dt, A, D, state, nthreads=0):
    """One step of Eq. 2 on the caller's float64 state [b,H,P,N] (updated in place).  Returns y [b,H,P]."""
    lib = _load()
    xq = _c(xq, np.int8); Bq = _c(Bq, np.int8); Cq = _c(Cq, np.int8)
    dt = _c(dt, np.float32); A = _c(A, np.float32); D = _c(D, np.float32)
    b, H, P = xq.shape
    G, N = Bq.shape[1], Bq.shape[2]
    assert state.dtype == np.float64 and state.flags.c_contiguous and state.shape == (b, H, P, N)
    assert Cq.shape == (b, G, N) and dt.shape == (b, H) and A.shape == (H,)
    shp = _Shape(b, 1, H, P, N, G, sc.m, sc.n)
    xs = _c(sc.x_scales, np.float32); he = _c(sc.head_cluster_end, np.int32)
    ce = _c(sc.chan_cluster_end, np.int32)
    Bs = _c(sc.B_scales, np.float32); Cs = _c(sc.C_scales, np.float32)
    y = np.empty((b, H, P), np.float64)
    used = lib.ssd_ref_decode_step(C.byref(shp), _p(xs, C.c_float), _p(he, C.c_int32), _p(ce, C.c_int32),
                                   _p(Bs, C.c_float), _p(Cs, C.c_float), _p(xq, C.c_int8),
                                   _p(Bq, C.c_int8), _p(Cq, C.c_int8), _p(dt, C.c_float), _p(A, C.c_float),
                                   _p(D, C.c_float), _p(state, C.c_double), _p(y, C.c_double),
                                   C.c_int(nthreads))
    if used < 0:
        raise ValueError("ssd_ref_decode_step: bad shape")
    return y
