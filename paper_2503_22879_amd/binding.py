"""ctypes binding of include/quamba_ssd.h: same names, argument marshalling only."""
from __future__ import annotations

import ctypes as C
import os
from dataclasses import dataclass

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.environ.get("QUAMBA_SSD_LIBRARY", os.path.join(_PKG, "libquamba_ssd.so"))
_lib = None

FLAG_GENERIC_KERNEL = 0x1
FLAG_PRECISE_STATE = 0x2
FLAG_NO_CHANNEL_SPLIT = 0x4
FLAG_NO_DECAY_SKIP = 0x8
FLAG_NO_SEQ_SPLIT = 0x10

EXPORTED_SYMBOLS = ("quamba_ssd_prefill_workspace_size", "quamba_ssd_prefill", "quamba_ssd_prefill_noalloc", "quamba_ssd_decode_step",
                    "quamba_ssd_decode_step_q8", "quamba_ssd_quantize_state", "quamba_state_scales",
                    "quamba_hadamard_quantize", "quamba_conv1d_q8", "quamba_mamba1_scan",
                    "quamba_mamba1_decode_step", "quamba_mamba1_scan_gated", "quamba_mamba1_decode_step_gated",
                    "quamba_ssd_prefill_gated", "quamba_ssd_decode_step_gated", "quamba_ssd_decode_step_q8_gated",
                    "quamba_reorder_params", "quamba_gather_rows", "quamba_quantize_x",
                    "quamba_quantize_groups", "quamba_strerror",
                    # measurement helpers of the benchmark harness (include/quamba_probe.h)
                    "quamba_probe_mfma", "quamba_probe_stream_rmw", "quamba_probe_stream_read", "quamba_probe_clock",
                    "quamba_probe_clock_xcd")


class QuambaError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {quamba_strerror(status)} (status {status})")


class Shape(C.Structure):
    """quamba_ssd_shape_t"""
    _fields_ = [("batch", C.c_int32), ("seqlen", C.c_int32), ("nheads", C.c_int32), ("headdim", C.c_int32),
                ("d_state", C.c_int32), ("ngroups", C.c_int32), ("chunk", C.c_int32),
                ("n_head_clusters", C.c_int32), ("n_chan_clusters", C.c_int32), ("flags", C.c_uint32)]


class _ScalesStruct(C.Structure):
    """quamba_ssd_scales_t"""
    _fields_ = [("x_scales", C.c_void_p), ("head_cluster_end", C.c_void_p), ("chan_cluster_end", C.c_void_p),
                ("B_scales", C.c_void_p), ("C_scales", C.c_void_p)]


class _GateStruct(C.Structure):
    """quamba_ssd_gate_t"""
    _fields_ = [("z", C.c_void_p), ("z_scale", C.c_float), ("dt_q", C.c_void_p), ("dt_scale", C.c_float),
                ("dt_bias", C.c_void_p)]


@dataclass
class Gate:
    """Optional 8-bit side inputs (device tensors): gate codes z with their scale, and / or the codes of the step
    size's pre-activation with their scale and the per-head bias."""
    z: object = None
    z_scale: float = 0.0
    dt_q: object = None
    dt_scale: float = 0.0
    dt_bias: object = None

    def struct(self, z_shape, dt_shape, nheads) -> _GateStruct:
        import torch
        return _GateStruct(_dp(self.z, torch.int8, z_shape, "gate.z"), float(self.z_scale),
                           _dp(self.dt_q, torch.int8, dt_shape, "gate.dt_q"), float(self.dt_scale),
                           _dp(self.dt_bias, torch.float32, (nheads,), "gate.dt_bias"))


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Load libquamba_ssd.so; raises if it has not been built (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(_LIB_PATH):
            raise FileNotFoundError(
                f"{_LIB_PATH} is missing: build it with `python -m paper_2503_22879_amd.build` "
                "(or __graft_entry__.build()); this package has no CPU fallback")
        # PyTorch ships its own HIP runtime.  Import it before the library is opened, so that the library's dependency
        # on libamdhip64 resolves to the runtime that owns the tensors and streams the callers pass in; opened the other
        # way round, the process holds two runtimes and launches on torch's streams are refused.
        try:
            import torch  # noqa: F401
        except ImportError:
            pass
        lib = C.CDLL(_LIB_PATH)
        lib.quamba_ssd_prefill_workspace_size.restype = C.c_size_t
        lib.quamba_ssd_prefill_workspace_size.argtypes = [C.POINTER(Shape)]
        lib.quamba_ssd_prefill.restype = C.c_int
        lib.quamba_ssd_prefill.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct)] + [C.c_void_p] * 10 + \
            [C.c_size_t, C.c_void_p]
        lib.quamba_ssd_prefill_noalloc.restype = C.c_int
        lib.quamba_ssd_prefill_noalloc.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct)] + [C.c_void_p] * 10
        lib.quamba_ssd_decode_step.restype = C.c_int
        lib.quamba_ssd_decode_step.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct)] + [C.c_void_p] * 9
        lib.quamba_mamba1_scan.restype = C.c_int
        lib.quamba_mamba1_scan.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct)] + [C.c_void_p] * 10
        lib.quamba_mamba1_decode_step.restype = C.c_int
        lib.quamba_mamba1_decode_step.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct)] + [C.c_void_p] * 9
        lib.quamba_mamba1_scan_gated.restype = C.c_int
        lib.quamba_mamba1_scan_gated.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct), C.POINTER(_GateStruct)] + \
            [C.c_void_p] * 10
        lib.quamba_mamba1_decode_step_gated.restype = C.c_int
        lib.quamba_mamba1_decode_step_gated.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct),
                                                        C.POINTER(_GateStruct)] + [C.c_void_p] * 9
        lib.quamba_conv1d_q8.restype = C.c_int
        lib.quamba_conv1d_q8.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct), C.c_void_p, C.c_void_p, C.c_void_p,
                                         C.c_float] + [C.c_void_p] * 6
        lib.quamba_hadamard_quantize.restype = C.c_int
        lib.quamba_hadamard_quantize.argtypes = [C.c_void_p, C.c_int64, C.c_int32, C.c_float, C.c_void_p, C.c_void_p]
        lib.quamba_ssd_prefill_gated.restype = C.c_int
        lib.quamba_ssd_prefill_gated.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct), C.POINTER(_GateStruct)] + \
            [C.c_void_p] * 10 + [C.c_size_t, C.c_void_p]
        lib.quamba_ssd_decode_step_gated.restype = C.c_int
        lib.quamba_ssd_decode_step_gated.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct),
                                                     C.POINTER(_GateStruct)] + [C.c_void_p] * 9
        lib.quamba_ssd_decode_step_q8_gated.restype = C.c_int
        lib.quamba_ssd_decode_step_q8_gated.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct),
                                                        C.POINTER(_GateStruct)] + [C.c_void_p] * 10
        lib.quamba_ssd_decode_step_q8.restype = C.c_int
        lib.quamba_ssd_decode_step_q8.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct)] + [C.c_void_p] * 10
        lib.quamba_ssd_quantize_state.restype = C.c_int
        lib.quamba_ssd_quantize_state.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct)] + [C.c_void_p] * 4
        lib.quamba_state_scales.restype = C.c_int
        lib.quamba_state_scales.argtypes = [C.c_int32] * 6 + [C.c_void_p] * 4
        lib.quamba_reorder_params.restype = C.c_int
        lib.quamba_reorder_params.argtypes = [C.c_int32] * 5 + [C.c_uint64, C.c_int32] + [C.c_void_p] * 10
        lib.quamba_gather_rows.restype = C.c_int
        lib.quamba_gather_rows.argtypes = [C.c_void_p, C.c_void_p, C.c_void_p, C.c_int64, C.c_int64]
        lib.quamba_quantize_x.restype = C.c_int
        lib.quamba_quantize_x.argtypes = [C.POINTER(Shape), C.POINTER(_ScalesStruct), C.c_int64, C.c_void_p,
                                          C.c_void_p]
        lib.quamba_quantize_groups.restype = C.c_int
        lib.quamba_quantize_groups.argtypes = [C.c_int64, C.c_int32, C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p]
        lib.quamba_strerror.restype = C.c_char_p
        lib.quamba_strerror.argtypes = [C.c_int]
        _lib = lib
    return _lib


def quamba_strerror(status: int) -> str:
    return load_library().quamba_strerror(int(status)).decode()


@dataclass
class HostScales:
    """Sort-and-cluster result on the host (numpy arrays), as quamba_reorder_params fills it."""
    x_scales: np.ndarray
    head_cluster_end: np.ndarray
    chan_cluster_end: np.ndarray
    B_scales: np.ndarray
    C_scales: np.ndarray

    def struct(self) -> _ScalesStruct:
        return _ScalesStruct(*(a.ctypes.data for a in (self.x_scales, self.head_cluster_end,
                                                       self.chan_cluster_end, self.B_scales, self.C_scales)))


class DeviceScales:
    """The same five tables as device tensors (kept alive by this object)."""

    def __init__(self, host: HostScales, device="cuda"):
        import torch
        self.tensors = [torch.from_numpy(np.ascontiguousarray(a)).to(device) for a in
                        (host.x_scales.astype(np.float32), host.head_cluster_end.astype(np.int32),
                         host.chan_cluster_end.astype(np.int32), host.B_scales.astype(np.float32),
                         host.C_scales.astype(np.float32))]

    def struct(self) -> _ScalesStruct:
        return _ScalesStruct(*(t.data_ptr() for t in self.tensors))


def _dp(t, dtype=None, shape=None, name="tensor"):
    """Device pointer of a torch tensor (None -> NULL), with the checks a C caller would have to make itself."""
    if t is None:
        return None
    if not t.is_cuda or not t.is_contiguous():
        raise ValueError(f"{name} must be a contiguous device tensor")
    if dtype is not None and t.dtype != dtype:
        raise ValueError(f"{name} must have dtype {dtype}, got {t.dtype}")
    if shape is not None and tuple(t.shape) != tuple(shape):
        raise ValueError(f"{name} must have shape {tuple(shape)}, got {tuple(t.shape)}")
    return t.data_ptr()


def _stream_ptr(stream):
    import torch
    if stream is None:
        stream = torch.cuda.current_stream()
    return getattr(stream, "cuda_stream", stream)


def quamba_ssd_prefill_workspace_size(shape: Shape) -> int:
    return int(load_library().quamba_ssd_prefill_workspace_size(C.byref(shape)))


def quamba_ssd_prefill(shape: Shape, scales, x, B, Cm, dt, A, D, init_state, y, final_state=None,
                       workspace=None, stream=None, gate: Gate | None = None) -> None:
    """Enqueue the chunked prefill on `stream` (default: torch's current stream).  Tensors are torch device tensors.
    With `gate`, quamba_ssd_prefill_gated is called (dt may then be None if the gate carries the step-size codes)."""
    import torch
    s = shape
    sc = scales.struct()
    if gate is not None:
        return _prefill_gated(s, sc, gate, x, B, Cm, dt, A, D, init_state, y, final_state, workspace, stream)
    ws_ptr = _dp(workspace, name="workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st_shape = (s.batch, s.nheads, s.headdim, s.d_state)
    rc = load_library().quamba_ssd_prefill(
        C.byref(s), C.byref(sc),
        _dp(x, torch.int8, (s.batch, s.seqlen, s.nheads, s.headdim), "x"),
        _dp(B, torch.int8, (s.batch, s.seqlen, s.ngroups, s.d_state), "B"),
        _dp(Cm, torch.int8, (s.batch, s.seqlen, s.ngroups, s.d_state), "C"),
        _dp(dt, torch.float32, (s.batch, s.seqlen, s.nheads), "dt"),
        _dp(A, torch.float32, (s.nheads,), "A"), _dp(D, torch.float32, (s.nheads,), "D"),
        _dp(init_state, torch.float32, st_shape, "init_state"),
        _dp(y, torch.float16, (s.batch, s.seqlen, s.nheads, s.headdim), "y"),
        _dp(final_state, torch.float32, st_shape, "final_state"),
        ws_ptr, ws_bytes, _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_ssd_prefill")


def quamba_ssd_prefill_noalloc(shape: Shape, scales, x, B, Cm, dt, A, D, init_state, y, final_state=None,
                               stream=None) -> None:
    """Enqueue the chunked prefill with the library's own fixed scratch area instead of a caller's workspace."""
    import torch
    s = shape
    sc = scales.struct()
    st_shape = (s.batch, s.nheads, s.headdim, s.d_state)
    rc = load_library().quamba_ssd_prefill_noalloc(
        C.byref(s), C.byref(sc),
        _dp(x, torch.int8, (s.batch, s.seqlen, s.nheads, s.headdim), "x"),
        _dp(B, torch.int8, (s.batch, s.seqlen, s.ngroups, s.d_state), "B"),
        _dp(Cm, torch.int8, (s.batch, s.seqlen, s.ngroups, s.d_state), "C"),
        _dp(dt, torch.float32, (s.batch, s.seqlen, s.nheads), "dt"),
        _dp(A, torch.float32, (s.nheads,), "A"), _dp(D, torch.float32, (s.nheads,), "D"),
        _dp(init_state, torch.float32, st_shape, "init_state"),
        _dp(y, torch.float16, (s.batch, s.seqlen, s.nheads, s.headdim), "y"),
        _dp(final_state, torch.float32, st_shape, "final_state"), _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_ssd_prefill_noalloc")


def _prefill_gated(s, sc, gate, x, B, Cm, dt, A, D, init_state, y, final_state, workspace, stream) -> None:
    import torch
    ws_ptr = _dp(workspace, name="workspace")
    ws_bytes = 0 if workspace is None else workspace.numel() * workspace.element_size()
    st_shape = (s.batch, s.nheads, s.headdim, s.d_state)
    g = gate.struct((s.batch, s.seqlen, s.nheads, s.headdim), (s.batch, s.seqlen, s.nheads), s.nheads)
    rc = load_library().quamba_ssd_prefill_gated(
        C.byref(s), C.byref(sc), C.byref(g),
        _dp(x, torch.int8, (s.batch, s.seqlen, s.nheads, s.headdim), "x"),
        _dp(B, torch.int8, (s.batch, s.seqlen, s.ngroups, s.d_state), "B"),
        _dp(Cm, torch.int8, (s.batch, s.seqlen, s.ngroups, s.d_state), "C"),
        _dp(dt, torch.float32, (s.batch, s.seqlen, s.nheads), "dt"),
        _dp(A, torch.float32, (s.nheads,), "A"), _dp(D, torch.float32, (s.nheads,), "D"),
        _dp(init_state, torch.float32, st_shape, "init_state"),
        _dp(y, torch.float16, (s.batch, s.seqlen, s.nheads, s.headdim), "y"),
        _dp(final_state, torch.float32, st_shape, "final_state"),
        ws_ptr, ws_bytes, _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_ssd_prefill_gated")


def quamba_ssd_decode_step(shape: Shape, scales, x, B, Cm, dt, A, D, state, y, stream=None,
                           gate: Gate | None = None) -> None:
    """Enqueue one decode step; `state` is updated in place.  With `gate`, quamba_ssd_decode_step_gated is called."""
    import torch
    s = shape
    sc = scales.struct()
    if gate is not None:
        g = gate.struct((s.batch, s.nheads, s.headdim), (s.batch, s.nheads), s.nheads)
        rc = load_library().quamba_ssd_decode_step_gated(
            C.byref(s), C.byref(sc), C.byref(g),
            _dp(x, torch.int8, (s.batch, s.nheads, s.headdim), "x"),
            _dp(B, torch.int8, (s.batch, s.ngroups, s.d_state), "B"),
            _dp(Cm, torch.int8, (s.batch, s.ngroups, s.d_state), "C"),
            _dp(dt, torch.float32, (s.batch, s.nheads), "dt"),
            _dp(A, torch.float32, (s.nheads,), "A"), _dp(D, torch.float32, (s.nheads,), "D"),
            _dp(state, torch.float32, (s.batch, s.nheads, s.headdim, s.d_state), "state"),
            _dp(y, torch.float16, (s.batch, s.nheads, s.headdim), "y"), _stream_ptr(stream))
        if rc != 0:
            raise QuambaError(rc, "quamba_ssd_decode_step_gated")
        return
    rc = load_library().quamba_ssd_decode_step(
        C.byref(s), C.byref(sc),
        _dp(x, torch.int8, (s.batch, s.nheads, s.headdim), "x"),
        _dp(B, torch.int8, (s.batch, s.ngroups, s.d_state), "B"),
        _dp(Cm, torch.int8, (s.batch, s.ngroups, s.d_state), "C"),
        _dp(dt, torch.float32, (s.batch, s.nheads), "dt"),
        _dp(A, torch.float32, (s.nheads,), "A"), _dp(D, torch.float32, (s.nheads,), "D"),
        _dp(state, torch.float32, (s.batch, s.nheads, s.headdim, s.d_state), "state"),
        _dp(y, torch.float16, (s.batch, s.nheads, s.headdim), "y"), _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_ssd_decode_step")


def quamba_ssd_decode_step_q8(shape: Shape, scales, state_scales, x, B, Cm, dt, A, D, state_q, y, stream=None,
                              gate: Gate | None = None) -> None:
    """Enqueue one decode step on the 8-bit cached state; `state_q` (int8) is updated in place.  With `gate` (z only),
    quamba_ssd_decode_step_q8_gated is called."""
    import torch
    s = shape
    sc = scales.struct()
    ncell = s.ngroups * s.n_head_clusters * s.n_chan_clusters
    if gate is not None:
        g = gate.struct((s.batch, s.nheads, s.headdim), (s.batch, s.nheads), s.nheads)
        rc = load_library().quamba_ssd_decode_step_q8_gated(
            C.byref(s), C.byref(sc), C.byref(g),
            _dp(state_scales, torch.float32, (ncell, s.d_state), "state_scales"),
            _dp(x, torch.int8, (s.batch, s.nheads, s.headdim), "x"),
            _dp(B, torch.int8, (s.batch, s.ngroups, s.d_state), "B"),
            _dp(Cm, torch.int8, (s.batch, s.ngroups, s.d_state), "C"),
            _dp(dt, torch.float32, (s.batch, s.nheads), "dt"),
            _dp(A, torch.float32, (s.nheads,), "A"), _dp(D, torch.float32, (s.nheads,), "D"),
            _dp(state_q, torch.int8, (s.batch, s.nheads, s.headdim, s.d_state), "state_q"),
            _dp(y, torch.float16, (s.batch, s.nheads, s.headdim), "y"), _stream_ptr(stream))
        if rc != 0:
            raise QuambaError(rc, "quamba_ssd_decode_step_q8_gated")
        return
    rc = load_library().quamba_ssd_decode_step_q8(
        C.byref(s), C.byref(sc), _dp(state_scales, torch.float32, (ncell, s.d_state), "state_scales"),
        _dp(x, torch.int8, (s.batch, s.nheads, s.headdim), "x"),
        _dp(B, torch.int8, (s.batch, s.ngroups, s.d_state), "B"),
        _dp(Cm, torch.int8, (s.batch, s.ngroups, s.d_state), "C"),
        _dp(dt, torch.float32, (s.batch, s.nheads), "dt"),
        _dp(A, torch.float32, (s.nheads,), "A"), _dp(D, torch.float32, (s.nheads,), "D"),
        _dp(state_q, torch.int8, (s.batch, s.nheads, s.headdim, s.d_state), "state_q"),
        _dp(y, torch.float16, (s.batch, s.nheads, s.headdim), "y"), _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_ssd_decode_step_q8")


def quamba_ssd_quantize_state(shape: Shape, scales, state_scales, state, state_q, stream=None) -> None:
    """Enqueue Eq. 1 on an fp32 device state with the scales of the 8-bit cache."""
    import torch
    s = shape
    sc = scales.struct()
    ncell = s.ngroups * s.n_head_clusters * s.n_chan_clusters
    st_shape = (s.batch, s.nheads, s.headdim, s.d_state)
    rc = load_library().quamba_ssd_quantize_state(
        C.byref(s), C.byref(sc), _dp(state_scales, torch.float32, (ncell, s.d_state), "state_scales"),
        _dp(state, torch.float32, st_shape, "state"), _dp(state_q, torch.int8, st_shape, "state_q"),
        _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_ssd_quantize_state")


def quamba_state_scales(nheads, headdim, ngroups, m, n, d_state, head_cluster_end, chan_cluster_end,
                        state_calib_absmax) -> np.ndarray:
    """Static scales of the 8-bit cached state from calibrated maxima [H,P,N] (host).  Returns [G*m*n, N] float32."""
    he = np.ascontiguousarray(head_cluster_end, np.int32).reshape(-1)
    ce = np.ascontiguousarray(chan_cluster_end, np.int32).reshape(-1)
    mx = np.ascontiguousarray(state_calib_absmax, np.float32).reshape(-1)
    if he.size != ngroups * m or ce.size != ngroups * m * n or mx.size != nheads * headdim * d_state:
        raise ValueError("arrays do not match the shape")
    out = np.empty((ngroups * m * n, d_state), np.float32)
    rc = load_library().quamba_state_scales(nheads, headdim, ngroups, m, n, d_state, he.ctypes.data, ce.ctypes.data,
                                            mx.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise QuambaError(rc, "quamba_state_scales")
    return out


def quamba_mamba1_scan(shape: Shape, scales: DeviceScales, x, B, Cm, dt, A, D, y, init_state=None, final_state=None,
                       stream=None, gate: Gate | None = None) -> None:
    """Enqueue the 8-bit Mamba1 selective scan (channel-major device tensors, time last).  With `gate`,
    quamba_mamba1_scan_gated is called (dt may then be None if the gate carries the step-size codes)."""
    import torch
    b, L, Dn, N = shape.batch, shape.seqlen, shape.headdim, shape.d_state
    sc = scales.struct()
    args = (_dp(x, torch.int8, (b, Dn, L), "x"), _dp(B, torch.int8, (b, N, L), "B"),
            _dp(Cm, torch.int8, (b, N, L), "C"), _dp(dt, torch.float32, (b, Dn, L), "dt"),
            _dp(A, torch.float32, (Dn, N), "A"), _dp(D, torch.float32, (Dn,), "D"),
            _dp(init_state, torch.float32, (b, Dn, N), "init_state"), _dp(y, torch.float16, (b, Dn, L), "y"),
            _dp(final_state, torch.float32, (b, Dn, N), "final_state"), _stream_ptr(stream))
    if gate is None:
        rc, name = load_library().quamba_mamba1_scan(C.byref(shape), C.byref(sc), *args), "quamba_mamba1_scan"
    else:
        g = gate.struct((b, Dn, L), (b, Dn, L), Dn)
        rc = load_library().quamba_mamba1_scan_gated(C.byref(shape), C.byref(sc), C.byref(g), *args)
        name = "quamba_mamba1_scan_gated"
    if rc != 0:
        raise QuambaError(rc, name)


def quamba_mamba1_decode_step(shape: Shape, scales: DeviceScales, x, B, Cm, dt, A, D, state, y, stream=None,
                              gate: Gate | None = None) -> None:
    """Enqueue one generation step of the Mamba1 recurrence on the fp32 state [b, D, N], in place.  With `gate`,
    quamba_mamba1_decode_step_gated is called."""
    import torch
    b, Dn, N = shape.batch, shape.headdim, shape.d_state
    sc = scales.struct()
    args = (_dp(x, torch.int8, (b, Dn), "x"), _dp(B, torch.int8, (b, N), "B"),
            _dp(Cm, torch.int8, (b, N), "C"), _dp(dt, torch.float32, (b, Dn), "dt"),
            _dp(A, torch.float32, (Dn, N), "A"), _dp(D, torch.float32, (Dn,), "D"),
            _dp(state, torch.float32, (b, Dn, N), "state"), _dp(y, torch.float16, (b, Dn), "y"), _stream_ptr(stream))
    if gate is None:
        rc, name = load_library().quamba_mamba1_decode_step(C.byref(shape), C.byref(sc), *args), "quamba_mamba1_decode_step"
    else:
        g = gate.struct((b, Dn), (b, Dn), Dn)
        rc = load_library().quamba_mamba1_decode_step_gated(C.byref(shape), C.byref(sc), C.byref(g), *args)
        name = "quamba_mamba1_decode_step_gated"
    if rc != 0:
        raise QuambaError(rc, name)


def quamba_conv1d_q8(shape: Shape, scales: DeviceScales, xBC, weight, bias, in_w_scale: float, x_out, B_out, C_out,
                     conv_state_in=None, conv_state_out=None, stream=None) -> None:
    """Enqueue the W8A8 causal convolution + SiLU + Eq. 1 that produces the scan's int8 x, B and C (device tensors)."""
    import torch
    b, L, H, P, G, N = shape.batch, shape.seqlen, shape.nheads, shape.headdim, shape.ngroups, shape.d_state
    Ct = H * P + 2 * G * N
    sc = scales.struct()
    rc = load_library().quamba_conv1d_q8(
        C.byref(shape), C.byref(sc), _dp(xBC, torch.int8, (b, L, Ct), "xBC"), _dp(weight, torch.int8, (Ct, 4), "weight"),
        _dp(bias, torch.float32, (Ct,), "bias"), float(in_w_scale),
        _dp(conv_state_in, torch.int8, (b, 3, Ct), "conv_state_in"), _dp(x_out, torch.int8, (b, L, H, P), "x_out"),
        _dp(B_out, torch.int8, (b, L, G, N), "B_out"), _dp(C_out, torch.int8, (b, L, G, N), "C_out"),
        _dp(conv_state_out, torch.int8, (b, 3, Ct), "conv_state_out"), _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_conv1d_q8")


def quamba_hadamard_quantize(y, s_y: float, out, stream=None) -> None:
    """Enqueue out = Eq.1((1/s_y) H_n y) over the last axis of the fp16 device tensor y (n = 2^k, 12 * 2^k or 20 * 2^k)."""
    import torch
    n = y.shape[-1]
    rows = y.numel() // max(1, n)
    if rows == 0 and n > 0:
        return                      # an empty tensor has no device pointer to pass
    rc = load_library().quamba_hadamard_quantize(_dp(y, torch.float16, name="y"), rows, n, float(s_y),
                                                 _dp(out, torch.int8, tuple(y.shape), "out"), _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_hadamard_quantize")


def quamba_reorder_params(nheads, headdim, ngroups, m, n, d_state, x_calib_absmax, B_calib_absmax,
                          C_calib_absmax, seed=0):
    """Offline sort-and-cluster on the host.  Returns (head_perm [H], chan_perm [H,P], HostScales)."""
    xm = np.ascontiguousarray(x_calib_absmax, np.float32).reshape(-1)
    bm = np.ascontiguousarray(B_calib_absmax, np.float32).reshape(-1)
    cm = np.ascontiguousarray(C_calib_absmax, np.float32).reshape(-1)
    if xm.size != nheads * headdim or bm.size != ngroups * d_state or cm.size != ngroups * d_state:
        raise ValueError("calibration arrays do not match the shape")
    head_perm = np.empty(nheads, np.int32)
    chan_perm = np.empty((nheads, headdim), np.int32)
    hs = HostScales(np.empty(ngroups * m * n, np.float32), np.empty(ngroups * m, np.int32),
                    np.empty(ngroups * m * n, np.int32), np.empty(ngroups, np.float32),
                    np.empty(ngroups, np.float32))
    rc = load_library().quamba_reorder_params(
        nheads, headdim, ngroups, m, n, seed, d_state, xm.ctypes.data, bm.ctypes.data, cm.ctypes.data,
        head_perm.ctypes.data, chan_perm.ctypes.data, hs.x_scales.ctypes.data, hs.head_cluster_end.ctypes.data,
        hs.chan_cluster_end.ctypes.data, hs.B_scales.ctypes.data, hs.C_scales.ctypes.data)
    if rc != 0:
        raise QuambaError(rc, "quamba_reorder_params")
    return head_perm, chan_perm, hs


def quamba_gather_rows(src: np.ndarray, new_to_old: np.ndarray) -> np.ndarray:
    """dst[i] = src[new_to_old[i]] along axis 0 (host)."""
    src = np.ascontiguousarray(src)
    idx = np.ascontiguousarray(new_to_old, np.int32)
    if idx.shape != (src.shape[0],):
        raise ValueError("need one index per row")
    dst = np.empty_like(src)
    row_bytes = src.nbytes // max(1, src.shape[0])
    rc = load_library().quamba_gather_rows(dst.ctypes.data, src.ctypes.data, idx.ctypes.data, src.shape[0],
                                           row_bytes)
    if rc != 0:
        raise QuambaError(rc, "quamba_gather_rows")
    return dst


def quamba_quantize_x(shape: Shape, host_scales: HostScales, x: np.ndarray) -> np.ndarray:
    """Eq. 1 with the m x n cluster scales; x [..., H, P] float32 in reordered order -> int8."""
    x = np.ascontiguousarray(x, np.float32)
    if x.shape[-2:] != (shape.nheads, shape.headdim):
        raise ValueError("x must end in [nheads, headdim]")
    tokens = x.size // (shape.nheads * shape.headdim)
    out = np.empty(x.shape, np.int8)
    sc = host_scales.struct()
    rc = load_library().quamba_quantize_x(C.byref(shape), C.byref(sc), tokens, x.ctypes.data, out.ctypes.data)
    if rc != 0:
        raise QuambaError(rc, "quamba_quantize_x")
    return out


def quamba_quantize_groups(v: np.ndarray, group_scales: np.ndarray) -> np.ndarray:
    """Eq. 1 with one scale per state group; v [..., G, N] float32 -> int8."""
    v = np.ascontiguousarray(v, np.float32)
    gs = np.ascontiguousarray(group_scales, np.float32)
    G, N = v.shape[-2], v.shape[-1]
    if gs.shape != (G,):
        raise ValueError("need one scale per group")
    out = np.empty(v.shape, np.int8)
    rc = load_library().quamba_quantize_groups(v.size // (G * N), G, N, gs.ctypes.data, v.ctypes.data,
                                               out.ctypes.data)
    if rc != 0:
        raise QuambaError(rc, "quamba_quantize_groups")
    return out


def quamba_probe_mfma(kind: int, iters: int, sink, stream=None, waves_per_simd: int = 2,
                      uniform_operands: bool = False) -> float:
    """Enqueue the register-resident matrix-core loop (kind 0: fp16, 1: int8); returns the operations of the launch."""
    import torch
    ops = C.c_double(0.0)
    lib = load_library()
    lib.quamba_probe_mfma.argtypes = [C.c_int, C.c_int, C.c_int, C.c_int, C.POINTER(C.c_double), C.c_void_p, C.c_void_p]
    rc = lib.quamba_probe_mfma(int(kind), int(iters), int(waves_per_simd), int(bool(uniform_operands)), C.byref(ops),
                               _dp(sink, torch.int32, name="sink"),
                               _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_probe_mfma")
    return ops.value


def quamba_probe_stream_rmw(buf, stream=None) -> int:
    """Enqueue one in-place read-modify-write pass over the device tensor buf; returns the bytes the launch moves."""
    lib = load_library()
    lib.quamba_probe_stream_rmw.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p]
    nbytes = buf.numel() * buf.element_size()
    rc = lib.quamba_probe_stream_rmw(_dp(buf, buf.dtype, name="buf"), nbytes, _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_probe_stream_rmw")
    return 2 * nbytes


def quamba_probe_stream_read(buf, sink, stream=None) -> int:
    """Enqueue one read-only pass over the device tensor buf; sink: int32 device tensor (>= 1 element); returns the
    bytes the launch moves."""
    import torch
    lib = load_library()
    lib.quamba_probe_stream_read.argtypes = [C.c_void_p, C.c_size_t, C.c_void_p, C.c_void_p]
    nbytes = buf.numel() * buf.element_size()
    rc = lib.quamba_probe_stream_read(_dp(buf, buf.dtype, name="buf"), nbytes, _dp(sink, torch.int32, name="sink"),
                                      _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_probe_stream_read")
    return nbytes


def quamba_probe_clock_xcd(out, spin_iters: int = 20000, stream=None) -> None:
    """Enqueue the per-XCD shader-clock probe; out: int64 device tensor [n, 3] (shader clocks, ticks of 10 ns, XCD id)."""
    import torch
    lib = load_library()
    lib.quamba_probe_clock_xcd.argtypes = [C.c_void_p, C.c_int, C.c_int, C.c_void_p]
    n = int(out.shape[0])
    rc = lib.quamba_probe_clock_xcd(_dp(out, torch.int64, (n, 3), "out"), n, int(spin_iters), _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_probe_clock_xcd")


def quamba_probe_clock(out, spin_iters: int = 20000, stream=None) -> None:
    """Enqueue the shader-clock probe; out: int64 device tensor of 2 (shader clocks, ticks of 10 ns)."""
    import torch
    lib = load_library()
    lib.quamba_probe_clock.argtypes = [C.c_void_p, C.c_int, C.c_void_p]
    rc = lib.quamba_probe_clock(_dp(out, torch.int64, (2,), "out"), int(spin_iters), _stream_ptr(stream))
    if rc != 0:
        raise QuambaError(rc, "quamba_probe_clock")
