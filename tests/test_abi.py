"""The C-ABI library loads, exports every function the header declares, and validates arguments before touching
the device (so these run without a GPU)."""
import ctypes as C
import os
import re

import pytest

import paper_2503_22879_amd as q

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _declared():
    names = set()
    for header in ("quamba_ssd.h", "quamba_probe.h"):
        text = open(os.path.join(ROOT, "include", header)).read()
        text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
        names |= set(re.findall(r"\b(quamba_[a-z_0-9]+)\s*\(", text))
    return sorted(names)


def test_every_declared_symbol_is_exported():
    lib = q.load_library()
    names = _declared()
    assert set(names) == set(q.EXPORTED_SYMBOLS)
    for n in names:
        assert getattr(lib, n) is not None


def test_strerror():
    assert q.quamba_strerror(0) == "ok"
    assert "NULL" in q.quamba_strerror(-1) and "unknown" in q.quamba_strerror(-99)


def _shape(**kw):
    d = dict(batch=1, seqlen=8, nheads=4, headdim=8, d_state=8, ngroups=2, chunk=4, n_head_clusters=1,
             n_chan_clusters=1, flags=0)
    d.update(kw)
    return q.Shape(**d)


def _call_prefill(shape, scales_ok=True, null_arg=None, ws_bytes=0):
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    from paper_2503_22879_amd.binding import _ScalesStruct
    sc = _ScalesStruct(p, p, p, p, p) if scales_ok else _ScalesStruct(p, None, p, p, p)
    args = [p] * 10          # x B C dt A D init y final workspace
    if null_arg is not None:
        args[null_arg] = None
    return lib.quamba_ssd_prefill(C.byref(shape), C.byref(sc), *args, ws_bytes, None)


def _call_decode(shape, null_arg=None):
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    from paper_2503_22879_amd.binding import _ScalesStruct
    sc = _ScalesStruct(p, p, p, p, p)
    args = [p] * 8           # x B C dt A D state y
    if null_arg is not None:
        args[null_arg] = None
    return lib.quamba_ssd_decode_step(C.byref(shape), C.byref(sc), *args, None)


@pytest.mark.parametrize("kw", [dict(batch=0), dict(seqlen=0), dict(nheads=5), dict(headdim=-1), dict(d_state=0),
                                dict(ngroups=0), dict(chunk=0), dict(n_head_clusters=0), dict(n_chan_clusters=0),
                                dict(headdim=512, d_state=512, flags=1)])
def test_prefill_rejects_bad_shapes_without_a_device(kw):
    assert _call_prefill(_shape(**kw)) == -2


def test_prefill_rejects_nulls_and_flags():
    for i in (0, 1, 2, 3, 4, 7):           # x B C dt A y are required
        assert _call_prefill(_shape(), null_arg=i) == -1
    assert _call_prefill(_shape(), scales_ok=False) == -1
    assert _call_prefill(_shape(flags=0x80)) == -5
    lib = q.load_library()
    assert lib.quamba_ssd_prefill(None, None, *([None] * 10), 0, None) == -1
    assert q.quamba_ssd_prefill_workspace_size(_shape()) == 0
    assert q.quamba_ssd_prefill_workspace_size(_shape(nheads=5)) == 0


def test_workspace_of_the_sequence_split():
    """Short batches of the matrix-core shape are cut along the sequence and need the segment states as workspace:
    (segments - 1) * batch * heads * (headdim * d_state + 1) floats; the flag, the generic kernel, long batches and short
    sequences need none.  (Without a GPU the library plans for 256 compute units.)"""
    mm = dict(headdim=64, d_state=128, chunk=256, n_head_clusters=1, n_chan_clusters=1)
    unit = 64 * 128 + 1
    # 24 heads, 2048 tokens = 16 chunks: 8 segments of 2 chunks
    s = _shape(batch=1, seqlen=2048, nheads=24, ngroups=1, **mm)
    assert q.quamba_ssd_prefill_workspace_size(s) == 4 * 7 * 24 * unit
    # 128 heads, 4096 tokens: whole heads, 4 segments
    s8 = _shape(batch=1, seqlen=4096, nheads=128, ngroups=8, **mm)
    assert q.quamba_ssd_prefill_workspace_size(s8) == 4 * 3 * 128 * unit
    # a ragged length: 19 chunks in 8 segments of 3 chunks -> 7 segments
    assert q.quamba_ssd_prefill_workspace_size(_shape(batch=1, seqlen=2333, nheads=24, ngroups=1, **mm)) == 4 * 6 * 24 * unit
    for kw in (dict(flags=q.FLAG_NO_SEQ_SPLIT), dict(flags=q.FLAG_GENERIC_KERNEL), dict(batch=4), dict(seqlen=1000)):
        d = dict(batch=1, seqlen=4096, nheads=128, ngroups=8, **mm)
        d.update(kw)
        assert q.quamba_ssd_prefill_workspace_size(_shape(**d)) == 0, kw
    assert q.quamba_ssd_prefill_workspace_size(_shape(batch=1, seqlen=512, nheads=24, ngroups=1, **mm)) == 0


def test_noalloc_prefill_validates_like_the_prefill():
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    from paper_2503_22879_amd.binding import _ScalesStruct
    sc = _ScalesStruct(p, p, p, p, p)
    ok = [p] * 9                               # x B C dt A D init y final
    assert lib.quamba_ssd_prefill_noalloc(None, C.byref(sc), *ok, None) == -1
    for i in (0, 1, 2, 3, 4, 7):               # x B C dt A y are required
        args = list(ok)
        args[i] = None
        assert lib.quamba_ssd_prefill_noalloc(C.byref(_shape()), C.byref(sc), *args, None) == -1
    assert lib.quamba_ssd_prefill_noalloc(C.byref(_shape(seqlen=0)), C.byref(sc), *ok, None) == -2
    assert lib.quamba_ssd_prefill_noalloc(C.byref(_shape(flags=0x80)), C.byref(sc), *ok, None) == -5


def test_decode_rejects_bad_arguments_without_a_device():
    assert _call_decode(_shape(nheads=5)) == -2
    assert _call_decode(_shape(batch=0)) == -2
    for i in (0, 1, 2, 3, 4, 6, 7):        # everything but D is required
        assert _call_decode(_shape(), null_arg=i) == -1
    assert _call_decode(_shape(seqlen=0, chunk=0), null_arg=0) == -1   # seqlen/chunk are ignored by decode


def test_q8_entry_points_reject_bad_arguments_without_a_device():
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    from paper_2503_22879_amd.binding import _ScalesStruct
    sc = _ScalesStruct(p, p, p, p, p)
    ok = [p] * 10                          # state_scales x B C dt A D state_q y stream(NULL below)
    for i in (0, 1, 2, 3, 4, 5, 7, 8):     # everything but D is required
        args = list(ok[:9]); args[i] = None
        assert lib.quamba_ssd_decode_step_q8(C.byref(_shape()), C.byref(sc), *args, None) == -1
    assert lib.quamba_ssd_decode_step_q8(C.byref(_shape(nheads=5)), C.byref(sc), *ok[:9], None) == -2
    assert lib.quamba_ssd_decode_step_q8(None, C.byref(sc), *ok[:9], None) == -1
    # tables that cannot fit the LDS of a compute unit
    assert lib.quamba_ssd_decode_step_q8(C.byref(_shape(d_state=8192, n_chan_clusters=4)), C.byref(sc), *ok[:9],
                                         None) == -2
    for i in range(3):                     # state_scales, state, state_q
        args = [p, p, p]; args[i] = None
        assert lib.quamba_ssd_quantize_state(C.byref(_shape()), C.byref(sc), *args, None) == -1
    assert lib.quamba_ssd_quantize_state(C.byref(_shape(batch=0)), C.byref(sc), p, p, p, None) == -2


def test_gated_entry_points_reject_bad_arguments_without_a_device():
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    from paper_2503_22879_amd.binding import _ScalesStruct, _GateStruct
    sc = _ScalesStruct(p, p, p, p, p)
    pre = [p] * 10                                   # x B C dt A D init y final workspace
    # dt may be NULL only when the gate carries the step-size codes
    args = list(pre); args[3] = None
    assert lib.quamba_ssd_prefill_gated(C.byref(_shape()), C.byref(sc), None, *args, 0, None) == -1
    g = _GateStruct(None, 0.0, p, 0.0, None)          # codes with a zero scale
    assert lib.quamba_ssd_prefill_gated(C.byref(_shape()), C.byref(sc), C.byref(g), *args, 0, None) == -5
    g = _GateStruct(p, float("nan"), None, 0.0, None)  # gate with a non-finite scale
    assert lib.quamba_ssd_prefill_gated(C.byref(_shape()), C.byref(sc), C.byref(g), *pre, 0, None) == -5
    dec = [p] * 8                                     # x B C dt A D state y
    g = _GateStruct(p, -1.0, None, 0.0, None)
    assert lib.quamba_ssd_decode_step_gated(C.byref(_shape()), C.byref(sc), C.byref(g), *dec, None) == -5
    args = list(dec); args[3] = None
    assert lib.quamba_ssd_decode_step_gated(C.byref(_shape()), C.byref(sc), None, *args, None) == -1
    g = _GateStruct(None, 0.0, p, 0.1, None)          # the 8-bit-state step refuses step-size codes
    assert lib.quamba_ssd_decode_step_q8_gated(C.byref(_shape()), C.byref(sc), C.byref(g), p, *dec, None) == -5


def test_binding_fails_loudly_without_library(monkeypatch):
    import paper_2503_22879_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", "/nonexistent/libquamba_ssd.so")
    with pytest.raises(FileNotFoundError):
        b.load_library()


def test_hadamard_rejects_bad_arguments_without_a_device():
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    f = lib.quamba_hadamard_quantize
    assert f(None, 1, 64, 1.0, p, None) == -1 and f(p, 1, 64, 1.0, None, None) == -1
    for n in (0, 1, 36, 3, 24, 40, 12 * 2048, 28 * 64, 32768, -64):     # 12 * 2^k and 20 * 2^k need k >= 2 and n <= 16384
        assert f(p, 1, n, 1.0, p, None) == -2
    assert f(p, -1, 64, 1.0, p, None) == -2 and f(p, 2 ** 31, 64, 1.0, p, None) == -2
    for s in (0.0, -2.0, float("inf"), float("nan")):
        assert f(p, 1, 64, s, p, None) == -5
    assert f(p, 0, 64, 1.0, p, None) == 0          # no rows: nothing is launched


def test_conv1d_rejects_bad_arguments_without_a_device():
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    from paper_2503_22879_amd.binding import _ScalesStruct
    sc = _ScalesStruct(p, p, p, p, p)

    def call(shape, scale=1e-3, null=None, st_in=None, st_out=None, scales=sc):
        args = [p, p, p]                      # in weight bias
        outs = [p, p, p]                      # x_out B_out C_out
        if null is not None:
            (args if null < 3 else outs)[null % 3] = None
        return lib.quamba_conv1d_q8(C.byref(shape), C.byref(scales), args[0], args[1], args[2], scale, st_in, outs[0],
                                    outs[1], outs[2], st_out, None)
    for i in (0, 1, 3, 4, 5):                 # bias (2) may be NULL
        assert call(_shape(), null=i) == -1
    assert call(_shape(), scales=_ScalesStruct(p, None, p, p, p)) == -1
    assert call(_shape(seqlen=0)) == -2 and call(_shape(nheads=5)) == -2
    for s in (0.0, -1.0, float("inf"), float("nan")):
        assert call(_shape(), scale=s) == -5
    assert call(_shape(seqlen=17), st_in=p, st_out=p) == -5      # one buffer for both states only on short pieces


def test_mamba1_rejects_bad_arguments_without_a_device():
    lib = q.load_library()
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    from paper_2503_22879_amd.binding import _ScalesStruct
    sc = _ScalesStruct(p, p, p, p, p)
    m1 = dict(nheads=1, ngroups=1, headdim=64, d_state=16, seqlen=32)

    def scan(shape, null=None):
        args = [p] * 9                        # x B C dt A D init y final
        if null is not None:
            args[null] = None
        return lib.quamba_mamba1_scan(C.byref(shape), C.byref(sc), *args, None)

    def step(shape, null=None):
        args = [p] * 8                        # x B C dt A D state y
        if null is not None:
            args[null] = None
        return lib.quamba_mamba1_decode_step(C.byref(shape), C.byref(sc), *args, None)
    for i in (0, 1, 2, 3, 4, 7):
        assert scan(_shape(**m1), null=i) == -1
    for i in (0, 1, 2, 3, 4, 6, 7):
        assert step(_shape(**m1), null=i) == -1
    for bad in (dict(nheads=2, ngroups=1), dict(n_head_clusters=2), dict(seqlen=0), dict(d_state=65)):
        assert scan(_shape(**dict(m1, **bad))) == -2
    assert step(_shape(**dict(m1, nheads=4, ngroups=2))) == -2
    assert scan(_shape(**dict(m1, flags=2))) == -5 and step(_shape(**dict(m1, flags=1))) == -5
    # the variants with the 8-bit side inputs: dt may be absent only when the gate carries its codes; bad scales
    from paper_2503_22879_amd.binding import _GateStruct

    def gated(fn, n, g, dt):
        args = [p] * n
        args[3] = dt
        return fn(C.byref(_shape(**m1)), C.byref(sc), None if g is None else C.byref(g), *args, None)
    for fn, n in ((lib.quamba_mamba1_scan_gated, 9), (lib.quamba_mamba1_decode_step_gated, 8)):
        assert gated(fn, n, None, None) == -1
        assert gated(fn, n, _GateStruct(p, 1.0, None, 0.0, None), None) == -1
        assert gated(fn, n, _GateStruct(None, 0.0, p, 0.0, None), None) == -5
        assert gated(fn, n, _GateStruct(p, float("inf"), None, 0.0, None), p) == -5
        assert gated(fn, n, _GateStruct(p, 0.0, p, 0.1, None), None) == -5


def test_probe_entry_points_validate_before_they_launch():
    """The measurement helpers of the benchmark (include/quamba_probe.h) reject bad arguments on a GPU-less host."""
    lib = q.load_library()
    ops = C.c_double(0.0)
    dummy = C.create_string_buffer(64)
    p = C.addressof(dummy)
    assert lib.quamba_probe_mfma(0, 10, 2, 0, None, C.c_void_p(p), None) == -1
    assert lib.quamba_probe_mfma(2, 10, 2, 0, C.byref(ops), C.c_void_p(p), None) == -5
    assert lib.quamba_probe_mfma(0, 0, 2, 0, C.byref(ops), C.c_void_p(p), None) == -5
    assert lib.quamba_probe_mfma(0, 10, 9, 1, C.byref(ops), C.c_void_p(p), None) == -5
    assert lib.quamba_probe_stream_rmw(None, C.c_size_t(64), None) == -1
    assert lib.quamba_probe_stream_rmw(C.c_void_p(p), C.c_size_t(24), None) == -5
    assert lib.quamba_probe_stream_read(None, C.c_size_t(64), C.c_void_p(p), None) == -1
    assert lib.quamba_probe_stream_read(C.c_void_p(p), C.c_size_t(64), None, None) == -1
    assert lib.quamba_probe_stream_read(C.c_void_p(p), C.c_size_t(0), C.c_void_p(p), None) == -5
    assert lib.quamba_probe_clock(None, 100, None) == -1
    assert lib.quamba_probe_clock(C.c_void_p(p), 0, None) == -5
    assert lib.quamba_probe_clock_xcd(None, 8, 100, None) == -1
    assert lib.quamba_probe_clock_xcd(C.c_void_p(p), 0, 100, None) == -5
    assert lib.quamba_probe_clock_xcd(C.c_void_p(p), 65, 100, None) == -5
    assert lib.quamba_probe_clock_xcd(C.c_void_p(p), 8, 0, None) == -5
