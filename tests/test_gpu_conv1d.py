"""GPU parity of the W8A8 causal convolution in front of the scan (quamba_conv1d_q8) against the oracle, through the
C ABI: the int8 codes of x, B and C and the carried conv state bit for bit."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import make_problem, make_conv_inputs, to_shape, host_scales

pytestmark = pytest.mark.gpu


def _split(codes, s):
    HP, GN = s.nheads * s.headdim, s.ngroups * s.d_state
    b, L, _ = codes.shape
    return (codes[:, :, :HP].reshape(b, L, s.nheads, s.headdim), codes[:, :, HP:HP + GN].reshape(b, L, s.ngroups, s.d_state),
            codes[:, :, HP + GN:].reshape(b, L, s.ngroups, s.d_state))


def _gpu(q, s, sc, inp, state_in=None, want_state=True, alias=False, offset=0):
    import torch
    b, L = inp["xBC"].shape[:2]
    shape = to_shape(q, s.with_(batch=b, seqlen=L))
    dsc = q.DeviceScales(host_scales(q, sc))
    Ct = inp["xBC"].shape[2]

    def dev(a):
        if offset == 0:
            return torch.from_numpy(np.ascontiguousarray(a)).cuda()
        buf = torch.zeros(a.size + offset, dtype=torch.from_numpy(a).dtype, device="cuda")   # unaligned view
        v = buf[offset:].view(a.shape)
        v.copy_(torch.from_numpy(np.ascontiguousarray(a)))
        return v
    xo = torch.full((b, L, s.nheads, s.headdim), 99, dtype=torch.int8, device="cuda")
    Bo = torch.full((b, L, s.ngroups, s.d_state), 99, dtype=torch.int8, device="cuda")
    Co = torch.full((b, L, s.ngroups, s.d_state), 99, dtype=torch.int8, device="cuda")
    st_in = None if state_in is None else torch.from_numpy(state_in.copy()).cuda()
    st_out = st_in if alias else (torch.full((b, 3, Ct), 99, dtype=torch.int8, device="cuda") if want_state else None)
    q.quamba_conv1d_q8(shape, dsc, dev(inp["xBC"]), torch.from_numpy(inp["weight"]).cuda(),
                       None if inp["bias"] is None else torch.from_numpy(inp["bias"]).cuda(), inp["in_w_scale"],
                       xo, Bo, Co, conv_state_in=st_in, conv_state_out=st_out)
    return xo.cpu().numpy(), Bo.cpu().numpy(), Co.cpu().numpy(), None if st_out is None else st_out.cpu().numpy()


def _check(q, s, sc, inp, state_in=None, **kw):
    os_ = oracle.output_scales(sc, s.nheads, s.headdim, s.ngroups, s.d_state)
    ref, ref_state = oracle.ref_conv1d_q8(inp["xBC"], inp["weight"], inp["in_w_scale"], inp["bias"], os_, state_in)
    rx, rB, rC = _split(ref, s)
    gx, gB, gC, gstate = _gpu(q, s, sc, inp, state_in, **kw)
    for name, g, r in (("x", gx, rx), ("B", gB, rB), ("C", gC, rC)):
        bad = np.argwhere(g != r)
        assert bad.size == 0, f"{name}: {len(bad)} codes differ, first at {bad[0]}: {g[tuple(bad[0])]} vs {r[tuple(bad[0])]}"
    if gstate is not None:
        assert np.array_equal(gstate, ref_state)
    return ref, ref_state


def test_codes_bit_exact_small_layer(gpu_lib):
    """Several channel blocks, several segments and a ragged last one; all three outputs and the state."""
    s = W.CONFIGS["m2_130m"].with_(batch=2, seqlen=77)
    sc, _, _ = make_problem(s.with_(seqlen=8), seed=1, calib_tokens=256)
    inp = make_conv_inputs(s, seed=1)
    ref, _ = _check(gpu_lib, s, sc, inp)
    assert len(np.unique(ref)) > 120 and (ref == 127).any()


def test_8b_shape_with_carried_state_in_pieces(gpu_lib):
    """The 8B layer's 10240 channels; a sequence run at once equals the same sequence run in pieces (decode-sized ones
    too) through the carried state, and both equal the oracle."""
    s = W.CONFIGS["m2_8b_b1"].with_(batch=2, seqlen=150)
    sc, _, _ = make_problem(s.with_(seqlen=8), seed=2, calib_tokens=256)
    inp = make_conv_inputs(s, seed=2)
    ref, ref_state = _check(gpu_lib, s, sc, inp)
    state = None
    for lo, hi in [(0, 1), (1, 3), (3, 64), (64, 149), (149, 150)]:
        piece = dict(inp, xBC=np.ascontiguousarray(inp["xBC"][:, lo:hi]))
        r, state = _check(gpu_lib, s, sc, piece, state)
        assert np.array_equal(r, ref[:, lo:hi])
    assert np.array_equal(state, ref_state)


def test_many_elements_against_the_exact_sequence(gpu_lib):
    """21 million outputs compared one by one.  The kernel takes most codes from the hardware's approximate exponential
    and reciprocal and falls back to the stated exact sequence wherever the two could round differently; a bound that
    was too optimistic would show here as single codes off by one."""
    s = W.CONFIGS["m2_8b_b1"].with_(batch=2, seqlen=1024)
    sc, _, _ = make_problem(s.with_(batch=1, seqlen=8), seed=12, calib_tokens=256)
    inp = make_conv_inputs(s, seed=12)
    ref, _ = _check(gpu_lib, s, sc, inp)
    assert len(np.unique(ref)) > 200


def test_decode_step_updates_state_in_place(gpu_lib):
    s = W.CONFIGS["m2_8b_decode"].with_(batch=5, seqlen=1)
    sc, _, _ = make_problem(s.with_(batch=1, seqlen=8), seed=3, calib_tokens=256)
    Ct = s.nheads * s.headdim + 2 * s.ngroups * s.d_state
    state = np.random.default_rng(3).integers(-128, 128, size=(5, 3, Ct), dtype=np.int8)
    for step in range(4):
        inp = make_conv_inputs(s, seed=3, stream=60 + step)
        _, state = _check(gpu_lib, s, sc, inp, state, alias=True)


def test_no_bias_no_state_output(gpu_lib):
    s = W.CONFIGS["m2_130m"].with_(batch=1, seqlen=40)
    sc, _, _ = make_problem(s.with_(seqlen=8), seed=4, calib_tokens=256)
    inp = dict(make_conv_inputs(s, seed=4), bias=None)
    _check(gpu_lib, s, sc, inp, want_state=False)


def test_any_shape_kernel_odd_sizes_and_unaligned_input(gpu_lib):
    """headdim and d_state that are no multiples of 16, and a 16-friendly shape whose input starts 1 byte off."""
    s = W.LayerShape("odd", 2, 45, 6, 20, 24, 2, 16, 2, 2)
    sc, _, _ = make_problem(s.with_(seqlen=8), seed=5, calib_tokens=128)
    st = np.random.default_rng(5).integers(-128, 128, size=(2, 3, 6 * 20 + 2 * 2 * 24), dtype=np.int8)
    _check(gpu_lib, s, sc, make_conv_inputs(s, seed=5), st)
    s2 = W.CONFIGS["m2_130m"].with_(batch=1, seqlen=33)
    sc2, _, _ = make_problem(s2.with_(seqlen=8), seed=6, calib_tokens=256)
    _check(gpu_lib, s2, sc2, make_conv_inputs(s2, seed=6), offset=1)


def test_extreme_codes_and_saturation(gpu_lib):
    """All-extreme inputs and filters: the largest window sums (4 * 128 * 128), both signs, deep exp underflow."""
    s = W.CONFIGS["m2_130m"].with_(batch=1, seqlen=35)
    sc, _, _ = make_problem(s.with_(seqlen=8), seed=7, calib_tokens=256)
    Ct = s.nheads * s.headdim + 2 * s.ngroups * s.d_state
    g = np.random.default_rng(7)
    inp = {"xBC": g.choice(np.array([-128, 127], np.int8), size=(1, 35, Ct)),
           "weight": g.choice(np.array([-128, 127], np.int8), size=(Ct, 4)),
           "bias": (g.standard_normal(Ct) * 5).astype(np.float32), "in_w_scale": 3e-3}
    ref, _ = _check(gpu_lib, s, sc, inp)
    assert (ref == 127).any() and (ref <= 0).any()


def test_rejects_aliased_state_on_long_sequences(gpu_lib):
    import torch
    s = W.CONFIGS["m2_130m"].with_(batch=1, seqlen=64)
    sc, _, _ = make_problem(s.with_(seqlen=8), seed=8, calib_tokens=128)
    inp = make_conv_inputs(s, seed=8)
    Ct = inp["xBC"].shape[2]
    with pytest.raises(gpu_lib.QuambaError):
        _gpu(gpu_lib, s, sc, inp, np.zeros((1, 3, Ct), np.int8), alias=True)


def test_bench_size_sampled_tokens(gpu_lib):
    """The bench launch (4 x 4096 tokens x 10240 channels): tokens sampled over the launch checked bit for bit; the
    oracle recomputes each sampled token from its own 4-token window."""
    import torch
    s = W.CONFIGS["m2_8b_b4"]
    sc, _, _ = make_problem(s.with_(batch=1, seqlen=8), seed=9, calib_tokens=256)
    inp = make_conv_inputs(s, seed=9)
    gx, gB, gC, gstate = _gpu(gpu_lib, s, sc, inp)
    got = np.concatenate([gx.reshape(s.batch, s.seqlen, -1), gB.reshape(s.batch, s.seqlen, -1),
                          gC.reshape(s.batch, s.seqlen, -1)], axis=2)
    os_ = oracle.output_scales(sc, s.nheads, s.headdim, s.ngroups, s.d_state)
    for t in [0, 1, 2, 3, 31, 32, 33, 1000, 2047, 2048, 4064, 4095]:
        lo = max(0, t - 3)
        win = np.ascontiguousarray(inp["xBC"][:, lo:t + 1])
        ref, _ = oracle.ref_conv1d_q8(win, inp["weight"], inp["in_w_scale"], inp["bias"], os_)
        assert np.array_equal(got[:, t], ref[:, -1]), f"token {t}"
    assert np.array_equal(gstate, inp["xBC"][:, -3:])
    assert not (got == 99).all(axis=2).any()
