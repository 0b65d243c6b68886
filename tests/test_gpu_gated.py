"""GPU parity of the gated entry points (output gate y * SiLU(z) on int8 z, step size from int8 codes of its
pre-activation) against the oracle: the fp64 scan on the oracle's own step size, followed by the oracle's gate."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import (make_problem, make_decode_inputs, make_gate_inputs, make_state_cache, to_shape, host_scales)

pytestmark = pytest.mark.gpu

Y_TOL = 2e-3      # max|y_gpu - y_ref| <= Y_TOL * max|y_ref|
H_TOL = 1e-4      # final fp32 state
GENERIC = 0x1
NO_SPLIT = 0x4


def _gate(q, g, use_z, use_dt):
    import torch
    return q.Gate(z=torch.from_numpy(g["z"]).cuda() if use_z else None, z_scale=g["z_scale"] if use_z else 0.0,
                  dt_q=torch.from_numpy(g["dt_q"]).cuda() if use_dt else None,
                  dt_scale=g["dt_scale"] if use_dt else 0.0,
                  dt_bias=torch.from_numpy(g["dt_bias"]).cuda() if use_dt else None)


@pytest.mark.parametrize("flags", [0, NO_SPLIT, GENERIC])
@pytest.mark.parametrize("use_z,use_dt", [(True, False), (False, True), (True, True)])
def test_prefill_gated(gpu_lib, flags, use_z, use_dt):
    """130M-shaped layer, ragged length (several chunks + a tail), with an initial state and the final state."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_130m"].with_(batch=2, seqlen=333)
    sc, prob, r = make_problem(s, 21)
    g = make_gate_inputs(s, r, 21)
    dt_ref = oracle.dt_from_codes(g["dt_q"], g["dt_scale"], g["dt_bias"]).astype(np.float32) if use_dt else prob["dt"]
    init = (0.05 * np.random.default_rng(3).standard_normal((2, s.nheads, s.headdim, s.d_state))).astype(np.float32)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], dt_ref, prob["A"], prob["D"],
                                       init_state=init.astype(np.float64))
    if use_z:
        yref = oracle.silu_gate(yref, g["z"], g["z_scale"])
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    y = torch.full((2, s.seqlen, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
    fin = torch.full((2, s.nheads, s.headdim, s.d_state), float("nan"), device="cuda")
    q.quamba_ssd_prefill(to_shape(q, s, flags=flags), q.DeviceScales(host_scales(q, sc)), t["x"], t["B"], t["C"],
                         None if use_dt else t["dt"], t["A"], t["D"], torch.from_numpy(init).cuda(), y, fin,
                         gate=_gate(q, g, use_z, use_dt))
    yg = y.cpu().numpy().astype(np.float64)
    hg = fin.cpu().numpy().astype(np.float64)
    assert np.isfinite(yg).all() and np.isfinite(hg).all()
    ey = np.abs(yg - yref).max() / np.abs(yref).max()
    eh = np.abs(hg - href).max() / np.abs(href).max()
    print(f"gated prefill flags={flags} z={use_z} dt_q={use_dt}: y err {ey:.3e}, state err {eh:.3e}")
    assert ey <= Y_TOL and eh <= H_TOL


@pytest.mark.parametrize("flags", [0, NO_SPLIT])
def test_prefill_gated_with_the_sequence_split(gpu_lib, flags):
    """130M-shaped layer at full length with both side inputs and a workspace: the launch is cut along the sequence
    (the state pass reads the step-size codes, the output pass applies the gate), with initial and final state."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_130m"]
    shape = to_shape(q, s, flags=flags)
    need = q.quamba_ssd_prefill_workspace_size(shape)
    assert need > 0
    sc, prob, r = make_problem(s, 23)
    g = make_gate_inputs(s, r, 23)
    dt_ref = oracle.dt_from_codes(g["dt_q"], g["dt_scale"], g["dt_bias"]).astype(np.float32)
    init = (0.05 * np.random.default_rng(4).standard_normal((1, s.nheads, s.headdim, s.d_state))).astype(np.float32)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], dt_ref, prob["A"], prob["D"],
                                       init_state=init.astype(np.float64))
    yref = oracle.silu_gate(yref, g["z"], g["z_scale"])
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    y = torch.full((1, s.seqlen, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
    fin = torch.full((1, s.nheads, s.headdim, s.d_state), float("nan"), device="cuda")
    ws = torch.empty(need, dtype=torch.uint8, device="cuda")
    q.quamba_ssd_prefill(shape, q.DeviceScales(host_scales(q, sc)), t["x"], t["B"], t["C"], None, t["A"], t["D"],
                         torch.from_numpy(init).cuda(), y, fin, ws, gate=_gate(q, g, True, True))
    yg = y.cpu().numpy().astype(np.float64)
    hg = fin.cpu().numpy().astype(np.float64)
    assert np.isfinite(yg).all() and np.isfinite(hg).all()
    ey = np.abs(yg - yref).max() / np.abs(yref).max()
    eh = np.abs(hg - href).max() / np.abs(href).max()
    print(f"gated prefill with the sequence split, flags={flags}: y err {ey:.3e}, state err {eh:.3e}")
    assert ey <= Y_TOL and eh <= H_TOL


def test_prefill_gated_8b_shape_sampled(gpu_lib):
    """The bench shape (batch 4 x 4096, one workgroup per head) with both side inputs, checked on sampled heads."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_b4"].with_(batch=2, seqlen=1024)
    sc, prob, r = make_problem(s, 22, calib_tokens=512)
    g = make_gate_inputs(s, r, 22)
    dt_ref = oracle.dt_from_codes(g["dt_q"], g["dt_scale"], g["dt_bias"]).astype(np.float32)
    pairs = [(0, 0), (0, 17), (1, 64), (1, 127)]
    yref, _, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], dt_ref, prob["A"], prob["D"], pairs=pairs,
                                    want_state=False)
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    y = torch.empty((2, s.seqlen, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    q.quamba_ssd_prefill(to_shape(q, s, flags=NO_SPLIT), q.DeviceScales(host_scales(q, sc)), t["x"], t["B"], t["C"],
                         None, t["A"], t["D"], None, y, None, gate=_gate(q, g, True, True))
    yg = y.cpu().numpy().astype(np.float64)
    scale = 0.0
    errs = []
    for i, (b, h) in enumerate(pairs):
        ref = oracle.silu_gate(yref[i], g["z"][b, :, h, :], g["z_scale"])
        errs.append(np.abs(yg[b, :, h, :] - ref).max())
        scale = max(scale, np.abs(ref).max())
    assert max(errs) <= Y_TOL * scale, (errs, scale)


@pytest.mark.parametrize("P,N,H,G", [(64, 128, 8, 2), (20, 24, 4, 2), (48, 32, 6, 3)])
@pytest.mark.parametrize("use_z,use_dt", [(True, False), (True, True)])
def test_decode_gated(gpu_lib, P, N, H, G, use_z, use_dt):
    import torch
    q = gpu_lib
    s = W.LayerShape("t", 3, 1, H, P, N, G, 64, 2, 3)
    sc, prob, r = make_problem(s.with_(seqlen=4), 23, calib_tokens=256)
    dsc = q.DeviceScales(host_scales(q, sc))
    st64 = W.draw_state(s, 23).astype(np.float64)
    st = torch.from_numpy(st64.astype(np.float32)).cuda()
    y = torch.empty((3, H, P), dtype=torch.float16, device="cuda")
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    for k in range(3):
        inp = make_decode_inputs(s, sc, r, 23, k)
        g = make_gate_inputs(s, r, 23, decode=True, step=k)
        dt_ref = oracle.dt_from_codes(g["dt_q"], g["dt_scale"], g["dt_bias"]).astype(np.float32) if use_dt else inp["dt"]
        d = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        q.quamba_ssd_decode_step(to_shape(q, s), dsc, d["x"], d["B"], d["C"], None if use_dt else d["dt"], A, D, st, y,
                                 gate=_gate(q, g, use_z, use_dt))
        yref = oracle.ref_decode_step(sc, inp["x"], inp["B"], inp["C"], dt_ref, prob["A"], prob["D"], st64)
        yref = oracle.silu_gate(yref, g["z"], g["z_scale"])
        yg = y.cpu().numpy().astype(np.float64)
        assert np.abs(yg - yref).max() <= Y_TOL * np.abs(yref).max(), f"step {k}"
        assert np.abs(st.cpu().numpy() - st64).max() <= H_TOL * np.abs(st64).max(), f"step {k}"


@pytest.mark.parametrize("P,N,H,G", [(64, 128, 8, 2), (20, 24, 4, 2)])
def test_decode_q8_gated(gpu_lib, P, N, H, G):
    """The 8-bit-state step with the gate: codes still bit for bit, y gated; dt codes are refused there."""
    import torch
    q = gpu_lib
    s = W.LayerShape("t", 3, 1, H, P, N, G, 64, 2, 3)
    sc, prob, r = make_problem(s.with_(seqlen=4), 24, calib_tokens=256)
    ss, codes, _ = make_state_cache(s, sc, r, 24, batch=3)
    dsc = q.DeviceScales(host_scales(q, sc))
    ssd = torch.from_numpy(ss).cuda()
    qs = torch.from_numpy(codes.copy()).cuda()
    ref = codes.copy()
    y = torch.empty((3, H, P), dtype=torch.float16, device="cuda")
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    for k in range(2):
        inp = make_decode_inputs(s, sc, r, 24, k)
        g = make_gate_inputs(s, r, 24, decode=True, step=k)
        d = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        q.quamba_ssd_decode_step_q8(to_shape(q, s), dsc, ssd, d["x"], d["B"], d["C"], d["dt"], A, D, qs, y,
                                    gate=_gate(q, g, True, False))
        yref = oracle.ref_decode_step_q8(sc, ss, inp["x"], inp["B"], inp["C"], inp["dt"], prob["A"], prob["D"], ref)
        yref = oracle.silu_gate(yref, g["z"], g["z_scale"])
        assert np.array_equal(qs.cpu().numpy(), ref)
        assert np.abs(y.cpu().numpy().astype(np.float64) - yref).max() <= Y_TOL * np.abs(yref).max()
    with pytest.raises(q.QuambaError):
        q.quamba_ssd_decode_step_q8(to_shape(q, s), dsc, ssd, d["x"], d["B"], d["C"], d["dt"], A, D, qs, y,
                                    gate=_gate(q, g, True, True))
