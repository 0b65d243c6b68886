"""GPU parity of the 8-bit Mamba1 selective scan (quamba_mamba1_scan, quamba_mamba1_decode_step) against the fp64
oracle, through the C ABI: y within 2e-3 of the largest |y| (fp32 scan, fp16 output), states within 1e-4."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import make_mamba1_problem, make_mamba1_gate, host_scales

pytestmark = pytest.mark.gpu

Y_TOL = 2e-3
S_TOL = 1e-4


def _shape(q, b, D, N, L, nranges, flags=0):
    return q.Shape(batch=b, seqlen=L, nheads=1, headdim=D, d_state=N, ngroups=1, chunk=1, n_head_clusters=1,
                   n_chan_clusters=nranges, flags=flags)


def _run(q, sc, p, b, D, N, L, nranges=4, flags=0, init=None, with_D=True, want_state=True):
    import torch
    shape = _shape(q, b, D, N, L, nranges, flags)
    dsc = q.DeviceScales(host_scales(q, sc))
    t = {k: torch.from_numpy(np.ascontiguousarray(p[k])).cuda() for k in ("x", "B", "C", "dt", "A", "D")}
    y = torch.full((b, D, L), float("nan"), dtype=torch.float16, device="cuda")
    fin = torch.full((b, D, N), float("nan"), device="cuda") if want_state else None
    ini = None if init is None else torch.from_numpy(init.astype(np.float32)).cuda()
    q.quamba_mamba1_scan(shape, dsc, t["x"], t["B"], t["C"], t["dt"], t["A"], t["D"] if with_D else None, y,
                         init_state=ini, final_state=fin)
    return y.cpu().numpy().astype(np.float64), None if fin is None else fin.cpu().numpy().astype(np.float64)


def _check(q, b, D, N, L, seed, nranges=4, flags=0, with_init=False, with_D=True):
    sc, p = make_mamba1_problem(b, D, N, L, seed, nranges)
    init = np.random.default_rng(seed).normal(0, 0.05, size=(b, D, N)).astype(np.float32) if with_init else None
    yref, sref = oracle.ref_mamba1_scan(p["xs"], sc.B_scales[0], sc.C_scales[0], p["x"], p["B"], p["C"], p["dt"], p["A"],
                                        p["D"] if with_D else None, init)
    y, fin = _run(q, sc, p, b, D, N, L, nranges, flags, init, with_D)
    assert np.isfinite(y).all() and np.isfinite(fin).all()
    ey = np.abs(y - yref).max() / np.abs(yref).max()
    es = np.abs(fin - sref).max() / np.abs(sref).max()
    assert ey <= Y_TOL, f"y error {ey:.3e}"
    assert es <= S_TOL, f"state error {es:.3e}"
    return ey, es


def test_wave_scan_kernel_several_tiles_and_a_ragged_one(gpu_lib):
    """2608 tokens = two full tiles of 1024 and one of 560 (35 live lanes); channels not a multiple of the 8 a
    workgroup owns (the last workgroup has waves without a channel)."""
    ey, es = _check(gpu_lib, b=2, D=8198, N=16, L=2608, seed=1, with_init=True)
    print(f"mamba1 scan, 8198 channels x 2608 tokens: y {ey:.2e} state {es:.2e}")


def test_wave_scan_kernel_small_shapes(gpu_lib):
    ey, es = _check(gpu_lib, b=1, D=203, N=16, L=1040, seed=2)
    print(f"mamba1 scan, 203 channels x 1040 tokens: y {ey:.2e} state {es:.2e}")
    _check(gpu_lib, b=3, D=64, N=16, L=16, seed=3, with_init=True, with_D=False)       # one lane of tokens


def test_any_shape_kernel_and_cross_check(gpu_lib):
    _check(gpu_lib, b=2, D=70, N=16, L=45, seed=4, with_init=True)                      # seqlen no multiple of 16
    _check(gpu_lib, b=1, D=33, N=24, L=64, seed=5, nranges=3)                           # other d_state
    _check(gpu_lib, b=1, D=130, N=16, L=256, seed=6, flags=gpu_lib.FLAG_GENERIC_KERNEL)  # forced, fast-path shape


def test_pieces_through_the_state_equal_one_run(gpu_lib):
    import torch
    b, D, N, L = 2, 256, 16, 2048
    sc, p = make_mamba1_problem(b, D, N, L, seed=7)
    y_all, s_all = _run(gpu_lib, sc, p, b, D, N, L)
    st = None
    ys = []
    for lo, hi in [(0, 1024), (1024, 1040), (1040, 2048)]:
        piece = dict(p, **{k: np.ascontiguousarray(p[k][:, :, lo:hi]) for k in ("x", "B", "C", "dt")})
        y, st = _run(gpu_lib, sc, piece, b, D, N, hi - lo, init=st)
        ys.append(y)
    yp = np.concatenate(ys, axis=2)
    scale = np.abs(y_all).max()
    assert np.abs(yp - y_all).max() <= 2 * 4.9e-4 * scale              # two fp16 roundings of nearly equal fp32 values
    assert np.abs(st - s_all).max() <= 1e-5 * np.abs(s_all).max()


def test_limits(gpu_lib):
    """dt = 0: y = D x exactly to fp16 rounding and the state does not move; strong decay: y -> dt C.B x + D x."""
    b, D, N, L = 1, 128, 16, 1024
    sc, p = make_mamba1_problem(b, D, N, L, seed=8)
    p0 = dict(p, dt=np.zeros_like(p["dt"]))
    init = np.random.default_rng(8).normal(0, 1, size=(b, D, N)).astype(np.float32)
    y, fin = _run(gpu_lib, sc, p0, b, D, N, L, init=np.zeros_like(init))
    want = (p["D"].astype(np.float64)[None, :, None] * p["x"] * p["xs"].astype(np.float64)[None, :, None]).astype(np.float16)
    assert np.array_equal(y.astype(np.float16), want) and not fin.any()
    _, fin2 = _run(gpu_lib, sc, dict(p0, D=np.zeros_like(p["D"])), b, D, N, L, init=init)
    assert np.array_equal(fin2.astype(np.float32), init)


def test_2p8b_shape_sampled(gpu_lib):
    """The Mamba1-2.8B-shaped layer the bench times (5120 channels, 16 states, 4 x 4096 tokens): the oracle scans 24
    sampled channels of every sequence in full."""
    import torch
    b, D, N, L = 4, 5120, 16, 4096
    sc, p = make_mamba1_problem(b, D, N, L, seed=9)
    y, fin = _run(gpu_lib, sc, p, b, D, N, L)
    pick = np.unique(np.concatenate([np.arange(0, D, 223), [D - 1, D - 2, 1]]))
    yref, sref = oracle.ref_mamba1_scan(p["xs"][pick], sc.B_scales[0], sc.C_scales[0], p["x"][:, pick], p["B"], p["C"],
                                        p["dt"][:, pick], p["A"][pick], p["D"][pick])
    ey = np.abs(y[:, pick] - yref).max() / np.abs(yref).max()
    es = np.abs(fin[:, pick] - sref).max() / np.abs(sref).max()
    assert ey <= Y_TOL and es <= S_TOL, (ey, es)
    assert np.isfinite(y).all()
    print(f"mamba1 scan 2.8B shape: y {ey:.2e} state {es:.2e}")


def test_decode_steps(gpu_lib):
    import torch
    q = gpu_lib
    for (b, D, N) in [(5, 5120, 16), (7, 203, 16), (3, 77, 24)]:  # 203: a last workgroup with idle lanes
        sc, p = make_mamba1_problem(b, D, N, 6, seed=10)
        shape = _shape(q, b, D, N, 1, 4)
        dsc = q.DeviceScales(host_scales(q, sc))
        st_ref = np.random.default_rng(10).normal(0, 0.1, size=(b, D, N))
        st = torch.from_numpy(st_ref.astype(np.float32)).cuda()
        st_ref = st_ref.astype(np.float32).astype(np.float64)
        A, Dk = torch.from_numpy(p["A"]).cuda(), torch.from_numpy(p["D"]).cuda()
        y = torch.empty((b, D), dtype=torch.float16, device="cuda")
        for t in range(6):
            sl = {k: np.ascontiguousarray(p[k][:, :, t]) for k in ("x", "B", "C", "dt")}
            q.quamba_mamba1_decode_step(shape, dsc, *(torch.from_numpy(sl[k]).cuda() for k in ("x", "B", "C", "dt")),
                                        A, Dk, st, y)
            yref, st_ref = oracle.ref_mamba1_scan(p["xs"], sc.B_scales[0], sc.C_scales[0], sl["x"][:, :, None],
                                                  sl["B"][:, :, None], sl["C"][:, :, None], sl["dt"][:, :, None], p["A"],
                                                  p["D"], st_ref)
            ey = np.abs(y.cpu().numpy().astype(np.float64) - yref[:, :, 0]).max() / np.abs(yref).max()
            es = np.abs(st.cpu().numpy().astype(np.float64) - st_ref).max() / np.abs(st_ref).max()
            assert ey <= Y_TOL and es <= S_TOL, (t, ey, es)


def _gate(q, g, use_z, use_dt, sl=None):
    import torch
    pick = (lambda v: torch.from_numpy(np.ascontiguousarray(v if sl is None else v[:, :, sl])).cuda())
    return q.Gate(z=pick(g["z"]) if use_z else None, z_scale=g["z_scale"] if use_z else 0.0,
                  dt_q=pick(g["dt_q"]) if use_dt else None, dt_scale=g["dt_scale"] if use_dt else 0.0,
                  dt_bias=torch.from_numpy(g["dt_bias"]).cuda() if use_dt else None)


def _dt_of_codes(g):
    """The oracle's softplus takes the bias along the last axis: channels last, then back to time last."""
    return np.moveaxis(oracle.dt_from_codes(np.moveaxis(g["dt_q"], 1, -1), g["dt_scale"], g["dt_bias"]), -1, 1)


@pytest.mark.parametrize("use_z,use_dt", [(True, False), (False, True), (True, True)])
@pytest.mark.parametrize("b,D,N,L,flags", [(2, 203, 16, 2608, 0), (2, 70, 16, 45, 0), (1, 33, 24, 64, 0),
                                           (1, 130, 16, 256, 1)])
def test_scan_with_side_inputs(gpu_lib, b, D, N, L, flags, use_z, use_dt):
    """Step size from int8 codes of its pre-activation plus a per-channel bias, and / or the output gate on int8 z
    (Section 3.2), on the wave-scan kernel (several tiles and a ragged one) and the any-shape kernel: the oracle's
    scan on the oracle's own step size, followed by the oracle's gate."""
    import torch
    q = gpu_lib
    sc, p = make_mamba1_problem(b, D, N, L, seed=11)
    g = make_mamba1_gate(b, D, L, seed=11)
    dt_ref = _dt_of_codes(g).astype(np.float32) if use_dt else p["dt"]
    init = np.random.default_rng(11).normal(0, 0.05, size=(b, D, N)).astype(np.float32)
    yref, sref = oracle.ref_mamba1_scan(p["xs"], sc.B_scales[0], sc.C_scales[0], p["x"], p["B"], p["C"], dt_ref, p["A"],
                                        p["D"], init)
    if use_z:
        yref = oracle.silu_gate(yref, g["z"], g["z_scale"])
    t = {k: torch.from_numpy(np.ascontiguousarray(p[k])).cuda() for k in ("x", "B", "C", "dt", "A", "D")}
    y = torch.full((b, D, L), float("nan"), dtype=torch.float16, device="cuda")
    fin = torch.full((b, D, N), float("nan"), device="cuda")
    q.quamba_mamba1_scan(_shape(q, b, D, N, L, 4, flags), q.DeviceScales(host_scales(q, sc)), t["x"], t["B"], t["C"],
                         None if use_dt else t["dt"], t["A"], t["D"], y, init_state=torch.from_numpy(init).cuda(),
                         final_state=fin, gate=_gate(q, g, use_z, use_dt))
    yg, sg = y.cpu().numpy().astype(np.float64), fin.cpu().numpy().astype(np.float64)
    assert np.isfinite(yg).all() and np.isfinite(sg).all()
    ey = np.abs(yg - yref).max() / np.abs(yref).max()
    es = np.abs(sg - sref).max() / np.abs(sref).max()
    print(f"mamba1 scan D={D} L={L} flags={flags} z={use_z} dt_q={use_dt}: y {ey:.2e} state {es:.2e}")
    assert ey <= Y_TOL and es <= S_TOL


def test_decode_steps_with_side_inputs(gpu_lib):
    import torch
    q = gpu_lib
    for (b, D, N) in [(5, 5120, 16), (7, 203, 16), (3, 77, 24)]:  # 203: a last workgroup with idle lanes
        sc, p = make_mamba1_problem(b, D, N, 4, seed=12)
        g = make_mamba1_gate(b, D, 4, seed=12)
        dt_all = _dt_of_codes(g).astype(np.float32)
        shape = _shape(q, b, D, N, 1, 4)
        dsc = q.DeviceScales(host_scales(q, sc))
        st_ref = np.random.default_rng(12).normal(0, 0.1, size=(b, D, N)).astype(np.float32)
        st = torch.from_numpy(st_ref).cuda()
        st_ref = st_ref.astype(np.float64)
        A, Dk = torch.from_numpy(p["A"]).cuda(), torch.from_numpy(p["D"]).cuda()
        y = torch.empty((b, D), dtype=torch.float16, device="cuda")
        for t in range(4):
            sl = {k: np.ascontiguousarray(p[k][:, :, t]) for k in ("x", "B", "C")}
            q.quamba_mamba1_decode_step(shape, dsc, *(torch.from_numpy(sl[k]).cuda() for k in ("x", "B", "C")), None,
                                        A, Dk, st, y, gate=_gate(q, g, True, True, sl=t))
            yref, st_ref = oracle.ref_mamba1_scan(p["xs"], sc.B_scales[0], sc.C_scales[0], sl["x"][:, :, None],
                                                  sl["B"][:, :, None], sl["C"][:, :, None], dt_all[:, :, t:t + 1],
                                                  p["A"], p["D"], st_ref)
            yref = oracle.silu_gate(yref[:, :, 0], g["z"][:, :, t], g["z_scale"])
            ey = np.abs(y.cpu().numpy().astype(np.float64) - yref).max() / np.abs(yref).max()
            es = np.abs(st.cpu().numpy().astype(np.float64) - st_ref).max() / np.abs(st_ref).max()
            assert ey <= Y_TOL and es <= S_TOL, (t, ey, es)
