"""GPU parity of quamba_ssd_decode_step against the fp64 oracle (through the C ABI)."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import make_problem, make_decode_inputs, to_shape, host_scales

pytestmark = pytest.mark.gpu

Y_TOL = 2e-3      # max|y_gpu - y_ref| <= Y_TOL * max|y_ref|
H_TOL = 1e-4      # max|h_gpu - h_ref| <= H_TOL * max|h_ref|


def _run_steps(q, s, steps, seed, batch, with_D=True, state_init=None, check_every=True):
    import torch
    sb = s.with_(batch=batch)
    sc, prob, r = make_problem(sb.with_(seqlen=4), seed, calib_tokens=512, with_D=with_D)
    dsc = q.DeviceScales(host_scales(q, sc))
    shape = to_shape(q, sb)
    A = torch.from_numpy(prob["A"]).cuda()
    D = torch.from_numpy(prob["D"]).cuda() if with_D else None
    st64 = (W.draw_state(sb, seed) if state_init is None else state_init).astype(np.float64)
    st = torch.from_numpy(st64.astype(np.float32)).cuda()
    y = torch.empty((batch, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    worst_y = worst_h = 0.0
    for k in range(steps):
        inp = make_decode_inputs(sb, sc, r, seed, k)
        t = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        q.quamba_ssd_decode_step(shape, dsc, t["x"], t["B"], t["C"], t["dt"], A, D, st, y)
        yref = oracle.ref_decode_step(sc, inp["x"], inp["B"], inp["C"], inp["dt"], prob["A"],
                                      prob["D"] if with_D else None, st64)
        if check_every or k == steps - 1:
            yg = y.cpu().numpy().astype(np.float64)
            hg = st.cpu().numpy().astype(np.float64)
            ey = np.abs(yg - yref).max() / np.abs(yref).max()
            eh = np.abs(hg - st64).max() / np.abs(st64).max()
            worst_y, worst_h = max(worst_y, ey), max(worst_h, eh)
            assert ey <= Y_TOL, f"step {k}: y error {ey:.3e}"
            assert eh <= H_TOL, f"step {k}: state error {eh:.3e}"
    return worst_y, worst_h


def test_decode_8b_shape_small_batch(gpu_lib):
    s = W.CONFIGS["m2_8b_decode"]
    ey, eh = _run_steps(gpu_lib, s, steps=8, seed=4, batch=3)
    print(f"decode 8B-shape b=3: y err {ey:.2e}, state err {eh:.2e}")


def test_decode_without_D_and_zero_state(gpu_lib):
    s = W.CONFIGS["m2_8b_decode"]
    z = np.zeros((2, s.nheads, s.headdim, s.d_state), np.float32)
    _run_steps(gpu_lib, s, steps=3, seed=5, batch=2, with_D=False, state_init=z)


@pytest.mark.parametrize("P,N,H,G", [(64, 16, 8, 1), (64, 64, 4, 2), (32, 256, 4, 4), (48, 32, 6, 3),
                                     (20, 24, 4, 2), (7, 5, 3, 1), (128, 128, 2, 1)])
def test_decode_other_shapes(gpu_lib, P, N, H, G):
    """Vector path for d_state in {16,32,64,128,256} (ragged headdim included) and the any-shape path."""
    s = W.LayerShape("t", 2, 1, H, P, N, G, 64, 2, 3)
    _run_steps(gpu_lib, s, steps=3, seed=6, batch=2)


def test_decode_full_batch(gpu_lib):
    """configs[4] at full size (batch 256, 1 GiB state), 32 steps: y of every sequence against the fp64 oracle at every
    step, the whole state at the end (the oracle's fp64 state is 2 GiB of host memory)."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_decode"]
    sc, prob, r = make_problem(s.with_(batch=1, seqlen=4), 4, calib_tokens=512)
    dsc = q.DeviceScales(host_scales(q, sc))
    shape = to_shape(q, s)
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    gen = torch.Generator(device="cuda"); gen.manual_seed(1234)
    st = torch.randn((s.batch, s.nheads, s.headdim, s.d_state), device="cuda", generator=gen) * 0.1
    st64 = st.cpu().numpy().astype(np.float64)
    y = torch.empty((s.batch, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    worst = 0.0
    for k in range(s.decode_steps):
        inp = make_decode_inputs(s, sc, r, 4, k)
        t = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        q.quamba_ssd_decode_step(shape, dsc, t["x"], t["B"], t["C"], t["dt"], A, D, st, y)
        yref = oracle.ref_decode_step(sc, inp["x"], inp["B"], inp["C"], inp["dt"], prob["A"], prob["D"], st64)
        yg = y.cpu().numpy().astype(np.float64)
        ey = np.abs(yg - yref).max() / np.abs(yref).max()
        worst = max(worst, ey)
        assert ey <= Y_TOL, f"step {k}: y error {ey:.3e}"
    hmax = np.abs(st64).max()
    eh = 0.0
    for b0 in range(0, s.batch, 32):   # in slices: the fp64 copy of the whole GPU state would be another 2 GiB
        eh = max(eh, np.abs(st[b0:b0 + 32].cpu().numpy().astype(np.float64) - st64[b0:b0 + 32]).max() / hmax)
    print(f"decode batch 256, 32 steps, all sequences: y err {worst:.2e}, state err {eh:.2e}")
    assert eh <= H_TOL
    assert torch.isfinite(st).all() and torch.isfinite(y).all()


def test_decode_is_deterministic(gpu_lib):
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_decode"].with_(batch=4)
    sc, prob, r = make_problem(s.with_(seqlen=4), 7, calib_tokens=256)
    dsc = q.DeviceScales(host_scales(q, sc))
    inp = {n: torch.from_numpy(v).cuda() for n, v in make_decode_inputs(s, sc, r, 7, 0).items()}
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    st0 = torch.from_numpy(W.draw_state(s, 7)).cuda()
    outs = []
    for _ in range(2):
        st = st0.clone(); y = torch.empty((4, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
        q.quamba_ssd_decode_step(to_shape(q, s), dsc, inp["x"], inp["B"], inp["C"], inp["dt"], A, D, st, y)
        outs.append((st.cpu(), y.cpu()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])
