"""GPU parity of the decode step on the 8-bit cached state (quamba_ssd_decode_step_q8, quamba_ssd_quantize_state)
against the oracle, through the C ABI: the int8 codes bit for bit, y within the fp16 output tolerance."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import make_problem, make_decode_inputs, make_state_cache, to_shape, host_scales

pytestmark = pytest.mark.gpu

Y_TOL = 2e-3      # max|y_gpu - y_ref| <= Y_TOL * max|y_ref|  (fp16 y, fp32 accumulation against fp64)


def _setup(q, s, seed, batch, with_D=True):
    import torch
    sb = s.with_(batch=batch)
    sc, prob, r = make_problem(sb.with_(seqlen=4), seed, calib_tokens=512, with_D=with_D)
    ss, codes, st = make_state_cache(sb, sc, r, seed, batch=batch)
    dev = dict(dsc=q.DeviceScales(host_scales(q, sc)), shape=to_shape(q, sb),
               ss=torch.from_numpy(ss).cuda(), A=torch.from_numpy(prob["A"]).cuda(),
               D=torch.from_numpy(prob["D"]).cuda() if with_D else None)
    return sb, sc, prob, r, ss, codes, st, dev


def _run_steps(q, s, steps, seed, batch, with_D=True):
    import torch
    sb, sc, prob, r, ss, codes, _, dev = _setup(q, s, seed, batch, with_D)
    qs = torch.from_numpy(codes.copy()).cuda()
    y = torch.full((batch, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
    ref = codes.copy()
    worst = 0.0
    changed = 0
    for k in range(steps):
        inp = make_decode_inputs(sb, sc, r, seed, k)
        t = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        before = ref.copy()
        q.quamba_ssd_decode_step_q8(dev["shape"], dev["dsc"], dev["ss"], t["x"], t["B"], t["C"], t["dt"], dev["A"],
                                    dev["D"], qs, y)
        yref = oracle.ref_decode_step_q8(sc, ss, inp["x"], inp["B"], inp["C"], inp["dt"], prob["A"],
                                         prob["D"] if with_D else None, ref)
        got = qs.cpu().numpy()
        bad = np.argwhere(got != ref)
        assert bad.size == 0, f"step {k}: {len(bad)} codes differ, first at {bad[0]}: {got[tuple(bad[0])]} vs {ref[tuple(bad[0])]}"
        yg = y.cpu().numpy().astype(np.float64)
        assert np.isfinite(yg).all()
        ey = np.abs(yg - yref).max() / np.abs(yref).max()
        worst = max(worst, ey)
        assert ey <= Y_TOL, f"step {k}: y error {ey:.3e}"
        changed += int((before != ref).sum())
    assert changed > 0                      # the steps did move the cache
    return worst


def test_q8_decode_8b_shape_small_batch(gpu_lib):
    s = W.CONFIGS["m2_8b_decode"]
    e = _run_steps(gpu_lib, s, steps=6, seed=4, batch=3)
    print(f"q8 decode 8B-shape b=3: y err {e:.2e}, codes bit-exact")


def test_q8_decode_without_D(gpu_lib):
    _run_steps(gpu_lib, W.CONFIGS["m2_8b_decode"], steps=2, seed=5, batch=2, with_D=False)


@pytest.mark.parametrize("P,N,H,G", [(64, 16, 8, 1), (64, 64, 4, 2), (32, 256, 4, 4), (48, 32, 6, 3),
                                     (20, 24, 4, 2), (7, 5, 3, 1), (128, 128, 2, 1), (40, 128, 4, 2)])
def test_q8_decode_other_shapes(gpu_lib, P, N, H, G):
    """Vector path for d_state in {16,32,64,128,256} (ragged headdim included) and the any-shape path."""
    s = W.LayerShape("t", 2, 1, H, P, N, G, 64, 2, 3)
    _run_steps(gpu_lib, s, steps=3, seed=6, batch=2)


def test_q8_decode_clamps_like_the_oracle(gpu_lib):
    """Scales calibrated far too small: most new codes saturate at +-127 on both sides."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_130m"]
    sb, sc, prob, r, ss, codes, _, dev = _setup(q, s, 8, 2)
    ss_small = (ss * np.float32(1e-3)).astype(np.float32)
    qs = torch.from_numpy(codes.copy()).cuda()
    y = torch.empty((2, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    inp = make_decode_inputs(sb, sc, r, 8, 0)
    t = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
    q.quamba_ssd_decode_step_q8(dev["shape"], dev["dsc"], torch.from_numpy(ss_small).cuda(), t["x"], t["B"], t["C"],
                                t["dt"], dev["A"], dev["D"], qs, y)
    ref = codes.copy()
    oracle.ref_decode_step_q8(sc, ss_small, inp["x"], inp["B"], inp["C"], inp["dt"], prob["A"], prob["D"], ref)
    assert np.array_equal(qs.cpu().numpy(), ref)
    assert (np.abs(ref.astype(int)) == 127).mean() > 0.3


def test_q8_decode_full_batch(gpu_lib):
    """configs[4] at full size (batch 256, 256 MiB of codes), 3 steps: the codes of every sequence bit for bit and
    every y at every step (the numpy oracle walks the batch in slices of 32 sequences)."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_decode"]
    sc, prob, r = make_problem(s.with_(batch=1, seqlen=4), 4, calib_tokens=512)
    ss, _, _ = make_state_cache(s.with_(batch=1), sc, r, 4, batch=1)
    dsc = q.DeviceScales(host_scales(q, sc))
    shape = to_shape(q, s)
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    gen = torch.Generator(device="cuda"); gen.manual_seed(4321)
    qs = torch.randint(-127, 128, (s.batch, s.nheads, s.headdim, s.d_state), device="cuda", generator=gen,
                       dtype=torch.int8)
    ref = qs.cpu().numpy()
    ssd = torch.from_numpy(ss).cuda()
    y = torch.empty((s.batch, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    for k in range(3):
        inp = make_decode_inputs(s, sc, r, 4, k)
        t = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        q.quamba_ssd_decode_step_q8(shape, dsc, ssd, t["x"], t["B"], t["C"], t["dt"], A, D, qs, y)
        got = qs.cpu().numpy()
        yg = y.cpu().numpy().astype(np.float64)
        for b0 in range(0, s.batch, 32):
            sl = slice(b0, b0 + 32)
            part = ref[sl]                       # a view: the oracle updates the reference codes in place
            yref = oracle.ref_decode_step_q8(sc, ss, inp["x"][sl], inp["B"][sl], inp["C"][sl], inp["dt"][sl],
                                             prob["A"], prob["D"], part)
            assert np.array_equal(got[sl], part), f"step {k}, sequences {b0}..{b0 + 31}"
            assert np.abs(yg[sl] - yref).max() <= Y_TOL * np.abs(yref).max(), f"step {k}, sequences {b0}..{b0 + 31}"
    assert torch.isfinite(y).all()


def _big_batch_steps(q, s, seed, steps, misalign=False):
    """Random codes as the cached state of a whole batch, `steps` steps, every code and every y against the oracle
    (in slices of 32 sequences).  misalign: x, B and C start one byte past a 4-byte boundary."""
    import torch
    sc, prob, r = make_problem(s.with_(batch=1, seqlen=4), seed, calib_tokens=512)
    ss, _, _ = make_state_cache(s.with_(batch=1), sc, r, seed, batch=1)
    dsc = q.DeviceScales(host_scales(q, sc))
    shape = to_shape(q, s)
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    gen = torch.Generator(device="cuda"); gen.manual_seed(1000 + seed)
    qs = torch.randint(-127, 128, (s.batch, s.nheads, s.headdim, s.d_state), device="cuda", generator=gen,
                       dtype=torch.int8)
    ref = qs.cpu().numpy()
    ssd = torch.from_numpy(ss).cuda()
    y = torch.empty((s.batch, s.nheads, s.headdim), dtype=torch.float16, device="cuda")

    def dev(v):
        t = torch.from_numpy(v).cuda()
        if not misalign or t.dtype != torch.int8:
            return t
        buf = torch.empty(t.numel() + 5, dtype=torch.int8, device="cuda")
        off = 1 + (-buf.data_ptr()) % 4          # data_ptr % 4 == 1
        view = buf[off:off + t.numel()].view(t.shape)
        view.copy_(t)
        assert view.data_ptr() % 4 == 1
        return view

    for k in range(steps):
        inp = make_decode_inputs(s, sc, r, seed, k)
        t = {n: dev(v) for n, v in inp.items()}
        q.quamba_ssd_decode_step_q8(shape, dsc, ssd, t["x"], t["B"], t["C"], t["dt"], A, D, qs, y)
        got = qs.cpu().numpy()
        yg = y.cpu().numpy().astype(np.float64)
        for b0 in range(0, s.batch, 32):
            sl = slice(b0, b0 + 32)
            part = ref[sl]                       # a view: the oracle updates the reference codes in place
            yref = oracle.ref_decode_step_q8(sc, ss, inp["x"][sl], inp["B"][sl], inp["C"][sl], inp["dt"][sl],
                                             prob["A"], prob["D"], part)
            assert np.array_equal(got[sl], part), f"step {k}, sequences {b0}..{b0 + 31}"
            assert np.abs(yg[sl] - yref).max() <= Y_TOL * np.abs(yref).max(), f"step {k}, sequences {b0}..{b0 + 31}"


@pytest.mark.parametrize("batch,H,P,N,G,misalign", [
    (250, 128, 32, 32, 4, False),    # 7 sequences per workgroup, a last slice of 5
    (512, 128, 128, 16, 8, False),   # 16 sequences per workgroup: more x codes per slice than one dword per thread
    (64, 128, 6, 16, 1, False),      # headdim not a multiple of 4: x byte by byte
    (130, 64, 64, 64, 2, False),     # 2 sequences per workgroup
    (96, 128, 64, 128, 8, True),     # x, B and C off the 4-byte grid: the any-shape kernel takes the step
])
def test_q8_decode_several_sequences_per_workgroup(gpu_lib, batch, H, P, N, G, misalign):
    """Batches large enough that a workgroup of the vector kernel owns slices of several sequences (the slice's side
    inputs are then requested one slice ahead), with ragged last slices and the x paths of the staging."""
    s = W.LayerShape("t", batch, 1, H, P, N, G, 64, 2, 3)
    _big_batch_steps(gpu_lib, s, seed=9, steps=2, misalign=misalign)


@pytest.mark.parametrize("P,N,H,G", [(64, 128, 8, 2), (20, 24, 4, 2), (7, 5, 3, 1), (33, 16, 4, 1)])
def test_quantize_state_bit_exact(gpu_lib, P, N, H, G):
    """fp32 state -> codes of the cache: the 4-wide path, the scalar path (d_state not a multiple of 4), clamping."""
    import torch
    q = gpu_lib
    s = W.LayerShape("t", 3, 1, H, P, N, G, 64, 2, 3)
    sb, sc, prob, r, ss, codes, st, dev = _setup(q, s, 9, 3)
    st = (st * np.float32(1.7)).astype(np.float32)                    # some values beyond the calibrated range
    out = torch.zeros((3, H, P, N), dtype=torch.int8, device="cuda")
    q.quamba_ssd_quantize_state(dev["shape"], dev["dsc"], dev["ss"], torch.from_numpy(st).cuda(), out)
    want = oracle.quantize_state(sc, ss, st, G)
    assert np.array_equal(out.cpu().numpy(), want)
    assert (np.abs(want.astype(int)) == 127).any()


def test_prefill_state_into_the_8bit_cache_and_on(gpu_lib):
    """The flow of a generation: prefill returns the fp32 state, it is quantized into the cache, decode steps run on
    the cache.  Every stage against its oracle, fed with the GPU's own previous stage (bit-exact stages compose)."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_130m"].with_(batch=2, seqlen=300)
    sc, prob, r = make_problem(s, 11)
    dsc = q.DeviceScales(host_scales(q, sc))
    shape = to_shape(q, s)
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    y = torch.empty((2, s.seqlen, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    fin = torch.empty((2, s.nheads, s.headdim, s.d_state), device="cuda")
    q.quamba_ssd_prefill(shape, dsc, t["x"], t["B"], t["C"], t["dt"], t["A"], t["D"], None, y, fin, None)
    fin_h = fin.cpu().numpy()
    ss = oracle.state_scales_from_absmax(sc, np.abs(fin_h).max(axis=0) * np.float32(1.2), s.ngroups)
    ssd = torch.from_numpy(ss).cuda()
    qs = torch.empty(fin.shape, dtype=torch.int8, device="cuda")
    q.quamba_ssd_quantize_state(shape, dsc, ssd, fin, qs)
    ref = oracle.quantize_state(sc, ss, fin_h, s.ngroups)
    assert np.array_equal(qs.cpu().numpy(), ref)
    yd = torch.empty((2, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    for k in range(3):
        inp = make_decode_inputs(s, sc, r, 11, k)
        d = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        q.quamba_ssd_decode_step_q8(shape, dsc, ssd, d["x"], d["B"], d["C"], d["dt"], t["A"], t["D"], qs, yd)
        yref = oracle.ref_decode_step_q8(sc, ss, inp["x"], inp["B"], inp["C"], inp["dt"], prob["A"], prob["D"], ref)
        assert np.array_equal(qs.cpu().numpy(), ref)
        assert np.abs(yd.cpu().numpy().astype(np.float64) - yref).max() <= Y_TOL * np.abs(yref).max()


def test_q8_decode_is_deterministic(gpu_lib):
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_decode"]
    sb, sc, prob, r, ss, codes, _, dev = _setup(q, s, 7, 4)
    inp = {n: torch.from_numpy(v).cuda() for n, v in make_decode_inputs(sb, sc, r, 7, 0).items()}
    outs = []
    for _ in range(2):
        qs = torch.from_numpy(codes.copy()).cuda()
        y = torch.empty((4, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
        q.quamba_ssd_decode_step_q8(dev["shape"], dev["dsc"], dev["ss"], inp["x"], inp["B"], inp["C"], inp["dt"],
                                    dev["A"], dev["D"], qs, y)
        outs.append((qs.cpu(), y.cpu()))
    assert torch.equal(outs[0][0], outs[1][0]) and torch.equal(outs[0][1], outs[1][1])


@pytest.mark.parametrize("batch,steps", [(3, 4), (32, 2)])
def test_q8_codes_against_the_fp64_step(gpu_lib, batch, steps):
    """The kernel's codes against Eq. 2 itself, with no fp32 operation order involved: the cached state is
    de-quantized in fp64, the pinned fp64 decode oracle takes one step, and every new code must be the Eq. 1 code of
    that exact state: within half a quantization step of it, saturated where it leaves +-127.  The only slack is the
    width of the kernel's own fp32 rounding around a tie (2e-3 of a step: the decision value h'/s is below 128 and
    carries a few fp32 roundings of 6e-8 each, plus the 3e-7 of the exponential)."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_decode"]
    sb, sc, prob, r, ss, codes, _, dev = _setup(q, s, 21, batch)
    cells = oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups)
    sv = ss.astype(np.float64)[cells]                                   # [H,P,N] scale of every state element
    qs = torch.from_numpy(codes.copy()).cuda()
    y = torch.full((batch, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
    cur = codes.copy()
    tie = 2e-3
    near_tie = 0
    for k in range(steps):
        inp = make_decode_inputs(sb, sc, r, 21, k)
        t = {n: torch.from_numpy(v).cuda() for n, v in inp.items()}
        q.quamba_ssd_decode_step_q8(dev["shape"], dev["dsc"], dev["ss"], t["x"], t["B"], t["C"], t["dt"], dev["A"],
                                    dev["D"], qs, y)
        h = np.ascontiguousarray(cur.astype(np.float64) * sv[None])     # inverse of Eq. 1, exact in fp64
        yref = oracle.ref_decode_step(sc, inp["x"], inp["B"], inp["C"], inp["dt"], prob["A"], prob["D"], h)
        rr = h / sv[None]                                                # exact decision value
        lo = np.clip(np.rint(rr - tie), -127, 127)
        hi = np.clip(np.rint(rr + tie), -127, 127)
        got = qs.cpu().numpy()
        bad = np.argwhere((got < lo) | (got > hi))
        assert bad.size == 0, (f"step {k}: {len(bad)} codes are not the Eq. 1 code of the fp64 state, first at "
                               f"{bad[0]}: code {got[tuple(bad[0])]}, exact value {rr[tuple(bad[0])]}")
        near_tie += int((lo != hi).sum())
        inside = np.abs(rr) < 126.5
        assert np.abs(got[inside] - rr[inside]).max() <= 0.5 + tie     # half a step inside the range
        assert (np.abs(rr) >= 127.5).sum() == 0 or np.all(np.abs(got[np.abs(rr) >= 127.5]) == 127)
        yg = y.cpu().numpy().astype(np.float64)
        assert np.isfinite(yg).all()
        assert np.abs(yg - yref).max() <= Y_TOL * np.abs(yref).max(), f"step {k}: y"
        cur = got.copy()
    print(f"q8 codes vs fp64 step, batch {batch}: all {cur.size * steps} codes are Eq. 1 codes of the exact state "
          f"({near_tie} within {tie} of a tie)")
