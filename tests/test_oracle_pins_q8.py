"""Pins of the 8-bit cached-state oracle (oracle/state_q8.py) against closed forms, the pinned fp64 decode oracle,
Eq. 1's error bound and brute force (no GPU, no HIP code).

A dropped term, a swapped B/C or p/n index, a wrong cell lookup, y taken from the re-quantized instead of the updated
state, a truncating instead of a rounding quantizer or a missing clamp each fail one of these.
"""
import numpy as np

import oracle
from oracle import Scales

from test_oracle_pins import _rand_scales

RNG = np.random.default_rng(2289)


def _rand_step(b=3, H=4, P=5, N=6, G=2, rng=RNG, lo=-127, hi=128):
    xq = rng.integers(lo, hi, (b, H, P), dtype=np.int8)
    Bq = rng.integers(lo, hi, (b, G, N), dtype=np.int8)
    Cq = rng.integers(lo, hi, (b, G, N), dtype=np.int8)
    dt = np.logaddexp(0, rng.standard_normal((b, H)) - 2).astype(np.float32)
    A = (-np.exp(rng.uniform(0, np.log(16), H))).astype(np.float32)
    D = rng.standard_normal(H).astype(np.float32)
    return xq, Bq, Cq, dt, A, D


def test_exp_f32_against_libm_and_special_values():
    z = np.concatenate([np.linspace(-80, 0, 20001), -np.logspace(-8, 1.9, 2000)]).astype(np.float32)
    got = oracle.exp_f32(z).astype(np.float64)
    want = np.exp(z.astype(np.float64))
    # one rounding of z * log2(e) costs |z| * 2^-24 in the exponent, the polynomial and its Horner steps 2e-7
    assert np.all(np.abs(got - want) / want < 2e-7 + 1e-7 * np.abs(z))
    assert oracle.exp_f32(np.float32(0.0)) == np.float32(1.0)          # idle decay is exactly 1
    assert oracle.exp_f32(np.float32(-200.0)) == np.float32(0.0)
    assert oracle.exp_f32(np.float32(-86.0)) > 0                     # t = -124.07: still a normal number
    assert got.dtype == np.float64 and oracle.exp_f32(z).dtype == np.float32
    assert np.all(np.diff(oracle.exp_f32(np.sort(z))) >= 0)              # monotone on the grid


def test_integer_closed_form_with_unit_scales():
    """s = s_x = s_B = s_C = 1, A = 0, dt = 1: code' = code + B[n] x[p] and y[p] = sum_n C[n] code' + D x[p], exactly."""
    b, H, P, N, G = 2, 4, 5, 7, 2
    sc = Scales.ones(G, H // G, P)
    ss = np.ones((G, N), np.float32)
    xq = RNG.integers(-5, 6, (b, H, P), dtype=np.int8)
    Bq = RNG.integers(-5, 6, (b, G, N), dtype=np.int8)
    Cq = RNG.integers(-9, 10, (b, G, N), dtype=np.int8)
    q0 = RNG.integers(-20, 21, (b, H, P, N), dtype=np.int8)
    dt = np.ones((b, H), np.float32)
    A = np.zeros(H, np.float32)
    D = np.array([2, -1, 0, 3], np.float32)
    q = q0.copy()
    y = oracle.ref_decode_step_q8(sc, ss, xq, Bq, Cq, dt, A, D, q)
    g = np.arange(H) // (H // G)
    want_q = q0.astype(np.int64) + Bq.astype(np.int64)[:, g][:, :, None, :] * xq.astype(np.int64)[:, :, :, None]
    assert np.array_equal(q.astype(np.int64), want_q)
    want_y = (want_q * Cq.astype(np.int64)[:, g][:, :, None, :]).sum(-1) + D.astype(np.int64)[None, :, None] * xq
    assert np.array_equal(y, want_y.astype(np.float64))


def test_clamp_and_y_from_the_unclamped_state():
    """Eq. 1 clamps the code to +-127; y is formed from the updated state before it is quantized."""
    sc = Scales.ones(1, 1, 2)
    ss = np.ones((1, 3), np.float32)
    q = np.array([[[[120, -120, 0], [127, -127, 5]]]], np.int8)           # [1,1,2,3]
    xq = np.array([[[10, -10]]], np.int8)
    Bq = np.array([[[3, -3, 1]]], np.int8)
    Cq = np.array([[[1, 1, 1]]], np.int8)
    y = oracle.ref_decode_step_q8(sc, ss, xq, Bq, Cq, np.ones((1, 1), np.float32), np.zeros(1, np.float32), None, q)
    assert q.tolist() == [[[[127, -127, 10], [97, -97, -5]]]]
    assert y.tolist() == [[[150 - 150 + 10, 97 - 97 - 5]]]


def test_matches_the_fp64_decode_oracle_within_eq1_error():
    """Against the pinned fp64 step on the de-quantized state: the updated state agrees to fp32 rounding, hence the
    new code is within half a quantization step of it (Eq. 1), and y agrees."""
    b, H, P, N, G, m, n = 3, 6, 7, 10, 2, 2, 3
    sc = _rand_scales(H, P, G, m, n)
    ss = RNG.uniform(0.02, 0.4, (G * m * n, N)).astype(np.float32)
    xq, Bq, Cq, dt, A, D = _rand_step(b, H, P, N, G)
    q0 = RNG.integers(-127, 128, (b, H, P, N), dtype=np.int8)
    cells = oracle.cell_index_table(sc, H, P, G)
    s = ss.astype(np.float64)[cells]
    h64 = np.ascontiguousarray(s[None] * q0)
    y64 = oracle.ref_decode_step(sc, xq, Bq, Cq, dt, A, D, h64)            # h64 becomes the exact new state
    q = q0.copy()
    y = oracle.ref_decode_step_q8(sc, ss, xq, Bq, Cq, dt, A, D, q)
    assert np.max(np.abs(y - y64)) <= 2e-6 * np.max(np.abs(y64))
    inside = np.abs(h64) <= 126.5 * s[None]
    assert inside.mean() > 0.5                                             # the test exercises both branches
    err = np.abs(q.astype(np.float64) * s[None] - h64)
    assert np.all(err[inside] <= 0.5 * s[None].repeat(b, 0)[inside] * (1 + 1e-5) + 1e-6 * np.abs(h64[inside]))
    assert np.all(np.abs(q[~inside]) >= 126)
    assert np.all(np.sign(q[~inside]) == np.sign(h64[~inside]))


def test_idle_step_keeps_every_code():
    """x = 0 and A = 0 (decay exactly 1): de-quantize then re-quantize must give the same code for any scale."""
    b, H, P, N, G, m, n = 2, 4, 6, 9, 2, 2, 2
    sc = _rand_scales(H, P, G, m, n)
    ss = RNG.uniform(1e-3, 30.0, (G * m * n, N)).astype(np.float32)
    _, Bq, Cq, dt, _, D = _rand_step(b, H, P, N, G)
    q0 = RNG.integers(-127, 128, (b, H, P, N), dtype=np.int8)
    q = q0.copy()
    oracle.ref_decode_step_q8(sc, ss, np.zeros((b, H, P), np.int8), Bq, Cq, dt, np.zeros(H, np.float32), D, q)
    assert np.array_equal(q, q0)


def test_decay_without_input_shrinks_codes_down_to_the_rounding_fixed_point():
    """Without input the codes never grow.  A decay factor below 1/2 takes every code to 0; above 1/2 a code of
    magnitude 1 is a fixed point of round-to-nearest (0.607 rounds back to 1): the cached state stops decaying one
    quantization step above zero, which is a property of re-quantizing every step, not of this implementation."""
    b, H, P, N, G = 1, 2, 3, 4, 1
    sc = Scales.ones(G, H, P)
    ss = np.full((1, N), 0.37, np.float32)
    q = RNG.integers(-127, 128, (b, H, P, N), dtype=np.int8)
    z = np.zeros((b, H, P), np.int8)
    Bq = np.ones((b, G, N), np.int8)
    dt = np.full((b, H), 0.5, np.float32)
    A = np.array([-1.0, -3.0], np.float32)
    prev = np.abs(q.astype(int))
    for _ in range(40):
        oracle.ref_decode_step_q8(sc, ss, z, Bq, Bq, dt, A, None, q)
        cur = np.abs(q.astype(int))
        assert np.all(cur <= prev)
        prev = cur
    assert not q[:, 1].any()                      # exp(-1.5) = 0.22 < 1/2
    assert np.all(np.abs(q[:, 0]) <= 1)           # exp(-0.5) = 0.61 > 1/2


def test_cells_are_the_cells_of_x_and_scales_are_cell_maxima():
    H, P, N, G, m, n = 8, 9, 5, 2, 2, 3
    sc = _rand_scales(H, P, G, m, n)
    cells = oracle.cell_index_table(sc, H, P, G)
    assert np.array_equal(sc.x_scales[cells], oracle.x_scale_table(sc, H, P, G))
    absmax = RNG.uniform(0, 4, (H, P, N)).astype(np.float32)
    absmax[:, :, 2] = 0                                                    # a state that never fires
    got = oracle.state_scales_from_absmax(sc, absmax, G)
    assert got.shape == (G * m * n, N) and got.dtype == np.float32
    hpg = H // G
    for c in range(G * m * n):                                             # brute force over the members of a cell
        g, rest = divmod(c, m * n)
        i, j = divmod(rest, n)
        h_lo = 0 if i == 0 else sc.head_cluster_end[g * m + i - 1]
        h_hi = sc.head_cluster_end[g * m + i]
        p_lo = 0 if j == 0 else sc.chan_cluster_end[c - 1]
        p_hi = sc.chan_cluster_end[c]
        # a boundary table may repeat an end: the lookup then never returns the empty cell
        members = absmax[g * hpg + h_lo:g * hpg + h_hi, p_lo:p_hi]
        for k in range(N):
            mx = members[:, :, k].max() if members.size else 0.0
            want = np.float32(mx) / np.float32(127) if mx > 0 else np.float32(1.0)
            assert got[c, k] == want, (c, k)


def test_quantize_state_rounds_to_nearest_even_and_clamps():
    sc = Scales.ones(1, 1, 1)
    ss = np.array([[0.5, 0.5, 0.5, 0.5, 0.5, 0.5]], np.float32)
    h = np.array([[[[1.25, 1.75, -1.25, 0.24, 200.0, -64.0]]]], np.float32)  # 2.5, 3.5, -2.5, 0.48, 400, -128
    assert oracle.quantize_state(sc, ss, h, 1).tolist() == [[[[2, 4, -2, 0, 127, -127]]]]
    H, P, N, G, m, n = 4, 6, 8, 2, 2, 2
    sc = _rand_scales(H, P, G, m, n)
    ss = RNG.uniform(0.01, 1.0, (G * m * n, N)).astype(np.float32)
    cells = oracle.cell_index_table(sc, H, P, G)
    hs = (RNG.uniform(-120, 120, (2, H, P, N)) * ss[cells][None]).astype(np.float32)
    q = oracle.quantize_state(sc, ss, hs, G)
    assert np.all(np.abs(q * ss[cells][None].astype(np.float64) - hs) <= 0.5 * ss[cells][None] * (1 + 1e-5))
