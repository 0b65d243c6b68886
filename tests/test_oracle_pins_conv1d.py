"""Pins of oracle/conv1d.py (W8A8 causal convolution + SiLU + Eq. 1 in front of the scan) against library routines
(scipy's lfilter and sigmoid), closed forms, causality and the carried state.  No GPU."""
import numpy as np
from scipy.signal import lfilter
from scipy.special import expit

import oracle


def _draw(seed, b=2, L=37, C=24):
    g = np.random.default_rng(seed)
    x = g.integers(-128, 128, size=(b, L, C), dtype=np.int8)
    w = g.integers(-128, 128, size=(C, 4), dtype=np.int8)
    bias = g.normal(0, 0.5, C).astype(np.float32)
    s_cw = np.float32(2.5e-4)
    s_out = np.exp(g.normal(-3.5, 0.5, C)).astype(np.float32)
    return x, w, bias, s_cw, s_out


def test_convolution_against_lfilter_and_library_sigmoid():
    x, w, bias, s_cw, _ = _draw(0)
    got = oracle.conv1d_silu_f64(x, w, s_cw, bias)
    b, L, C = x.shape
    for c in range(C):
        # lfilter: y[t] = sum_j taps[j] x[t - j]; the current token meets the LAST stored tap, the oldest the first
        taps = w[c, ::-1].astype(np.float64)
        for i in range(b):
            v = lfilter(taps, [1.0], x[i, :, c].astype(np.float64)) * float(s_cw) + float(bias[c])
            assert np.allclose(got[i, :, c], v * expit(v), rtol=1e-12, atol=1e-300)
    # single-tap filters: the last tap is the identity, the first delays by three tokens
    ident = np.zeros((C, 4), np.int8); ident[:, 3] = 1
    delay = np.zeros((C, 4), np.int8); delay[:, 0] = 1
    vi = x.astype(np.float64)
    assert np.allclose(oracle.conv1d_silu_f64(x, ident, 1.0), vi * expit(vi))
    vd = np.concatenate([np.zeros((b, 3, C)), vi[:, :-3]], axis=1)
    assert np.allclose(oracle.conv1d_silu_f64(x, delay, 1.0), vd * expit(vd))


def test_codes_follow_the_real_valued_definition_within_half_a_step():
    x, w, bias, s_cw, s_out = _draw(1, L=300)
    codes, _ = oracle.ref_conv1d_q8(x, w, s_cw, bias, s_out)
    real = oracle.conv1d_silu_f64(x, w, s_cw, bias)
    r = real / s_out.astype(np.float64)
    inside = (r > -128.4) & (r < 127.4)
    err = np.abs(codes.astype(np.float64) - r)
    assert inside.mean() > 0.5 and err[inside].max() <= 0.5 + 1e-4             # Eq. 1 error bound (fp32 slack)
    assert np.all(codes[r >= 127.5] == 127) and (r >= 127.5).any()             # the clamp, reached by this draw
    assert len(np.unique(codes)) > 100
    # SiLU is bounded below by -0.2785: no code can be lower than that over the scale
    assert np.all(codes.astype(np.float64) >= np.floor(-0.2785 / s_out)[None, None, :] - 1)


def test_exact_cases_ties_and_underflow():
    C = 6
    w = np.zeros((C, 4), np.int8); w[:, 3] = 1
    one = np.ones(C, np.float32)
    # for v >= 17.4 the factor 1 + exp(-v) rounds to 1 in fp32 and SiLU(v) = v exactly: half-integers are ties
    x = np.array([[[41, 43, 45, 47, 49, 51]]], np.int8)
    codes, _ = oracle.ref_conv1d_q8(x, w, 0.5, None, one)
    assert codes.tolist() == [[[20, 22, 22, 24, 24, 26]]]                       # 20.5 21.5 22.5 23.5 24.5 25.5 to even
    # SiLU(0) = 0; very negative v: exp underflows, the output is (minus) zero, never NaN
    zero, _ = oracle.ref_conv1d_q8(np.zeros((1, 5, C), np.int8), w, 1.0, None, one)
    assert not zero.any()
    neg, _ = oracle.ref_conv1d_q8(np.full((1, 2, C), -128, np.int8), w, 3.0, None, one * np.float32(1e-3))
    assert not neg.any()
    # bias alone: code = Eq. 1 (SiLU(bias) / s)
    bias = np.array([-3.0, -1.2784645, -0.5, 0.5, 2.0, 9.0], np.float32)
    s = np.float32(0.01)
    got, _ = oracle.ref_conv1d_q8(np.zeros((1, 1, C), np.int8), w, 1.0, bias, one * s)
    want = np.clip(np.rint(bias.astype(np.float64) * expit(bias.astype(np.float64)) / 0.01), -128, 127)
    assert got[0, 0].tolist() == want.tolist() and got[0, 0, 1] == -28              # the minimum of SiLU, -0.2785
    # both clamps: +127 from a large positive value; -128 is out of reach of SiLU (>= -0.2785) unless s is tiny
    big, _ = oracle.ref_conv1d_q8(np.full((1, 1, C), 127, np.int8), w, 1.0, None, one * np.float32(0.5))
    assert np.all(big == 127)
    low, _ = oracle.ref_conv1d_q8(np.full((1, 1, C), -1, np.int8), w, 1.0, None, one * np.float32(1e-3))
    assert np.all(low == -128)                                                      # SiLU(-1) = -0.2689 -> -268.9


def test_causality_and_carried_state():
    x, w, bias, s_cw, s_out = _draw(2, b=3, L=50)
    full, st_full = oracle.ref_conv1d_q8(x, w, s_cw, bias, s_out)
    # the future does not leak into the past
    x2 = x.copy(); x2[:, 20:] = np.random.default_rng(9).integers(-128, 128, size=x2[:, 20:].shape, dtype=np.int8)
    other, _ = oracle.ref_conv1d_q8(x2, w, s_cw, bias, s_out)
    assert np.array_equal(other[:, :20], full[:, :20]) and not np.array_equal(other[:, 20:], full[:, 20:])
    # the state is the last three input tokens, and running in pieces with it equals running at once
    assert np.array_equal(st_full, x[:, -3:])
    st = None
    pieces = []
    for lo, hi in [(0, 1), (1, 3), (3, 4), (4, 31), (31, 50)]:                   # pieces shorter than the filter too
        c, st = oracle.ref_conv1d_q8(x[:, lo:hi], w, s_cw, bias, s_out, st)
        pieces.append(c)
    assert np.array_equal(np.concatenate(pieces, axis=1), full) and np.array_equal(st, st_full)
    # a piece shorter than the state keeps the tail of the old state in front
    _, s1 = oracle.ref_conv1d_q8(x[:, :1], w, s_cw, bias, s_out)
    assert np.array_equal(s1[:, 2], x[:, 0]) and not s1[:, :2].any()
    # channels are independent (depthwise): permuting channels permutes the output
    perm = np.random.default_rng(3).permutation(x.shape[2])
    pc, _ = oracle.ref_conv1d_q8(x[:, :, perm], w[perm], s_cw, bias[perm], s_out[perm])
    assert np.array_equal(pc, full[:, :, perm])


def test_output_scales_layout():
    sc = oracle.Scales(m=2, n=2, x_scales=np.arange(1, 9, dtype=np.float32) / 100,
                       head_cluster_end=np.array([1, 2, 1, 2], np.int32),
                       chan_cluster_end=np.array([2, 4, 1, 4, 3, 4, 2, 4], np.int32),
                       B_scales=np.array([0.5, 0.25], np.float32), C_scales=np.array([0.125, 2.0], np.float32))
    H, P, G, N = 4, 4, 2, 3
    s = oracle.output_scales(sc, H, P, G, N)
    assert s.shape == (H * P + 2 * G * N,) and s.dtype == np.float32
    assert np.array_equal(s[:H * P].reshape(H, P), oracle.x_scale_table(sc, H, P, G))
    assert s[H * P:].tolist() == [0.5] * 3 + [0.25] * 3 + [0.125] * 3 + [2.0] * 3
