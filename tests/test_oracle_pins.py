"""Pins of the CPU oracle against what the paper and the mathematics fix (no GPU, no HIP code).

Each test is chosen so that a plausible mistake in oracle/ssd_ref.c — a dropped term, pre- vs
post-update state in y, a wrong scale lookup, a transposed B/C, dt missing from B-dot — fails it.
"""
import os

import numpy as np
import pytest

import oracle
from oracle import Scales

RNG = np.random.default_rng(12345)


def _rand_problem(b=2, L=24, H=4, P=5, N=6, G=2, rng=RNG, with_D=True):
    xq = rng.integers(-127, 128, (b, L, H, P), dtype=np.int8)
    Bq = rng.integers(-127, 128, (b, L, G, N), dtype=np.int8)
    Cq = rng.integers(-127, 128, (b, L, G, N), dtype=np.int8)
    dt = np.logaddexp(0, rng.standard_normal((b, L, H)) - 2).astype(np.float32)
    A = (-np.exp(rng.uniform(0, np.log(16), H))).astype(np.float32)
    D = rng.standard_normal(H).astype(np.float32) if with_D else None
    return xq, Bq, Cq, dt, A, D


def _rand_scales(H, P, G, m, n, rng=RNG):
    hpg = H // G
    he, ce = [], []
    for g in range(G):
        cuts = np.sort(rng.integers(0, hpg + 1, m - 1)) if m > 1 else np.array([], int)
        he += list(cuts) + [hpg]
        for _ in range(m):
            cc = np.sort(rng.integers(1, P + 1, n - 1)) if n > 1 else np.array([], int)
            ce += list(cc) + [P]
    return Scales(m, n, rng.uniform(0.01, 0.2, G * m * n).astype(np.float32),
                  np.array(he, np.int32), np.array(ce, np.int32),
                  rng.uniform(0.01, 0.1, G).astype(np.float32),
                  rng.uniform(0.01, 0.1, G).astype(np.float32))


def _dequant(sc, xq, Bq, Cq):
    b, L, H, P = xq.shape
    G = Bq.shape[2]
    sx = oracle.x_scale_table(sc, H, P, G).astype(np.float64)
    x = xq.astype(np.float64) * sx
    B = Bq.astype(np.float64) * sc.B_scales.astype(np.float64)[None, None, :, None]
    C = Cq.astype(np.float64) * sc.C_scales.astype(np.float64)[None, None, :, None]
    return x, B, C


# --- independent evaluations written here, not in oracle/ ------------------------------------

def _dual_form(x, B, C, dt, A, D, h0=None):
    """O(L^2) 'attention' form of the SSD duality (Section 3.2, Mamba2 paragraph):
    y_t = sum_{s<=t} (C_t.B_s) exp(A sum_{r=s+1..t} dt_r) dt_s x_s + D x_t (+ C_t.(decay h0))."""
    b, L, H, P = x.shape
    G = B.shape[2]
    hpg = H // G
    y = np.zeros_like(x)
    for bi in range(b):
        for h in range(H):
            g = h // hpg
            a = dt[bi, :, h].astype(np.float64) * float(A[h])
            cs = np.cumsum(a)
            for t in range(L):
                acc = np.zeros(P)
                for s in range(t + 1):
                    w = np.exp(cs[t] - cs[s]) * float(dt[bi, s, h]) * np.dot(C[bi, t, g], B[bi, s, g])
                    acc += w * x[bi, s, h]
                if h0 is not None:
                    acc += np.exp(cs[t]) * (h0[bi, h] @ C[bi, t, g])
                y[bi, t, h] = acc + (float(D[h]) if D is not None else 0.0) * x[bi, t, h]
    return y


def _chunked_form(x, B, C, dt, A, D, Q, h0=None):
    """Chunked SSD: intra-chunk quadratic part + chunk states + sequential pass over chunks."""
    b, L, H, P = x.shape
    G, N = B.shape[2], B.shape[3]
    hpg = H // G
    y = np.zeros_like(x)
    fin = np.zeros((b, H, P, N))
    for bi in range(b):
        for h in range(H):
            g = h // hpg
            Hs = np.zeros((P, N)) if h0 is None else h0[bi, h].copy()
            for c0 in range(0, L, Q):
                c1 = min(L, c0 + Q)
                a = dt[bi, c0:c1, h].astype(np.float64) * float(A[h])
                cum = np.cumsum(a)
                d = dt[bi, c0:c1, h].astype(np.float64)
                Bc, Cc, xc = B[bi, c0:c1, g], C[bi, c0:c1, g], x[bi, c0:c1, h]
                Gm = Cc @ Bc.T
                dec = np.exp(np.minimum(cum[:, None] - cum[None, :], 0.0))
                Lm = np.tril(Gm * dec * d[None, :])
                yin = Lm @ xc + np.exp(cum)[:, None] * (Cc @ Hs.T)
                y[bi, c0:c1, h] = yin + (float(D[h]) if D is not None else 0.0) * xc
                w = np.exp(cum[-1] - cum) * d
                Hs = np.exp(cum[-1]) * Hs + (xc * w[:, None]).T @ Bc
            fin[bi, h] = Hs
    return y, fin


# --- the pins --------------------------------------------------------------------------------

@pytest.mark.parametrize("Q", [1, 4, 7, 24])
def test_sequential_equals_chunked_and_dual(Q):
    xq, Bq, Cq, dt, A, D = _rand_problem()
    sc = _rand_scales(4, 5, 2, 2, 3)
    y, st, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D)
    x, B, C = _dequant(sc, xq, Bq, Cq)
    yc, fc = _chunked_form(x, B, C, dt, A, D, Q)
    np.testing.assert_allclose(y, yc, rtol=0, atol=1e-11 * np.abs(y).max())
    np.testing.assert_allclose(st, fc, rtol=0, atol=1e-11 * np.abs(st).max())
    if Q == 1:
        yd = _dual_form(x, B, C, dt, A, D)
        np.testing.assert_allclose(y, yd, rtol=0, atol=1e-11 * np.abs(y).max())


def test_init_state_enters_through_decay_and_C():
    xq, Bq, Cq, dt, A, D = _rand_problem(b=1, L=10)
    sc = _rand_scales(4, 5, 2, 1, 2)
    h0 = RNG.standard_normal((1, 4, 5, 6))
    y, st, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D, init_state=h0)
    x, B, C = _dequant(sc, xq, Bq, Cq)
    yd = _dual_form(x, B, C, dt, A, D, h0=h0)
    np.testing.assert_allclose(y, yd, rtol=0, atol=1e-11 * np.abs(y).max())


def test_integer_case_is_exact_causal_linear_attention():
    """A = 0, dt = 1, all scales 1: y_t = sum_{s<=t} (C_t.B_s) x_s + D x_t in exact integers."""
    b, L, H, P, N, G = 1, 40, 2, 3, 4, 1
    rng = np.random.default_rng(7)
    xq = rng.integers(-9, 10, (b, L, H, P), dtype=np.int8)
    Bq = rng.integers(-9, 10, (b, L, G, N), dtype=np.int8)
    Cq = rng.integers(-9, 10, (b, L, G, N), dtype=np.int8)
    dt = np.ones((b, L, H), np.float32)
    A = np.zeros(H, np.float32)
    D = np.array([2.0, -3.0], np.float32)
    sc = Scales.ones(G, H // G, P)
    y, st, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D)
    exp_y = np.zeros((L, H, P), np.int64)
    state = np.zeros((H, P, N), np.int64)
    for t in range(L):
        state += xq[0, t].astype(np.int64)[:, :, None] * Bq[0, t, 0].astype(np.int64)[None, None, :]
        exp_y[t] = state @ Cq[0, t, 0].astype(np.int64) + D.astype(np.int64)[:, None] * xq[0, t]
    assert np.array_equal(y[0], exp_y.astype(np.float64))
    assert np.array_equal(st[0], state.astype(np.float64))


def test_dt_zero_gives_D_times_x_plus_C_h0():
    xq, Bq, Cq, dt, A, D = _rand_problem(b=1, L=6)
    sc = _rand_scales(4, 5, 2, 2, 2)
    dt0 = np.zeros_like(dt)
    y, st, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt0, A, D)
    x, B, C = _dequant(sc, xq, Bq, Cq)
    np.testing.assert_array_equal(y, D.astype(np.float64)[None, None, :, None] * x)
    assert not st.any()
    h0 = RNG.standard_normal((1, 4, 5, 6))
    y2, st2, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt0, A, D, init_state=h0)
    Cexp = np.repeat(C, 2, axis=2)                                   # [b,L,H,N]
    np.testing.assert_allclose(y2 - y, np.einsum("blhn,bhpn->blhp", Cexp, h0), atol=1e-12)
    np.testing.assert_array_equal(st2, h0)
    # small dt: the SSM part vanishes linearly
    yk = [oracle.ref_prefill(sc, xq, Bq, Cq, np.full_like(dt, e), A, D)[0] - y for e in (1e-3, 1e-4)]
    ratio = np.abs(yk[0]).max() / np.abs(yk[1]).max()
    assert 9.0 < ratio < 11.0


def test_constant_inputs_geometric_series():
    """x, B, C, dt constant: h_t = dt B x (1 - r^(t+1))/(1 - r), r = exp(dt A)."""
    L, P, N = 50, 2, 3
    xq = np.full((1, L, 1, P), 0, np.int8); xq[..., 0] = 50; xq[..., 1] = -20
    Bq = np.tile(np.array([10, -4, 7], np.int8), (1, L, 1, 1))
    Cq = np.tile(np.array([3, 9, -5], np.int8), (1, L, 1, 1))
    dtv, Av, Dv = 0.05, -2.5, 0.75
    dt = np.full((1, L, 1), dtv, np.float32)
    sc = Scales(1, 1, np.array([0.02], np.float32), np.array([1], np.int32), np.array([P], np.int32),
                np.array([0.5], np.float32), np.array([0.25], np.float32))
    y, st, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, np.array([Av], np.float32), np.array([Dv], np.float32))
    dtd = float(np.float32(dtv))
    r = np.exp(dtd * Av)
    x = np.float64(np.float32(0.02)) * np.array([50.0, -20.0])
    B = 0.5 * np.array([10.0, -4, 7]); Cv = 0.25 * np.array([3.0, 9, -5])
    for t in (0, 1, 17, L - 1):
        geo = (1 - r ** (t + 1)) / (1 - r)
        np.testing.assert_allclose(y[0, t, 0], np.dot(Cv, B) * dtd * x * geo + Dv * x, rtol=1e-12)
    np.testing.assert_allclose(st[0, 0], dtd * np.outer(x, B) * (1 - r ** L) / (1 - r), rtol=1e-12)


def test_impulse_response_uses_post_update_state():
    """x nonzero only at t0: y_t = (C_t.B_t0) dt_t0 exp(A sum_{r=t0+1..t} dt_r) x_t0 for t >= t0."""
    xq, Bq, Cq, dt, A, _ = _rand_problem(b=1, L=12, H=2, G=1, with_D=False)
    t0 = 4
    keep = xq[0, t0].copy(); xq[:] = 0; xq[0, t0] = keep
    sc = _rand_scales(2, 5, 1, 1, 1)
    y, _, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, None)
    x, B, C = _dequant(sc, xq, Bq, Cq)
    assert not y[0, :t0].any()
    for h in range(2):
        for t in range(t0, 12):
            dec = np.exp(float(A[h]) * dt[0, t0 + 1:t + 1, h].astype(np.float64).sum())
            ref = np.dot(C[0, t, 0], B[0, t0, 0]) * float(dt[0, t0, h]) * dec * x[0, t0, h]
            np.testing.assert_allclose(y[0, t, h], ref, rtol=1e-12, atol=1e-15)
    assert np.abs(y[0, t0]).max() > 0      # the step's own input already shows in y_t0


def test_linearity_in_scales_and_codes():
    xq, Bq, Cq, dt, A, D = _rand_problem(b=1, L=16)
    xq = (xq // 2).astype(np.int8)
    sc = _rand_scales(4, 5, 2, 2, 2)
    y, st, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D)
    sc2 = Scales(sc.m, sc.n, sc.x_scales * 2, sc.head_cluster_end, sc.chan_cluster_end, sc.B_scales, sc.C_scales)
    y2, st2, _ = oracle.ref_prefill(sc2, xq, Bq, Cq, dt, A, D)
    np.testing.assert_allclose(y2, 2 * y, rtol=1e-13)
    y3, _, _ = oracle.ref_prefill(sc, (2 * xq).astype(np.int8), Bq, Cq, dt, A, D)
    np.testing.assert_allclose(y3, 2 * y, rtol=1e-13)
    sc4 = Scales(sc.m, sc.n, sc.x_scales, sc.head_cluster_end, sc.chan_cluster_end, sc.B_scales * 4, sc.C_scales / 4)
    y4, st4, _ = oracle.ref_prefill(sc4, xq, Bq, Cq, dt, A, D)
    np.testing.assert_allclose(y4, y, rtol=1e-12)
    np.testing.assert_allclose(st4, 4 * st, rtol=1e-12)


def test_scale_lookup_follows_cluster_boundaries():
    """dt = 0, D = 1, code 1 everywhere: y is the (h,p) -> scale map itself."""
    H, P, G, m, n = 6, 7, 2, 2, 3
    he = np.array([1, 3, 2, 3], np.int32)           # group 0: heads {0},{1,2}; group 1: {3,4},{5}
    ce = np.array([2, 5, 7,  1, 1, 7,  3, 6, 7,  7, 7, 7], np.int32)
    xs = np.arange(1, 13, dtype=np.float32)
    sc = Scales(m, n, xs, he, ce, np.ones(G, np.float32), np.ones(G, np.float32))
    xq = np.ones((1, 1, H, P), np.int8)
    z = np.zeros((1, 1, G, 4), np.int8)
    y, _, _ = oracle.ref_prefill(sc, xq, z, z, np.zeros((1, 1, H), np.float32), -np.ones(H, np.float32),
                                 np.ones(H, np.float32))
    exp = np.array([[1, 1, 2, 2, 2, 3, 3],
                    [4, 6, 6, 6, 6, 6, 6],
                    [4, 6, 6, 6, 6, 6, 6],
                    [7, 7, 7, 8, 8, 8, 9],
                    [7, 7, 7, 8, 8, 8, 9],
                    [10, 10, 10, 10, 10, 10, 10]], np.float64)
    np.testing.assert_array_equal(y[0, 0], exp)
    np.testing.assert_array_equal(oracle.x_scale_table(sc, H, P, G), exp.astype(np.float32))


def test_state_group_of_a_head():
    """Heads read the B/C of group h // (H/G): zero every group but one and watch which heads respond."""
    xq, Bq, Cq, dt, A, _ = _rand_problem(b=1, L=8, H=6, G=3, with_D=False)
    sc = _rand_scales(6, 5, 3, 1, 1)
    Bz = np.zeros_like(Bq); Bz[:, :, 1] = Bq[:, :, 1]
    y, _, _ = oracle.ref_prefill(sc, xq, Bz, Cq, dt, A, None)
    assert not y[:, :, [0, 1, 4, 5]].any() and y[:, :, [2, 3]].any()


def test_permutation_invariance_bit_identical():
    """Channel-order preservation (Section 4.1): permuting heads inside a state group and channels
    inside a head, together with their parameters and scales, permutes y and the state identically."""
    b, L, H, P, N, G = 1, 12, 4, 6, 5, 2
    xq, Bq, Cq, dt, A, D = _rand_problem(b, L, H, P, N, G)
    sx = RNG.uniform(0.01, 0.2, (H, P)).astype(np.float32)

    def per_channel(sxt):     # one cluster per head and per channel needs m = hpg, n = P
        return Scales(2, P, sxt.reshape(-1), np.tile(np.array([1, 2], np.int32), G),
                      np.tile(np.arange(1, P + 1, dtype=np.int32), H),
                      np.array([0.03, 0.07], np.float32), np.array([0.05, 0.02], np.float32))

    y, st, _ = oracle.ref_prefill(per_channel(sx), xq, Bq, Cq, dt, A, D)
    hp = np.array([1, 0, 3, 2])
    cp = np.stack([RNG.permutation(P) for _ in range(H)])
    xq2 = np.take_along_axis(xq[:, :, hp], np.broadcast_to(cp, (b, L, H, P)), axis=-1)
    sx2 = np.take_along_axis(sx[hp], cp, axis=-1)
    y2, st2, _ = oracle.ref_prefill(per_channel(sx2), xq2, Bq, Cq, dt[:, :, hp], A[hp], D[hp])
    assert np.array_equal(y2, np.take_along_axis(y[:, :, hp], np.broadcast_to(cp, (b, L, H, P)), axis=-1))
    assert np.array_equal(st2, np.take_along_axis(st[:, hp], np.broadcast_to(cp[None, :, :, None], (b, H, P, N)), axis=2))


def test_prefill_then_decode_equals_longer_prefill():
    xq, Bq, Cq, dt, A, D = _rand_problem(b=2, L=20)
    sc = _rand_scales(4, 5, 2, 2, 2)
    yfull, stfull, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D)
    k = 3
    y0, st0, _ = oracle.ref_prefill(sc, xq[:, :-k], Bq[:, :-k], Cq[:, :-k], dt[:, :-k], A, D)
    np.testing.assert_array_equal(y0, yfull[:, :-k])
    state = st0.copy()
    for i in range(20 - k, 20):
        yi = oracle.ref_decode_step(sc, xq[:, i], Bq[:, i], Cq[:, i], dt[:, i], A, D, state)
        np.testing.assert_array_equal(yi, yfull[:, i])
    np.testing.assert_array_equal(state, stfull)
    # and a prefill of length 1 from an initial state is the decode step
    y1, st1, _ = oracle.ref_prefill(sc, xq[:, -1:], Bq[:, -1:], Cq[:, -1:], dt[:, -1:], A, D,
                                    init_state=oracle.ref_prefill(sc, xq[:, :-1], Bq[:, :-1], Cq[:, :-1],
                                                                  dt[:, :-1], A, D)[1])
    np.testing.assert_array_equal(y1[:, 0], yfull[:, -1])


def test_pairs_subset_matches_full():
    xq, Bq, Cq, dt, A, D = _rand_problem(b=2, L=9)
    sc = _rand_scales(4, 5, 2, 2, 2)
    y, st, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D)
    pairs = [(1, 3), (0, 0), (1, 1)]
    ys, sts, _ = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D, pairs=pairs)
    for i, (bi, h) in enumerate(pairs):
        np.testing.assert_array_equal(ys[i], y[bi, :, h])
        np.testing.assert_array_equal(sts[i], st[bi, h])


def test_threads_do_not_change_results():
    xq, Bq, Cq, dt, A, D = _rand_problem(b=2, L=9)
    sc = _rand_scales(4, 5, 2, 2, 2)
    y1, s1, u1 = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D, nthreads=1)
    y4, s4, u4 = oracle.ref_prefill(sc, xq, Bq, Cq, dt, A, D, nthreads=4)
    assert u1 == 1 and u4 == 4
    assert np.array_equal(y1, y4) and np.array_equal(s1, s4)


# --- Eq. 1 -----------------------------------------------------------------------------------

def test_quantizer_golden_cases():
    path = os.path.join(os.path.dirname(__file__), "golden", "eq1_quantizer_cases.txt")
    rows = [ln.split() for ln in open(path) if ln.strip() and not ln.startswith("#")]
    for s in (np.float32(1.0), np.float32(0.25), np.float32(8.0)):      # exact powers of two: X/s is exact
        X = np.array([float(r[0]) for r in rows], np.float32) * s
        np.testing.assert_array_equal(oracle.quantize(X, s), np.array([int(r[1]) for r in rows], np.int8))


def test_quantizer_scale_maps_max_to_127():
    X = RNG.standard_normal(1000).astype(np.float32) * 3.7
    s = oracle.group_scales(np.abs(X)[None, :])[0]
    q = oracle.quantize(X, s)
    assert q[np.argmax(np.abs(X))] in (127, -127) and np.abs(q).max() == 127
    assert np.abs(q.astype(np.float64) * float(s) - X).max() <= 0.5 * float(s) * (1 + 1e-6)
    assert oracle.group_scales(np.zeros((1, 4), np.float32))[0] == 1.0
