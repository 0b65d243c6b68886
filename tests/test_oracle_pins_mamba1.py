"""Pins of oracle/mamba1.py (the Mamba1 selective scan on 8-bit operands): the already pinned Mamba2 oracle on the
inputs where the two coincide, closed-form geometric series where they do not, brute force, limits.  No GPU."""
import numpy as np

import oracle


def _draw(seed, b=2, D=12, N=5, L=40):
    g = np.random.default_rng(seed)
    return dict(xq=g.integers(-128, 128, size=(b, D, L), dtype=np.int8),
                Bq=g.integers(-128, 128, size=(b, N, L), dtype=np.int8),
                Cq=g.integers(-128, 128, size=(b, N, L), dtype=np.int8),
                dt=np.log1p(np.exp(g.normal(-2.5, 1, size=(b, D, L)))).astype(np.float32),
                A=-np.exp(g.uniform(0, 2.5, size=(D, N))).astype(np.float32),
                D=g.normal(0, 1, D).astype(np.float32),
                xs=np.exp(g.normal(-3, 0.5, D)), sB=0.013, sC=0.021)


def test_reduces_to_the_mamba2_scan_when_a_head_shares_its_decay():
    """With A constant over the states and the channels of a head, and the step size shared inside a head, Eq. 2 in the
    Mamba1 form is the Mamba2 SSD with one state group; that oracle (C, pinned on its own) must agree."""
    g = np.random.default_rng(0)
    b, H, P, N, L = 2, 3, 4, 6, 33
    d = _draw(0, b, H * P, N, L)
    A_h = -np.exp(g.uniform(0, 2, H)).astype(np.float32)
    dt_h = np.log1p(np.exp(g.normal(-2, 1, size=(b, L, H)))).astype(np.float32)
    A1 = np.repeat(A_h, P)[:, None].repeat(N, 1)
    dt1 = np.repeat(dt_h.transpose(0, 2, 1), P, axis=1)                              # [b, H*P, L]
    xs = np.exp(g.normal(-3, 0.5, (H, P))).astype(np.float32)
    init = g.normal(0, 0.1, size=(b, H * P, N))
    # the same problem in the Mamba2 oracle's layout: one cell per (head, channel) so that every channel has its scale
    sc = oracle.Scales(m=H, n=P, x_scales=xs.reshape(-1), head_cluster_end=np.arange(1, H + 1, dtype=np.int32),
                       chan_cluster_end=np.tile(np.arange(1, P + 1, dtype=np.int32), H),
                       B_scales=np.array([d["sB"]], np.float32), C_scales=np.array([d["sC"]], np.float32))
    x2 = d["xq"].reshape(b, H, P, L).transpose(0, 3, 1, 2)
    B2 = d["Bq"].transpose(0, 2, 1)[:, :, None, :]
    C2 = d["Cq"].transpose(0, 2, 1)[:, :, None, :]
    # the Mamba2 oracle has one D per head: give every channel of a head the same D
    Dhead = d["D"][:H]
    y1, st1 = oracle.ref_mamba1_scan(xs.reshape(-1), np.float32(d["sB"]), np.float32(d["sC"]), d["xq"], d["Bq"], d["Cq"],
                                     dt1, A1, np.repeat(Dhead, P), init)
    y2, st2, _ = oracle.ref_prefill(sc, x2, B2, C2, dt_h, A_h, Dhead, init_state=init.reshape(b, H, P, N))
    assert np.allclose(y1, y2.transpose(0, 2, 3, 1).reshape(b, H * P, L), rtol=1e-11, atol=1e-12)
    assert np.allclose(st1, st2.reshape(b, H * P, N), rtol=1e-11, atol=1e-14)


def test_per_channel_per_state_decay_closed_form():
    """Constant inputs: h_t[d,n] = u_d (1 - a^t) / (1 - a) with a = exp(dt A[d,n]), u_d = dt s_B B s_x x; every (d, n)
    has its own a, which the Mamba2 pin cannot see."""
    b, D, N, L = 1, 5, 4, 25
    g = np.random.default_rng(1)
    A = -np.exp(g.uniform(-1, 2, size=(D, N)))
    dtv = np.array([0.05, 0.1, 0.2, 0.4, 0.8])
    xs = np.array([0.5, 0.25, 1.0, 2.0, 0.125])
    xq = np.full((b, D, L), 3, np.int8) * np.array([1, -1, 2, 5, -7], np.int8)[None, :, None]
    Bq = np.broadcast_to(np.array([2, -3, 4, 1], np.int8)[None, :, None], (b, N, L)).copy()
    Cq = np.broadcast_to(np.array([1, 5, -2, 3], np.int8)[None, :, None], (b, N, L)).copy()
    dt = np.broadcast_to(dtv[None, :, None], (b, D, L)).copy()
    Dk = np.array([0.3, -1.0, 0.0, 2.0, 0.5])
    y, st = oracle.ref_mamba1_scan(xs, 0.1, 0.01, xq, Bq, Cq, dt, A, Dk)
    a = np.exp(dtv[:, None] * A)                                                     # [D,N]
    x = xq[0, :, 0] * xs
    u = dtv[:, None] * x[:, None] * (0.1 * Bq[0, :, 0])[None, :]
    for t in range(L):
        h = u * (1 - a ** (t + 1)) / (1 - a)
        want = (h * (0.01 * Cq[0, :, 0])[None, :]).sum(1) + Dk * x
        assert np.allclose(y[0, :, t], want, rtol=1e-12)
    assert np.allclose(st[0], u * (1 - a ** L) / (1 - a), rtol=1e-12)


def test_brute_force_limits_and_continuation():
    d = _draw(2)
    y, st = oracle.ref_mamba1_scan(d["xs"], d["sB"], d["sC"], d["xq"], d["Bq"], d["Cq"], d["dt"], d["A"], d["D"])
    b, Dn, L = d["xq"].shape
    N = d["Bq"].shape[1]
    # brute force: the unrolled sum y_t = sum_{s<=t} sum_n C_t[n] exp(A[d,n] sum_{s<r<=t} dt_r) dt_s B_s[n] x_s + D x_t
    for (bi, di, t) in [(0, 0, 0), (1, 7, 13), (0, 11, 39), (1, 3, 1)]:
        acc = 0.0
        for s in range(t + 1):
            span = d["dt"][bi, di, s + 1:t + 1].astype(np.float64).sum()
            for n in range(N):
                acc += (d["sC"] * d["Cq"][bi, n, t]) * np.exp(float(d["A"][di, n]) * span) * float(d["dt"][bi, di, s]) * \
                    (d["sB"] * d["Bq"][bi, n, s]) * (d["xs"][di] * d["xq"][bi, di, s])
        acc += float(d["D"][di]) * d["xs"][di] * d["xq"][bi, di, t]
        assert np.isclose(y[bi, di, t], acc, rtol=1e-10, atol=1e-12)
    # dt = 0: the state never changes and y = C h_init + D x; without a state y = D x
    z = np.zeros_like(d["dt"])
    y0, s0 = oracle.ref_mamba1_scan(d["xs"], d["sB"], d["sC"], d["xq"], d["Bq"], d["Cq"], z, d["A"], d["D"])
    assert np.allclose(y0, d["D"].astype(np.float64)[None, :, None] * d["xq"] * d["xs"][None, :, None], rtol=1e-14)
    assert not s0.any()
    # A = 0: no decay, the state is the running sum
    yA, sA = oracle.ref_mamba1_scan(d["xs"], d["sB"], d["sC"], d["xq"], d["Bq"], d["Cq"], d["dt"], np.zeros_like(d["A"]), None)
    want = np.einsum("bdl,bnl->bdn", d["dt"].astype(np.float64) * d["xq"] * d["xs"][None, :, None], d["sB"] * d["Bq"].astype(np.float64))
    assert np.allclose(sA, want, rtol=1e-12)
    # running in two pieces through the state equals running at once
    cut = 17
    f = lambda k, lo, hi: d[k][:, :, lo:hi]
    y1, s1 = oracle.ref_mamba1_scan(d["xs"], d["sB"], d["sC"], f("xq", 0, cut), f("Bq", 0, cut), f("Cq", 0, cut), f("dt", 0, cut), d["A"], d["D"])
    y2, s2 = oracle.ref_mamba1_scan(d["xs"], d["sB"], d["sC"], f("xq", cut, L), f("Bq", cut, L), f("Cq", cut, L), f("dt", cut, L), d["A"], d["D"], s1)
    assert np.allclose(np.concatenate([y1, y2], axis=2), y, rtol=1e-13, atol=1e-15) and np.allclose(s2, st, rtol=1e-13)
    # channels are independent; the scales are per channel
    assert np.array_equal(oracle.channel_scales([0.5, 0.25, 2.0], [2, 3, 7], 7), [0.5, 0.5, 0.25, 2.0, 2.0, 2.0, 2.0])
