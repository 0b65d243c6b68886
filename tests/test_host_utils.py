"""The library's host-side utilities (sort-and-cluster, gather, Eq. 1) against the numpy oracle.  No GPU."""
import numpy as np
import pytest

import oracle
import paper_2503_22879_amd as q
import workloads as W
from helpers import to_shape


@pytest.mark.parametrize("name", ["tiny", "m2_130m", "m2_2p7b", "m2_8b_b1"])
def test_reorder_matches_oracle_reading(name):
    """Same documented reading of the clustering on both sides -> identical tables on the synthetic calibration
    sets (the partition is not unique in general; test_snc_oracle.py pins what is)."""
    s = W.CONFIGS[name]
    xm, bm, cm = W.draw_calibration(s, tokens=512)
    hp, cp, hs = q.quamba_reorder_params(s.nheads, s.headdim, s.ngroups, s.m, s.n, s.d_state, xm, bm, cm)
    r = oracle.sort_and_cluster(xm, s.ngroups, s.m, s.n)
    assert np.array_equal(hp, r["head_perm"]) and np.array_equal(cp, r["chan_perm"])
    assert np.array_equal(hs.head_cluster_end, r["head_cluster_end"])
    assert np.array_equal(hs.chan_cluster_end, r["chan_cluster_end"])
    assert np.array_equal(hs.x_scales, r["x_scales"])
    assert np.array_equal(hs.B_scales, oracle.group_scales(bm))
    assert np.array_equal(hs.C_scales, oracle.group_scales(cm))


def test_reorder_validity_on_random_profiles():
    rng = np.random.default_rng(99)
    for _ in range(10):
        G = int(rng.choice([1, 2, 4])); hpg = int(rng.integers(1, 9)); P = int(rng.integers(1, 40))
        m = int(rng.integers(1, 6)); n = int(rng.integers(1, 6)); H = G * hpg
        xm = rng.lognormal(0, 1.5, (H, P)).astype(np.float32)
        hp, cp, hs = q.quamba_reorder_params(H, P, G, m, n, 4, xm, np.ones((G, 4)), np.ones((G, 4)))
        assert sorted(hp.tolist()) == list(range(H)) and np.array_equal(hp // hpg, np.arange(H) // hpg)
        he = hs.head_cluster_end.reshape(G, m); ce = hs.chan_cluster_end.reshape(G, m, n)
        assert np.all(np.diff(he, axis=1) >= 0) and np.all(he[:, -1] == hpg)
        assert np.all(np.diff(ce, axis=2) >= 0) and np.all(ce[:, :, -1] == P)
        sc = oracle.Scales(m, n, hs.x_scales, hs.head_cluster_end, hs.chan_cluster_end, hs.B_scales, hs.C_scales)
        tab = oracle.x_scale_table(sc, H, P, G)
        re = np.take_along_axis(xm[hp], cp, axis=1)
        assert np.all(np.diff(re, axis=1) >= 0)
        assert np.all(tab * np.float32(127) >= re * np.float32(1 - 1e-6))


def test_quantizers_bit_exact_against_oracle():
    s = W.CONFIGS["m2_130m"].with_(seqlen=64)
    xm, bm, cm = W.draw_calibration(s, tokens=256)
    hp, cp, hs = q.quamba_reorder_params(s.nheads, s.headdim, s.ngroups, s.m, s.n, s.d_state, xm, bm, cm)
    raw = W.apply_reorder(W.draw_layer(s), hp, cp)
    sc = oracle.Scales(s.m, s.n, hs.x_scales, hs.head_cluster_end, hs.chan_cluster_end, hs.B_scales, hs.C_scales)
    tab = oracle.x_scale_table(sc, s.nheads, s.headdim, s.ngroups)
    xq = q.quamba_quantize_x(to_shape(q, s), hs, raw["x"])
    assert np.array_equal(xq, oracle.quantize(raw["x"], tab))
    assert np.abs(xq.astype(np.int32)).max() == 127 or np.abs(xq.astype(np.int32)).max() == 128
    for k, sg in (("B", hs.B_scales), ("C", hs.C_scales)):
        assert np.array_equal(q.quamba_quantize_groups(raw[k], sg), oracle.quantize(raw[k], sg[:, None]))
    # ties and clamping
    v = np.array([[[0.5, 1.5, 2.5, -0.5, -1.5, 300.0, -300.0, 126.5]]], np.float32)
    assert q.quamba_quantize_groups(v, np.ones(1, np.float32)).ravel().tolist() == [0, 2, 2, 0, -2, 127, -128, 126]


def test_gather_rows_and_compute_invariance():
    """Reordering the producer's rows offline equals reordering its output (Section 4.2)."""
    rng = np.random.default_rng(4)
    W_in = rng.standard_normal((12, 5)).astype(np.float32)     # rows = output channels of the in-projection
    u = rng.standard_normal((5, 3)).astype(np.float32)
    perm = rng.permutation(12).astype(np.int32)
    assert np.array_equal(q.quamba_gather_rows(W_in, perm) @ u, (W_in @ u)[perm])
    assert np.array_equal(q.quamba_gather_rows(np.arange(12, dtype=np.int64), perm), perm.astype(np.int64))
    with pytest.raises(q.QuambaError) as e:
        q.quamba_gather_rows(W_in, np.full(12, 12, np.int32))
    assert e.value.status == -5


def test_reorder_rejects_bad_input():
    ok = np.ones((4, 8), np.float32)
    with pytest.raises(q.QuambaError) as e:
        q.quamba_reorder_params(4, 8, 3, 2, 2, 4, ok, np.ones((3, 4)), np.ones((3, 4)))
    assert e.value.status == -2
    bad = ok.copy(); bad[1, 2] = np.nan
    with pytest.raises(q.QuambaError) as e:
        q.quamba_reorder_params(4, 8, 2, 2, 2, 4, bad, np.ones((2, 4)), np.ones((2, 4)))
    assert e.value.status == -5


def test_state_scales_bit_exact_against_oracle_and_argument_checks():
    """quamba_state_scales: cell maxima / 127 over the cells the lookup assigns (Appendix E), same as the oracle's."""
    rng = np.random.default_rng(5)
    for name in ("tiny", "m2_130m"):
        s = W.CONFIGS[name]
        xm, bm, cm = W.draw_calibration(s, tokens=256)
        hp, cp, hs = q.quamba_reorder_params(s.nheads, s.headdim, s.ngroups, s.m, s.n, s.d_state, xm, bm, cm)
        sc = oracle.Scales(s.m, s.n, hs.x_scales, hs.head_cluster_end, hs.chan_cluster_end, hs.B_scales, hs.C_scales)
        mx = W.reorder_state(W.draw_cached_state_calibration(s, 3, sequences=2), hp, cp)
        mx[:, :, 1] = 0                                           # a state that never fires: scale 1
        got = q.quamba_state_scales(s.nheads, s.headdim, s.ngroups, s.m, s.n, s.d_state, hs.head_cluster_end,
                                    hs.chan_cluster_end, mx)
        want = oracle.state_scales_from_absmax(sc, mx, s.ngroups)
        assert got.dtype == np.float32 and np.array_equal(got, want)
        assert np.all(got[:, 1] == 1.0) and np.all(got > 0)
    H, P, G, m, n, N = 4, 6, 2, 2, 2, 3
    he = np.array([1, 2, 2, 2], np.int32); ce = np.array([3, 6] * 4, np.int32)
    mx = rng.uniform(0, 1, (H, P, N)).astype(np.float32)
    assert q.quamba_state_scales(H, P, G, m, n, N, he, ce, mx).shape == (G * m * n, N)
    bad = mx.copy(); bad[0, 0, 0] = -1
    with pytest.raises(q.QuambaError):
        q.quamba_state_scales(H, P, G, m, n, N, he, ce, bad)
    with pytest.raises(q.QuambaError):
        q.quamba_state_scales(H, P, G, m, n, N, np.array([3, 2, 2, 2], np.int32), ce, mx)      # beyond the group
    with pytest.raises(q.QuambaError):
        q.quamba_state_scales(H, P, G, m, n, N, he, np.array([4, 3] * 4, np.int32), mx)       # decreasing
    with pytest.raises(q.QuambaError):
        q.quamba_state_scales(5, P, G, m, n, N, he, ce, np.zeros((5, P, N), np.float32))      # H % G


def test_the_host_quantizers_reject_scales_that_are_not_positive_and_finite():
    """Eq. 1 divides by the scale: zero, negative, infinite and NaN scales are refused before anything is written."""
    import paper_2503_22879_amd as q
    v = np.ones((2, 3, 4), np.float32)
    for bad in (0.0, -1.0, np.inf, np.nan):
        gs = np.array([1.0, bad, 1.0], np.float32)
        with pytest.raises(q.QuambaError):
            q.quamba_quantize_groups(v, gs)
    assert q.quamba_quantize_groups(v, np.ones(3, np.float32)).dtype == np.int8
    shape = q.Shape(batch=1, seqlen=1, nheads=2, headdim=4, d_state=4, ngroups=1, chunk=1, n_head_clusters=1,
                    n_chan_clusters=2, flags=0)
    for bad in (0.0, -2.0, np.nan):
        hs = q.HostScales(np.array([1.0, bad], np.float32), np.array([2], np.int32), np.array([2, 4], np.int32),
                          np.ones(1, np.float32), np.ones(1, np.float32))
        with pytest.raises(q.QuambaError):
            q.quamba_quantize_x(shape, hs, np.ones((1, 2, 4), np.float32))
