"""Invariants of the oracle's sort-and-cluster (Section 4.1).  The partition itself has several
valid answers ("parity unpinned"); what is unique or required is checked here."""
import numpy as np
import pytest

import oracle
import workloads as W


def _check_valid(r, xmax, G, m, n):
    H, P = xmax.shape
    hpg = H // G
    hp, cp = r["head_perm"], r["chan_perm"]
    assert sorted(hp.tolist()) == list(range(H))
    assert np.array_equal(hp // hpg, np.arange(H) // hpg)            # heads stay in their state group
    for i in range(H):
        assert sorted(cp[i].tolist()) == list(range(P))
        v = xmax[hp[i]][cp[i]]
        assert np.all(np.diff(v) >= 0)                               # channels sorted by calibrated max
    he = r["head_cluster_end"].reshape(G, m)
    ce = r["chan_cluster_end"].reshape(G, m, n)
    assert np.all(np.diff(he, axis=1) >= 0) and np.all(he[:, -1] == hpg) and np.all(he >= 0)
    assert np.all(np.diff(ce, axis=2) >= 0) and np.all(ce[:, :, -1] == P) and np.all(ce >= 0)
    sc = oracle.Scales(m, n, r["x_scales"], r["head_cluster_end"], r["chan_cluster_end"],
                       np.ones(G, np.float32), np.ones(G, np.float32))
    tab = oracle.x_scale_table(sc, H, P, G)
    re = np.take_along_axis(xmax[hp], cp, axis=1)
    assert np.all(tab * np.float32(127) >= re * np.float32(1 - 1e-6))  # no clipping on calibration data
    # every scale is attained: it is exactly (max of its cell)/127
    for g in range(G):
        for i in range(m):
            h0 = 0 if i == 0 else he[g, i - 1]
            for j in range(n):
                c0 = 0 if j == 0 else ce[g, i, j - 1]
                cell = re[g * hpg + h0: g * hpg + he[g, i], c0: ce[g, i, j]]
                want = np.float32(1.0) if cell.size == 0 or cell.max() == 0 else np.float32(cell.max() / np.float32(127))
                assert r["x_scales"].reshape(G, m, n)[g, i, j] == want
    return tab, re


@pytest.mark.parametrize("name,G,m,n", [("tiny", 1, 1, 4), ("m2_130m", 1, 4, 4), ("m2_8b_b1", 8, 4, 4)])
def test_invariants_on_synthetic_calibration(name, G, m, n):
    s = W.CONFIGS[name]
    xmax, _, _ = W.draw_calibration(s, tokens=512)
    r = oracle.sort_and_cluster(xmax, G, m, n)
    tab, re = _check_valid(r, xmax, G, m, n)
    # quantization error on calibration-like data: no worse than one scale for the whole tensor
    data = re[None] * np.random.default_rng(3).uniform(-1, 1, (64,) + re.shape).astype(np.float32)
    one = np.float32(re.max() / 127)
    e_snc = np.mean((oracle.quantize(data, tab).astype(np.float64) * tab - data) ** 2)
    e_one = np.mean((oracle.quantize(data, one).astype(np.float64) * one - data) ** 2)
    assert e_snc < e_one


def test_planted_clusters_are_recovered():
    """4 well-separated head families x 4 channel levels, shuffled: clusters must be the families."""
    rng = np.random.default_rng(11)
    H, P, G, m, n = 16, 32, 1, 4, 4
    fam_gain = np.array([1.0, 10.0, 100.0, 1000.0])
    level = np.repeat(np.array([1.0, 2.0, 4.0, 8.0]), P // 4)
    fam = rng.permutation(np.repeat(np.arange(4), H // 4))
    xmax = np.empty((H, P), np.float32)
    for h in range(H):
        xmax[h] = (fam_gain[fam[h]] * level * rng.uniform(0.97, 1.0, P))[rng.permutation(P)]
    r = oracle.sort_and_cluster(xmax, G, m, n)
    _check_valid(r, xmax, G, m, n)
    assert r["head_cluster_end"].tolist() == [4, 8, 12, 16]
    assert np.array_equal(fam[r["head_perm"]], np.repeat(np.arange(4), 4))     # ascending magnitude
    assert r["chan_cluster_end"].reshape(4, 4).tolist() == [[8, 16, 24, 32]] * 4


def test_degenerate_inputs():
    r = oracle.sort_and_cluster(np.zeros((2, 4), np.float32), 1, 4, 2)    # fewer heads than clusters, all zero
    _check_valid(r, np.zeros((2, 4), np.float32), 1, 4, 2)
    assert np.all(r["x_scales"] == 1.0)
    r = oracle.sort_and_cluster(np.ones((4, 2), np.float32), 2, 1, 4)     # fewer channels than clusters
    _check_valid(r, np.ones((4, 2), np.float32), 2, 1, 4)


def test_kmeans_1d_against_brute_force():
    from itertools import combinations
    from oracle.snc import _kmeans_1d
    rng = np.random.default_rng(5)
    for _ in range(20):
        P, k = 9, 3
        v = np.sort(rng.lognormal(0, 1, P))

        def sse(ends):
            a, tot = 0, 0.0
            for e in ends:
                seg = v[a:e]; tot += ((seg - seg.mean()) ** 2).sum(); a = e
            return tot
        best = min((sse(list(c) + [P]) for c in combinations(range(1, P), k - 1)))
        assert abs(sse(_kmeans_1d(v, k)) - best) <= 1e-12 * max(1.0, best)
