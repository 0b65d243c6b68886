"""TEST INFRASTRUCTURE: the offline side of the method, written out step by step in numpy/Python.

* quantize            — symmetric uniform quantizer, Eq. 1 (Section 3.1).
* sort_and_cluster    — Section 4.1 "Sort-and-cluster" (and the caption of the clustering figure):
                        calibrated channel maxima -> sort channels inside every head -> cluster the
                        heads of each state group into m clusters -> cluster the sorted channel
                        positions of each head cluster into n ranges -> m x n scales.
* group_scales        — Section 4.1 "Per-state-group quantization": one scale per state group.

The paper only says "unsupervised clustering"; the reading taken here (the same one the product
documents) is: heads — Lloyd k-means on the sorted-maximum vectors with a deterministic start
(heads ranked by vector sum, start centroids at evenly spaced ranks), at most 50 rounds, an empty
cluster takes the point farthest from its centroid; channels — the exact 1-D k-means partition of
the cluster's max-profile into contiguous ranges, by dynamic programming.  Any partition yields
the same scan output, so the partition itself is "parity unpinned"; tests pin its invariants
(valid permutations, heads stay inside their state group, monotone boundaries, no clipping of
the calibration maxima, a planted cluster structure is recovered, error no worse than one scale).
"""
from __future__ import annotations

import numpy as np

F32 = np.float32


def quantize(X: np.ndarray, s, nbits: int = 8) -> np.ndarray:
    """Eq. 1: clamp(round(X / s), -2^(N-1), 2^(N-1)-1); division and rounding (half to even) in fp32."""
    q = np.rint(np.asarray(X, F32) / np.asarray(s, F32))
    lo, hi = -(1 << (nbits - 1)), (1 << (nbits - 1)) - 1
    return np.clip(q, lo, hi).astype(np.int8)


def _scale_from_max(mx: float, nbits: int = 8) -> np.float32:
    """s = max|X| / (2^(N-1) - 1) (Eq. 1); an all-zero group gets s = 1."""
    mx = F32(mx)
    return F32(1.0) if mx == 0 else F32(mx / F32((1 << (nbits - 1)) - 1))


def group_scales(absmax: np.ndarray) -> np.ndarray:
    """absmax [G,N] calibrated maxima -> one scale per state group [G]."""
    absmax = np.asarray(absmax, F32)
    return np.array([_scale_from_max(absmax[g].max()) for g in range(absmax.shape[0])], F32)


def _sqdist(a: np.ndarray, b: np.ndarray) -> float:
    d = 0.0
    for u, v in zip(a, b):
        d += (float(u) - float(v)) ** 2
    return d


def _lloyd(vecs: np.ndarray, k: int, rounds: int = 50) -> np.ndarray:
    """Deterministic Lloyd k-means of the rows of vecs [cnt,P] (fp64).  Returns labels [cnt]."""
    cnt = vecs.shape[0]
    if k <= 1:
        return np.zeros(cnt, np.int64)
    sums = np.array([float(sum(float(t) for t in v)) for v in vecs])
    rank = np.argsort(sums, kind="stable")
    cent = np.stack([vecs[rank[(i * (cnt - 1)) // (k - 1)]] for i in range(k)]).astype(np.float64)
    labels = np.full(cnt, -1, np.int64)
    for _ in range(rounds):
        new = np.empty(cnt, np.int64)
        dist = np.empty(cnt, np.float64)
        for i in range(cnt):
            best, bd = 0, _sqdist(vecs[i], cent[0])
            for c in range(1, k):
                d = _sqdist(vecs[i], cent[c])
                if d < bd:
                    best, bd = c, d
            new[i], dist[i] = best, bd
        for c in range(k):                       # an empty cluster takes the farthest point
            if not np.any(new == c):
                cand = [i for i in range(cnt) if np.sum(new == new[i]) > 1]
                far = max(cand, key=lambda i: (dist[i], -i))
                new[far], dist[far] = c, 0.0
        if np.array_equal(new, labels):
            break
        labels = new
        for c in range(k):
            mem = [i for i in range(cnt) if labels[i] == c]
            acc = np.zeros(vecs.shape[1], np.float64)
            for i in mem:
                acc += vecs[i]
            cent[c] = acc / len(mem)
    return labels


def _kmeans_1d(profile: np.ndarray, k: int) -> list:
    """Exact 1-D k-means of profile[0..P) into k contiguous non-empty ranges; returns exclusive ends."""
    P = len(profile)
    k = min(k, P)
    s1 = np.zeros(P + 1); s2 = np.zeros(P + 1)
    for i, v in enumerate(profile):
        s1[i + 1] = s1[i] + float(v)
        s2[i + 1] = s2[i] + float(v) * float(v)

    def cost(a, e):
        t = s1[e] - s1[a]
        return (s2[e] - s2[a]) - t * t / (e - a)

    INF = float("inf")
    dp = [[INF] * (P + 1) for _ in range(k + 1)]
    arg = [[0] * (P + 1) for _ in range(k + 1)]
    dp[0][0] = 0.0
    for j in range(1, k + 1):
        for e in range(j, P + 1):
            for a in range(j - 1, e):
                if dp[j - 1][a] == INF:
                    continue
                c = dp[j - 1][a] + cost(a, e)
                if c < dp[j][e]:
                    dp[j][e], arg[j][e] = c, a
    ends, e = [], P
    for j in range(k, 0, -1):
        ends.append(e)
        e = arg[j][e]
    return ends[::-1]


def sort_and_cluster(xmax: np.ndarray, ngroups: int, m: int, n: int) -> dict:
    """Section 4.1 on calibrated maxima xmax [H,P] (original head/channel order).

    Returns head_perm [H] (new -> old), chan_perm [H,P] (row i: sorted position -> old channel of
    NEW head i), x_scales [G*m*n], head_cluster_end [G*m], chan_cluster_end [G*m*n].
    """
    xmax = np.asarray(xmax, F32)
    H, P = xmax.shape
    assert H % ngroups == 0
    hpg = H // ngroups
    order = np.stack([np.argsort(xmax[h], kind="stable") for h in range(H)])      # step 1: sort channels
    sorted_max = np.take_along_axis(xmax, order, axis=1).astype(np.float64)        # head embeddings
    head_perm = np.empty(H, np.int32)
    chan_perm = np.empty((H, P), np.int32)
    x_scales = np.ones(ngroups * m * n, F32)
    head_end = np.empty(ngroups * m, np.int32)
    chan_end = np.full(ngroups * m * n, P, np.int32)
    for g in range(ngroups):
        heads = np.arange(g * hpg, (g + 1) * hpg)
        k = min(m, hpg)
        labels = _lloyd(sorted_max[heads], k)                                     # step 2: cluster heads
        cents = []
        for c in range(k):
            mem = heads[labels == c]
            cents.append((float(sorted_max[mem].mean(axis=0).sum()), int(mem.min()), c))
        pos = 0
        for i, (_, _, c) in enumerate(sorted(cents)):                             # clusters by magnitude
            mem = heads[labels == c]
            head_perm[g * hpg + pos: g * hpg + pos + len(mem)] = mem
            pos += len(mem)
            head_end[g * m + i] = pos
            profile = sorted_max[mem].max(axis=0)                                 # step 3: cluster channels
            ends = _kmeans_1d(profile, n)
            base = (g * m + i) * n
            for j in range(n):
                e = ends[j] if j < len(ends) else P
                chan_end[base + j] = e
                a = 0 if j == 0 else chan_end[base + j - 1]
                x_scales[base + j] = _scale_from_max(profile[a:e].max()) if e > a else F32(1.0)
        for i in range(k, m):
            head_end[g * m + i] = hpg
    chan_perm[:] = order[head_perm]
    return {"head_perm": head_perm, "chan_perm": chan_perm, "x_scales": x_scales,
            "head_cluster_end": head_end, "chan_cluster_end": chan_end}
