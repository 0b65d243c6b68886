// Host-side, offline part of the library: sort-and-cluster (Section 4.1), the permutation tables used by the
// cluster-aware weight reordering (Section 4.2), the static-scale quantizer of Eq. 1, and the static scales of the
// 8-bit cached state (Appendix E).  No device code.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <limits>
#include <numeric>
#include <vector>

#include "quamba_ssd.h"

namespace {

// Eq. 1 with N = 8: s = max|X| / 127.  A cell that never fires keeps codes at zero with s = 1.
inline float scale_of_max(float mx) { return mx == 0.0f ? 1.0f : mx / 127.0f; }

struct HeadVec {
    int old_index;
    const double *v;  // sorted calibrated maxima, length P
    double sum;
};

double sqdist(const double *a, const double *b, int P)
{
    double d = 0.0;
    for (int i = 0; i < P; ++i) {
        const double t = a[i] - b[i];
        d += t * t;
    }
    return d;
}

// Lloyd k-means of `hv` into k clusters.  Start: heads ranked by vector sum, centroids at evenly spaced ranks.
// A cluster that ends a round empty takes the point farthest from its own centroid (from a cluster that
// keeps at least one other member).  Stops when labels repeat or after 50 rounds.
std::vector<int> lloyd(const std::vector<HeadVec> &hv, int P, int k)
{
    const int cnt = (int)hv.size();
    std::vector<int> label(cnt, 0);
    if (k <= 1) return label;
    std::vector<int> rank(cnt);
    std::iota(rank.begin(), rank.end(), 0);
    std::stable_sort(rank.begin(), rank.end(), [&](int a, int b) { return hv[a].sum < hv[b].sum; });
    std::vector<double> cent((size_t)k * P);
    for (int c = 0; c < k; ++c) {
        const int r = rank[(size_t)c * (cnt - 1) / (k - 1)];
        std::copy(hv[r].v, hv[r].v + P, cent.begin() + (size_t)c * P);
    }
    std::fill(label.begin(), label.end(), -1);
    std::vector<int> next(cnt), pop(k);
    std::vector<double> dist(cnt);
    for (int round = 0; round < 50; ++round) {
        for (int i = 0; i < cnt; ++i) {
            int best = 0;
            double bd = sqdist(hv[i].v, &cent[0], P);
            for (int c = 1; c < k; ++c) {
                const double d = sqdist(hv[i].v, &cent[(size_t)c * P], P);
                if (d < bd) { bd = d; best = c; }
            }
            next[i] = best;
            dist[i] = bd;
        }
        for (int c = 0; c < k; ++c) {
            std::fill(pop.begin(), pop.end(), 0);
            for (int i = 0; i < cnt; ++i) ++pop[next[i]];
            if (pop[c]) continue;
            int far = -1;
            for (int i = 0; i < cnt; ++i)
                if (pop[next[i]] > 1 && (far < 0 || dist[i] > dist[far])) far = i;
            next[far] = c;
            dist[far] = 0.0;
        }
        if (next == label) break;
        label = next;
        for (int c = 0; c < k; ++c) {
            double *ctr = &cent[(size_t)c * P];
            std::fill(ctr, ctr + P, 0.0);
            int members = 0;
            for (int i = 0; i < cnt; ++i)
                if (label[i] == c) {
                    for (int j = 0; j < P; ++j) ctr[j] += hv[i].v[j];
                    ++members;
                }
            for (int j = 0; j < P; ++j) ctr[j] /= members;
        }
    }
    return label;
}

// Exact 1-D k-means of a profile into at most k contiguous non-empty ranges (dynamic programming over prefix
// sums; the earliest split wins ties).  Returns the exclusive range ends.
std::vector<int> kmeans_1d(const std::vector<double> &profile, int k)
{
    const int P = (int)profile.size();
    k = std::min(k, P);
    std::vector<double> s1(P + 1, 0.0), s2(P + 1, 0.0);
    for (int i = 0; i < P; ++i) {
        s1[i + 1] = s1[i] + profile[i];
        s2[i + 1] = s2[i] + profile[i] * profile[i];
    }
    auto cost = [&](int a, int e) {
        const double t = s1[e] - s1[a];
        return (s2[e] - s2[a]) - t * t / (e - a);
    };
    const double INF = std::numeric_limits<double>::infinity();
    std::vector<std::vector<double>> dp(k + 1, std::vector<double>(P + 1, INF));
    std::vector<std::vector<int>> from(k + 1, std::vector<int>(P + 1, 0));
    dp[0][0] = 0.0;
    for (int j = 1; j <= k; ++j)
        for (int e = j; e <= P; ++e)
            for (int a = j - 1; a < e; ++a) {
                if (dp[j - 1][a] == INF) continue;
                const double c = dp[j - 1][a] + cost(a, e);
                if (c < dp[j][e]) { dp[j][e] = c; from[j][e] = a; }
            }
    std::vector<int> ends(k);
    for (int j = k, e = P; j >= 1; --j) {
        ends[j - 1] = e;
        e = from[j][e];
    }
    return ends;
}

inline int8_t quantize_one(float v, float s)
{
    float q = std::nearbyintf(v / s);  // default rounding mode: half to even
    q = std::min(127.0f, std::max(-128.0f, q));
    return (int8_t)q;
}

}  // namespace

extern "C" int quamba_reorder_params(int32_t nheads, int32_t headdim, int32_t ngroups, int32_t m, int32_t n,
                                     uint64_t /*seed*/, int32_t d_state, const float *x_calib_absmax,
                                     const float *B_calib_absmax, const float *C_calib_absmax, int32_t *head_perm,
                                     int32_t *chan_perm, float *x_scales, int32_t *head_cluster_end,
                                     int32_t *chan_cluster_end, float *B_scales, float *C_scales)
{
    if (!x_calib_absmax || !B_calib_absmax || !C_calib_absmax || !head_perm || !chan_perm || !x_scales ||
        !head_cluster_end || !chan_cluster_end || !B_scales || !C_scales)
        return QUAMBA_ENULL;
    if (nheads <= 0 || headdim <= 0 || ngroups <= 0 || m <= 0 || n <= 0 || d_state <= 0 || nheads % ngroups)
        return QUAMBA_ESHAPE;
    const int H = nheads, P = headdim, G = ngroups, hpg = H / G;
    for (size_t i = 0; i < (size_t)H * P; ++i)
        if (!(x_calib_absmax[i] >= 0.0f) || !std::isfinite(x_calib_absmax[i])) return QUAMBA_EINVAL;
    for (size_t i = 0; i < (size_t)G * d_state; ++i)
        if (!(B_calib_absmax[i] >= 0.0f) || !std::isfinite(B_calib_absmax[i]) || !(C_calib_absmax[i] >= 0.0f) ||
            !std::isfinite(C_calib_absmax[i]))
            return QUAMBA_EINVAL;

    // Per-state-group scales of B and C.
    for (int g = 0; g < G; ++g) {
        float mb = 0.0f, mc = 0.0f;
        for (int k = 0; k < d_state; ++k) {
            mb = std::max(mb, B_calib_absmax[(size_t)g * d_state + k]);
            mc = std::max(mc, C_calib_absmax[(size_t)g * d_state + k]);
        }
        B_scales[g] = scale_of_max(mb);
        C_scales[g] = scale_of_max(mc);
    }

    // Sort the channels of every head by calibrated maximum (ascending, stable).
    std::vector<int> order((size_t)H * P);
    std::vector<double> sorted((size_t)H * P);
    for (int h = 0; h < H; ++h) {
        int *o = &order[(size_t)h * P];
        const float *mx = x_calib_absmax + (size_t)h * P;
        std::iota(o, o + P, 0);
        std::stable_sort(o, o + P, [&](int a, int b) { return mx[a] < mx[b]; });
        for (int j = 0; j < P; ++j) sorted[(size_t)h * P + j] = (double)mx[o[j]];
    }

    std::fill(x_scales, x_scales + (size_t)G * m * n, 1.0f);
    std::fill(chan_cluster_end, chan_cluster_end + (size_t)G * m * n, P);
    for (int g = 0; g < G; ++g) {
        std::vector<HeadVec> hv(hpg);
        for (int i = 0; i < hpg; ++i) {
            const int h = g * hpg + i;
            double s = 0.0;
            for (int j = 0; j < P; ++j) s += sorted[(size_t)h * P + j];
            hv[i] = HeadVec{h, &sorted[(size_t)h * P], s};
        }
        const int k = std::min(m, hpg);
        const std::vector<int> label = lloyd(hv, P, k);

        // Order the clusters by mean vector sum (then by first member), heads inside a cluster by old index.
        struct Cl { double key; int first; int id; };
        std::vector<Cl> cl;
        for (int c = 0; c < k; ++c) {
            double s = 0.0;
            int members = 0, first = -1;
            for (int i = 0; i < hpg; ++i)
                if (label[i] == c) { s += hv[i].sum; ++members; if (first < 0) first = hv[i].old_index; }
            cl.push_back(Cl{s / members, first, c});
        }
        std::sort(cl.begin(), cl.end(), [](const Cl &a, const Cl &b) {
            return a.key != b.key ? a.key < b.key : a.first < b.first;
        });

        int pos = 0;
        for (int ci = 0; ci < k; ++ci) {
            std::vector<double> profile(P, 0.0);
            for (int i = 0; i < hpg; ++i)
                if (label[i] == cl[ci].id) {
                    head_perm[g * hpg + pos++] = hv[i].old_index;
                    for (int j = 0; j < P; ++j) profile[j] = std::max(profile[j], hv[i].v[j]);
                }
            head_cluster_end[g * m + ci] = pos;
            const std::vector<int> ends = kmeans_1d(profile, n);
            const size_t base = ((size_t)g * m + ci) * n;
            int a = 0;
            for (int j = 0; j < n; ++j) {
                const int e = j < (int)ends.size() ? ends[j] : P;
                chan_cluster_end[base + j] = e;
                float mx = 0.0f;
                for (int q = a; q < e; ++q) mx = std::max(mx, (float)profile[q]);
                x_scales[base + j] = e > a ? scale_of_max(mx) : 1.0f;
                a = e;
            }
        }
        for (int ci = k; ci < m; ++ci) head_cluster_end[g * m + ci] = hpg;
    }
    for (int i = 0; i < H; ++i)
        std::memcpy(chan_perm + (size_t)i * P, &order[(size_t)head_perm[i] * P], sizeof(int32_t) * P);
    return QUAMBA_OK;
}

extern "C" int quamba_gather_rows(void *dst, const void *src, const int32_t *new_to_old, int64_t rows,
                                  int64_t row_bytes)
{
    if (!dst || !src || !new_to_old) return QUAMBA_ENULL;
    if (rows < 0 || row_bytes <= 0) return QUAMBA_ESHAPE;
    for (int64_t i = 0; i < rows; ++i)
        if (new_to_old[i] < 0 || new_to_old[i] >= rows) return QUAMBA_EINVAL;
    for (int64_t i = 0; i < rows; ++i)
        std::memcpy((char *)dst + i * row_bytes, (const char *)src + (int64_t)new_to_old[i] * row_bytes,
                    (size_t)row_bytes);
    return QUAMBA_OK;
}

extern "C" int quamba_quantize_x(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *sc, int64_t tokens,
                                 const float *x, int8_t *xq)
{
    if (!shape || !sc || !x || !xq || !sc->x_scales || !sc->head_cluster_end || !sc->chan_cluster_end)
        return QUAMBA_ENULL;
    const int H = shape->nheads, P = shape->headdim, G = shape->ngroups, m = shape->n_head_clusters,
              n = shape->n_chan_clusters;
    if (tokens < 0 || H <= 0 || P <= 0 || G <= 0 || m <= 0 || n <= 0 || H % G) return QUAMBA_ESHAPE;
    const int hpg = H / G;
    std::vector<float> table((size_t)H * P);
    for (int h = 0; h < H; ++h) {
        const int g = h / hpg, hl = h % hpg;
        int i = 0;
        while (i < m - 1 && hl >= sc->head_cluster_end[g * m + i]) ++i;
        const size_t base = ((size_t)g * m + i) * n;
        for (int p = 0, j = 0; p < P; ++p) {
            while (j < n - 1 && p >= sc->chan_cluster_end[base + j]) ++j;
            table[(size_t)h * P + p] = sc->x_scales[base + j];
        }
    }
    const size_t row = (size_t)H * P;
    for (size_t k = 0; k < row; ++k)
        if (!(table[k] > 0.0f) || !std::isfinite(table[k])) return QUAMBA_EINVAL;  // Eq. 1 divides by the scale
    for (int64_t t = 0; t < tokens; ++t)
        for (size_t k = 0; k < row; ++k) xq[t * row + k] = quantize_one(x[t * row + k], table[k]);
    return QUAMBA_OK;
}

extern "C" int quamba_quantize_groups(int64_t tokens, int32_t ngroups, int32_t d_state, const float *group_scales,
                                      const float *v, int8_t *vq)
{
    if (!group_scales || !v || !vq) return QUAMBA_ENULL;
    if (tokens < 0 || ngroups <= 0 || d_state <= 0) return QUAMBA_ESHAPE;
    for (int g = 0; g < ngroups; ++g)
        if (!(group_scales[g] > 0.0f) || !std::isfinite(group_scales[g])) return QUAMBA_EINVAL;
    for (int64_t t = 0; t < tokens; ++t)
        for (int g = 0; g < ngroups; ++g) {
            const size_t o = ((size_t)t * ngroups + g) * d_state;
            for (int k = 0; k < d_state; ++k) vq[o + k] = quantize_one(v[o + k], group_scales[g]);
        }
    return QUAMBA_OK;
}

extern "C" int quamba_state_scales(int32_t nheads, int32_t headdim, int32_t ngroups, int32_t m, int32_t n,
                                   int32_t d_state, const int32_t *head_cluster_end, const int32_t *chan_cluster_end,
                                   const float *state_calib_absmax, float *state_scales)
{
    if (!head_cluster_end || !chan_cluster_end || !state_calib_absmax || !state_scales) return QUAMBA_ENULL;
    const int H = nheads, P = headdim, G = ngroups, N = d_state;
    if (H <= 0 || P <= 0 || G <= 0 || m <= 0 || n <= 0 || N <= 0 || H % G) return QUAMBA_ESHAPE;
    const int hpg = H / G;
    for (int c = 0; c < G * m; ++c) {
        const int prev = c % m ? head_cluster_end[c - 1] : 0;
        if (head_cluster_end[c] < prev || head_cluster_end[c] > hpg) return QUAMBA_EINVAL;
    }
    for (int c = 0; c < G * m * n; ++c) {
        const int prev = c % n ? chan_cluster_end[c - 1] : 0;
        if (chan_cluster_end[c] < prev || chan_cluster_end[c] > P) return QUAMBA_EINVAL;
    }
    const size_t total = (size_t)H * P * N;
    for (size_t i = 0; i < total; ++i)
        if (!(state_calib_absmax[i] >= 0.0f) || !std::isfinite(state_calib_absmax[i])) return QUAMBA_EINVAL;
    // maximum per (cell, state) over the heads and channel positions the lookup assigns to the cell
    std::vector<float> mx((size_t)G * m * n * N, 0.0f);
    for (int h = 0; h < H; ++h) {
        const int g = h / hpg, hl = h % hpg;
        int i = 0;
        while (i < m - 1 && hl >= head_cluster_end[g * m + i]) ++i;
        const size_t base = ((size_t)g * m + i) * n;
        for (int p = 0, j = 0; p < P; ++p) {
            while (j < n - 1 && p >= chan_cluster_end[base + j]) ++j;
            float *row = &mx[(base + j) * N];
            const float *src = state_calib_absmax + ((size_t)h * P + p) * N;
            for (int k = 0; k < N; ++k) row[k] = std::max(row[k], src[k]);
        }
    }
    for (size_t i = 0; i < mx.size(); ++i) state_scales[i] = scale_of_max(mx[i]);
    return QUAMBA_OK;
}
