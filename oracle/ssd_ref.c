/*
 * TEST INFRASTRUCTURE — the CPU oracle of the 8-bit Mamba2 selective scan.
 *
 * A plain, slow, sequential fp64 evaluation of the selective SSM of the Quamba2 paper
 * (arXiv 2503.22879) on de-quantized int8 inputs.  Only tests, the smoke check and the
 * benchmark's CPU-baseline leg may build or call this file; the product (the HIP library)
 * shares no code with it.
 *
 * What is computed, per batch entry b and head h (state group g = h / (H/G)):
 *
 *     h_t = exp(dt_t * A_h) * h_{t-1} + dt_t * B_t x_t^T        (Eq. 2 with the
 *     y_t = C_t . h_t + D_h * x_t                                 discretisation of Sec. 3.2:
 *                                                                 A-dot = exp(dt A), B-dot ~ dt B)
 *
 * with x = s_x(h,p) * xq (the m x n sort-and-cluster scales of Sec. 4.1), B = s_B[g] * Bq and
 * C = s_C[g] * Cq (one scale per state group, Sec. 4.1 "Per-state-group quantization"),
 * de-quantized as the inverse of Eq. 1.  y uses the state AFTER the update of step t (Eq. 2).
 * Time is walked one step at a time; there is no chunking, blocking or re-association.  The only
 * parallelism is an OpenMP loop over the independent (b,h) pairs.
 *
 * Pins (tests/test_oracle_pins.py): closed forms (constant inputs -> geometric series; impulse
 * response), exact integer arithmetic when A = 0, dt = 1 and all scales are 1, dt = 0 -> y = D x
 * (+ C h0), linearity in the scales, head/channel permutation invariance, and agreement with two
 * independent evaluations written in the tests (the chunked form and the O(L^2) dual form).
 */
#include <math.h>
#include <stddef.h>
#include <stdint.h>
#include <stdlib.h>
#ifdef _OPENMP
#include <omp.h>
#endif

typedef struct {
    int32_t batch, seqlen, nheads, headdim, d_state, ngroups;
    int32_t m; /* head clusters per state group   */
    int32_t n; /* channel clusters per head cluster */
} ssd_ref_shape;

/* Scale of channel p of head h (both in sorted/clustered order): walk the cluster boundaries. */
static double x_scale_of(const ssd_ref_shape *s, const float *x_scales, const int32_t *head_cluster_end,
                         const int32_t *chan_cluster_end, int h, int p)
{
    const int hpg = s->nheads / s->ngroups;
    const int g = h / hpg, hl = h % hpg;
    int i = 0;
    while (i < s->m - 1 && hl >= head_cluster_end[g * s->m + i]) ++i;
    const int base = (g * s->m + i) * s->n;
    int j = 0;
    while (j < s->n - 1 && p >= chan_cluster_end[base + j]) ++j;
    return (double)x_scales[base + j];
}

/* One time step of Eq. 2 for one (b,h): updates state[P][N] in place, writes y[P]. */
static void ssd_ref_step(int P, int N, const double *sx /*[P]*/, double sB, double sC, const int8_t *xq /*[P]*/,
                         const int8_t *Bq /*[N]*/, const int8_t *Cq /*[N]*/, double dt, double A, double D,
                         double *state, double *y)
{
    const double dA = exp(dt * A);
    for (int p = 0; p < P; ++p) {
        const double xv = sx[p] * (double)xq[p];
        double acc = 0.0;
        double *hp = state + (size_t)p * N;
        for (int n = 0; n < N; ++n) {
            const double Bv = sB * (double)Bq[n];
            const double Cv = sC * (double)Cq[n];
            hp[n] = dA * hp[n] + dt * Bv * xv;
            acc += Cv * hp[n];
        }
        y[p] = acc + D * xv;
    }
}

/*
 * Prefill.  Layouts (row-major): xq [b,L,H,P], Bq/Cq [b,L,G,N], dt [b,L,H], A/D [H] (D may be NULL),
 * init_state [b,H,P,N] fp64 or NULL (= 0).  `pairs` lists npairs (b,h) couples as 2*npairs ints, or
 * NULL for all of them in (b,h) order.  Outputs are packed per listed pair: y_out [npairs,L,P],
 * state_out [npairs,P,N] (either may be NULL).  Returns the number of threads used, <0 on bad input.
 */
int ssd_ref_prefill(const ssd_ref_shape *s, const float *x_scales, const int32_t *head_cluster_end,
                    const int32_t *chan_cluster_end, const float *B_scales, const float *C_scales,
                    const int8_t *xq, const int8_t *Bq, const int8_t *Cq, const float *dt, const float *A,
                    const float *D, const double *init_state, const int32_t *pairs, int64_t npairs,
                    double *y_out, double *state_out, int nthreads)
{
    if (!s || s->ngroups <= 0 || s->nheads % s->ngroups) return -1;
    const int L = s->seqlen, H = s->nheads, P = s->headdim, N = s->d_state, G = s->ngroups;
    const int hpg = H / G;
    const int64_t total = pairs ? npairs : (int64_t)s->batch * H;
    int used = 1;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
    used = nthreads;
#pragma omp parallel for schedule(dynamic, 1) num_threads(nthreads)
#endif
    for (int64_t u = 0; u < total; ++u) {
        const int b = pairs ? pairs[2 * u] : (int)(u / H);
        const int h = pairs ? pairs[2 * u + 1] : (int)(u % H);
        const int g = h / hpg;
        double *state = (double *)calloc((size_t)P * N, sizeof(double));
        double *sx = (double *)malloc((size_t)P * sizeof(double));
        double *yrow = (double *)malloc((size_t)P * sizeof(double));
        for (int p = 0; p < P; ++p) sx[p] = x_scale_of(s, x_scales, head_cluster_end, chan_cluster_end, h, p);
        if (init_state) {
            const double *src = init_state + ((size_t)b * H + h) * P * N;
            for (size_t k = 0; k < (size_t)P * N; ++k) state[k] = src[k];
        }
        const double sB = (double)B_scales[g], sC = (double)C_scales[g];
        for (int t = 0; t < L; ++t) {
            const size_t bt = (size_t)b * L + t;
            ssd_ref_step(P, N, sx, sB, sC, xq + (bt * H + h) * P, Bq + (bt * G + g) * N, Cq + (bt * G + g) * N,
                         (double)dt[bt * H + h], (double)A[h], D ? (double)D[h] : 0.0, state, yrow);
            if (y_out)
                for (int p = 0; p < P; ++p) y_out[((size_t)u * L + t) * P + p] = yrow[p];
        }
        if (state_out)
            for (size_t k = 0; k < (size_t)P * N; ++k) state_out[(size_t)u * P * N + k] = state[k];
        free(state);
        free(sx);
        free(yrow);
    }
    return used;
}

/*
 * Decode: one step of Eq. 2 for every (b,h) on a caller-held fp64 state [b,H,P,N], updated in place.
 * xq [b,H,P], Bq/Cq [b,G,N], dt [b,H]; y_out [b,H,P].  seqlen of the shape is ignored.
 */
int ssd_ref_decode_step(const ssd_ref_shape *s, const float *x_scales, const int32_t *head_cluster_end,
                        const int32_t *chan_cluster_end, const float *B_scales, const float *C_scales,
                        const int8_t *xq, const int8_t *Bq, const int8_t *Cq, const float *dt, const float *A,
                        const float *D, double *state, double *y_out, int nthreads)
{
    if (!s || s->ngroups <= 0 || s->nheads % s->ngroups) return -1;
    const int H = s->nheads, P = s->headdim, N = s->d_state, G = s->ngroups;
    const int hpg = H / G;
    const int64_t total = (int64_t)s->batch * H;
    int used = 1;
#ifdef _OPENMP
    if (nthreads <= 0) nthreads = omp_get_max_threads();
    used = nthreads;
#pragma omp parallel for schedule(static) num_threads(nthreads)
#endif
    for (int64_t u = 0; u < total; ++u) {
        const int b = (int)(u / H), h = (int)(u % H), g = h / hpg;
        double *sx = (double *)malloc((size_t)P * sizeof(double));
        for (int p = 0; p < P; ++p) sx[p] = x_scale_of(s, x_scales, head_cluster_end, chan_cluster_end, h, p);
        ssd_ref_step(P, N, sx, (double)B_scales[g], (double)C_scales[g], xq + (size_t)u * P,
                     Bq + ((size_t)b * G + g) * N, Cq + ((size_t)b * G + g) * N, (double)dt[u], (double)A[h],
                     D ? (double)D[h] : 0.0, state + (size_t)u * P * N, y_out + (size_t)u * P);
        free(sx);
    }
    return used;
}
