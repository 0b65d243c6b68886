/*
 * quamba_ssd — the 8-bit Mamba2 selective scan (SSD) of Quamba2 (arXiv 2503.22879) for AMD MI355X (gfx950).
 *
 * C ABI, plain pointers and sizes.  The library computes, for every batch entry b and head h (state group
 * g = h / (nheads / ngroups)), the selective SSM of the paper's Eq. 2 with the discretisation of Section 3.2
 * (A-dot_t = exp(dt_t A_h), B-dot_t = dt_t B_t):
 *
 *      h_t = exp(dt_t A_h) h_{t-1} + dt_t B_t x_t^T ,      y_t = C_t . h_t + D_h x_t
 *
 * on quantized operands (Eq. 1, symmetric 8-bit, static scales):
 *      x = s_x(h,p) * xq   — sort-and-cluster scales of Section 4.1: inside each state group the heads are split into
 *                            m head clusters, and inside each head cluster the (sorted) channel positions are split
 *                            into n ranges; one scale per (group, head cluster, channel range);
 *      B = s_B[g] * Bq, C = s_C[g] * Cq — one scale per state group (Section 4.1, per-state-group quantization).
 * All tensors are in the SORTED/CLUSTERED head and channel order that the offline weight reordering of
 * Section 4.2 makes the projections produce; quamba_reorder_params() computes that order and the scale tables.
 *
 * Conventions for every entry point
 *   - returns QUAMBA_OK (0) or a negative quamba_status; never throws, never allocates device memory;
 *   - prefill/decode only ENQUEUE work on the caller's stream (a hipStream_t passed as void*, NULL = default stream)
 *     and never synchronise; the caller owns every buffer and keeps it alive until the stream has drained;
 *   - all tensors are dense row-major in the stated shape; pointers named "device" must be device-accessible,
 *     pointers named "host" must be host memory; the two structs are host structs (their members may be device
 *     pointers as stated);
 *   - arguments are validated before anything is enqueued, so validation errors can be observed without a GPU.
 *     Cluster boundary tables live on the device and are trusted (not read back).
 */
#ifndef QUAMBA_SSD_H_
#define QUAMBA_SSD_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum quamba_status {
    QUAMBA_OK = 0,
    QUAMBA_ENULL = -1,      /* a required pointer is NULL                                   */
    QUAMBA_ESHAPE = -2,     /* a dimension is non-positive, inconsistent or unsupported      */
    QUAMBA_EWORKSPACE = -3, /* a shape needs more scratch memory than an entry point with a fixed scratch area has */
    QUAMBA_EHIP = -4,       /* the HIP runtime refused the launch (no device, bad stream ...) */
    QUAMBA_EINVAL = -5      /* an argument value is invalid (unknown flag, bad permutation ...) */
} quamba_status;

/* flags of quamba_ssd_shape_t */
#define QUAMBA_FLAG_GENERIC_KERNEL 0x1u /* prefill: use the shape-agnostic sequential kernel even where the
                                           chunked MFMA kernel applies (a cross-check, not a fast path)      */
#define QUAMBA_FLAG_PRECISE_STATE 0x2u  /* prefill: compute chunk states with a two-term fp16 product so       
                                           that final_state meets 1e-4 of its max; implied when final_state
                                           is requested, settable to get the same arithmetic without it       */
#define QUAMBA_FLAG_NO_CHANNEL_SPLIT 0x4u /* prefill: keep one workgroup per (sequence, head) even when the batch
                                           has fewer heads than the device has compute units (by default such
                                           batches give every head two workgroups of 32 channels each); the
                                           results of the two launch shapes agree to rounding                  */

#define QUAMBA_FLAG_NO_DECAY_SKIP 0x8u  /* prefill: also compute the products whose decay factor exp(sum of dt*A)
                                           over the tokens between their operands is below 2^-32 (by default the
                                           chunked kernel leaves such 32-token blocks out: the carried-state term of
                                           an output block, score blocks far below the diagonal, a block's share of
                                           the chunk state; what is left out is below 2.4e-10 of the term's own
                                           undecayed size, five orders under the tightest tolerance)          */

#define QUAMBA_FLAG_NO_SEQ_SPLIT 0x10u  /* prefill: walk every sequence with one workgroup (or pair of workgroups) from
                                           its first to its last token even when the batch is too short to fill the
                                           chip (by default such batches are cut into up to 8 segments: a first
                                           launch computes the state at the end of every segment, a second one gives
                                           every segment its own workgroups; the results agree to rounding)       */

typedef struct quamba_ssd_shape_t {
    int32_t batch;           /* sequences                                                             */
    int32_t seqlen;          /* tokens per sequence (ignored by decode)                               */
    int32_t nheads;          /* H, multiple of ngroups                                                */
    int32_t headdim;         /* P, channels per head                                                  */
    int32_t d_state;         /* N, states per group                                                   */
    int32_t ngroups;         /* G, state groups sharing B and C                                       */
    int32_t chunk;           /* Q, SSD chunk length for prefill (ignored by decode)                   */
    int32_t n_head_clusters; /* m, head clusters per state group                                      */
    int32_t n_chan_clusters; /* n, channel ranges per head cluster                                    */
    uint32_t flags;          /* QUAMBA_FLAG_*                                                         */
} quamba_ssd_shape_t;

/* Sort-and-cluster result in the reordered index space (Section 4.1).  For prefill/decode every member is a
 * DEVICE pointer; quamba_reorder_params() fills HOST arrays of the same sizes. */
typedef struct quamba_ssd_scales_t {
    const float *x_scales;           /* [ngroups*m*n]  scale of (group, head cluster, channel range)              */
    const int32_t *head_cluster_end; /* [ngroups*m]    exclusive end head index of each head cluster, counted
                                                       inside its group (0..H/G], non-decreasing, last == H/G      */
    const int32_t *chan_cluster_end; /* [ngroups*m*n]  exclusive end channel position (0..P], non-decreasing,
                                                       last of each head cluster == P                              */
    const float *B_scales;           /* [ngroups] */
    const float *C_scales;           /* [ngroups] */
} quamba_ssd_scales_t;

/*
 * Bytes of device workspace with which quamba_ssd_prefill runs this shape fastest on the current device (may be 0).
 * Non-zero only for batches short enough for the sequence split of the matrix-core kernel
 * (QUAMBA_FLAG_NO_SEQ_SPLIT): the states at the segment boundaries, (segments - 1) * batch * nheads *
 * (headdim * d_state + 1) floats.  A call with a NULL, smaller or not 16-byte aligned workspace is not an error: it
 * takes the unsplit launch (same results to rounding, slower on such batches).  The workspace is scratch: written
 * and read by the call's own launches, contents undefined afterwards; calls that share one workspace must not
 * overlap.  Returns 0 for an invalid shape; quamba_ssd_prefill reports the error.
 */
size_t quamba_ssd_prefill_workspace_size(const quamba_ssd_shape_t *shape);

/*
 * Chunked prefill of the 8-bit SSD (Eq. 2 over a whole sequence; the chunked matmul form is the SSD algorithm the
 * paper's Section 3.2 "Mamba2" refers to, applied to the quantized operands of Section 4.1).
 *   x  device int8  [batch, seqlen, nheads, headdim]     B, C  device int8 [batch, seqlen, ngroups, d_state]
 *   dt device fp32  [batch, seqlen, nheads]  final step size (softplus and bias already applied), >= 0
 *   A  device fp32  [nheads], <= 0           D  device fp32 [nheads] or NULL (no skip term)
 *   init_state  device fp32 [batch, nheads, headdim, d_state] or NULL (zero state)
 *   y           device fp16 [batch, seqlen, nheads, headdim]   (written, round-to-nearest-even)
 *   final_state device fp32 [batch, nheads, headdim, d_state] or NULL (not returned); may alias init_state (an update
 *               in place; such a call is never cut along the sequence)
 *   workspace   device scratch of workspace_bytes, 16-byte aligned; NULL or fewer bytes than
 *               quamba_ssd_prefill_workspace_size(shape) select the launch that needs none
 * Any seqlen >= 1 is accepted; a last partial chunk is processed as if padded with dt = 0, x = 0 steps (identity
 * steps of Eq. 2) whose outputs are not written.  Errors: ENULL, ESHAPE (nheads % ngroups, non-positive sizes,
 * headdim*d_state too large for the generic kernel), EHIP.
 * Operand ranges of the matrix-core kernel (headdim 64, d_state 128), which narrows its operands to fp16 after fixed
 * power-of-two scalings and does not check them (they live on the device; outside them the result becomes inf or
 * NaN without an error; QUAMBA_FLAG_GENERIC_KERNEL computes in fp32 and has none of the three limits):
 *   - 0 <= dt <= 16 (a softplus output far above any trained step size; the decayed scores times dt/4 must stay
 *     below 65504) and A <= 0 (every decay exponent is formed for a non-rising prefix sum);
 *   - every scale of `scales` finite and > 0 (an initial state is divided by s_x s_B);
 *   - |state| / (s_x s_B) < 8e6 at every chunk boundary (the fp16 copy of the carried state): holds for full-scale
 *     codes whenever |A_h| dt stays above about 3e-4 per token on average, and for any init_state of that size.
 */
int quamba_ssd_prefill(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *x,
                       const int8_t *B, const int8_t *C, const float *dt, const float *A, const float *D,
                       const float *init_state, uint16_t *y, float *final_state, void *workspace,
                       size_t workspace_bytes, void *hip_stream);

/*
 * quamba_ssd_prefill for callers that cannot provide a workspace and must not allocate: code under HIP graph
 * capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments and results as quamba_ssd_prefill
 * without the workspace; the scratch memory of the sequence split is a fixed area of 16 MiB inside the library's
 * device image (one per GPU, held until the process ends), enough for every shape the matrix-core kernel takes.
 * The call allocates nothing and synchronises nothing.  All calls on one GPU share that area: calls that overlap in
 * time on the same GPU (different streams) race on it and must be ordered by the caller; nothing in it has to be
 * cleared between calls (a call writes what it reads).
 * Errors: as quamba_ssd_prefill, and EWORKSPACE for a shape whose split would need more than the fixed area.
 */
int quamba_ssd_prefill_noalloc(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *x,
                               const int8_t *B, const int8_t *C, const float *dt, const float *A, const float *D,
                               const float *init_state, uint16_t *y, float *final_state, void *hip_stream);

/*
 * Single-token decode: one application of Eq. 2 on a persistent state, the step the paper identifies as the
 * generation bottleneck at large batch (Appendix E, "The cached state sizes").
 *   x device int8 [batch, nheads, headdim]    B, C device int8 [batch, ngroups, d_state]
 *   dt device fp32 [batch, nheads]            A, D as in prefill (D may be NULL)
 *   state device fp32 [batch, nheads, headdim, d_state], read and overwritten IN PLACE (the only in/out buffer)
 *   y device fp16 [batch, nheads, headdim]
 * seqlen and chunk of the shape are ignored.  Errors: ENULL, ESHAPE, EHIP.
 */
int quamba_ssd_decode_step(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *x,
                           const int8_t *B, const int8_t *C, const float *dt, const float *A, const float *D,
                           float *state, uint16_t *y, void *hip_stream);

/*
 * Optional 8-bit side inputs of the SSD kernels (Section 5.2 lists x, the step size, B, C and z as the kernel's 8-bit
 * loads).  Host struct of device pointers.
 *   z        int8, laid out like x ([batch, seqlen, nheads, headdim] for prefill, [batch, nheads, headdim] for decode),
 *            reordered like x; the output becomes y * SiLU(z_scale * z) (Section 3.2: the optional residual branch z
 *            multiplies the SSM output y = C h + D x before the output projection).  NULL: no gate.
 *   dt_q     int8, laid out like dt: Eq. 1 codes of the step size's pre-activation; the step size becomes
 *            softplus(dt_scale * dt_q + dt_bias[h]) (Section 3.2) and the fp32 `dt` argument is ignored (may be
 *            NULL).  NULL: `dt` is used as is.
 *   dt_bias  fp32 [nheads] or NULL (zero); only read with dt_q.
 */
typedef struct quamba_ssd_gate_t {
    const int8_t *z;
    float z_scale;
    const int8_t *dt_q;
    float dt_scale;
    const float *dt_bias;
} quamba_ssd_gate_t;

/*
 * quamba_ssd_prefill / quamba_ssd_decode_step / quamba_ssd_decode_step_q8 with the side inputs above; `gate` may be
 * NULL (then they are the plain entry points).  Everything else as documented there.  The 8-bit-state step takes the
 * gate only: its re-quantization decision is defined on the caller's fp32 dt, so dt_q must be NULL there (EINVAL).
 * Errors: as the plain entry points, plus EINVAL for non-finite or non-positive scales.
 */
int quamba_ssd_prefill_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                             const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B, const int8_t *C,
                             const float *dt, const float *A, const float *D, const float *init_state, uint16_t *y,
                             float *final_state, void *workspace, size_t workspace_bytes, void *hip_stream);
int quamba_ssd_decode_step_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                 const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B, const int8_t *C,
                                 const float *dt, const float *A, const float *D, float *state, uint16_t *y,
                                 void *hip_stream);
int quamba_ssd_decode_step_q8_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                    const quamba_ssd_gate_t *gate, const float *state_scales, const int8_t *x,
                                    const int8_t *B, const int8_t *C, const float *dt, const float *A, const float *D,
                                    int8_t *state_q, uint16_t *y, void *hip_stream);

/*
 * The same decode step on an 8-BIT CACHED STATE (Appendix E, "Quantizing cached SSM states"): the state is cached as
 * int8 codes whose scales reuse the m x n (head cluster, channel range) cells of x and differ per state, i.e.
 * d_state x m x n scales per state group.  One step de-quantizes the state (inverse of Eq. 1), applies Eq. 2, forms y
 * from the updated state, and re-quantizes the state (Eq. 1) in place.
 *   state_scales device fp32 [ngroups*m*n, d_state], all > 0 (quamba_state_scales produces them)
 *   state_q      device int8 [batch, nheads, headdim, d_state], read and overwritten IN PLACE
 *   everything else as in quamba_ssd_decode_step; dt >= 0 and A <= 0 are required (the decay is computed for
 *   dt*A <= 0 only).
 * The new code is decided in fp32, every operation rounded to nearest even on its own, in this order:
 *   xv = s_x(h,p)*x;  dtx = dt*xv;  Bv = s_B[g]*B[n];  u = dtx*Bv;  sd = dA*s[cell,n];  d = sd*code;  hn = d + u;
 *   r = hn*(1/s[cell,n]);  code' = clamp(rint(r), -127, 127)   with ties to even,
 * where dA = exp(dt*A) is evaluated as t = (dt*A)*log2(e) (fp32 constant 0x3FB8AA3B), k = rint(t), f = t - k,
 * 2^f by Horner's rule on the fp32-rounded coefficients (ln 2)^i / i!, i = 7..0 (multiply and add rounded
 * separately), times 2^k; 0 when t < -125.  y = sum_n (s_C[g]*C[n])*hn + D*xv in fp32, rounded to fp16.
 * The codes of the cached state stay within [-127, 127]: narrower on the negative side than Eq. 1's 8-bit range
 * [-128, 127], on purpose.  The scales are (calibrated maximum) / 127, so the grid is symmetric, and an element is
 * re-quantized at every step: a code of -128 would let a saturated negative state sit one step beyond the
 * calibrated maximum where a positive one cannot.
 * Errors: ENULL, ESHAPE, EHIP.
 */
int quamba_ssd_decode_step_q8(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                              const float *state_scales, const int8_t *x, const int8_t *B, const int8_t *C,
                              const float *dt, const float *A, const float *D, int8_t *state_q, uint16_t *y,
                              void *hip_stream);

/*
 * Eq. 1 on a device fp32 state with the scales of the cached state (what a prefill's final state goes through before
 * it is cached in 8 bits): state_q = clamp(rint(state * (1/s[cell,n])), -127, 127), the reciprocal and the product
 * rounded to fp32 one after the other, ties to even.
 *   state device fp32 [batch, nheads, headdim, d_state]   state_q device int8, same shape (must not overlap state)
 * Errors: ENULL, ESHAPE, EHIP.
 */
int quamba_ssd_quantize_state(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                              const float *state_scales, const float *state, int8_t *state_q, void *hip_stream);

/*
 * Static scales of the 8-bit cached state from calibrated maxima (absolute-maximum calibration, Appendix C,
 * "Quantization setup"; cells of Appendix E).  HOST function, all pointers host memory.
 *   head_cluster_end [ngroups*m], chan_cluster_end [ngroups*m*n]: as in quamba_ssd_scales_t
 *   state_calib_absmax [nheads*headdim*d_state]: calibrated max |h| per state element, heads and channels in the
 *                      reordered order
 *   state_scales [ngroups*m*n*d_state] (written): (max over the heads and channel positions of the cell) / 127,
 *                      1.0 for an empty or all-zero cell
 * Errors: ENULL, ESHAPE, EINVAL (negative or non-finite maxima, boundaries out of range or decreasing).
 */
int quamba_state_scales(int32_t nheads, int32_t headdim, int32_t ngroups, int32_t m, int32_t n, int32_t d_state,
                        const int32_t *head_cluster_end, const int32_t *chan_cluster_end,
                        const float *state_calib_absmax, float *state_scales);

/*
 * Quantized Hadamard transform of the SSD output (Section 4.2, "Offline Hadamard matrix fusion" and "Efficient
 * 4-bit/8-bit Mamba blocks"): out = Eq. 1 of (1/s_y) H_n y for every row, H_n a Hadamard matrix of order n (entries +-1,
 * no normalisation), the 8-bit input of an output projection whose weight carries H_n offline.
 *   y   device fp16 [rows, n] (the flattened [.., nheads*headdim] output of the scan, gated or not)
 *   out device int8 [rows, n]; must not overlap y
 *   n   2^k (2 <= n <= 16384), or 12 * 2^k or 20 * 2^k with k >= 2 (48 <= n <= 16384: the widths 1536, 3072, 5120 of the
 *       Mamba blocks);  s_y > 0 the static scale of the transformed output
 * n = 2^k: H_n is the Sylvester matrix, evaluated in fp32 as the radix-2 butterfly network with strides 1, 2, 4, ..., n/2
 * in this order (stage h replaces (v[i], v[i+h]), i & h == 0, by (v[i] + v[i+h], v[i] - v[i+h])), every operation
 * rounded on its own.  n = m * 2^k, m = 12 or 20: H_n = H_m (x) H_{2^k} (Kronecker product, H_m on the slow index), H_m =
 * I + S by Paley's first construction with q = m - 1: S[0][b] = 1, S[a][0] = -1, S[a][b] = chi(a - b mod q) for a, b >= 1
 * (chi = +1 on the non-zero squares mod q, -1 on the others, 0 at 0); the butterfly network runs inside every block of
 * 2^k consecutive values, then element (a, j) is the sum over the blocks b = 0, 1, ..., m-1 of H_m[a][b] * block_b[j],
 * accumulated in this order with every addition rounded to fp32.
 * Then code = clamp(rint(v * (1/s_y)), -128, 127) with 1/s_y and the product rounded to fp32, ties to even.
 * Errors: ENULL, ESHAPE (unsupported n, rows < 0 or > 2^31 - 1), EINVAL (s_y), EHIP.
 */
int quamba_hadamard_quantize(const uint16_t *y, int64_t rows, int32_t n, float s_y, int8_t *out, void *hip_stream);

/*
 * The 8-bit Mamba1 selective scan (Section 3.2, Eq. 2 with the Mamba1 parameterisation: per-channel step size, A a
 * [channels, states] matrix, B_t and C_t shared by all channels; Section 4.2 lists the 8-bit selective-scan kernel):
 *   h_t[d,n] = exp(dt_t[d] A[d,n]) h_{t-1}[d,n] + dt_t[d] B_t[n] x_t[d],    y_t[d] = sum_n C_t[n] h_t[d,n] + D[d] x_t[d]
 * with x = s_x(d) x_code, one scale per channel range (sort-and-cluster of Section 4.1 for a block without heads),
 * B = s_B B_code, C = s_C C_code (one state group).  Tensors are channel-major with time last, as in the Mamba1 block.
 * shape: nheads = 1, ngroups = 1, n_head_clusters = 1; headdim = number of channels D; d_state = N; n_chan_clusters =
 * number of channel ranges; scales: x_scales [n_chan_clusters], chan_cluster_end [n_chan_clusters] (exclusive ends on
 * the sorted channel positions), head_cluster_end [1] = {1}, B_scales [1], C_scales [1]  (all device).
 *   x  device int8 [batch, D, seqlen]        B, C  device int8 [batch, N, seqlen]       dt  device fp32 [batch, D, seqlen]
 *   A  device fp32 [D, N] (<= 0)             D     device fp32 [D] or NULL
 *   init_state  device fp32 [batch, D, N] or NULL (zero)      final_state  device fp32 [batch, D, N] or NULL
 *   y  device fp16 [batch, D, seqlen]
 * d_state = 16, seqlen a multiple of 16 and 16-byte aligned tensors take the wave-scan kernel; other shapes (d_state
 * <= 64) or QUAMBA_FLAG_GENERIC_KERNEL a one-thread-per-channel kernel.  fp32 throughout; y rounded to fp16.
 * Errors: ENULL, ESHAPE, EINVAL, EHIP.
 */
int quamba_mamba1_scan(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *x,
                       const int8_t *B, const int8_t *C, const float *dt, const float *A, const float *D,
                       const float *init_state, uint16_t *y, float *final_state, void *hip_stream);

/*
 * One generation step of the same recurrence on a persistent fp32 state, in place.
 *   x device int8 [batch, D];  B, C device int8 [batch, N];  dt device fp32 [batch, D];  state device fp32 [batch, D, N]
 *   (in/out);  y device fp16 [batch, D];  A, D, shape (seqlen ignored) and scales as above; any d_state.
 */
int quamba_mamba1_decode_step(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *x,
                              const int8_t *B, const int8_t *C, const float *dt, const float *A, const float *D,
                              float *state, uint16_t *y, void *hip_stream);

/*
 * quamba_mamba1_scan / quamba_mamba1_decode_step with the 8-bit side inputs of quamba_ssd_gate_t (Section 3.2: the step
 * size is softplus of a quantized projection plus a bias, and the branch z gates the output); `gate` may be NULL.
 *   gate->z        int8, laid out like x ([batch, D, seqlen] / [batch, D]): y becomes y * SiLU(z_scale * z)
 *   gate->dt_q     int8, laid out like dt: the step size becomes softplus(dt_scale * dt_q + dt_bias[d]); `dt` is then
 *                  ignored and may be NULL
 *   gate->dt_bias  fp32 [D] (one per channel) or NULL
 * The wave-scan kernel additionally needs z and dt_q 16-byte aligned.  Errors as the plain entry points, plus EINVAL for
 * non-finite or non-positive scales.
 */
int quamba_mamba1_scan_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                             const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B, const int8_t *C,
                             const float *dt, const float *A, const float *D, const float *init_state, uint16_t *y,
                             float *final_state, void *hip_stream);
int quamba_mamba1_decode_step_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                    const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B, const int8_t *C,
                                    const float *dt, const float *A, const float *D, float *state, uint16_t *y,
                                    void *hip_stream);

/*
 * W8A8 causal convolution in front of the scan (Section 4.2, "Efficient 4-bit/8-bit Mamba blocks": the W8A8 causal
 * convolution kernel; "Offline Hadamard matrix fusion" / reordering: its channels come in the sorted order, so its
 * outputs are the SSD kernel's operands as they are).  Depthwise over time, 4 taps, over the concatenated channels
 * [x | B | C] (Ct = nheads*headdim + 2*ngroups*d_state), then bias, SiLU and Eq. 1:
 *   acc[t,c] = sum_{k=0..3} weight[c,k] * in[t-3+k, c]      (exact integers; tap 3 meets the current token; tokens
 *                                                            before the sequence come from conv_state_in, else zero)
 *   out[t,c] = Eq. 1 of SiLU(in_w_scale * acc + bias[c]) / s_out[c]
 * with s_out the cell scale of (head, channel position) for x (Section 4.1, sort-and-cluster) and the state group's
 * scale for B and C (per-state-group quantization).  The code is decided in fp32, every operation rounded on its own:
 *   v = float(acc) * in_w_scale;  v = v + bias[c];  e = exp(-|v|);  den = 1 + e;  num = v >= 0 ? v : v * e;
 *   a = num / den;  r = a * (1 / s_out[c]);  code = clamp(rint(r), -128, 127), ties to even;
 * both divisions correctly rounded, and exp evaluated as t = z * log2(e) (fp32 constant 0x3FB8AA3B), k = rint(t),
 * f = t - k, a degree-7 Horner polynomial in f with separately rounded multiplies and adds (coefficients the fp32
 * roundings of (ln 2)^i / i!), scaled by 2^k, and 0 for t < -125.
 *   in             device int8 [batch, seqlen, Ct]          weight  device int8 [Ct, 4]
 *   bias           device fp32 [Ct] or NULL                 in_w_scale = (input scale) * (weight scale) > 0
 *   conv_state_in  device int8 [batch, 3, Ct] or NULL (the 3 input tokens before the sequence, oldest first)
 *   conv_state_out device int8 [batch, 3, Ct] or NULL: the last 3 input tokens after this call (for seqlen < 3 the tail
 *                  of the old state moves up); may be the same buffer as conv_state_in only when seqlen <= 16
 *   x_out device int8 [batch, seqlen, nheads, headdim];  B_out, C_out device int8 [batch, seqlen, ngroups, d_state]
 * shape: batch, seqlen, nheads, headdim, d_state, ngroups and the cluster counts are used; scales as for the prefill.
 * Shapes with headdim and d_state multiples of 16 and 16-byte aligned tensors take the vector kernel, others a
 * one-thread-per-channel kernel with the same results.
 * Errors: ENULL, ESHAPE, EINVAL (in_w_scale; aliased states with seqlen > 16), EHIP.
 */
int quamba_conv1d_q8(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *in,
                     const int8_t *weight, const float *bias, float in_w_scale, const int8_t *conv_state_in,
                     int8_t *x_out, int8_t *B_out, int8_t *C_out, int8_t *conv_state_out, void *hip_stream);

/*
 * Offline sort-and-cluster (Section 4.1) and the index tables for cluster-aware weight reordering (Section 4.2).
 * HOST function, all pointers host memory.
 *   x_calib_absmax [nheads*headdim]  calibrated per-channel max|x| in the model's original order
 *   B_calib_absmax, C_calib_absmax [ngroups*d_state] calibrated per-state max|B|, max|C|
 * Outputs:
 *   head_perm [nheads]          new head index -> old head index (heads never leave their state group)
 *   chan_perm [nheads*headdim]  row i (NEW head i): sorted channel position -> old channel of that head
 *   x_scales, head_cluster_end, chan_cluster_end, B_scales, C_scales: as in quamba_ssd_scales_t
 * Steps: sort each head's channels by calibrated max (ascending); per state group, k-means (Lloyd, deterministic
 * start, <= 50 rounds) of the heads on their sorted-max vectors into m clusters, clusters ordered by magnitude;
 * per head cluster, exact 1-D k-means of the max-profile over sorted positions into n contiguous ranges; every
 * scale = (max of its cell) / 127 (Eq. 1, N = 8), 1.0 for an empty or all-zero cell.  `seed` is reserved (the
 * default procedure draws no random numbers).  Errors: ENULL, ESHAPE, EINVAL (negative or non-finite maxima).
 */
int quamba_reorder_params(int32_t nheads, int32_t headdim, int32_t ngroups, int32_t m, int32_t n, uint64_t seed,
                          int32_t d_state, const float *x_calib_absmax, const float *B_calib_absmax,
                          const float *C_calib_absmax, int32_t *head_perm, int32_t *chan_perm, float *x_scales,
                          int32_t *head_cluster_end, int32_t *chan_cluster_end, float *B_scales, float *C_scales);

/*
 * Apply a permutation to the rows of any host matrix: dst row i = src row new_to_old[i] (Section 4.2: in-projection
 * output columns as rows of W^T, conv channels, norm weights, out-projection input rows, A, D, dt_bias).
 * dst and src must not overlap.  Errors: ENULL, ESHAPE, EINVAL (index out of range).
 */
int quamba_gather_rows(void *dst, const void *src, const int32_t *new_to_old, int64_t rows, int64_t row_bytes);

/*
 * Eq. 1 on the host, with the static scales above (fp32 division, round half to even, clamp to [-128,127]).
 *   quamba_quantize_x:      x [tokens, nheads, headdim] fp32, already in reordered order -> xq int8, same shape;
 *                           scales is a struct of HOST pointers.
 *   quamba_quantize_groups: v [tokens, ngroups, d_state] fp32 -> int8 with group_scales [ngroups] (B or C).
 * Errors: ENULL, ESHAPE, EINVAL (a scale that is not finite and > 0: Eq. 1 divides by it).
 */
int quamba_quantize_x(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *host_scales, int64_t tokens,
                      const float *x, int8_t *xq);
int quamba_quantize_groups(int64_t tokens, int32_t ngroups, int32_t d_state, const float *group_scales,
                           const float *v, int8_t *vq);

/* Static description of a quamba_status value. */
const char *quamba_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* QUAMBA_SSD_H_ */
