/*
 * quamba_probe — measurement helpers of the benchmark harness (NOT part of the method): small kernels that measure what
 * this machine attains for the two resources the rooflines are priced against, and the shader clock it runs at.
 * The benchmark reports its kernels' fractions of these measured figures beside the fractions of the published peaks.
 * They live in the same library so that the harness needs no second build product; nothing in the scan calls them.
 *
 * Conventions as in quamba_ssd.h: plain pointers and sizes, work is only ENQUEUED on the caller's stream (a
 * hipStream_t passed as void*), nothing is allocated, nothing synchronises; returns QUAMBA_OK or a negative status.
 */
#ifndef QUAMBA_PROBE_H_
#define QUAMBA_PROBE_H_

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

/* Register-resident matrix-core loop: waves_per_simd (1..8) waves on every SIMD of the device each issue `iters` rounds of 4 independent
 * v_mfma_f32_32x32x16_f16 (kind 0) or v_mfma_i32_32x32x32_i8 (kind 1) on operands that never leave its registers
 * (no memory traffic inside the loop), so the elapsed time of the launch gives the matrix-core rate the machine
 * sustains.  uniform_operands != 0 gives every lane the same operand values (the matrix cores then draw less power and
 * the board stays below its cap: the figure comes out near the published peak); 0 gives every lane its own values, as
 * a real contraction has them.  *ops_out (host) receives the number of multiply-add operations x 2 the launch performs
 * (32*32*16*2 per fp16 instruction, 32*32*32*2 per int8 instruction).  sink (device, >= 4 bytes) receives one word so
 * that the loop cannot be removed.  Errors: QUAMBA_ENULL, QUAMBA_EINVAL (kind, iters <= 0, waves_per_simd), QUAMBA_EHIP. */
int quamba_probe_mfma(int kind, int iters, int waves_per_simd, int uniform_operands, double *ops_out, uint32_t *sink,
                      void *stream);

/* In-place streaming pass over buf (device, n_bytes a multiple of 16): every 16-byte piece is read, changed and
 * written back once (non-temporal), the access pattern of the decode state update without its arithmetic.  The launch
 * moves 2 * n_bytes.  Errors: QUAMBA_ENULL, QUAMBA_EINVAL (n_bytes == 0, not a multiple of 16, or beyond 2^31 workgroups of 32 KiB), QUAMBA_EHIP. */
int quamba_probe_stream_rmw(void *buf, size_t n_bytes, void *stream);

/* Read-only streaming pass over buf (device, n_bytes a multiple of 16): 16 workgroups per compute unit stride over
 * the buffer with 16-byte loads; nothing is written (sink, device, >= 4 bytes, receives one word in a case that
 * practically never occurs, so that the loads cannot be removed).  The launch moves n_bytes: the rate HBM reads
 * alone reach, the ceiling of a kernel that reads more than it writes.
 * Errors: QUAMBA_ENULL, QUAMBA_EINVAL (n_bytes == 0 or not a multiple of 16), QUAMBA_EHIP. */
int quamba_probe_stream_read(const void *buf, size_t n_bytes, uint32_t *sink, void *stream);

/* Shader clock: one wave reads the shader-clock counter and the constant 100 MHz counter, spins for about
 * spin_iters dependent vector operations, reads both again and writes the two differences to out[0] (shader clocks)
 * and out[1] (ticks of 10 ns) (device, 16 bytes).  Enqueued on a second stream while a kernel runs back to back on
 * the first, it takes a free wave slot when one opens and shows the clock the power management holds the chip at under
 * that load (a probe that runs alone behind the launches reads the idle clock again within microseconds).
 * Errors: QUAMBA_ENULL, QUAMBA_EINVAL, QUAMBA_EHIP. */
int quamba_probe_clock(int64_t *out, int spin_iters, void *stream);

/* The same probe on n workgroups of one wave each, which the hardware hands to the XCDs in turn: out (device,
 * n x 3 x 8 bytes) receives per workgroup the shader clocks, the ticks of 10 ns and the id of the XCD the wave ran on
 * (hardware register XCC_ID).  The XCDs of one chip run at different clocks under a power-limited load, and a launch
 * that gives every XCD the same work ends with the slowest one; n = 8 covers the 8 XCDs of an MI355X.
 * Errors: QUAMBA_ENULL, QUAMBA_EINVAL (n outside 1..64, spin_iters <= 0), QUAMBA_EHIP. */
int quamba_probe_clock_xcd(int64_t *out, int n, int spin_iters, void *stream);

#ifdef __cplusplus
}
#endif
#endif /* QUAMBA_PROBE_H_ */
