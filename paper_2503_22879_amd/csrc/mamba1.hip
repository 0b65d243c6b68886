// The 8-bit Mamba1 selective scan (Section 3.2, Eq. 2 in the Mamba1 parameterisation; the framework's 8-bit
// selective-scan kernel of Section 4.2): per sequence b, channel d, state n
//     h_t[d,n] = exp(Delta_t[d] A[d,n]) h_{t-1}[d,n] + Delta_t[d] B_t[n] x_t[d],   y_t[d] = sum_n C_t[n] h_t[d,n] + D[d] x_t[d]
// on int8 x (one scale per channel range), int8 B and C (one scale each).  Tensors are channel-major with time last:
// x, Delta, y [b, D, L]; B, C [b, N, L]; A [D, N]; states [b, D, N].
//
// There is no contraction to put on the matrix cores: every (token, channel, state) element needs its own
// exponential, so the kernel is bound by the vector ALU (about 14 instruction slots per element, 4 of them the
// quarter-rate exponential) and is organised to keep that unit busy.  A wave owns one channel at a time and a tile of
// 1024 tokens, 16 consecutive tokens per lane: per state it forms the 16 decay factors and inputs of its tokens,
// reduces them to one (product, state) pair, scans the pairs over the 64 lanes with data-parallel-primitive row shifts
// and broadcasts (the operator of a first-order linear recurrence), and replays its 16 tokens from the scanned-in state
// while accumulating y.  The tile's B and C codes sit in LDS, shared by the workgroup's eight channels; the state at the
// end of a tile is carried to the next tile through LDS.
#include <algorithm>

#include "quamba_internal.h"

namespace quamba {
namespace {

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / 64;
constexpr int kE = 16;              // tokens per lane
constexpr int kTile = 64 * kE;      // tokens per tile
constexpr float kLog2e = 1.44269504088896340736f;
constexpr int kDecodeSeqs = 4;      // sequences per thread and trip of the decode step
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_fetch(float old, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v),
                                                                 CTRL, ROW_MASK, 0xf, false));
}

// Inclusive scan of (P, h) pairs over the 64 lanes.  One step applies the pair fetched from an earlier lane first and
// the lane's own after it: (Ps, hs) then (P, h) -> (Ps P, P hs + h), as two instructions whose first source is the
// shifted lane: h += hs * P, then P *= Ps.  Lanes without a source lane (and rows the mask leaves out) are not
// written, which is the identity.  Shifts by 1, 2, 4, 8 inside rows of 16 lanes, then lane 15 of rows 0 and 2 into
// rows 1 and 3, then lane 31 into rows 2 and 3.  The two idle cycles in front of each step are the wait a
// data-parallel-primitive read needs after a vector write of the same register.
#define QUAMBA_SCAN_STEP(ctrl)                                                       \
    "s_nop 1\n\t"                                                                    \
    "v_fmac_f32_dpp %0, %0, %1 " ctrl " bank_mask:0xf\n\t"                           \
    "v_mul_f32_dpp %1, %1, %1 " ctrl " bank_mask:0xf\n\t"
__device__ __forceinline__ void wave_scan(float &P, float &h)
{
    asm volatile(QUAMBA_SCAN_STEP("row_shr:1 row_mask:0xf") QUAMBA_SCAN_STEP("row_shr:2 row_mask:0xf")
                 QUAMBA_SCAN_STEP("row_shr:4 row_mask:0xf") QUAMBA_SCAN_STEP("row_shr:8 row_mask:0xf")
                 QUAMBA_SCAN_STEP("row_bcast:15 row_mask:0xa") QUAMBA_SCAN_STEP("row_bcast:31 row_mask:0xc")
                 "s_nop 1"
                 : "+v"(h), "+v"(P));
}
#undef QUAMBA_SCAN_STEP

// log(1 + exp(v)) = max(v, 0) + log(1 + e), e = 2^(-|v| log2 e), on the hardware's base-2 exponential and logarithm.
__device__ __forceinline__ float softplus_fast(float v)
{
    const float e = __builtin_amdgcn_exp2f(-__builtin_fabsf(v) * kLog2e);
    // below 1/32 the rounding of 1 + e would cost more than the series' fifth-order remainder
    const float series = e * fmaf(e, fmaf(e, fmaf(e, -0.25f, 0.33333334f), -0.5f), 1.0f);
    const float viaLog = __builtin_amdgcn_logf(1.0f + e) * 0.69314718055994530942f;
    return fmaxf(v, 0.0f) + (e < 0.03125f ? series : viaLog);
}

__device__ __forceinline__ float byte_to_float(uint32_t w, int k) { return (float)(int)(int8_t)(w >> (8 * k)); }

// u * (fp16 half HI of w) and (fp16 half HI of w) * g + acc as one mixed-precision multiply-add each: the fp16 operand
// is widened inside the instruction.
__device__ __forceinline__ float mix_mul(int hi, float u, uint32_t w)  // hi is a constant after unrolling
{
    float d;
    if (hi) asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,1,0] op_sel_hi:[0,1,0]" : "=v"(d) : "v"(u), "v"(w));
    else asm("v_fma_mix_f32 %0, %1, %2, 0 op_sel:[0,0,0] op_sel_hi:[0,1,0]" : "=v"(d) : "v"(u), "v"(w));
    return d;
}
__device__ __forceinline__ float mix_fma(int hi, uint32_t w, float g, float acc)
{
    float d;
    if (hi) asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[1,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(g), "v"(acc));
    else asm("v_fma_mix_f32 %0, %1, %2, %3 op_sel:[0,0,0] op_sel_hi:[1,0,0]" : "=v"(d) : "v"(w), "v"(g), "v"(acc));
    return d;
}

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

// N = 16 states, seqlen a multiple of 16, 16-byte aligned tensors.  grid = (D / kWaves, batch); wave w of a workgroup
// owns channel blockIdx.x * kWaves + w.  The loop over states stays rolled: the 16 tokens of a lane already give every
// instruction 16 independent copies, and unrolling further only costs registers.  The tile's B and C codes are
// converted to fp16 once, when they are staged (exact: 8-bit integers), so that the products that consume them take
// them as fp16 operands of a mixed-precision multiply-add instead of converting them again for every channel.
__global__ __launch_bounds__(kThreads, 4) void mamba1_scan_kernel(SsdArgs a, const float *A, const float *init,
                                                                  float *fin)
{
    constexpr int N = 16;
    __shared__ u32x4 s_B[N][64][2];  // [state][lane]: the lane's 16 token codes of the tile as fp16 pairs
    __shared__ u32x4 s_C[N][64][2];
    __shared__ float s_carry[kWaves][N];  // per wave: the state in front of the current tile
    __shared__ float s_silu[256];         // SiLU(z_scale * code), indexed by the gate code's byte
    const int D = a.s.headdim, L = a.s.seqlen;
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int d = blockIdx.x * kWaves + wave;
    const bool own = d < D;  // wave-uniform; waves without a channel only help staging
    const int dd = own ? d : D - 1;
    const float sB = a.B_scales[0], sC = a.C_scales[0];
    const float sx = x_scale_lookup(a, 0, dd);
    const float sxB = sx * sB;
    const float *Ad = A + (size_t)dd * N;

    if (lane < N) s_carry[wave][lane] = (init && own) ? init[((size_t)b * D + d) * N + lane] : 0.0f;
    if (a.z && threadIdx.x < 256) s_silu[threadIdx.x] = silu_of_code(a.z_scale, (int8_t)threadIdx.x);

    for (int t0 = 0; t0 < L; t0 += kTile) {
        // the tile's B and C codes: 2 * 16 rows of 1024 codes, 16 codes per thread and trip
        __syncthreads();
        for (int i = threadIdx.x; i < 2 * N * 64; i += kThreads) {
            const int which = i / (N * 64), n = (i / 64) % N, l = i % 64;
            const int t = t0 + kE * l;
            u32x4 v = {0, 0, 0, 0};
            if (t < L) v = *reinterpret_cast<const u32x4 *>((which ? a.C : a.B) + ((size_t)b * N + n) * L + t);
            f16x8 lo, hi;
#pragma unroll
            for (int k = 0; k < 8; ++k) {
                lo[k] = (_Float16)byte_to_float(v[k >> 2], k & 3);
                hi[k] = (_Float16)byte_to_float(v[2 + (k >> 2)], k & 3);
            }
            u32x4 *dst = which ? s_C[n][l] : s_B[n][l];
            dst[0] = __builtin_bit_cast(u32x4, lo);
            dst[1] = __builtin_bit_cast(u32x4, hi);
        }
        __syncthreads();
        if (!own) continue;

        const int t = t0 + kE * lane;
        const bool live = t < L;  // whole groups of 16 tokens: seqlen is a multiple of 16
        const size_t row = ((size_t)b * D + d) * L + t;
        u32x4 xq = {0, 0, 0, 0}, zq = {0, 0, 0, 0};
        float dt[kE];
        if (live) {
            xq = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.x + row));
            if (a.z) zq = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.z + row));  // used after the scan
            if (a.dt_q) {  // step size = softplus(s_dt code + bias[d]) (Section 3.2), 16 codes in one load
                const u32x4 dq = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.dt_q + row));
                const float bias = a.dt_bias ? a.dt_bias[d] : 0.0f;
#pragma unroll
                for (int i = 0; i < kE; ++i) dt[i] = softplus_fast(fmaf(a.dt_scale, byte_to_float(dq[i >> 2], i & 3), bias));
            } else {
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v = reinterpret_cast<const f32x4 *>(a.dt + row)[q];  // plain: four loads share a sector
                    dt[4 * q] = v[0]; dt[4 * q + 1] = v[1]; dt[4 * q + 2] = v[2]; dt[4 * q + 3] = v[3];
                }
            }
        } else {
#pragma unroll
            for (int i = 0; i < kE; ++i) dt[i] = 0.0f;  // identity steps: decay 1, input 0
        }
        float u[kE], y[kE];
        float dtsum = 0.0f;
#pragma unroll
        for (int i = 0; i < kE; ++i) {
            u[i] = dt[i] * (sxB * byte_to_float(xq[i >> 2], i & 3));  // Delta_t x_t with B's scale folded in
            y[i] = 0.0f;
            dtsum += dt[i];
        }
#pragma unroll 1
        for (int n = 0; n < N; ++n) {
            const float A2 = Ad[n] * kLog2e;
            const u32x4 b0 = s_B[n][lane][0], b1 = s_B[n][lane][1];
            const float Hc = s_carry[wave][n];
            float dec[kE], in[kE];
            float h = 0.0f;
#pragma unroll
            for (int i = 0; i < kE; ++i) {
                dec[i] = __builtin_amdgcn_exp2f(dt[i] * A2);
                in[i] = mix_mul(i & 1, u[i], i < 8 ? b0[(i & 7) >> 1] : b1[(i & 7) >> 1]);
                h = fmaf(dec[i], h, in[i]);
            }
            float P = __builtin_amdgcn_exp2f(dtsum * A2);  // the product of the lane's 16 decay factors
            wave_scan(P, h);
            // the state in front of this lane's tokens: the pairs of all earlier lanes applied to the carried state
            const float Pex = dpp_fetch<0x138, 0xf>(1.0f, P);  // wave_shr:1
            const float hex = dpp_fetch<0x138, 0xf>(0.0f, h);
            float hh = fmaf(Pex, Hc, hex);
            if (lane == 63) s_carry[wave][n] = fmaf(P, Hc, h);  // the state after the tile
            const u32x4 c0 = s_C[n][lane][0], c1 = s_C[n][lane][1];
#pragma unroll
            for (int i = 0; i < kE; ++i) {
                hh = fmaf(dec[i], hh, in[i]);
                y[i] = mix_fma(i & 1, i < 8 ? c0[(i & 7) >> 1] : c1[(i & 7) >> 1], hh, y[i]);
            }
        }
        if (live) {
            const float Dx = (a.D ? a.D[d] : 0.0f) * sx;
#pragma unroll
            for (int i = 0; i < kE; ++i) y[i] = fmaf(Dx, byte_to_float(xq[i >> 2], i & 3), sC * y[i]);
            if (a.z) {  // y * SiLU(z) on the gate codes of the lane's 16 tokens (Section 3.2), from the table
#pragma unroll
                for (int i = 0; i < kE; ++i) y[i] *= s_silu[(zq[i >> 2] >> (8 * (i & 3))) & 255u];
            }
            u32x4 o[2];
#pragma unroll
            for (int i = 0; i < kE; i += 2)
                o[i >> 3][(i >> 1) & 3] = (uint32_t)f32_to_f16_bits(y[i]) | ((uint32_t)f32_to_f16_bits(y[i + 1]) << 16);
            u32x4 *yp = reinterpret_cast<u32x4 *>(a.y + row);
            __builtin_nontemporal_store(o[0], yp);
            __builtin_nontemporal_store(o[1], yp + 1);
        }
    }
    if (fin && own && lane < N) fin[((size_t)b * D + d) * N + lane] = s_carry[wave][lane];
}

// Any d_state <= 64 and any seqlen: one thread per (sequence, channel), token by token.
constexpr int kMaxStates = 64;
__global__ __launch_bounds__(64) void mamba1_scan_any_kernel(SsdArgs a, const float *A, const float *init, float *fin)
{
    const int D = a.s.headdim, L = a.s.seqlen, N = a.s.d_state;
    const int d = blockIdx.x * 64 + threadIdx.x, b = blockIdx.y;
    if (d >= D) return;
    float h[kMaxStates], A2[kMaxStates];
    for (int n = 0; n < N; ++n) {
        h[n] = init ? init[((size_t)b * D + d) * N + n] : 0.0f;
        A2[n] = A[(size_t)d * N + n] * kLog2e;
    }
    const float sx = x_scale_lookup(a, 0, d), sB = a.B_scales[0], sC = a.C_scales[0];
    const float Dk = a.D ? a.D[d] : 0.0f;
    for (int t = 0; t < L; ++t) {
        const size_t row = ((size_t)b * D + d) * L + t;
        const float dt = step_size(a, row, d), xv = sx * (float)a.x[row];
        const float u = dt * xv * sB;
        float y = 0.0f;
        for (int n = 0; n < N; ++n) {
            const size_t bc = ((size_t)b * N + n) * L + t;
            h[n] = fmaf(__builtin_amdgcn_exp2f(dt * A2[n]), h[n], u * (float)a.B[bc]);
            y = fmaf((float)a.C[bc], h[n], y);
        }
        const float gate = a.z ? silu_of_code(a.z_scale, a.z[row]) : 1.0f;
        a.y[row] = f32_to_f16_bits(fmaf(Dk, xv, sC * y) * gate);
    }
    if (fin)
        for (int n = 0; n < N; ++n) fin[((size_t)b * D + d) * N + n] = h[n];
}

// One generation step on the fp32 state [b, D, N], in place.  N = 16: four lanes share a (sequence, channel) row,
// each moves 16 contiguous bytes of it (consecutive lanes, consecutive addresses), and the four partial sums of y meet
// by data-parallel-primitive moves inside the quad.
__global__ __launch_bounds__(256) void mamba1_decode16_kernel(SsdArgs a, const float *A)
{
    constexpr int kSeq = kDecodeSeqs;  // sequences per thread and trip: the loads of a trip are in flight together
    const int D = a.s.headdim, nb = a.s.batch;
    const int q = blockIdx.x * 256 + threadIdx.x;  // (channel, quarter of its 16 states)
    const int j = q & 3;
    const bool live = (q >> 2) < D;
    const int d = live ? q >> 2 : D - 1;  // lanes past the end redo the last channel and store nothing
    // per channel, once for all sequences of the thread: scale, skip coefficient, the quarter's row of A
    const float sx = x_scale_lookup(a, 0, d);
    const float sxB = sx * a.B_scales[0], sC = a.C_scales[0];
    const float Dx = (a.D ? a.D[d] : 0.0f) * sx;
    const f32x4 A2 = *(reinterpret_cast<const f32x4 *>(A + (size_t)d * 16) + j) * kLog2e;
    for (int b0 = blockIdx.y * kSeq; b0 < nb; b0 += gridDim.y * kSeq) {
        f32x4 h[kSeq];
        float dt[kSeq], xc[kSeq];
        uint32_t bq[kSeq], cq[kSeq];
#pragma unroll
        for (int s = 0; s < kSeq; ++s) {
            const int b = min(b0 + s, nb - 1);  // sequences past the end redo the last one and store nothing
            const size_t idx = (size_t)b * D + d;
            h[s] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.state + idx * 16) + j);
            dt[s] = step_size(a, idx, d);
            xc[s] = (float)a.x[idx];
            bq[s] = *reinterpret_cast<const uint32_t *>(a.B + (size_t)b * 16 + 4 * j);
            cq[s] = *reinterpret_cast<const uint32_t *>(a.C + (size_t)b * 16 + 4 * j);
        }
#pragma unroll
        for (int s = 0; s < kSeq; ++s) {
            const bool store = live && b0 + s < nb;
            const size_t idx = (size_t)min(b0 + s, nb - 1) * D + d;
            const float u = dt[s] * (sxB * xc[s]);
            float y = 0.0f;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                h[s][k] = fmaf(__builtin_amdgcn_exp2f(dt[s] * A2[k]), h[s][k], u * byte_to_float(bq[s], k));
                y = fmaf(byte_to_float(cq[s], k), h[s][k], y);
            }
            if (store) __builtin_nontemporal_store(h[s], reinterpret_cast<f32x4 *>(a.state + idx * 16) + j);
            y = group_sum<4>(y);
            if (j == 0 && store) {
                const float gate = a.z ? silu_of_code(a.z_scale, a.z[idx]) : 1.0f;
                a.y[idx] = f32_to_f16_bits(fmaf(Dx, xc[s], sC * y) * gate);
            }
        }
    }
}

// Any d_state: one thread per (sequence, channel).
__global__ __launch_bounds__(256) void mamba1_decode_any_kernel(SsdArgs a, const float *A)
{
    const int D = a.s.headdim, N = a.s.d_state;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)a.s.batch * D) return;
    const int b = (int)(idx / D), d = (int)(idx - (size_t)b * D);
    const float dt = step_size(a, idx, d), xv = x_scale_lookup(a, 0, d) * (float)a.x[idx];
    const float u = dt * xv * a.B_scales[0];
    float *st = a.state + idx * N;
    const float *Ar = A + (size_t)d * N;
    const int8_t *Bq = a.B + (size_t)b * N, *Cq = a.C + (size_t)b * N;
    float y = 0.0f;
    for (int n = 0; n < N; ++n) {
        const float hn = fmaf(__builtin_amdgcn_exp2f(dt * Ar[n] * kLog2e), st[n], u * (float)Bq[n]);
        st[n] = hn;
        y = fmaf((float)Cq[n], hn, y);
    }
    const float gate = a.z ? silu_of_code(a.z_scale, a.z[idx]) : 1.0f;
    a.y[idx] = f32_to_f16_bits(fmaf(a.D ? a.D[d] : 0.0f, xv, a.C_scales[0] * y) * gate);
}

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

}  // namespace

bool mamba1_scan_supports_any(const quamba_ssd_shape_t &s) { return s.d_state <= kMaxStates; }

hipError_t launch_mamba1_scan(const SsdArgs &a, const float *A, const float *init, float *fin, hipStream_t stream)
{
    const int D = a.s.headdim;
    const bool fast = !(a.s.flags & QUAMBA_FLAG_GENERIC_KERNEL) && a.s.d_state == 16 && a.s.seqlen % 16 == 0 &&
                      aligned16(a.x) && aligned16(a.B) && aligned16(a.C) && aligned16(a.dt) && aligned16(a.y) &&
                      aligned16(a.z) && aligned16(a.dt_q);
    if (fast) {
        const dim3 grid((unsigned)((D + kWaves - 1) / kWaves), (unsigned)a.s.batch);
        hipLaunchKernelGGL(mamba1_scan_kernel, grid, dim3(kThreads), 0, stream, a, A, init, fin);
    } else {
        const dim3 grid((unsigned)((D + 63) / 64), (unsigned)a.s.batch);
        hipLaunchKernelGGL(mamba1_scan_any_kernel, grid, dim3(64), 0, stream, a, A, init, fin);
    }
    return hipGetLastError();
}

hipError_t launch_mamba1_decode(const SsdArgs &a, const float *A, hipStream_t stream)
{
    const size_t total = (size_t)a.s.batch * a.s.headdim;
    if (a.s.d_state == 16 && aligned16(a.state) && aligned16(A) && reinterpret_cast<uintptr_t>(a.B) % 4 == 0 &&
        reinterpret_cast<uintptr_t>(a.C) % 4 == 0) {
        // x: the (channel, quarter) pairs; y: groups of kDecodeSeqs sequences (a thread loops if the batch has more
        // groups than the grid's y dimension may hold)
        const dim3 grid((unsigned)((4 * (size_t)a.s.headdim + 255) / 256),
                        (unsigned)std::min((a.s.batch + kDecodeSeqs - 1) / kDecodeSeqs, 65535));
        hipLaunchKernelGGL(mamba1_decode16_kernel, grid, dim3(256), 0, stream, a, A);
    } else {
        hipLaunchKernelGGL(mamba1_decode_any_kernel, dim3((unsigned)((total + 255) / 256)), dim3(256), 0, stream, a, A);
    }
    return hipGetLastError();
}

}  // namespace quamba
