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
// while accumulating y.  The tile's B and C codes sit in LDS, shared by the workgroup's channels; the state at the end
// of a tile is carried to the next tile in scalar registers.
#include "quamba_internal.h"

namespace quamba {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kE = 16;              // tokens per lane
constexpr int kTile = 64 * kE;      // tokens per tile
constexpr float kLog2e = 1.44269504088896340736f;
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

template <int CTRL, int ROW_MASK>
__device__ __forceinline__ float dpp_fetch(float old, float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(__builtin_bit_cast(int, old), __builtin_bit_cast(int, v),
                                                                 CTRL, ROW_MASK, 0xf, false));
}

// One step of the scan of (P, h) pairs: the pair fetched from an earlier lane is applied first, the lane's own after
// it: (Ps, hs) then (P, h) -> (Ps P, P hs + h).  Lanes without a source (or in rows the mask leaves out) fetch the
// identity (1, 0).
template <int CTRL, int ROW_MASK>
__device__ __forceinline__ void scan_step(float &P, float &h)
{
    const float Ps = dpp_fetch<CTRL, ROW_MASK>(1.0f, P);
    const float hs = dpp_fetch<CTRL, ROW_MASK>(0.0f, h);
    h = fmaf(P, hs, h);
    P = P * Ps;
}

// Inclusive scan over the 64 lanes: shifts by 1, 2, 4, 8 inside rows of 16 lanes, then lane 15 of rows 0 and 2
// into rows 1 and 3, then lane 31 into rows 2 and 3.
__device__ __forceinline__ void wave_scan(float &P, float &h)
{
    scan_step<0x111, 0xf>(P, h);  // row_shr:1
    scan_step<0x112, 0xf>(P, h);  // row_shr:2
    scan_step<0x114, 0xf>(P, h);  // row_shr:4
    scan_step<0x118, 0xf>(P, h);  // row_shr:8
    scan_step<0x142, 0xa>(P, h);  // row_bcast:15 into rows 1, 3
    scan_step<0x143, 0xc>(P, h);  // row_bcast:31 into rows 2, 3
}

__device__ __forceinline__ float byte_to_float(uint32_t w, int k) { return (float)(int)(int8_t)(w >> (8 * k)); }

// N = 16 states, seqlen a multiple of 16, 16-byte aligned tensors.  grid = (D / (kWaves * CPW), batch); wave w of a
// workgroup owns channels d0 + w * CPW .. + CPW - 1.  The loops over channels and states stay rolled: the 16 tokens
// of a lane already give every instruction 16 independent copies, and unrolling further only costs registers.
template <int CPW>
__global__ __launch_bounds__(kThreads, 4) void mamba1_scan_kernel(SsdArgs a, const float *A, const float *init,
                                                                  float *fin)
{
    constexpr int N = 16;
    __shared__ u32x4 s_B[N][64];  // [state][lane]: the lane's 16 token codes of the tile
    __shared__ u32x4 s_C[N][64];
    __shared__ float s_carry[kWaves][CPW][N];  // per wave: the state in front of the current tile
    const int D = a.s.headdim, L = a.s.seqlen;
    const int b = blockIdx.y;
    const int lane = threadIdx.x & 63;
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
    const int d0 = (blockIdx.x * kWaves + wave) * CPW;
    const float sB = a.B_scales[0], sC = a.C_scales[0];

    for (int i = lane; i < CPW * N; i += 64) {
        const int c = i / N, n = i - c * N;
        s_carry[wave][c][n] = (init && d0 + c < D) ? init[((size_t)b * D + d0 + c) * N + n] : 0.0f;
    }

    for (int t0 = 0; t0 < L; t0 += kTile) {
        // the tile's B and C codes: 2 * 16 rows of 1024 bytes, 16 bytes per thread and trip
        __syncthreads();
        for (int i = threadIdx.x; i < 2 * N * 64; i += kThreads) {
            const int which = i / (N * 64), n = (i / 64) % N, l = i % 64;
            const int t = t0 + kE * l;
            u32x4 v = {0, 0, 0, 0};
            if (t < L) v = *reinterpret_cast<const u32x4 *>((which ? a.C : a.B) + ((size_t)b * N + n) * L + t);
            (which ? s_C : s_B)[n][l] = v;
        }
        __syncthreads();

        const int t = t0 + kE * lane;
        const bool live = t < L;  // whole groups of 16 tokens: seqlen is a multiple of 16
#pragma unroll 1
        for (int c = 0; c < CPW; ++c) {
            const int d = d0 + c;
            if (d >= D) break;
            const size_t row = ((size_t)b * D + d) * L + t;
            u32x4 xq = {0, 0, 0, 0};
            float dt[kE];
            if (live) {
                xq = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(a.x + row));
#pragma unroll
                for (int q = 0; q < 4; ++q) {
                    const f32x4 v = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(a.dt + row) + q);
                    dt[4 * q] = v[0]; dt[4 * q + 1] = v[1]; dt[4 * q + 2] = v[2]; dt[4 * q + 3] = v[3];
                }
            } else {
#pragma unroll
                for (int i = 0; i < kE; ++i) dt[i] = 0.0f;  // identity steps: decay 1, input 0
            }
            const float sx = x_scale_lookup(a, 0, d);
            const float sxB = sx * sB;
            float u[kE], y[kE];
#pragma unroll
            for (int i = 0; i < kE; ++i) {
                u[i] = dt[i] * (sxB * byte_to_float(xq[i >> 2], i & 3));  // Delta_t x_t with B's scale folded in
                y[i] = 0.0f;
            }
            const float *Ad = A + (size_t)d * N;
#pragma unroll 1
            for (int n = 0; n < N; ++n) {
                const float A2 = Ad[n] * kLog2e;
                const u32x4 bq = s_B[n][lane], cq = s_C[n][lane];
                const float Hc = s_carry[wave][c][n];
                float dec[kE], in[kE];
                float P = 1.0f, h = 0.0f;
#pragma unroll
                for (int i = 0; i < kE; ++i) {
                    dec[i] = __builtin_amdgcn_exp2f(dt[i] * A2);
                    in[i] = u[i] * byte_to_float(bq[i >> 2], i & 3);
                    h = fmaf(dec[i], h, in[i]);
                    P = P * dec[i];
                }
                wave_scan(P, h);
                // the state in front of this lane's tokens: the pairs of all earlier lanes applied to the carried state
                const float Pex = dpp_fetch<0x138, 0xf>(1.0f, P);  // wave_shr:1
                const float hex = dpp_fetch<0x138, 0xf>(0.0f, h);
                float hh = fmaf(Pex, Hc, hex);
                if (lane == 63) s_carry[wave][c][n] = fmaf(P, Hc, h);  // the state after the tile
#pragma unroll
                for (int i = 0; i < kE; ++i) {
                    hh = fmaf(dec[i], hh, in[i]);
                    y[i] = fmaf(byte_to_float(cq[i >> 2], i & 3), hh, y[i]);
                }
            }
            if (live) {
                const float Dx = (a.D ? a.D[d] : 0.0f) * sx;
                u32x4 o[2];
#pragma unroll
                for (int i = 0; i < kE; i += 2) {
                    const uint32_t lo = f32_to_f16_bits(fmaf(Dx, byte_to_float(xq[i >> 2], i & 3), sC * y[i]));
                    const uint32_t hi = f32_to_f16_bits(fmaf(Dx, byte_to_float(xq[(i + 1) >> 2], (i + 1) & 3), sC * y[i + 1]));
                    o[i >> 3][(i >> 1) & 3] = lo | (hi << 16);
                }
                u32x4 *yp = reinterpret_cast<u32x4 *>(a.y + row);
                __builtin_nontemporal_store(o[0], yp);
                __builtin_nontemporal_store(o[1], yp + 1);
            }
        }
    }
    if (fin)
        for (int i = lane; i < CPW * N; i += 64) {
            const int c = i / N, n = i - c * N;
            if (d0 + c < D) fin[((size_t)b * D + d0 + c) * N + n] = s_carry[wave][c][n];
        }
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
        const float dt = a.dt[row], xv = sx * (float)a.x[row];
        const float u = dt * xv * sB;
        float y = 0.0f;
        for (int n = 0; n < N; ++n) {
            const size_t bc = ((size_t)b * N + n) * L + t;
            h[n] = fmaf(__builtin_amdgcn_exp2f(dt * A2[n]), h[n], u * (float)a.B[bc]);
            y = fmaf((float)a.C[bc], h[n], y);
        }
        a.y[row] = f32_to_f16_bits(fmaf(Dk, xv, sC * y));
    }
    if (fin)
        for (int n = 0; n < N; ++n) fin[((size_t)b * D + d) * N + n] = h[n];
}

// One generation step on the fp32 state [b, D, N], in place: one thread per (sequence, channel); with N = 16 a thread
// moves its 64 contiguous bytes of state with four 16-byte loads and stores.
template <int NT>
__global__ __launch_bounds__(256) void mamba1_decode_kernel(SsdArgs a, const float *A)
{
    const int D = a.s.headdim, N = NT ? NT : a.s.d_state;
    const size_t idx = (size_t)blockIdx.x * 256 + threadIdx.x;
    if (idx >= (size_t)a.s.batch * D) return;
    const int b = (int)(idx / D), d = (int)(idx - (size_t)b * D);
    const float dt = a.dt[idx], xv = x_scale_lookup(a, 0, d) * (float)a.x[idx];
    const float u = dt * xv * a.B_scales[0];
    float *st = a.state + idx * N;
    const float *Ar = A + (size_t)d * N;
    const int8_t *Bq = a.B + (size_t)b * N, *Cq = a.C + (size_t)b * N;
    float y = 0.0f;
    if (NT == 16) {
        f32x4 h[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) h[q] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(st) + q);
#pragma unroll
        for (int n = 0; n < 16; ++n) {
            const float hn = fmaf(__builtin_amdgcn_exp2f(dt * Ar[n] * kLog2e), h[n >> 2][n & 3], u * (float)Bq[n]);
            h[n >> 2][n & 3] = hn;
            y = fmaf((float)Cq[n], hn, y);
        }
#pragma unroll
        for (int q = 0; q < 4; ++q) __builtin_nontemporal_store(h[q], reinterpret_cast<f32x4 *>(st) + q);
    } else {
        for (int n = 0; n < N; ++n) {
            const float hn = fmaf(__builtin_amdgcn_exp2f(dt * Ar[n] * kLog2e), st[n], u * (float)Bq[n]);
            st[n] = hn;
            y = fmaf((float)Cq[n], hn, y);
        }
    }
    a.y[idx] = f32_to_f16_bits(fmaf(a.D ? a.D[d] : 0.0f, xv, a.C_scales[0] * y));
}

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

}  // namespace

bool mamba1_scan_supports_any(const quamba_ssd_shape_t &s) { return s.d_state <= kMaxStates; }

hipError_t launch_mamba1_scan(const SsdArgs &a, const float *A, const float *init, float *fin, hipStream_t stream)
{
    const int D = a.s.headdim;
    const bool fast = !(a.s.flags & QUAMBA_FLAG_GENERIC_KERNEL) && a.s.d_state == 16 && a.s.seqlen % 16 == 0 &&
                      aligned16(a.x) && aligned16(a.B) && aligned16(a.C) && aligned16(a.dt) && aligned16(a.y);
    if (fast) {
        // four channels per wave when that still fills the device, else one
        if ((int64_t)a.s.batch * D >= 16384) {
            const dim3 grid((unsigned)((D + kWaves * 4 - 1) / (kWaves * 4)), (unsigned)a.s.batch);
            hipLaunchKernelGGL(mamba1_scan_kernel<4>, grid, dim3(kThreads), 0, stream, a, A, init, fin);
        } else {
            const dim3 grid((unsigned)((D + kWaves - 1) / kWaves), (unsigned)a.s.batch);
            hipLaunchKernelGGL(mamba1_scan_kernel<1>, grid, dim3(kThreads), 0, stream, a, A, init, fin);
        }
    } else {
        const dim3 grid((unsigned)((D + 63) / 64), (unsigned)a.s.batch);
        hipLaunchKernelGGL(mamba1_scan_any_kernel, grid, dim3(64), 0, stream, a, A, init, fin);
    }
    return hipGetLastError();
}

hipError_t launch_mamba1_decode(const SsdArgs &a, const float *A, hipStream_t stream)
{
    const size_t total = (size_t)a.s.batch * a.s.headdim;
    const dim3 grid((unsigned)((total + 255) / 256));
    if (a.s.d_state == 16 && aligned16(a.state))
        hipLaunchKernelGGL(mamba1_decode_kernel<16>, grid, dim3(256), 0, stream, a, A);
    else
        hipLaunchKernelGGL(mamba1_decode_kernel<0>, grid, dim3(256), 0, stream, a, A);
    return hipGetLastError();
}

}  // namespace quamba
