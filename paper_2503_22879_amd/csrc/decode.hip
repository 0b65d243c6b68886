// Single-token decode of the 8-bit SSD: one step of Eq. 2 on the persistent fp32 state, in place.
//
// The step is a pure stream over the state (read 4 B + write 4 B per element, 3 FMAs), so the kernel is built
// around HBM: one workgroup per (sequence, head), every lane owns 16-byte pieces of state rows, all of a lane's
// loads are issued before any arithmetic, the d_state reduction of y stays in registers (cross-lane adds), and
// the de-quantized per-row input x is staged through a few hundred bytes of LDS by each wave for its own rows.
#include "quamba_internal.h"

namespace quamba {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
typedef float f32x4 __attribute__((ext_vector_type(4)));

// De-quantized x of this head into LDS: xv[p] = s_x(h,p) * xq[p] (inverse of Eq. 1 with the m x n table).
__device__ __forceinline__ void stage_x(const SsdArgs &a, int bh, int h, float *xv)
{
    const int P = a.s.headdim;
    for (int p = threadIdx.x; p < P; p += kThreads)
        xv[p] = x_scale_lookup(a, h, p) * (float)a.x[(size_t)bh * P + p];
}

// Fast path: d_state = N (multiple of 4, N/4 a power of two <= 64).  A row of N floats is covered by N/4 lanes with
// one float4 each; a wave covers 64/(N/4) rows per load instruction and keeps ROWS such instructions in flight.
// FULL: headdim is a multiple of the rows one pass of the workgroup covers, so no row needs clamping or masking and
// the row addresses are one base plus compile-time offsets.
template <int N, int ROWS, bool FULL>
__global__ __launch_bounds__(kThreads) void decode_vec_kernel(SsdArgs a)
{
    constexpr int LPR = N / 4;     // lanes per row
    constexpr int RPI = 64 / LPR;  // rows per wave-wide load
    extern __shared__ float lds[];
    const int P = a.s.headdim, H = a.s.nheads, G = a.s.ngroups;
    float *xv = lds;  // [P]

    const int bh = blockIdx.x;
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane % LPR, sub = lane / LPR;

    float *st = a.state + (size_t)bh * P * N + 4 * j;

    const float dt = step_size(a, bh, h);
    const float dA = expf(dt * a.A[h]);
    const float Dh = a.D ? a.D[h] : 0.0f;
    const float sB = a.B_scales[g] * dt, sC = a.C_scales[g];
    const char4 bq = *reinterpret_cast<const char4 *>(a.B + ((size_t)b * G + g) * N + 4 * j);
    const char4 cq = *reinterpret_cast<const char4 *>(a.C + ((size_t)b * G + g) * N + 4 * j);
    const float4 Bv = make_float4(sB * bq.x, sB * bq.y, sB * bq.z, sB * bq.w);  // dt * B_t (B-dot of Sec. 3.2)
    const float4 Cv = make_float4(sC * cq.x, sC * cq.y, sC * cq.z, sC * cq.w);

    for (int p0 = wave * RPI * ROWS; p0 < P; p0 += kWaves * RPI * ROWS) {
        // all of the lane's loads first, unconditionally (rows past the end re-read the last row and are not stored)
        f32x4 v[ROWS];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int p = FULL ? p0 + i * RPI + sub : min(p0 + i * RPI + sub, P - 1);
            v[i] = __builtin_nontemporal_load(reinterpret_cast<const f32x4 *>(st + (size_t)p * N));
        }
        // de-quantized x of the rows of this trip, staged by the wave for itself while its state loads are in
        // flight: no workgroup barrier, the waves never wait for each other (LDS accesses of one wave stay in order)
        for (int r = lane; r < RPI * ROWS; r += 64) {
            const int p = p0 + r;
            if (FULL || p < P) xv[p] = x_scale_lookup(a, h, p) * (float)a.x[(size_t)bh * P + p];
        }
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "wavefront");
        __builtin_amdgcn_wave_barrier();
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "wavefront");
        float part[ROWS];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int p = FULL ? p0 + i * RPI + sub : min(p0 + i * RPI + sub, P - 1);
            const float x = xv[p];
            v[i].x = fmaf(dA, v[i].x, Bv.x * x);
            v[i].y = fmaf(dA, v[i].y, Bv.y * x);
            v[i].z = fmaf(dA, v[i].z, Bv.z * x);
            v[i].w = fmaf(dA, v[i].w, Bv.w * x);
            if (FULL || p0 + i * RPI + sub < P)
                __builtin_nontemporal_store(v[i], reinterpret_cast<f32x4 *>(st + (size_t)p * N));
            part[i] = fmaf(Cv.x, v[i].x, fmaf(Cv.y, v[i].y, fmaf(Cv.z, v[i].z, Cv.w * v[i].w)));
        }
#pragma unroll
        for (int i = 0; i < ROWS; ++i) part[i] = group_sum<LPR>(part[i]);
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int p = p0 + i * RPI + sub;
            if (j == 0 && (FULL || p < P)) {
                const float gate = a.z ? silu_of_code(a.z_scale, a.z[(size_t)bh * P + p]) : 1.0f;  // y * SiLU(z)
                a.y[(size_t)bh * P + p] = f32_to_f16_bits(fmaf(Dh, xv[p], part[i]) * gate);
            }
        }
    }
}

// Any d_state: one wave per row, lanes stride over the states.
__global__ __launch_bounds__(kThreads) void decode_any_kernel(SsdArgs a)
{
    extern __shared__ float lds[];
    const int P = a.s.headdim, H = a.s.nheads, G = a.s.ngroups, N = a.s.d_state;
    float *xv = lds;
    float *ys = lds + P;
    const int bh = blockIdx.x;
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    stage_x(a, bh, h, xv);
    __syncthreads();
    const float dt = step_size(a, bh, h);
    const float dA = expf(dt * a.A[h]);
    const float Dh = a.D ? a.D[h] : 0.0f;
    const float sB = a.B_scales[g] * dt, sC = a.C_scales[g];
    const int8_t *Bq = a.B + ((size_t)b * G + g) * N;
    const int8_t *Cq = a.C + ((size_t)b * G + g) * N;
    float *st = a.state + (size_t)bh * P * N;
    for (int p = wave; p < P; p += kWaves) {
        const float x = xv[p];
        float part = 0.0f;
        for (int n = lane; n < N; n += 64) {
            const float hn = fmaf(dA, st[(size_t)p * N + n], sB * (float)Bq[n] * x);
            st[(size_t)p * N + n] = hn;
            part = fmaf(sC * (float)Cq[n], hn, part);
        }
        part = group_sum<64>(part);
        if (lane == 0) ys[p] = fmaf(Dh, x, part);
    }
    __syncthreads();
    for (int p = threadIdx.x; p < P; p += kThreads) {
        const float gate = a.z ? silu_of_code(a.z_scale, a.z[(size_t)bh * P + p]) : 1.0f;  // y * SiLU(z)
        a.y[(size_t)bh * P + p] = f32_to_f16_bits(ys[p] * gate);
    }
}

template <int N>
hipError_t launch_vec(const SsdArgs &a, hipStream_t stream)
{
    constexpr int LPR = N / 4, RPI = 64 / LPR;
    constexpr int ROWS = (RPI * 4 * kWaves <= 64) ? 4 : (RPI <= 8 ? 2 : 1);  // rows per lane in flight per trip
    const dim3 grid((unsigned)(a.s.batch * a.s.nheads));
    const size_t lds = sizeof(float) * (size_t)a.s.headdim;
    if (a.s.headdim % (kWaves * RPI * ROWS) == 0)
        hipLaunchKernelGGL((decode_vec_kernel<N, ROWS, true>), grid, dim3(kThreads), lds, stream, a);
    else
        hipLaunchKernelGGL((decode_vec_kernel<N, ROWS, false>), grid, dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

}  // namespace

hipError_t launch_decode(const SsdArgs &a, hipStream_t stream)
{
    const bool aligned = (reinterpret_cast<uintptr_t>(a.state) % 16 == 0) &&
                         (reinterpret_cast<uintptr_t>(a.B) % 4 == 0) && (reinterpret_cast<uintptr_t>(a.C) % 4 == 0);
    if (aligned) {
        switch (a.s.d_state) {
            case 256: return launch_vec<256>(a, stream);
            case 128: return launch_vec<128>(a, stream);
            case 64: return launch_vec<64>(a, stream);
            case 32: return launch_vec<32>(a, stream);
            case 16: return launch_vec<16>(a, stream);
            default: break;
        }
    }
    const dim3 grid((unsigned)(a.s.batch * a.s.nheads));
    const size_t lds = sizeof(float) * 2 * (size_t)a.s.headdim;
    hipLaunchKernelGGL(decode_any_kernel, grid, dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

}  // namespace quamba
