// Shape-agnostic prefill: the recurrence of Eq. 2 walked token by token in fp32, one workgroup per (sequence, head).
// It accepts every shape the library does (any headdim, d_state, seqlen; no chunking at all) and serves as the
// fallback where the chunked MFMA kernel does not apply, and as an on-device cross-check of it.
//
// Layout of the work: the head's state [P,N] lives in LDS for the whole sequence; tokens are staged kTB at a time
// (de-quantized x, dt*s_B*B, s_C*C, exp(dt*A)) so that global loads and the fp16 y stores are coalesced; each wave
// owns the state rows p = wave, wave+4, ... and walks the kTB staged steps for them with its lanes spread over
// d_state, reducing y across lanes in a fixed order (deterministic, no atomics).
#include "quamba_internal.h"

namespace quamba {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kTB = 16;  // tokens staged per round

__device__ __forceinline__ float wave_sum(float v)
{
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) v += __shfl_xor(v, off, 64);
    return v;
}

__global__ __launch_bounds__(kThreads) void prefill_generic_kernel(SsdArgs a)
{
    extern __shared__ float lds[];
    const int L = a.s.seqlen, H = a.s.nheads, P = a.s.headdim, N = a.s.d_state, G = a.s.ngroups;
    float *st = lds;              // [P][N]
    float *sx = st + P * N;       // [P]
    float *xs = sx + P;           // [kTB][P]   de-quantized x
    float *ys = xs + kTB * P;     // [kTB][P]
    float *Bs = ys + kTB * P;     // [kTB][N]   dt * s_B * Bq
    float *Cs = Bs + kTB * N;     // [kTB][N]   s_C * Cq
    float *dAs = Cs + kTB * N;    // [kTB]

    const int bh = blockIdx.x;
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;

    for (int p = tid; p < P; p += kThreads) sx[p] = x_scale_lookup(a, h, p);
    for (int e = tid; e < P * N; e += kThreads)
        st[e] = a.init_state ? a.init_state[(size_t)bh * P * N + e] : 0.0f;
    const float Ah = a.A[h], Dh = a.D ? a.D[h] : 0.0f;
    const float sB = a.B_scales[g], sC = a.C_scales[g];
    __syncthreads();

    for (int t0 = 0; t0 < L; t0 += kTB) {
        const int nt = min(kTB, L - t0);
        const size_t tok0 = (size_t)b * L + t0;
        for (int e = tid; e < nt * P; e += kThreads) {
            const int t = e / P, p = e - t * P;
            xs[e] = sx[p] * (float)a.x[((tok0 + t) * H + h) * P + p];
        }
        for (int e = tid; e < nt * N; e += kThreads) {
            const int t = e / N, n = e - t * N;
            const float dt = step_size(a, (tok0 + t) * H + h, h);
            Bs[e] = dt * sB * (float)a.B[((tok0 + t) * G + g) * N + n];
            Cs[e] = sC * (float)a.C[((tok0 + t) * G + g) * N + n];
        }
        for (int t = tid; t < nt; t += kThreads) dAs[t] = expf(step_size(a, (tok0 + t) * H + h, h) * Ah);
        __syncthreads();
        for (int p = wave; p < P; p += kWaves) {
            for (int t = 0; t < nt; ++t) {
                const float x = xs[t * P + p], dA = dAs[t];
                float part = 0.0f;
                for (int n = lane; n < N; n += 64) {
                    const float hn = fmaf(dA, st[p * N + n], Bs[t * N + n] * x);
                    st[p * N + n] = hn;
                    part = fmaf(Cs[t * N + n], hn, part);
                }
                part = wave_sum(part);
                if (lane == 0) ys[t * P + p] = fmaf(Dh, x, part);
            }
        }
        __syncthreads();
        for (int e = tid; e < nt * P; e += kThreads) {
            const int t = e / P, p = e - t * P;
            const size_t o = ((tok0 + t) * H + h) * P + p;
            const float gate = a.z ? silu_of_code(a.z_scale, a.z[o]) : 1.0f;  // y * SiLU(z), Section 3.2
            const _Float16 v = (_Float16)(ys[e] * gate);
            a.y[o] = __builtin_bit_cast(uint16_t, v);
        }
    }
    if (a.state) {
        __syncthreads();
        for (int e = tid; e < P * N; e += kThreads) a.state[(size_t)bh * P * N + e] = st[e];
    }
}

}  // namespace

size_t prefill_generic_lds_bytes(const quamba_ssd_shape_t &s)
{
    const size_t P = (size_t)s.headdim, N = (size_t)s.d_state;
    return sizeof(float) * (P * N + P + 2 * kTB * P + 2 * kTB * N + kTB);
}

hipError_t launch_prefill_generic(const SsdArgs &a, hipStream_t stream)
{
    const size_t lds = prefill_generic_lds_bytes(a.s);
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(prefill_generic_kernel),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL(prefill_generic_kernel, dim3((unsigned)(a.s.batch * a.s.nheads)), dim3(kThreads), lds, stream,
                       a);
    return hipGetLastError();
}

}  // namespace quamba
