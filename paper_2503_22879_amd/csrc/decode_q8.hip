// Single-token decode on an 8-bit cached state (Appendix E, "Quantizing cached SSM states"), in place, and the
// quantizer that turns an fp32 state into that cache.
//
// The cached state is int8 codes; the scale of code (h, p, n) belongs to the (head cluster, channel range) cell of
// (h, p) -- the m x n cells of x (Section 4.1) -- and to the state n.  A step reads a code, de-quantizes it (inverse of
// Eq. 1), applies Eq. 2, adds the element to y, and writes the re-quantized code (Eq. 1) back: 1 B read + 1 B written
// per state element instead of 4 B + 4 B, with about 11 vector instructions per element, which puts the kernel near
// the point where the vector ALU and HBM take the same time.  One workgroup per (sequence, head); a lane owns 16
// consecutive states of a row (one 16-byte load), the head's scale rows and their reciprocals sit in LDS.
//
// The new code is an integer decided by fp32 arithmetic, so every operation that leads to it is rounded on its own, in
// a fixed order (the header states it); the compiler must not contract multiplies and adds, and the exponential of
// the decay is a fixed sequence of such operations instead of a library call.
#include "quamba_internal.h"

// no fused multiply-add unless written as one: the quantization decision depends on the individual roundings
#pragma clang fp contract(off)

namespace quamba {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float from_bits(uint32_t u) { return __builtin_bit_cast(float, u); }

// exp(z) for z <= 0 as separately rounded fp32 steps: t = z log2(e), k = rint(t), f = t - k in [-1/2, 1/2],
// 2^f = sum_i ((ln 2)^i / i!) f^i (i = 7..0, Horner, multiply then add), result 2^f 2^k; t < -125 gives 0 so that
// no result is subnormal.  Constants are the fp32 roundings of log2(e) and of the Taylor coefficients.
__device__ __forceinline__ float exp_steps(float z)
{
    const float t = z * from_bits(0x3FB8AA3Bu);
    const float k = __builtin_rintf(t);
    const float f = t - k;
    float p = from_bits(0x377FE5FEu);
    p = p * f; p = p + from_bits(0x39218489u);
    p = p * f; p = p + from_bits(0x3AAEC3FFu);
    p = p * f; p = p + from_bits(0x3C1D955Bu);
    p = p * f; p = p + from_bits(0x3D635847u);
    p = p * f; p = p + from_bits(0x3E75FDF0u);
    p = p * f; p = p + from_bits(0x3F317218u);
    p = p * f; p = p + 1.0f;
    return t < -125.0f ? 0.0f : __builtin_ldexpf(p, (int)k);
}

// Eq. 1: clamp to [-127, 127], then round to nearest even by adding 1.5 * 2^23 (the sum's unit in the last place is
// 1): the code is the low byte of the sum's bit pattern, in two's complement.  Clamping first gives the same code as
// clamping after rounding because the bounds are integers.
__device__ __forceinline__ uint32_t code_bits(float r)
{
    const float c = __builtin_fminf(__builtin_fmaxf(r, -127.0f), 127.0f);
    return __builtin_bit_cast(uint32_t, c + 12582912.0f);
}

// low bytes of four patterns -> one dword
__device__ __forceinline__ uint32_t pack4(uint32_t m0, uint32_t m1, uint32_t m2, uint32_t m3)
{
    const uint32_t lo = __builtin_amdgcn_perm(m1, m0, 0x0c0c0400u);  // bytes: m0.b0, m1.b0, 0, 0
    const uint32_t hi = __builtin_amdgcn_perm(m3, m2, 0x04000c0cu);  // bytes: 0, 0, m2.b0, m3.b0
    return lo | hi;
}

__device__ __forceinline__ float code_to_float(uint32_t w, int e) { return (float)(int)(int8_t)(w >> (8 * e)); }

// LDS of a workgroup: xv[P] de-quantized x, cl[P] channel range of every row, s_tab[n][N] the head's scale rows,
// inv_tab[n][N] their reciprocals (correctly rounded divisions, done once per workgroup).
// floats in front of the scale tables: xv and cl, rounded up so that the tables' rows can be read 16 bytes at a time
__host__ __device__ inline size_t table_offset(int P) { return ((size_t)2 * P + 3) & ~(size_t)3; }

struct Tables {
    float *xv;
    int *cl;
    float *s_tab;
    float *inv_tab;
};

__device__ __forceinline__ Tables stage_tables(const SsdArgs &a, const float *state_scales, int bh, int h, float *lds,
                                               bool with_x)
{
    const int P = a.s.headdim, N = a.s.d_state, nc = a.s.n_chan_clusters;
    Tables t;
    t.xv = lds;
    t.cl = reinterpret_cast<int *>(lds + P);
    t.s_tab = lds + table_offset(P);
    t.inv_tab = t.s_tab + nc * N;
    int base = 0;
    for (int p = threadIdx.x; p < P; p += kThreads) {
        const int cell = cell_lookup(a, h, p, &base);
        t.cl[p] = cell - base;
        if (with_x) t.xv[p] = a.x_scales[cell] * (float)a.x[(size_t)bh * P + p];
    }
    cell_lookup(a, h, 0, &base);  // threads beyond P need the head's first cell too
    const float *src = state_scales + (size_t)base * N;
    for (int i = threadIdx.x; i < nc * N; i += kThreads) {
        const float s = src[i];
        t.s_tab[i] = s;
        t.inv_tab[i] = __fdiv_rn(1.0f, s);
    }
    __syncthreads();
    return t;
}

// d_state = N with N/16 a power of two <= 64: a row of N codes is covered by N/16 lanes with 16 bytes each; a wave
// covers 64/(N/16) rows per load instruction and keeps ROWS such loads in flight.  FULL: headdim is a multiple of the
// rows one trip of the workgroup covers (no clamping or masking of rows).
template <int N, int ROWS, bool FULL>
__global__ __launch_bounds__(kThreads) void decode_q8_vec_kernel(SsdArgs a, const float *state_scales, int8_t *state_q)
{
    constexpr int LPR = N / 16, RPI = 64 / LPR;
    extern __shared__ float lds[];
    const int P = a.s.headdim, H = a.s.nheads, G = a.s.ngroups;
    const int bh = blockIdx.x;
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane % LPR, sub = lane / LPR;

    // the lane's state loads go first: rows past the end re-read the last row and are not stored
    int8_t *st = state_q + (size_t)bh * P * N + 16 * j;
    const Tables t = stage_tables(a, state_scales, bh, h, lds, true);

    const float dt = a.dt[bh];
    const float dA = exp_steps(dt * a.A[h]);
    const float Dh = a.D ? a.D[h] : 0.0f;
    const float sB = a.B_scales[g], sC = a.C_scales[g];
    const u32x4 bq = *reinterpret_cast<const u32x4 *>(a.B + ((size_t)b * G + g) * N + 16 * j);
    const u32x4 cq = *reinterpret_cast<const u32x4 *>(a.C + ((size_t)b * G + g) * N + 16 * j);
    float Bv[16], Cv[16];
#pragma unroll
    for (int e = 0; e < 16; ++e) {
        Bv[e] = sB * code_to_float(bq[e >> 2], e & 3);
        Cv[e] = sC * code_to_float(cq[e >> 2], e & 3);
    }

    for (int p0 = wave * RPI * ROWS; p0 < P; p0 += kWaves * RPI * ROWS) {
        u32x4 w[ROWS];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int p = FULL ? p0 + i * RPI + sub : min(p0 + i * RPI + sub, P - 1);
            w[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(st + (size_t)p * N));
        }
        float part[ROWS];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int p = FULL ? p0 + i * RPI + sub : min(p0 + i * RPI + sub, P - 1);
            const float dtx = dt * t.xv[p];
            const float *srow = t.s_tab + t.cl[p] * N + 16 * j;
            const float *irow = t.inv_tab + t.cl[p] * N + 16 * j;
            float acc = 0.0f;
            u32x4 out;
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 s4 = *reinterpret_cast<const f32x4 *>(srow + 4 * q4);
                const f32x4 i4 = *reinterpret_cast<const f32x4 *>(irow + 4 * q4);
                uint32_t m[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    const int e = 4 * q4 + k;
                    const float hp = s4[k] * code_to_float(w[i][q4], k);  // inverse of Eq. 1
                    const float d = dA * hp;                               // Eq. 2: decay ...
                    const float u = dtx * Bv[e];                           // ... plus B-dot x
                    const float hn = d + u;
                    acc = __builtin_fmaf(Cv[e], hn, acc);                  // y from the updated state
                    m[k] = code_bits(hn * i4[k]);                          // Eq. 1
                }
                out[q4] = pack4(m[0], m[1], m[2], m[3]);
            }
            if (FULL || p0 + i * RPI + sub < P)
                __builtin_nontemporal_store(out, reinterpret_cast<u32x4 *>(st + (size_t)p * N));
            part[i] = acc;
        }
#pragma unroll
        for (int i = 0; i < ROWS; ++i) part[i] = group_sum<LPR>(part[i]);
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            const int p = p0 + i * RPI + sub;
            if (j == 0 && (FULL || p < P))
                a.y[(size_t)bh * P + p] = f32_to_f16_bits(__builtin_fmaf(Dh, t.xv[p], part[i]));
        }
    }
}

// Any d_state: one wave per row, lanes stride over the states, byte accesses.
__global__ __launch_bounds__(kThreads) void decode_q8_any_kernel(SsdArgs a, const float *state_scales, int8_t *state_q)
{
    extern __shared__ float lds[];
    const int P = a.s.headdim, H = a.s.nheads, G = a.s.ngroups, N = a.s.d_state;
    const int bh = blockIdx.x;
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const Tables t = stage_tables(a, state_scales, bh, h, lds, true);
    const float dt = a.dt[bh];
    const float dA = exp_steps(dt * a.A[h]);
    const float Dh = a.D ? a.D[h] : 0.0f;
    const float sB = a.B_scales[g], sC = a.C_scales[g];
    const int8_t *Bq = a.B + ((size_t)b * G + g) * N;
    const int8_t *Cq = a.C + ((size_t)b * G + g) * N;
    for (int p = wave; p < P; p += kWaves) {
        int8_t *row = state_q + ((size_t)bh * P + p) * N;
        const float dtx = dt * t.xv[p];
        const float *srow = t.s_tab + t.cl[p] * N, *irow = t.inv_tab + t.cl[p] * N;
        float acc = 0.0f;
        for (int n = lane; n < N; n += 64) {
            const float hp = srow[n] * (float)row[n];
            const float d = dA * hp;
            const float u = dtx * (sB * (float)Bq[n]);
            const float hn = d + u;
            acc = __builtin_fmaf(sC * (float)Cq[n], hn, acc);
            row[n] = (int8_t)(code_bits(hn * irow[n]) & 0xffu);
        }
        acc = group_sum<64>(acc);
        if (lane == 0) a.y[(size_t)bh * P + p] = f32_to_f16_bits(__builtin_fmaf(Dh, t.xv[p], acc));
    }
}

// fp32 state (a.state) -> int8 codes with the scales of the cache: one workgroup per (sequence, head), four states
// per thread and trip when d_state is a multiple of 4, one otherwise.
template <bool VEC4>
__global__ __launch_bounds__(kThreads) void quantize_state_kernel(SsdArgs a, const float *state_scales, int8_t *state_q)
{
    extern __shared__ float lds[];
    const int P = a.s.headdim, H = a.s.nheads, N = a.s.d_state;
    const int bh = blockIdx.x;
    const int h = bh % H;
    const Tables t = stage_tables(a, state_scales, bh, h, lds, false);
    const float *src = a.state + (size_t)bh * P * N;
    int8_t *dst = state_q + (size_t)bh * P * N;
    if (VEC4) {
        const int n4 = N / 4;
        for (int i = threadIdx.x; i < P * n4; i += kThreads) {
            const int p = i / n4, n = 4 * (i - p * n4);
            const f32x4 v = *reinterpret_cast<const f32x4 *>(src + (size_t)p * N + n);
            const f32x4 i4 = *reinterpret_cast<const f32x4 *>(t.inv_tab + t.cl[p] * N + n);
            *reinterpret_cast<uint32_t *>(dst + (size_t)p * N + n) =
                pack4(code_bits(v[0] * i4[0]), code_bits(v[1] * i4[1]), code_bits(v[2] * i4[2]), code_bits(v[3] * i4[3]));
        }
    } else {
        for (int i = threadIdx.x; i < P * N; i += kThreads) {
            const int p = i / N, n = i - p * N;
            dst[i] = (int8_t)(code_bits(src[i] * t.inv_tab[t.cl[p] * N + n]) & 0xffu);
        }
    }
}

template <typename K>
hipError_t launch(K kernel, const SsdArgs &a, const float *ss, int8_t *q, size_t lds, hipStream_t stream)
{
    if (lds > 64 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, dim3((unsigned)(a.s.batch * a.s.nheads)), dim3(kThreads), lds, stream, a, ss, q);
    return hipGetLastError();
}

template <int N>
hipError_t launch_vec(const SsdArgs &a, const float *ss, int8_t *q, size_t lds, hipStream_t stream)
{
    constexpr int RPI = 64 / (N / 16);
    const int P = a.s.headdim;
    if (P % (kWaves * RPI * 2) == 0) return launch(decode_q8_vec_kernel<N, 2, true>, a, ss, q, lds, stream);
    if (P % (kWaves * RPI) == 0) return launch(decode_q8_vec_kernel<N, 1, true>, a, ss, q, lds, stream);
    return launch(decode_q8_vec_kernel<N, 1, false>, a, ss, q, lds, stream);
}

}  // namespace

size_t decode_q8_lds_bytes(const quamba_ssd_shape_t &s)
{
    return sizeof(float) * (table_offset(s.headdim) + 2 * (size_t)s.n_chan_clusters * s.d_state);
}

hipError_t launch_decode_q8(const SsdArgs &a, const float *state_scales, int8_t *state_q, hipStream_t stream)
{
    const size_t lds = decode_q8_lds_bytes(a.s);
    const bool al = reinterpret_cast<uintptr_t>(state_q) % 16 == 0 && reinterpret_cast<uintptr_t>(a.B) % 16 == 0 &&
                    reinterpret_cast<uintptr_t>(a.C) % 16 == 0;
    if (al) {
        switch (a.s.d_state) {
            case 16: return launch_vec<16>(a, state_scales, state_q, lds, stream);
            case 32: return launch_vec<32>(a, state_scales, state_q, lds, stream);
            case 64: return launch_vec<64>(a, state_scales, state_q, lds, stream);
            case 128: return launch_vec<128>(a, state_scales, state_q, lds, stream);
            case 256: return launch_vec<256>(a, state_scales, state_q, lds, stream);
            default: break;
        }
    }
    return launch(decode_q8_any_kernel, a, state_scales, state_q, lds, stream);
}

hipError_t launch_quantize_state(const SsdArgs &a, const float *state_scales, int8_t *state_q, hipStream_t stream)
{
    const size_t lds = decode_q8_lds_bytes(a.s);
    const bool vec = a.s.d_state % 4 == 0 && reinterpret_cast<uintptr_t>(a.state) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(state_q) % 4 == 0;
    return vec ? launch(quantize_state_kernel<true>, a, state_scales, state_q, lds, stream)
               : launch(quantize_state_kernel<false>, a, state_scales, state_q, lds, stream);
}

}  // namespace quamba
