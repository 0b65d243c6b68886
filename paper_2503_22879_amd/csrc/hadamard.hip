// Quantized Hadamard transform of the SSD output (Section 4.2): out = Eq.1((1/s_y) H_n y) per row of n = 2^k values,
// the 8-bit input of the output projection whose weight carries the matching H_n offline.
//
// The transform is the radix-2 butterfly network with strides 1, 2, 4, ..., n/2 in this order, in fp32, every add and
// subtract rounded on its own (the codes are integers decided by these roundings, so the order is part of the
// definition; the header states it).  One workgroup per row at a time.  For n >= 1024 a thread keeps 32 values in
// registers and the network runs in three phases of up to 5 strides each, with the values redistributed through LDS
// in between so that the strides of a phase are register-local: phase A on 32 consecutive values (strides 1..16),
// phase B on values 32 apart (strides 32..512), phase C on values 1024 apart (strides 1024..n/2) for groups of
// consecutive values, so that the codes leave as dwords.  The row is read once (fp16, 64 contiguous bytes per thread)
// and written once (int8): 3 bytes of HBM traffic and 17 vector instructions (13 butterflies, a scale, a clamp, a
// rounding add; no packed fp32) per value.  At n = 8192 the vector ALU, the LDS exchanges and HBM each take 40-60 us
// when alone; a row's fp32 image (37 KB of LDS) limits a compute unit to 4 rows in flight, so they overlap only partly.
#include <atomic>

#include "quamba_internal.h"

#pragma clang fp contract(off)

namespace quamba {
namespace {

typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));

constexpr float kMagic = 12582912.0f;  // 1.5 * 2^23: adding it rounds to nearest even, the code is the sum's low byte

// Eq. 1 with the bounds of an 8-bit code for one value (the paths without packing).
__device__ __forceinline__ uint32_t code_byte(float r)
{
    const float c = __builtin_amdgcn_fmed3f(r, -128.0f, 127.0f);
    return __builtin_bit_cast(uint32_t, c + kMagic) & 0xffu;
}

// The same for K = 2 or 4 values packed into the low bytes of a dword: the rounding add writes its low byte straight
// into byte k of the result through the sub-dword destination select.
template <int K>
__device__ __forceinline__ uint32_t codes_packed(const float (&r)[4])
{
    float c[4];
#pragma unroll
    for (int k = 0; k < K; ++k) c[k] = __builtin_amdgcn_fmed3f(r[k], -128.0f, 127.0f);
    uint32_t out;
    asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD"
        : "=v"(out) : "v"(c[0]), "v"(kMagic));
    asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
        : "+v"(out) : "v"(c[1]), "v"(kMagic));
    if (K == 4) {
        asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
            : "+v"(out) : "v"(c[2]), "v"(kMagic));
        asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
            : "+v"(out) : "v"(c[3]), "v"(kMagic));
    }
    return out;
}

// In-register butterflies of one phase: v[e], e = 0..31, strides 1..2^(BITS-1) on the register index.
template <int BITS, int FIRST = 1>
__device__ __forceinline__ void butterflies(float (&v)[32])
{
#pragma unroll
    for (int h = FIRST; h < (1 << BITS); h <<= 1)
#pragma unroll
        for (int e = 0; e < 32; ++e)
            if ((e & h) == 0) {
                const float a = v[e], b = v[e + h];
                v[e] = a + b;
                v[e + h] = a - b;
            }
}

// n = 2^LOGN, 10 <= LOGN <= 14, n/32 threads, as many workgroups as stay resident; each loops over rows
// blockIdx.x, blockIdx.x + gridDim.x, ... and loads its next row (16 registers of packed fp16) while it works on the
// current one, so the HBM latency of a row is hidden behind the arithmetic of the row before.  The loads are plain,
// not non-temporal: a lane's four 16-byte loads walk through one 64-byte sector, which has to stay in the vector cache
// between them (with non-temporal loads every one of the four fetched the sector again and the loads alone took 69 us
// instead of 39 at the 8B layer's size).
// Rows of fewer than 8192 values share a workgroup (8 rows of 1024, 4 of 2048, 2 of 4096), each with its own threads
// and its own piece of LDS, so that a workgroup always has 256 or 512 threads; the rows of a workgroup move through
// the phases together.
template <int LOGN>
constexpr int rows_per_workgroup() { return LOGN >= 13 ? 1 : 1 << (13 - LOGN); }

template <int LOGN>
__global__ __launch_bounds__((1 << (LOGN - 5)) * rows_per_workgroup<LOGN>()) void hadamard_quantize_kernel(
    const uint16_t *y, int8_t *out, int rows, float inv_s)
{
    constexpr int N = 1 << LOGN;
    constexpr int RPW = rows_per_workgroup<LOGN>(), T = N / 32;
    // phase C: a thread holds CONSEC consecutive values at NE places GS apart (4 x 8, n/8 apart; 2 x 16, 1024 apart for
    // n = 16384); the places' index bits that are strides >= 1024 still have their butterflies to come
    constexpr int NE = LOGN == 14 ? 16 : 8;
    constexpr int CONSEC = 32 / NE;
    constexpr int GS = N / NE;
    constexpr int CFIRST = LOGN >= 13 ? 1 : 1 << (13 - LOGN);  // first register stride of phase C that is a stride >= 1024
    extern __shared__ float lds_all[];  // per row 1152 floats per block of 1024 values
    const int t = threadIdx.x % T, rw = threadIdx.x / T;
    float *lds = lds_all + rw * (N / 1024) * 1152;
    const int t_lo = t & 31, t_hi = t >> 5;
    float v[32];
    u32x4 nx[4];
    const long long stride = (long long)gridDim.x * RPW;  // rows between two rounds of a thread

    long long r = (long long)blockIdx.x * RPW + rw;  // the launch has no more workgroups than groups of RPW rows
#pragma unroll
    for (int q = 0; q < 4; ++q) nx[q] = (u32x4){0, 0, 0, 0};
    if (r < rows) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(y + (size_t)r * N + 32 * t);
#pragma unroll
        for (int q = 0; q < 4; ++q) nx[q] = src[q];
    }
    // every thread of the workgroup makes the same number of rounds (the barriers below are the workgroup's); a thread
    // whose row lies past the end works on zeros and stores nothing
    for (long long r0 = (long long)blockIdx.x * RPW; r0 < rows; r0 += stride, r += stride) {
        // phase A: values 32 t + e;
        // stride 1 straight from the packed fp16 pairs: the mixed-precision fused multiply-add takes both halves of a
        // dword as fp16 sources, lo * 1.0 +- hi in fp32 with one rounding (conversion of fp16 to fp32 is exact, so
        // this is the fp32 add or subtract of the converted values)
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w = nx[q][i];
                asm("v_fma_mix_f32 %0, %1, 1.0, %1 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(v[8 * q + 2 * i]) : "v"(w));
                asm("v_fma_mix_f32 %0, %1, 1.0, -%1 op_sel:[0,0,1] op_sel_hi:[1,0,1]"
                    : "=v"(v[8 * q + 2 * i + 1]) : "v"(w));
            }
        if (r + stride < rows) {
            const u32x4 *src = reinterpret_cast<const u32x4 *>(y + (size_t)(r + stride) * N + 32 * t);
#pragma unroll
            for (int q = 0; q < 4; ++q) nx[q] = src[q];
        }
        butterflies<5, 2>(v);
        // Through LDS, transposed inside every block of 1024 values: value 32 a + k of the block (thread a's k-th
        // value) goes to 36 k + a, so that the 32 values the next phase needs in one thread (k fixed, a = 0..31) are
        // 32 consecutive floats, read 16 bytes at a time; the pitch of 36 floats keeps 16 lanes' 16-byte reads on
        // distinct banks, and the writes of consecutive threads are consecutive floats.
        {
            float *pa = lds + t_lo + 1152 * t_hi;
#pragma unroll
            for (int k = 0; k < 32; ++k) pa[36 * k] = v[k];
            __syncthreads();
            // phase B: values i = t_lo + 32 e + 1024 t_hi, e = 0..31
            const f32x4 *pb = reinterpret_cast<const f32x4 *>(lds + 36 * t_lo + 1152 * t_hi);
#pragma unroll
            for (int q = 0; q < 8; ++q) {
                const f32x4 w = pb[q];
                v[4 * q] = w[0]; v[4 * q + 1] = w[1]; v[4 * q + 2] = w[2]; v[4 * q + 3] = w[3];
            }
        }
        butterflies<5>(v);
        __syncthreads();  // all reads of the transposed layout are done before the plain one overwrites it
        {
            float *pb = lds + t_lo + 1024 * t_hi;
#pragma unroll
            for (int e = 0; e < 32; ++e) pb[32 * e] = v[e];
        }
        __syncthreads();

        // phase C: CONSEC consecutive values at CONSEC t + GS e', e' = 0..NE-1; register index k * NE + e', so the
        // strides GS .. n/2 are its low bits, of which those below 1024 are already done
#pragma unroll
        for (int ep = 0; ep < NE; ++ep)
#pragma unroll
            for (int k = 0; k < CONSEC; ++k) v[k * NE + ep] = (lds + CONSEC * t)[k + GS * ep];
        butterflies<(LOGN == 14 ? 4 : 3), CFIRST>(v);

        // Eq. 1 and the store: CONSEC consecutive codes per e'
        int8_t *orow = out + (size_t)r * N + CONSEC * t;
#pragma unroll
        for (int ep = 0; ep < NE; ++ep) {
            if (r >= rows) break;
            if (CONSEC >= 4) {
#pragma unroll
                for (int k = 0; k < CONSEC; k += 4) {
                    const float sc[4] = {v[k * NE + ep] * inv_s, v[(k + 1) * NE + ep] * inv_s,
                                         v[(k + 2) * NE + ep] * inv_s, v[(k + 3) * NE + ep] * inv_s};
                    __builtin_nontemporal_store(codes_packed<4>(sc),
                                                reinterpret_cast<uint32_t *>(orow + GS * ep + k));
                }
            } else {
                const float sc[4] = {v[ep] * inv_s, v[NE + ep] * inv_s, 0.0f, 0.0f};
                *reinterpret_cast<uint16_t *>(orow + GS * ep) = (uint16_t)codes_packed<2>(sc);
            }
        }
        __syncthreads();  // phase C has read the row before the next row's phase A writes
    }
}

// Any power of two n <= 16384: the network stage by stage in LDS.
__global__ __launch_bounds__(256) void hadamard_quantize_small_kernel(const uint16_t *y, int8_t *out, int n, float inv_s)
{
    extern __shared__ float lds[];
    const size_t row = (size_t)blockIdx.x * n;
    for (int i = threadIdx.x; i < n; i += 256) {
        const _Float16 hv = __builtin_bit_cast(_Float16, y[row + i]);
        lds[i] = (float)hv;
    }
    __syncthreads();
    for (int h = 1; h < n; h <<= 1) {
        for (int k = threadIdx.x; k < n / 2; k += 256) {
            const int i = ((k & ~(h - 1)) << 1) | (k & (h - 1));  // k-th index with bit h clear
            const float a = lds[i], b = lds[i + h];
            lds[i] = a + b;
            lds[i + h] = a - b;
        }
        __syncthreads();
    }
    for (int i = threadIdx.x; i < n; i += 256) out[row + i] = (int8_t)code_byte(lds[i] * inv_s);
}

// Orders m * 2^k, m = 12 or 20: H_n = H_m (x) H_{2^k} with H_m from Paley's first construction (q = m - 1 prime, 3 mod 4):
// H_m = I + S, S = [[0, 1^T], [-1, Q]], Q[i, j] = chi(i - j), chi the quadratic character mod q.  chi is a bit mask of
// the non-zero squares mod q, built at compile time.
constexpr uint32_t square_mask(int q)
{
    uint32_t mask = 0;
    for (int v = 1; v < q; ++v) mask |= 1u << ((v * v) % q);
    return mask;
}
template <int M>
constexpr float paley_sign(int a, int b)  // H_M[a][b] as +-1.0f
{
    constexpr int q = M - 1;
    if (a == 0 || a == b) return 1.0f;
    if (b == 0) return -1.0f;
    const int d = ((a - b) % q + q) % q;
    return (square_mask(q) >> d) & 1u ? 1.0f : -1.0f;
}

// One workgroup per row: the butterfly network inside every block of p = 2^k values stage by stage in LDS, then for
// every position j the M-point transform across the blocks, accumulated over the blocks in ascending order (the order
// the header states), Eq. 1, and the codes of 4 consecutive positions per store.
template <int M>
__global__ __launch_bounds__(256) void hadamard_quantize_mixed_kernel(const uint16_t *y, int8_t *out, int p, float inv_s,
                                                                     int out_aligned)
{
    extern __shared__ float lds[];
    const int n = M * p;
    const size_t row = (size_t)blockIdx.x * n;
    for (int i = threadIdx.x; i < n; i += 256) {
        const _Float16 hv = __builtin_bit_cast(_Float16, y[row + i]);
        lds[i] = (float)hv;
    }
    __syncthreads();
    for (int h = 1; h < p; h <<= 1) {
        for (int k = threadIdx.x; k < n / 2; k += 256) {
            const int i = ((k & ~(h - 1)) << 1) | (k & (h - 1));  // k-th index with bit h clear; h < p stays in a block
            const float a = lds[i], b = lds[i + h];
            lds[i] = a + b;
            lds[i + h] = a - b;
        }
        __syncthreads();
    }
    for (int j4 = threadIdx.x; j4 < p / 4; j4 += 256) {
        f32x4 t[M];
#pragma unroll
        for (int b = 0; b < M; ++b) t[b] = *reinterpret_cast<const f32x4 *>(lds + b * p + 4 * j4);
#pragma unroll
        for (int a = 0; a < M; ++a) {
            f32x4 acc = t[0] * paley_sign<M>(a, 0);
#pragma unroll
            for (int b = 1; b < M; ++b) acc = acc + t[b] * paley_sign<M>(a, b);
            const float sc[4] = {acc[0] * inv_s, acc[1] * inv_s, acc[2] * inv_s, acc[3] * inv_s};
            int8_t *dst = out + row + (size_t)a * p + 4 * j4;
            const uint32_t w = codes_packed<4>(sc);
            if (out_aligned) {
                *reinterpret_cast<uint32_t *>(dst) = w;
            } else {
#pragma unroll
                for (int k = 0; k < 4; ++k) dst[k] = (int8_t)(w >> (8 * k));
            }
        }
    }
}

// The same orders with the register-blocked phases of the power-of-two kernel (p = 2^LOGP values per block, 7 <= LOGP
// <= 10, 16-byte aligned rows): phase A, strides 1..16 on the 32 consecutive values a thread loads; exchange through
// LDS, transposed inside super-blocks of 1024 values like the power-of-two kernel's first exchange; phase B, strides
// 32..p/2 on values 32 apart (a thread's 32 values span 1024 / p blocks, the butterflies stay inside each); exchange
// in plain order; phase C, for 2 consecutive positions the M-point sum over the blocks in ascending order, Eq. 1, one
// 2-byte store per block.  A row need not fill its last super-block: the missing part is never written, and what
// phase B reads of it stays in register groups of its own that are not used.
template <int M, int LOGP>
__global__ void hadamard_quantize_mixed_fast_kernel(const uint16_t *y, int8_t *out, float inv_s)
{
    constexpr int P = 1 << LOGP, N = M * P, T = N / 32, NSB = (N + 1023) / 1024;
    extern __shared__ float lds[];  // NSB * 1152 floats
    const int t = threadIdx.x;
    const size_t row = (size_t)blockIdx.x * N;
    float v[32];
    if (t < T) {
        const u32x4 *src = reinterpret_cast<const u32x4 *>(y + row + 32 * t);
        u32x4 nx[4];
#pragma unroll
        for (int q = 0; q < 4; ++q) nx[q] = src[q];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const uint32_t w = nx[q][i];
                asm("v_fma_mix_f32 %0, %1, 1.0, %1 op_sel:[0,0,1] op_sel_hi:[1,0,1]" : "=v"(v[8 * q + 2 * i]) : "v"(w));
                asm("v_fma_mix_f32 %0, %1, 1.0, -%1 op_sel:[0,0,1] op_sel_hi:[1,0,1]"
                    : "=v"(v[8 * q + 2 * i + 1]) : "v"(w));
            }
        butterflies<5, 2>(v);
        float *pa = lds + (t & 31) + 1152 * (t >> 5);
#pragma unroll
        for (int k = 0; k < 32; ++k) pa[36 * k] = v[k];
    }
    __syncthreads();
    const int t_lo = t & 31, t_hi = t >> 5;
    if (t_hi < NSB) {
        // phase B: values i = t_lo + 32 e + 1024 t_hi, e = 0..31; e's low LOGP - 5 bits are the strides 32..p/2
        const f32x4 *pb = reinterpret_cast<const f32x4 *>(lds + 36 * t_lo + 1152 * t_hi);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
            const f32x4 w = pb[q];
            v[4 * q] = w[0]; v[4 * q + 1] = w[1]; v[4 * q + 2] = w[2]; v[4 * q + 3] = w[3];
        }
        butterflies<LOGP - 5>(v);
    }
    __syncthreads();  // all reads of the transposed layout are done before the plain one overwrites it
    if (t_hi < NSB) {
        float *pb = lds + t_lo + 1024 * t_hi;
#pragma unroll
        for (int e = 0; e < 32; ++e)
            if (1024 * t_hi + 32 * e < N) pb[32 * e] = v[e];  // uniform per wave half: whole groups of 32 lanes
    }
    __syncthreads();
    if (t < P / 2) {
        // phase C: positions 2 t and 2 t + 1 of every block
        float t0[M], t1[M];
#pragma unroll
        for (int b = 0; b < M; ++b) {
            t0[b] = lds[b * P + 2 * t];
            t1[b] = lds[b * P + 2 * t + 1];
        }
#pragma unroll
        for (int a = 0; a < M; ++a) {
            float a0 = t0[0] * paley_sign<M>(a, 0), a1 = t1[0] * paley_sign<M>(a, 0);
#pragma unroll
            for (int b = 1; b < M; ++b) {
                a0 = a0 + t0[b] * paley_sign<M>(a, b);
                a1 = a1 + t1[b] * paley_sign<M>(a, b);
            }
            const float sc[4] = {a0 * inv_s, a1 * inv_s, 0.0f, 0.0f};
            *reinterpret_cast<uint16_t *>(out + row + (size_t)a * P + 2 * t) = (uint16_t)codes_packed<2>(sc);
        }
    }
}

template <int M, int LOGP>
hipError_t launch_mixed_fast(const uint16_t *y, int64_t rows, float inv_s, int8_t *out, hipStream_t stream)
{
    constexpr int P = 1 << LOGP, N = M * P, NSB = (N + 1023) / 1024;
    constexpr int need = N / 32 > 32 * NSB ? N / 32 : 32 * NSB;
    constexpr int threads = ((need > P / 2 ? need : P / 2) + 63) / 64 * 64;
    constexpr int lds = NSB * 1152 * (int)sizeof(float);
    static_assert(threads <= 1024 && lds <= 160 * 1024, "launch shape");
    if (lds > 48 * 1024) {  // raise the kernel's LDS limit once per device
        static std::atomic<uint32_t> done{0};
        int dev = 0;
        hipError_t e = hipGetDevice(&dev);
        if (e != hipSuccess) return e;
        if (dev < 0 || dev >= 32 || !(done.load() >> dev & 1u)) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(hadamard_quantize_mixed_fast_kernel<M, LOGP>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
            if (dev >= 0 && dev < 32) done.fetch_or(1u << dev);
        }
    }
    hipLaunchKernelGGL((hadamard_quantize_mixed_fast_kernel<M, LOGP>), dim3((unsigned)rows), dim3(threads), lds, stream, y,
                       out, inv_s);
    return hipGetLastError();
}

template <int LOGN>
hipError_t launch_fast(const uint16_t *y, int64_t rows, float inv_s, int8_t *out, hipStream_t stream)
{
    constexpr int N = 1 << LOGN, RPW = rows_per_workgroup<LOGN>();
    constexpr int lds = RPW * (N / 1024) * 1152 * (int)sizeof(float);
    // twice the workgroups that fit the device at once (measured best; one round of exactly resident workgroups
    // is 10% slower), asked of the runtime once per order and device
    static std::atomic<int> resident[16];  // zero-initialised; concurrent first calls compute the same value
    int dev = 0;
    hipError_t e = hipGetDevice(&dev);
    if (e != hipSuccess) return e;
    if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
    if (!resident[dev].load()) {
        if (lds > 48 * 1024) {
            e = hipFuncSetAttribute(reinterpret_cast<const void *>(hadamard_quantize_kernel<LOGN>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, lds);
            if (e != hipSuccess) return e;
        }
        int per_cu = 0, cus = 0;
        e = hipOccupancyMaxActiveBlocksPerMultiprocessor(&per_cu, hadamard_quantize_kernel<LOGN>, RPW * N / 32, lds);
        if (e != hipSuccess) return e;
        e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
        if (e != hipSuccess) return e;
        resident[dev].store(per_cu > 0 && cus > 0 ? 2 * per_cu * cus : 2048);
    }
    const int res = resident[dev].load();
    const int64_t groups = (rows + RPW - 1) / RPW;
    const unsigned grid = (unsigned)(groups < res ? groups : res);
    hipLaunchKernelGGL(hadamard_quantize_kernel<LOGN>, dim3(grid), dim3(RPW * N / 32), lds, stream, y, out, (int)rows,
                       inv_s);
    return hipGetLastError();
}

}  // namespace

bool hadamard_order_supported(int n)
{
    if (n < 2 || n > 16384) return false;
    if ((n & (n - 1)) == 0) return true;
    for (int m : {12, 20})
        if (n % m == 0 && ((n / m) & (n / m - 1)) == 0 && n / m >= 4) return true;
    return false;
}

hipError_t launch_hadamard_quantize(const uint16_t *y, int64_t rows, int n, float s_y, int8_t *out, hipStream_t stream)
{
    if (rows == 0) return hipSuccess;
    const float inv_s = 1.0f / s_y;  // correctly rounded fp32 division on the host
    if (n & (n - 1)) {
        const int m = (n % 12 == 0 && ((n / 12) & (n / 12 - 1)) == 0) ? 12 : 20;
        if (reinterpret_cast<uintptr_t>(y) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 2 == 0) {
            switch (n) {  // the register-blocked kernel for blocks of 128 .. 1024 values
                case 12 * 128: return launch_mixed_fast<12, 7>(y, rows, inv_s, out, stream);
                case 12 * 256: return launch_mixed_fast<12, 8>(y, rows, inv_s, out, stream);
                case 12 * 512: return launch_mixed_fast<12, 9>(y, rows, inv_s, out, stream);
                case 12 * 1024: return launch_mixed_fast<12, 10>(y, rows, inv_s, out, stream);
                case 20 * 128: return launch_mixed_fast<20, 7>(y, rows, inv_s, out, stream);
                case 20 * 256: return launch_mixed_fast<20, 8>(y, rows, inv_s, out, stream);
                case 20 * 512: return launch_mixed_fast<20, 9>(y, rows, inv_s, out, stream);
                default: break;
            }
        }
        const int lds = n * (int)sizeof(float);
        const int aligned = reinterpret_cast<uintptr_t>(out) % 4 == 0;
        if (m == 12) {
            if (lds > 48 * 1024) {
                const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(hadamard_quantize_mixed_kernel<12>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
                if (e != hipSuccess) return e;
            }
            hipLaunchKernelGGL(hadamard_quantize_mixed_kernel<12>, dim3((unsigned)rows), dim3(256), lds, stream, y, out,
                               n / 12, inv_s, aligned);
        } else {
            if (lds > 48 * 1024) {
                const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(hadamard_quantize_mixed_kernel<20>),
                                                         hipFuncAttributeMaxDynamicSharedMemorySize, lds);
                if (e != hipSuccess) return e;
            }
            hipLaunchKernelGGL(hadamard_quantize_mixed_kernel<20>, dim3((unsigned)rows), dim3(256), lds, stream, y, out,
                               n / 20, inv_s, aligned);
        }
        return hipGetLastError();
    }
    const bool al = reinterpret_cast<uintptr_t>(y) % 16 == 0 && reinterpret_cast<uintptr_t>(out) % 4 == 0;
    if (al) {
        switch (n) {
            case 1024: return launch_fast<10>(y, rows, inv_s, out, stream);
            case 2048: return launch_fast<11>(y, rows, inv_s, out, stream);
            case 4096: return launch_fast<12>(y, rows, inv_s, out, stream);
            case 8192: return launch_fast<13>(y, rows, inv_s, out, stream);
            case 16384: return launch_fast<14>(y, rows, inv_s, out, stream);
            default: break;
        }
    }
    const int lds = n * (int)sizeof(float);
    if (lds > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(hadamard_quantize_small_kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(hadamard_quantize_small_kernel, dim3((unsigned)rows), dim3(256), lds, stream, y, out, n, inv_s);
    return hipGetLastError();
}

}  // namespace quamba
