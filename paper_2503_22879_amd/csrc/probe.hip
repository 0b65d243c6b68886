// Measurement helpers of the benchmark harness (not part of the method): what this machine attains for the matrix
// cores and for an in-place HBM stream, and the shader clock it runs at.  See include/quamba_probe.h.
#include <hip/hip_runtime.h>

#include "quamba_probe.h"
#include "quamba_ssd.h"

namespace {

typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kProbeThreads = 256;     // 4 waves per workgroup
constexpr int kChains = 4;             // independent accumulators per wave

template <int KIND>
__global__ __launch_bounds__(kProbeThreads) void mfma_probe_kernel(int iters, int uniform, uint32_t *sink)
{
    // uniform: every lane holds the same operand values (few bits toggle between lanes: the matrix cores draw less
    // power and the board stays below its cap); otherwise the operands differ from lane to lane
    const int lane = uniform ? 3 : (int)(threadIdx.x & 63);
    uint32_t keep = 0;
    if (KIND == 0) {
        f16x8 a, b;
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            a[i] = (_Float16)(0.001f * (float)(lane + i));
            b[i] = (_Float16)(0.002f * (float)(lane - i));
        }
        f32x16 acc[kChains];
#pragma unroll
        for (int c = 0; c < kChains; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][r] = 0.0f;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, acc[c], 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < kChains; ++c) keep += __builtin_bit_cast(uint32_t, acc[c][c]);
    } else {
        i32x4 a, b;
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            a[i] = 0x01020304 * (lane + i);
            b[i] = 0x04030201 * (lane - i);
        }
        i32x16 acc[kChains];
#pragma unroll
        for (int c = 0; c < kChains; ++c)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[c][r] = 0;
        for (int it = 0; it < iters; ++it) {
#pragma unroll
            for (int c = 0; c < kChains; ++c) acc[c] = __builtin_amdgcn_mfma_i32_32x32x32_i8(a, b, acc[c], 0, 0, 0);
        }
#pragma unroll
        for (int c = 0; c < kChains; ++c) keep += (uint32_t)acc[c][c];
    }
    if (keep == 0x9e3779b9u) sink[0] = keep;  // practically never: keeps the loop alive
}

// Every workgroup owns a contiguous run of 256 x kRmwPieces 16-byte pieces: all its loads are issued before the first
// store, so that a wave keeps kRmwPieces pieces per lane in flight (the shape that streams fastest on this machine).
constexpr int kRmwPieces = 8;
__global__ __launch_bounds__(256) void stream_rmw_kernel(u32x4 *buf, size_t n16)
{
    const size_t base = (size_t)blockIdx.x * 256 * kRmwPieces + threadIdx.x;
    if (base - threadIdx.x + 256 * kRmwPieces <= n16) {  // a whole run (all workgroups but possibly the last)
        u32x4 v[kRmwPieces];
#pragma unroll
        for (int i = 0; i < kRmwPieces; ++i) v[i] = __builtin_nontemporal_load(buf + base + (size_t)i * 256);
#pragma unroll
        for (int i = 0; i < kRmwPieces; ++i) {
            v[i] += (u32x4){1u, 2u, 3u, 4u};  // every dword changes: the whole piece is read and written
            __builtin_nontemporal_store(v[i], buf + base + (size_t)i * 256);
        }
    } else {
        for (size_t j = base; j < n16; j += 256) {
            u32x4 v = __builtin_nontemporal_load(buf + j);
            v += (u32x4){1u, 2u, 3u, 4u};
            __builtin_nontemporal_store(v, buf + j);
        }
    }
}

// Read-only pass: every workgroup strides over the buffer (consecutive lanes on consecutive 16-byte pieces) and folds
// what it reads into one word that is stored only in a case that practically never occurs.
__global__ __launch_bounds__(256) void stream_read_kernel(const u32x4 *buf, size_t n16, uint32_t *sink)
{
    const size_t stride = (size_t)gridDim.x * 256;
    u32x4 s = {0u, 0u, 0u, 0u};
    for (size_t i = (size_t)blockIdx.x * 256 + threadIdx.x; i < n16; i += stride) s += buf[i];
    const uint32_t keep = s[0] ^ s[1] ^ s[2] ^ s[3];
    if (keep == 0x9e3779b9u) sink[0] = keep;
}

__global__ __launch_bounds__(64) void clock_probe_kernel(int64_t *out, int spin_iters)
{
    const long long c0 = __builtin_amdgcn_s_memtime();
    const long long r0 = __builtin_amdgcn_s_memrealtime();
    float v = (float)threadIdx.x;
    for (int i = 0; i < spin_iters; ++i) v = __builtin_fmaf(v, 1.0000001f, 1.0e-7f);
    asm volatile("" : "+v"(v));
    const long long c1 = __builtin_amdgcn_s_memtime();
    const long long r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0) {
        out[0] = c1 - c0;
        out[1] = r1 - r0;
    }
    if (v == 12345.678f) out[0] = 0;
}

// One wave per workgroup; the hardware hands consecutive workgroup ids to the XCDs in turn, so n workgroups sample n
// XCDs (the id register read back says which).
__global__ __launch_bounds__(64) void clock_probe_xcd_kernel(int64_t *out, int spin_iters)
{
    const long long c0 = __builtin_amdgcn_s_memtime();
    const long long r0 = __builtin_amdgcn_s_memrealtime();
    float v = (float)threadIdx.x;
    for (int i = 0; i < spin_iters; ++i) v = __builtin_fmaf(v, 1.0000001f, 1.0e-7f);
    asm volatile("" : "+v"(v));
    const long long c1 = __builtin_amdgcn_s_memtime();
    const long long r1 = __builtin_amdgcn_s_memrealtime();
    if (threadIdx.x == 0) {
        int64_t *o = out + 3 * (size_t)blockIdx.x;
        o[0] = c1 - c0;
        o[1] = r1 - r0;
        o[2] = (int64_t)(__builtin_amdgcn_s_getreg(20 | (0 << 6) | (3 << 11)) & 0xf);  // XCC_ID, bits 3:0
    }
    if (v == 12345.678f) out[0] = 0;
}

int device_cus()
{
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess) return 256;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) return 256;
    return n;
}

}  // namespace

extern "C" int quamba_probe_mfma(int kind, int iters, int waves_per_simd, int uniform_operands, double *ops_out,
                                 uint32_t *sink, void *stream)
{
    if (!ops_out || !sink) return QUAMBA_ENULL;
    if ((kind != 0 && kind != 1) || iters <= 0 || waves_per_simd < 1 || waves_per_simd > 8) return QUAMBA_EINVAL;
    const int blocks = device_cus() * waves_per_simd;  // a workgroup is 4 waves, one per SIMD of its compute unit
    const double per_inst = kind == 0 ? 32.0 * 32.0 * 16.0 * 2.0 : 32.0 * 32.0 * 32.0 * 2.0;
    *ops_out = per_inst * kChains * (double)iters * (kProbeThreads / 64) * blocks;
    if (kind == 0)
        hipLaunchKernelGGL(mfma_probe_kernel<0>, dim3(blocks), dim3(kProbeThreads), 0, (hipStream_t)stream, iters,
                           uniform_operands, sink);
    else
        hipLaunchKernelGGL(mfma_probe_kernel<1>, dim3(blocks), dim3(kProbeThreads), 0, (hipStream_t)stream, iters,
                           uniform_operands, sink);
    return hipGetLastError() == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_probe_stream_rmw(void *buf, size_t n_bytes, void *stream)
{
    if (!buf) return QUAMBA_ENULL;
    if (n_bytes == 0 || n_bytes % 16) return QUAMBA_EINVAL;
    const size_t n16 = n_bytes / 16;
    const size_t blocks = (n16 + 256 * kRmwPieces - 1) / (256 * kRmwPieces);
    if (blocks > 0x7fffffffull) return QUAMBA_EINVAL;
    hipLaunchKernelGGL(stream_rmw_kernel, dim3((unsigned)blocks), dim3(256), 0, (hipStream_t)stream,
                       static_cast<u32x4 *>(buf), n16);
    return hipGetLastError() == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_probe_stream_read(const void *buf, size_t n_bytes, uint32_t *sink, void *stream)
{
    if (!buf || !sink) return QUAMBA_ENULL;
    if (n_bytes == 0 || n_bytes % 16) return QUAMBA_EINVAL;
    int dev = 0, cus = 256;
    if (hipGetDevice(&dev) != hipSuccess) return QUAMBA_EHIP;
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    hipLaunchKernelGGL(stream_read_kernel, dim3((unsigned)(cus * 16)), dim3(256), 0, (hipStream_t)stream,
                       static_cast<const u32x4 *>(buf), n_bytes / 16, sink);
    return hipGetLastError() == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_probe_clock_xcd(int64_t *out, int n, int spin_iters, void *stream)
{
    if (!out) return QUAMBA_ENULL;
    if (n <= 0 || n > 64 || spin_iters <= 0) return QUAMBA_EINVAL;
    hipLaunchKernelGGL(clock_probe_xcd_kernel, dim3((unsigned)n), dim3(64), 0, (hipStream_t)stream, out, spin_iters);
    return hipGetLastError() == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_probe_clock(int64_t *out, int spin_iters, void *stream)
{
    if (!out) return QUAMBA_ENULL;
    if (spin_iters <= 0) return QUAMBA_EINVAL;
    hipLaunchKernelGGL(clock_probe_kernel, dim3(1), dim3(64), 0, (hipStream_t)stream, out, spin_iters);
    return hipGetLastError() == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}
