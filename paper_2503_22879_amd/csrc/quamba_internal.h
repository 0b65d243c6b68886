// Internal launch interface between the C-ABI layer and the HIP kernels (not installed).
#pragma once
#include <hip/hip_runtime.h>

#include "quamba_ssd.h"

namespace quamba {

// Device pointers of one call, shared by all kernels.
struct SsdArgs {
    quamba_ssd_shape_t s;
    const float *x_scales;
    const int32_t *head_cluster_end;
    const int32_t *chan_cluster_end;
    const float *B_scales;
    const float *C_scales;
    const int8_t *x;
    const int8_t *B;
    const int8_t *C;
    const float *dt;
    const float *A;
    const float *D;            // may be null
    const float *init_state;   // may be null (prefill)
    float *state;              // decode: in/out; prefill: final state or null
    uint16_t *y;               // fp16 bits
    // optional 8-bit side inputs (quamba_ssd_gate_t); all null / zero when absent
    const int8_t *z;           // gate codes, laid out like x
    float z_scale;
    const int8_t *dt_q;        // codes of the step size's pre-activation, laid out like dt (dt is then unused)
    float dt_scale;
    const float *dt_bias;      // [nheads] or null
    // Sequence split of the chunked prefill (matrix-core kernels only; nseg == 1: none).  The sequence is cut into nseg
    // segments of seg_chunks 128-token chunks (the last takes the rest).  A first kernel walks segments 0 .. nseg-2
    // without producing outputs and leaves, per segment, the state it ends with when started from zero (segment 0:
    // from init_state) and the sum of dt*A*log2(e) over its tokens; the prefill kernel then gives every segment its
    // own workgroups, which start from the combination of those.
    int32_t nseg;
    int32_t seg_chunks;
    float *seg_state;          // [nseg-1][batch*nheads][headdim][d_state], in the kernel's accumulator units
    float *seg_decay;          // [nseg-1][batch*nheads]
    int32_t pace_first;        // matrix-core prefill: first workgroup id of the second dispatch round when the two
                               // workgroups of a compute unit are to be kept at the same pace (see the kernel), else
                               // INT_MAX
};

// Plan of the sequence split for a shape on the current device: segments (1 = no split), chunks per segment, and
// whether every head is cut into two workgroups of 32 channels each.
struct PrefillPlan {
    int nseg;
    int seg_chunks;
    bool channel_split;
};
PrefillPlan prefill_mfma_plan(const quamba_ssd_shape_t &s);
size_t prefill_mfma_workspace_bytes(const quamba_ssd_shape_t &s);

// Step size of (token or sequence) index idx of head h: the caller's fp32 dt, or softplus(s_dt * code + bias[h])
// (Section 3.2: Delta = softplus(F(x)) with the bias) when the pre-activation comes as int8 codes.
__device__ __forceinline__ float step_size(const SsdArgs &a, size_t idx, int h)
{
    if (!a.dt_q) return a.dt[idx];
    const float v = a.dt_scale * (float)a.dt_q[idx] + (a.dt_bias ? a.dt_bias[h] : 0.0f);
    return fmaxf(v, 0.0f) + log1pf(expf(-fabsf(v)));  // log(1 + exp(v)) without overflow
}

// SiLU(z) = z / (1 + exp(-z)) of a gate code (Section 3.2: the optional branch z multiplies the SSM output).
__device__ __forceinline__ float silu_of_code(float z_scale, int code)
{
    const float z = z_scale * (float)code;
    return z * __frcp_rn(1.0f + __expf(-z));
}

// Index of the (group, head cluster, channel range) cell of channel position p of head h in the cluster boundary
// tables (Section 4.1: m x n cells per group).  The cluster index is the number of boundaries at or below the
// position, so all boundary loads are independent (three dependent memory round trips in total instead of one per
// boundary).
__device__ __forceinline__ int cell_lookup(const SsdArgs &a, int h, int p, int *first_cell_of_head = nullptr)
{
    const int hpg = a.s.nheads / a.s.ngroups;
    const int g = h / hpg, hl = h - g * hpg;
    const int m = a.s.n_head_clusters, n = a.s.n_chan_clusters;
    int i = 0;
    for (int k = 0; k < m - 1; ++k) i += hl >= a.head_cluster_end[g * m + k] ? 1 : 0;
    const int base = (g * m + i) * n;  // the head cluster's n cells are base .. base + n - 1
    if (first_cell_of_head) *first_cell_of_head = base;
    int j = 0;
    for (int k = 0; k < n - 1; ++k) j += p >= a.chan_cluster_end[base + k] ? 1 : 0;
    return base + j;
}

// Scale of channel position p of head h (Section 4.1: one scale per cell).
__device__ __forceinline__ float x_scale_lookup(const SsdArgs &a, int h, int p)
{
    return a.x_scales[cell_lookup(a, h, p)];
}

// fp32 -> fp16 bits, round to nearest even.
__device__ __forceinline__ uint16_t f32_to_f16_bits(float v)
{
    const _Float16 h = (_Float16)v;
    return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ float from_bits(uint32_t u) { return __builtin_bit_cast(float, u); }

// exp(z) for z <= 0 as separately rounded fp32 steps: t = z log2(e), k = rint(t), f = t - k in [-1/2, 1/2],
// 2^f = sum_i ((ln 2)^i / i!) f^i (i = 7..0, Horner, multiply then add), result 2^f 2^k; t < -125 gives 0 so that
// no result is subnormal.  Constants are the fp32 roundings of log2(e) and of the Taylor coefficients.  Used where an
// integer code depends on the result, so that it is the same fixed sequence of roundings on every machine.
__device__ __forceinline__ float exp_steps(float z)
{
#pragma clang fp contract(off)
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

template <int CTRL>
__device__ __forceinline__ float dpp_move(float v)
{
    return __builtin_bit_cast(float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, 0xf, 0xf, true));
}

// Sum over groups of LANES consecutive lanes (LANES a power of two <= 64); every lane of a group gets the sum.
// Steps inside a row of 16 lanes are data-parallel-primitive moves fused into the adds (no LDS traffic): swap
// inside pairs, swap pairs inside quads, mirror inside 8, mirror inside 16; the step across rows is one swizzle.
template <int LANES>
__device__ __forceinline__ float group_sum(float v)
{
    if (LANES >= 2) v += dpp_move<0xB1>(v);   // quad_perm [1,0,3,2]
    if (LANES >= 4) v += dpp_move<0x4E>(v);   // quad_perm [2,3,0,1]
    if (LANES >= 8) v += dpp_move<0x141>(v);  // row_half_mirror
    if (LANES >= 16) v += dpp_move<0x140>(v); // row_mirror
    if (LANES >= 32)  // lane ^ 16
        v += __builtin_bit_cast(float, __builtin_amdgcn_ds_swizzle(__builtin_bit_cast(int, v), 0x401F));
    if (LANES >= 64) v += __shfl_xor(v, 32, 64);
    return v;
}

hipError_t launch_decode(const SsdArgs &a, hipStream_t stream);
// 8-bit cached state (Appendix E): the step on int8 codes in place, and the quantizer of an fp32 state (a.state)
hipError_t launch_decode_q8(const SsdArgs &a, const float *state_scales, int8_t *state_q, hipStream_t stream);
hipError_t launch_quantize_state(const SsdArgs &a, const float *state_scales, int8_t *state_q, hipStream_t stream);
size_t decode_q8_lds_bytes(const quamba_ssd_shape_t &s);
// Quantized Hadamard transform of rows of n = 2^k fp16 values (Section 4.2)
hipError_t launch_hadamard_quantize(const uint16_t *y, int64_t rows, int n, float s_y, int8_t *out, hipStream_t stream);
bool hadamard_order_supported(int n);  // 2^k, or 12 * 2^k / 20 * 2^k with k >= 2, up to 16384
// W8A8 causal convolution in front of the scan (4 taps, SiLU, Eq. 1 to the scan's operands)
struct ConvArgs {
    quamba_ssd_shape_t s;
    const float *x_scales;
    const int32_t *head_cluster_end;
    const int32_t *chan_cluster_end;
    const float *B_scales;
    const float *C_scales;
    const int8_t *in;         // [b, L, HP + 2 GN]
    const int8_t *weight;     // [HP + 2 GN, 4]
    const float *bias;        // [HP + 2 GN] or null
    float in_w_scale;
    const int8_t *state_in;   // [b, 3, HP + 2 GN] or null
    int8_t *state_out;        // same shape, or null
    int8_t *x_out, *B_out, *C_out;
    int seg;                  // tokens per workgroup (set by the launcher)
};
hipError_t launch_conv1d_q8(const ConvArgs &a, hipStream_t stream);
int conv1d_segments(const quamba_ssd_shape_t &s);  // workgroups along one sequence (1: state_in may equal state_out)
// Mamba1 selective scan: shape has nheads = ngroups = 1, headdim = channels; A is [channels, d_state]
hipError_t launch_mamba1_scan(const SsdArgs &a, const float *A, const float *init, float *fin, hipStream_t stream);
hipError_t launch_mamba1_decode(const SsdArgs &a, const float *A, hipStream_t stream);
bool mamba1_scan_supports_any(const quamba_ssd_shape_t &s);
hipError_t launch_prefill_generic(const SsdArgs &a, hipStream_t stream);
bool prefill_mfma_supports(const quamba_ssd_shape_t &s);
hipError_t launch_prefill_mfma(const SsdArgs &a, void *workspace, hipStream_t stream);
size_t prefill_generic_lds_bytes(const quamba_ssd_shape_t &s);

}  // namespace quamba
