// W8A8 causal convolution in front of the scan (Section 4.2, "Efficient 4-bit/8-bit Mamba blocks"): the depthwise
// 4-tap convolution over time of the block's concatenated channels [x | B | C], bias, SiLU, and Eq. 1 to the 8-bit
// operands of the SSD kernel -- x with the sort-and-cluster cell scales, B and C with their per-state-group scales
// (Section 4.1) -- written straight into the scan's three input tensors.  The channel order is the sorted order
// the offline reordering gives the convolution's weights (Section 4.2), so nothing is permuted here.
//
// A thread owns 16 consecutive channels (one 16-byte load per token) and walks a segment of 16 or 32 tokens.  Per channel it
// keeps the last four input codes in one dword (byte k = tap k, the newest in byte 3): a byte permute shifts the new
// code in, one 4-way int8 dot product with the channel's packed taps gives the exact integer sum.  The code is an
// integer decided by fp32 arithmetic; the decision sequence (stated in the header) is evaluated with every operation
// rounded on its own.
#include "quamba_internal.h"

#pragma clang fp contract(off)

namespace quamba {
namespace {

constexpr int kSegLong = 32;   // tokens per workgroup of the vector kernel when that still gives the device enough waves,
constexpr int kSegShort = 16;  // else this many
constexpr int kWaveSlots = 4096;  // resident waves at this kernel's register budget (1024 SIMDs x 4)
constexpr int kAhead = 4;      // tokens whose loads are in flight
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

// r = SiLU(acc * s_cw + bias) * inv in the stated order: the value Eq. 1 rounds.
__device__ __forceinline__ float activation_over_scale(int acc, float s_cw, float bias, float inv)
{
    float v = (float)acc * s_cw;
    v = v + bias;
    const float e = exp_steps(-__builtin_fabsf(v));
    const float den = 1.0f + e;
    const float num = v >= 0.0f ? v : v * e;
    const float a = __fdiv_rn(num, den);
    return a * inv;
}

// The same value through the hardware's approximate base-2 exponential and reciprocal (1 unit in the last place
// each): v / (1 + 2^(-v log2 e)) * inv.  It shares v and the rounded exponent argument with the exact sequence above
// (whose e is 2^-|t| for the same t), so the two differ only by the roundings after that point: by less than
// 1e-6 of the value (derivation in the design notes).  Deeply negative v gives 2^t = inf and the result -0.
__device__ __forceinline__ float activation_over_scale_fast(int acc, float s_cw, float bias, float inv)
{
    float v = (float)acc * s_cw;
    v = v + bias;
    const float E = __builtin_amdgcn_exp2f(-v * from_bits(0x3FB8AA3Bu));
    const float w = __builtin_amdgcn_rcpf(1.0f + E);
    const float a = v * w;
    return a * inv;
}

// True when a clamped pre-rounding value c from the fast evaluation might round to another integer than the exact
// sequence's value: when it lies within 2e-6 |c| + 1e-6 (twice the bound on their difference) of a half-integer.
__device__ __forceinline__ bool near_rounding_boundary(float c)
{
    const float d = c - __builtin_rintf(c);
    return __builtin_fabsf(d) >= __builtin_fmaf(-2e-6f, __builtin_fabsf(c), 0.499999f);
}

// Eq. 1 for four clamped values into one dword: the rounding add (1.5 * 2^23) writes its low byte into byte k.
__device__ __forceinline__ uint32_t codes4(float c0, float c1, float c2, float c3)  // values already clamped
{
    const float magic = 12582912.0f;
    uint32_t out;
    asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_0 dst_unused:UNUSED_PAD src0_sel:DWORD src1_sel:DWORD"
        : "=v"(out) : "v"(c0), "v"(magic));
    asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_1 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
        : "+v"(out) : "v"(c1), "v"(magic));
    asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_2 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
        : "+v"(out) : "v"(c2), "v"(magic));
    asm("v_add_f32_sdwa %0, %1, %2 dst_sel:BYTE_3 dst_unused:UNUSED_PRESERVE src0_sel:DWORD src1_sel:DWORD"
        : "+v"(out) : "v"(c3), "v"(magic));
    return out;
}

__device__ __forceinline__ uint32_t code1(float r)
{
    const float c = __builtin_amdgcn_fmed3f(r, -128.0f, 127.0f);
    return __builtin_bit_cast(uint32_t, c + 12582912.0f) & 0xffu;
}

// Eq. 1 scale of concatenated channel c (x: cell of (head, position); B, C: the state group's scale), and where its
// code goes: *dst is the output tensor, *row its row length, *col the column.
__device__ __forceinline__ float channel_scale(const ConvArgs &a, int c, int8_t **dst, int *row, int *col)
{
    const int HP = a.s.nheads * a.s.headdim, GN = a.s.ngroups * a.s.d_state;
    if (c < HP) {
        *dst = a.x_out; *row = HP; *col = c;
        SsdArgs t;
        t.s = a.s; t.x_scales = a.x_scales; t.head_cluster_end = a.head_cluster_end;
        t.chan_cluster_end = a.chan_cluster_end;
        const int h = c / a.s.headdim;
        return x_scale_lookup(t, h, c - h * a.s.headdim);
    }
    if (c < HP + GN) {
        *dst = a.B_out; *row = GN; *col = c - HP;
        return a.B_scales[(c - HP) / a.s.d_state];
    }
    *dst = a.C_out; *row = GN; *col = c - HP - GN;
    return a.C_scales[(c - HP - GN) / a.s.d_state];
}

// Input code of token tau (may be negative: then from the carried state, whose row 3 + tau it is, or zero).
__device__ __forceinline__ const int8_t *token_row(const ConvArgs &a, int b, int tau, int Ct)
{
    if (tau >= 0) return a.in + ((size_t)b * a.s.seqlen + tau) * Ct;
    return a.state_in ? a.state_in + ((size_t)b * 3 + (3 + tau)) * Ct : nullptr;
}

// Vector kernel: headdim, d_state multiples of 16 and 16-byte aligned tensors.  grid = (channel blocks of 64 x 16,
// segments, batch); one wave per workgroup, no LDS, no barrier.
__global__ __launch_bounds__(64) void conv1d_q8_vec_kernel(ConvArgs a)
{
    const int HP = a.s.nheads * a.s.headdim, GN = a.s.ngroups * a.s.d_state, Ct = HP + 2 * GN;
    const int c0 = 16 * (blockIdx.x * 64 + threadIdx.x);
    if (c0 >= Ct) return;
    const int b = blockIdx.z, L = a.s.seqlen;
    const int t0 = blockIdx.y * a.seg, t1 = min(t0 + a.seg, L);

    // per-channel constants: packed taps, bias, reciprocal output scale (one correctly rounded division each)
    uint32_t w[16];
    float bias[16], inv[16];
    int8_t *dst; int row, col;
    {
        const u32x4 *wp = reinterpret_cast<const u32x4 *>(a.weight + (size_t)c0 * 4);
#pragma unroll
        for (int q = 0; q < 4; ++q) {
            const u32x4 v = wp[q];
            w[4 * q] = v[0]; w[4 * q + 1] = v[1]; w[4 * q + 2] = v[2]; w[4 * q + 3] = v[3];
        }
        if (a.bias) {
            const f32x4 *bp = reinterpret_cast<const f32x4 *>(a.bias + c0);  // c0 is a multiple of 16: 64-byte aligned
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const f32x4 v = bp[q];
                bias[4 * q] = v[0]; bias[4 * q + 1] = v[1]; bias[4 * q + 2] = v[2]; bias[4 * q + 3] = v[3];
            }
        } else {
#pragma unroll
            for (int j = 0; j < 16; ++j) bias[j] = 0.0f;
        }
        // The 16 channels share one output tensor and one head or state group (16 divides headdim and d_state), so
        // one lookup finds the first channel's cell; the channel ranges of a head are ascending, so the following
        // channels only step to the next range when they pass its end.
        if (c0 < HP) {
            SsdArgs t;
            t.s = a.s; t.x_scales = a.x_scales; t.head_cluster_end = a.head_cluster_end;
            t.chan_cluster_end = a.chan_cluster_end;
            const int h = c0 / a.s.headdim, p0 = c0 - h * a.s.headdim;
            int base;
            int cell = cell_lookup(t, h, p0, &base);
            const int last = base + a.s.n_chan_clusters - 1;
            int end = cell < last ? a.chan_cluster_end[cell] : a.s.headdim;
            float iv = __fdiv_rn(1.0f, a.x_scales[cell]);
#pragma unroll
            for (int j = 0; j < 16; ++j) {
                while (p0 + j >= end) {  // at most n - 1 steps over the 16 channels together
                    ++cell;
                    end = cell < last ? a.chan_cluster_end[cell] : a.s.headdim;
                    iv = __fdiv_rn(1.0f, a.x_scales[cell]);
                }
                inv[j] = iv;
            }
            dst = a.x_out; row = HP; col = c0;
        } else {
            const bool isB = c0 < HP + GN;
            const int cg = c0 - HP - (isB ? 0 : GN);
            const float iv = __fdiv_rn(1.0f, (isB ? a.B_scales : a.C_scales)[cg / a.s.d_state]);
#pragma unroll
            for (int j = 0; j < 16; ++j) inv[j] = iv;
            dst = isB ? a.B_out : a.C_out; row = GN; col = cg;
        }
    }

    // the window before the segment: tokens t0-3 .. t0-1 in bytes 1..3 (byte 0 is shifted out by the first token)
    uint32_t win[16];
#pragma unroll
    for (int j = 0; j < 16; ++j) win[j] = 0;
#pragma unroll
    for (int k = 0; k < 3; ++k) {
        const int8_t *rp = token_row(a, b, t0 - 3 + k, Ct);
        u32x4 v = {0, 0, 0, 0};
        if (rp) v = *reinterpret_cast<const u32x4 *>(rp + c0);
#pragma unroll
        for (int j = 0; j < 16; ++j)  // bytes: win.b1, win.b2, win.b3, new.b(j & 3)
            win[j] = __builtin_amdgcn_perm(v[j >> 2], win[j], 0x04030201u + ((uint32_t)(j & 3) << 24));
    }

    const int8_t *ip = a.in + ((size_t)b * L + t0) * Ct + c0;
    u32x4 nx[kAhead];
#pragma unroll
    for (int u = 0; u < kAhead; ++u)
        nx[u] = t0 + u < t1 ? __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(ip + (size_t)u * Ct))
                            : (u32x4){0, 0, 0, 0};
    int8_t *op = dst + ((size_t)b * L + t0) * row + col;

    for (int t = t0; t < t1; t += kAhead) {
#pragma unroll
        for (int u = 0; u < kAhead; ++u) {
            if (t + u >= t1) break;
            const u32x4 cur = nx[u];
            if (t + u + kAhead < t1)
                nx[u] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(ip + (size_t)(t - t0 + u + kAhead) * Ct));
            // Codes from the fast evaluation wherever it provably rounds like the exact sequence; channels in which any
            // lane sits too close to a rounding boundary (about 1 % of the channel-tokens of a wave) are redone with
            // the exact sequence below, so every code is the exact sequence's code.
            u32x4 o;
            uint32_t redo = 0;  // wave-uniform: bit j = channel j needs the exact sequence
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                float r[4];
#pragma unroll
                for (int i = 0; i < 4; ++i) {
                    const int j = 4 * q + i;
                    win[j] = __builtin_amdgcn_perm(cur[q], win[j], 0x04030201u + ((uint32_t)i << 24));
                    const int acc = __builtin_amdgcn_sdot4((int)win[j], (int)w[j], 0, false);
                    r[i] = __builtin_amdgcn_fmed3f(activation_over_scale_fast(acc, a.in_w_scale, bias[j], inv[j]),
                                                   -128.0f, 127.0f);
                    redo |= (__builtin_amdgcn_ballot_w64(near_rounding_boundary(r[i])) != 0 ? 1u : 0u) << j;
                }
                o[q] = codes4(r[0], r[1], r[2], r[3]);
            }
            if (redo) {
#pragma unroll
                for (int j = 0; j < 16; ++j)
                    if (redo & (1u << j)) {
                        const int acc = __builtin_amdgcn_sdot4((int)win[j], (int)w[j], 0, false);
                        const uint32_t code = code1(activation_over_scale(acc, a.in_w_scale, bias[j], inv[j]));
                        o[j >> 2] = (o[j >> 2] & ~(0xffu << (8 * (j & 3)))) | (code << (8 * (j & 3)));
                    }
            }
            __builtin_nontemporal_store(o, reinterpret_cast<u32x4 *>(op + (size_t)(t - t0 + u) * row));
        }
    }

    // the state to carry on: the last three input tokens = bytes 1..3 of the windows after the last token
    if (a.state_out && t1 == L) {
#pragma unroll
        for (int k = 0; k < 3; ++k) {
            u32x4 o;
#pragma unroll
            for (int q = 0; q < 4; ++q) {
                const uint32_t lo = __builtin_amdgcn_perm(win[4 * q + 1], win[4 * q], 0x0c0c0400u + 0x00000101u * (k + 1));
                const uint32_t hi = __builtin_amdgcn_perm(win[4 * q + 3], win[4 * q + 2], 0x04000c0cu + 0x01010000u * (k + 1));
                o[q] = lo | hi;
            }
            *reinterpret_cast<u32x4 *>(a.state_out + ((size_t)b * 3 + k) * Ct + c0) = o;
        }
    }
}

// Any shape: one thread per channel, the whole sequence.
__global__ __launch_bounds__(256) void conv1d_q8_any_kernel(ConvArgs a)
{
    const int HP = a.s.nheads * a.s.headdim, GN = a.s.ngroups * a.s.d_state, Ct = HP + 2 * GN;
    const int c = blockIdx.x * 256 + threadIdx.x;
    if (c >= Ct) return;
    const int b = blockIdx.y, L = a.s.seqlen;
    int8_t *dst; int row, col;
    const float inv = __fdiv_rn(1.0f, channel_scale(a, c, &dst, &row, &col));
    const float bias = a.bias ? a.bias[c] : 0.0f;
    int wt[4];
    for (int k = 0; k < 4; ++k) wt[k] = a.weight[(size_t)c * 4 + k];
    int x0 = 0, x1 = 0, x2 = 0;  // tokens t-3, t-2, t-1
    if (a.state_in) {
        x0 = a.state_in[((size_t)b * 3 + 0) * Ct + c];
        x1 = a.state_in[((size_t)b * 3 + 1) * Ct + c];
        x2 = a.state_in[((size_t)b * 3 + 2) * Ct + c];
    }
    for (int t = 0; t < L; ++t) {
        const int x3 = a.in[((size_t)b * L + t) * Ct + c];
        const int acc = wt[0] * x0 + wt[1] * x1 + wt[2] * x2 + wt[3] * x3;
        dst[((size_t)b * L + t) * row + col] = (int8_t)code1(activation_over_scale(acc, a.in_w_scale, bias, inv));
        x0 = x1; x1 = x2; x2 = x3;
    }
    if (a.state_out) {
        a.state_out[((size_t)b * 3 + 0) * Ct + c] = (int8_t)x0;
        a.state_out[((size_t)b * 3 + 1) * Ct + c] = (int8_t)x1;
        a.state_out[((size_t)b * 3 + 2) * Ct + c] = (int8_t)x2;
    }
}

bool vec_ok(const ConvArgs &a)
{
    auto al = [](const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; };
    return a.s.headdim % 16 == 0 && a.s.d_state % 16 == 0 && al(a.in) && al(a.weight) && al(a.bias) && al(a.state_in) &&
           al(a.state_out) && al(a.x_out) && al(a.B_out) && al(a.C_out);
}

}  // namespace

// Tokens per workgroup: the long segment amortises the per-segment set-up and the 3-token halo better, the short one
// is taken when the long one would leave wave slots empty.
int conv1d_segment_tokens(const quamba_ssd_shape_t &s)
{
    const int64_t Ct = (int64_t)s.nheads * s.headdim + 2LL * s.ngroups * s.d_state;
    const int64_t waves = ((Ct / 16 + 63) / 64) * s.batch * ((s.seqlen + kSegLong - 1) / kSegLong);
    return waves >= kWaveSlots ? kSegLong : kSegShort;
}

int conv1d_segments(const quamba_ssd_shape_t &s)
{
    const int seg = conv1d_segment_tokens(s);
    return (s.seqlen + seg - 1) / seg;
}

hipError_t launch_conv1d_q8(const ConvArgs &a, hipStream_t stream)
{
    const int Ct = a.s.nheads * a.s.headdim + 2 * a.s.ngroups * a.s.d_state;
    if (vec_ok(a)) {
        ConvArgs v = a;
        v.seg = conv1d_segment_tokens(a.s);
        const dim3 grid((unsigned)((Ct / 16 + 63) / 64), (unsigned)conv1d_segments(a.s), (unsigned)a.s.batch);
        hipLaunchKernelGGL(conv1d_q8_vec_kernel, grid, dim3(64), 0, stream, v);
    } else {
        const dim3 grid((unsigned)((Ct + 255) / 256), (unsigned)a.s.batch);
        hipLaunchKernelGGL(conv1d_q8_any_kernel, grid, dim3(256), 0, stream, a);
    }
    return hipGetLastError();
}

}  // namespace quamba
