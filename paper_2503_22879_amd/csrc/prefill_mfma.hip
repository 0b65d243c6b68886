// Chunked prefill of the 8-bit SSD on the gfx950 matrix cores.
//
// One workgroup (4 waves) owns one (sequence, head) and walks its chunks of Q = 256 tokens in order; the head's
// state never leaves the chip.  Per chunk, with a_t = dt_t A_h, cum_t its inclusive prefix sum inside the chunk,
// 32-token blocks tb / sb, and m_sb = cum at the last token of block sb (so cum_t <= m_sb <= cum_s whenever s lies
// in block sb and t in a later block: every exponent below is <= 0):
//
//   G^T[s,t]   = sum_n Bq[s,n] Cq[t,n]                                   int8 MFMA 32x32x32, int32 (exact)
//   x'[s,p]    = xq[s,p] * exp(m_sb - cum_s) * dt_s                      fp16, staged once per chunk in LDS
//   off-diagonal block pair (sb < tb):  Y^T[p,t] += x'^T[p,s] * (G^T[s,t] * exp(cum_t - m_sb))      fp16 MFMA
//   diagonal block (sb = tb):           Y^T[p,t] += xq^T[p,s] * (G^T[s,t] * exp(cum_t - cum_s) dt_s [s <= t])
//   carried state:                      Y^T[p,t] += exp(cum_t) * sum_n H[p,n] Cq[t,n]               fp16 MFMA
//   state, block by block:              H <- exp(m_sb - m_{sb-1}) H + sum_{s in sb} x'[s,:]^T Bq[s,:] fp16 MFMA
//   y[t,p]     = s_x(h,p) * (s_B s_C * Y[t,p] + D_h xq[t,p])             fp32 epilogue, fp16 store
//
// which is Eq. 2 with A-dot = exp(dt A), B-dot = dt B (Section 3.2) regrouped; the quantization scales of
// Section 4.1 enter only in the epilogue because x enters linearly and channel-wise and B, C have one scale per
// state group.  int8 codes are exact in fp16; G (|G| <= 2^21) is scaled by 2^-7 in fp32 before it is narrowed.
// The MFMA output layout (a lane holds one column and 16 rows) equals the operand layout (a lane holds one
// row/column and 8 or 16 consecutive k) up to a fixed permutation of k, so G^T tiles feed the next MFMA straight
// from registers; x^T and B^T are stored in LDS with that permutation (bits 2 and 3 of the token index swapped).
#include "quamba_internal.h"

namespace quamba {
namespace {

typedef int i32x4 __attribute__((ext_vector_type(4)));
typedef int i32x16 __attribute__((ext_vector_type(16)));
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef float f32x16 __attribute__((ext_vector_type(16)));
typedef _Float16 f16x2 __attribute__((ext_vector_type(2)));
typedef _Float16 f16x4 __attribute__((ext_vector_type(4)));
typedef _Float16 f16x8 __attribute__((ext_vector_type(8)));
typedef uint32_t u32x2 __attribute__((ext_vector_type(2)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

constexpr int kP = 64, kN = 128, kQ = 256, kBlk = 32, kNBlk = kQ / kBlk;
constexpr int kThreads = 256;
constexpr int kXqStride = 264;  // bytes per row of xq^T [p][token]
constexpr int kBtStride = 264;  // bytes per row of Bq^T [n][token]
constexpr int kXsStride = 264;  // halves per row of x'^T [p][token]
constexpr int kHsStride = 136;  // halves per row of H [p][n]
constexpr int kYsStride = 72;   // halves per row of the per-wave y staging tile [t][p]
constexpr float kNarrow = 1.0f / 128.0f;  // applied to G and H before narrowing to fp16; undone in the epilogue

// LDS map (bytes)
constexpr int kOffCum = 0;                                  // float[256]
constexpr int kOffDt = kOffCum + 4 * kQ;                    // float[256]
constexpr int kOffSx = kOffDt + 4 * kQ;                     // float[64]
constexpr int kOffWt = kOffSx + 4 * kP;                     // float[4] (+pad)
constexpr int kOffXq = kOffWt + 64;                         // int8 [64][264]
constexpr int kOffBt = kOffXq + kP * kXqStride;             // int8 [128][264]
constexpr int kOffHs = kOffBt + kN * kBtStride;             // fp16 [64][136]
constexpr int kOffYs = kOffHs + 2 * kP * kHsStride;         // fp16 [4][32][72]
constexpr int kOffXs = kOffYs + 2 * 4 * kBlk * kYsStride;   // fp16 [64][264]
constexpr int kOffXl = kOffXs + 2 * kP * kXsStride;         // fp16 [64][264]  (two-term state path only)
constexpr int kLdsFast = kOffXl;
constexpr int kLdsPrecise = kOffXl + 2 * kP * kXsStride;
static_assert(kOffXq % 16 == 0 && kOffBt % 16 == 0 && kOffHs % 16 == 0 && kOffYs % 16 == 0 && kOffXs % 16 == 0 &&
                  kOffXl % 16 == 0, "LDS arrays must be 16-byte aligned");
static_assert(kLdsPrecise <= 160 * 1024, "exceeds the LDS of a gfx950 compute unit");

// Storage position of token s of the chunk inside an LDS row: bits 2 and 3 swapped (see file comment).
__device__ __forceinline__ int tok_pos(int s) { return (s & ~12) | ((s & 4) << 1) | ((s & 8) >> 1); }

// 8 int8 codes (two dwords, lowest address first) -> 8 exact fp16 values: byte^0x80 placed under the fp16
// pattern of 1024 gives 1024 + (code + 128); subtract 1152.
__device__ __forceinline__ f16x8 i8x8_to_f16(uint32_t w0, uint32_t w1)
{
    const f16x2 bias = {(_Float16)1152.0f, (_Float16)1152.0f};
    w0 ^= 0x80808080u;
    w1 ^= 0x80808080u;
    union { f16x8 v; f16x2 h[4]; } r;
    r.h[0] = __builtin_bit_cast(f16x2, __builtin_amdgcn_perm(0x64646464u, w0, 0x04010400u)) - bias;
    r.h[1] = __builtin_bit_cast(f16x2, __builtin_amdgcn_perm(0x64646464u, w0, 0x04030402u)) - bias;
    r.h[2] = __builtin_bit_cast(f16x2, __builtin_amdgcn_perm(0x64646464u, w1, 0x04010400u)) - bias;
    r.h[3] = __builtin_bit_cast(f16x2, __builtin_amdgcn_perm(0x64646464u, w1, 0x04030402u)) - bias;
    return r.v;
}

// 4x4 byte transpose: r[k] holds 4 consecutive columns of row k; c[j] gets column j of rows 0..3.
__device__ __forceinline__ void transpose4x4(const uint32_t r[4], uint32_t c[4])
{
    const uint32_t t0 = __builtin_amdgcn_perm(r[1], r[0], 0x05010400u);
    const uint32_t t1 = __builtin_amdgcn_perm(r[1], r[0], 0x07030602u);
    const uint32_t t2 = __builtin_amdgcn_perm(r[3], r[2], 0x05010400u);
    const uint32_t t3 = __builtin_amdgcn_perm(r[3], r[2], 0x07030602u);
    c[0] = __builtin_amdgcn_perm(t2, t0, 0x05040100u);
    c[1] = __builtin_amdgcn_perm(t2, t0, 0x07060302u);
    c[2] = __builtin_amdgcn_perm(t3, t1, 0x05040100u);
    c[3] = __builtin_amdgcn_perm(t3, t1, 0x07060302u);
}

__device__ __forceinline__ f16x8 pack_f16x8(const float v[8])
{
    f16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (_Float16)v[j];
    return r;
}

template <bool PRECISE>
__global__ __launch_bounds__(kThreads) void prefill_mfma_kernel(SsdArgs a)
{
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *s_cum = reinterpret_cast<float *>(smem + kOffCum);
    float *s_dt = reinterpret_cast<float *>(smem + kOffDt);
    float *s_sx = reinterpret_cast<float *>(smem + kOffSx);
    float *s_wt = reinterpret_cast<float *>(smem + kOffWt);
    unsigned char *s_xq = smem + kOffXq;
    unsigned char *s_bt = smem + kOffBt;
    _Float16 *s_hs = reinterpret_cast<_Float16 *>(smem + kOffHs);
    _Float16 *s_xs = reinterpret_cast<_Float16 *>(smem + kOffXs);
    _Float16 *s_xl = reinterpret_cast<_Float16 *>(smem + kOffXl);

    const int L = a.s.seqlen, H = a.s.nheads, G = a.s.ngroups;
    const int bh = blockIdx.x;
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
    const int l32 = lane & 31, hb = lane >> 5;
    _Float16 *s_ys = reinterpret_cast<_Float16 *>(smem + kOffYs) + wave * kBlk * kYsStride;

    const float Ah = a.A[h];
    const float Dh = a.D ? a.D[h] : 0.0f;
    const float sB = a.B_scales[g], sC = a.C_scales[g];
    const float y_scale = sB * sC * (1.0f / kNarrow);

    if (tid < kP) s_sx[tid] = x_scale_lookup(a, h, tid);
    __syncthreads();

    // Carried state in x-code * B-code units (true state = s_x(p) s_B * st).  Wave w owns states n in
    // [32w, 32w+32); st[pt][r]: p = 32 pt + l32, n = 32 w + 8 (r/4) + 4 hb + r%4.
    f32x16 st[2];
#pragma unroll
    for (int pt = 0; pt < 2; ++pt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st[pt][r] = 0.0f;
    if (a.init_state) {
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            const int p = pt * 32 + l32;
            const float inv = 1.0f / (s_sx[p] * sB);
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int n0 = 32 * wave + 8 * rg + 4 * hb;
                const f32x4 v = *reinterpret_cast<const f32x4 *>(a.init_state + ((size_t)bh * kP + p) * kN + n0);
#pragma unroll
                for (int i = 0; i < 4; ++i) st[pt][4 * rg + i] = v[i] * inv;
            }
        }
    }

    const int nchunks = (L + kQ - 1) / kQ;
    for (int c = 0; c < nchunks; ++c) {
        const int t0 = c * kQ;
        const int nv = min(kQ, L - t0);  // valid tokens of this chunk
        const size_t tokbase = (size_t)b * L + t0;

        // ---- global loads of the chunk's x and B codes (consumed after the scan) ----
        uint32_t xr[4][4], br[8][4];
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int item = tid + kThreads * i, p4 = item & 15, s4 = item >> 4;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int s = 4 * s4 + k;
                xr[i][k] = s < nv ? *reinterpret_cast<const uint32_t *>(a.x + ((tokbase + s) * H + h) * kP + 4 * p4) : 0u;
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int item = tid + kThreads * i, n4 = item & 31, s4 = item >> 5;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const int s = 4 * s4 + k;
                br[i][k] = s < nv ? *reinterpret_cast<const uint32_t *>(a.B + ((tokbase + s) * G + g) * kN + 4 * n4) : 0u;
            }
        }

        // ---- dt and the inclusive prefix sum of dt*A over the chunk ----
        const float dtv = tid < nv ? a.dt[(tokbase + tid) * H + h] : 0.0f;
        float scan = dtv * Ah;
#pragma unroll
        for (int off = 1; off < 64; off <<= 1) {
            const float o = __shfl_up(scan, off, 64);
            if (lane >= off) scan += o;
        }
        if (lane == 63) s_wt[wave] = scan;

        // carried state -> LDS as fp16 (operand of the C.H product of this chunk)
#pragma unroll
        for (int pt = 0; pt < 2; ++pt)
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                f16x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = (_Float16)(st[pt][4 * rg + i] * kNarrow);
                *reinterpret_cast<f16x4 *>(s_hs + (pt * 32 + l32) * kHsStride + 32 * wave + 8 * rg + 4 * hb) = v;
            }
        __syncthreads();
        {
            float offs = 0.0f;
            for (int w = 0; w < wave; ++w) offs += s_wt[w];
            s_cum[tid] = scan + offs;
            s_dt[tid] = dtv;
        }
        __syncthreads();

        // ---- x^T (codes and scaled fp16) and B^T (codes) into LDS, token positions permuted ----
#pragma unroll
        for (int i = 0; i < 4; ++i) {
            const int item = tid + kThreads * i, p4 = item & 15, s4 = item >> 4;
            const int s0 = 4 * s4, q = tok_pos(s0);
            const float m = s_cum[(s0 & ~31) + 31];
            float colf[4], c128[4];
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                colf[k] = __expf(m - s_cum[s0 + k]) * s_dt[s0 + k];
                c128[k] = -128.0f * colf[k];
            }
            uint32_t col[4];
            transpose4x4(xr[i], col);
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                const int p = 4 * p4 + j;
                *reinterpret_cast<uint32_t *>(s_xq + p * kXqStride + q) = col[j];
                const uint32_t u = col[j] ^ 0x80808080u;
                float v[4];
#pragma unroll
                for (int k = 0; k < 4; ++k) v[k] = fmaf((float)((u >> (8 * k)) & 0xffu), colf[k], c128[k]);
                f16x4 hi;
#pragma unroll
                for (int k = 0; k < 4; ++k) hi[k] = (_Float16)v[k];
                *reinterpret_cast<f16x4 *>(s_xs + p * kXsStride + q) = hi;
                if (PRECISE) {
                    f16x4 lo;
#pragma unroll
                    for (int k = 0; k < 4; ++k) lo[k] = (_Float16)(v[k] - (float)hi[k]);
                    *reinterpret_cast<f16x4 *>(s_xl + p * kXsStride + q) = lo;
                }
            }
        }
#pragma unroll
        for (int i = 0; i < 8; ++i) {
            const int item = tid + kThreads * i, n4 = item & 31, s4 = item >> 5;
            const int q = tok_pos(4 * s4);
            uint32_t col[4];
            transpose4x4(br[i], col);
#pragma unroll
            for (int j = 0; j < 4; ++j) *reinterpret_cast<uint32_t *>(s_bt + (4 * n4 + j) * kBtStride + q) = col[j];
        }
        __syncthreads();

        // ---- outputs: each wave owns the 32-token blocks tb = wave and 7 - wave (equal causal work) ----
        for (int which = 0; which < 2; ++which) {
            const int tb = which ? (kNBlk - 1 - wave) : wave;
            if (tb * kBlk >= nv) continue;
            const int tl = tb * kBlk + l32;  // this lane's token inside the chunk
            const bool t_ok = tl < nv;
            i32x4 ct[4];
            {
                const int8_t *crow = a.C + ((tokbase + tl) * G + g) * kN + hb * 64;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk)
                    ct[kk] = t_ok ? *reinterpret_cast<const i32x4 *>(crow + 16 * kk) : (i32x4){0, 0, 0, 0};
            }
            const float cum_t = s_cum[tl];

            // carried-state term: Y^T[p,t] = exp(cum_t) * sum_n H[p,n] Cq[t,n]
            f32x16 acc[2];
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[pt][r] = 0.0f;
#pragma unroll
            for (int kk = 0; kk < 8; ++kk) {
                const f16x8 cf = i8x8_to_f16((uint32_t)ct[kk >> 1][2 * (kk & 1)], (uint32_t)ct[kk >> 1][2 * (kk & 1) + 1]);
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) {
                    const f16x8 hf = *reinterpret_cast<const f16x8 *>(s_hs + (pt * 32 + l32) * kHsStride + hb * 64 + 8 * kk);
                    acc[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(hf, cf, acc[pt], 0, 0, 0);
                }
            }
            {
                const float e = __expf(cum_t);
#pragma unroll
                for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[pt][r] *= e;
            }

            // intra-chunk term, block pairs (sb <= tb)
            for (int sb = 0; sb <= tb; ++sb) {
                const int sl = sb * kBlk + l32;
                i32x4 bq[4];
                {
                    const int8_t *brow = a.B + ((tokbase + sl) * G + g) * kN + hb * 64;
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk)
                        bq[kk] = sl < nv ? *reinterpret_cast<const i32x4 *>(brow + 16 * kk) : (i32x4){0, 0, 0, 0};
                }
                i32x16 gi;
#pragma unroll
                for (int r = 0; r < 16; ++r) gi[r] = 0;
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) gi = __builtin_amdgcn_mfma_i32_32x32x32_i8(bq[kk], ct[kk], gi, 0, 0, 0);

                float lv[16];
                if (sb < tb) {
                    const float rowf = __expf(cum_t - s_cum[sb * kBlk + kBlk - 1]) * kNarrow;
#pragma unroll
                    for (int r = 0; r < 16; ++r) lv[r] = (float)gi[r] * rowf;
                } else {
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int s0 = 8 * rg + 4 * hb;  // four consecutive tokens of the block
                        const f32x4 cs = *reinterpret_cast<const f32x4 *>(s_cum + sb * kBlk + s0);
                        const f32x4 ds = *reinterpret_cast<const f32x4 *>(s_dt + sb * kBlk + s0);
#pragma unroll
                        for (int i = 0; i < 4; ++i) {
                            const float w = __expf(fminf(cum_t - cs[i], 0.0f)) * ds[i] * kNarrow;
                            lv[4 * rg + i] = (s0 + i <= l32) ? (float)gi[4 * rg + i] * w : 0.0f;
                        }
                    }
                }
                const f16x8 l0 = pack_f16x8(lv), l1 = pack_f16x8(lv + 8);
#pragma unroll
                for (int ks = 0; ks < 2; ++ks) {
                    const int col = sb * kBlk + 16 * ks + 8 * hb;
#pragma unroll
                    for (int pt = 0; pt < 2; ++pt) {
                        f16x8 xa;
                        if (sb < tb) {
                            xa = *reinterpret_cast<const f16x8 *>(s_xs + (pt * 32 + l32) * kXsStride + col);
                        } else {
                            const u32x2 w = *reinterpret_cast<const u32x2 *>(s_xq + (pt * 32 + l32) * kXqStride + col);
                            xa = i8x8_to_f16(w[0], w[1]);
                        }
                        acc[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(xa, ks ? l1 : l0, acc[pt], 0, 0, 0);
                    }
                }
            }

            // epilogue: scales, skip term, fp16, transposed through the wave's LDS tile, coalesced 16-byte stores
            const int tq = tok_pos(tl);
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    f16x4 o;
#pragma unroll
                    for (int i = 0; i < 4; ++i) {
                        const int p = pt * 32 + 8 * rg + 4 * hb + i;
                        const float xc = (float)(signed char)s_xq[p * kXqStride + tq];
                        o[i] = (_Float16)(s_sx[p] * fmaf(y_scale, acc[pt][4 * rg + i], Dh * xc));
                    }
                    *reinterpret_cast<f16x4 *>(s_ys + l32 * kYsStride + pt * 32 + 8 * rg + 4 * hb) = o;
                }
            __builtin_amdgcn_wave_barrier();
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                const int row = 8 * i + (lane >> 3), c8 = lane & 7;
                const u32x4 v = *reinterpret_cast<const u32x4 *>(s_ys + row * kYsStride + 8 * c8);
                const int tok = tb * kBlk + row;
                if (tok < nv) *reinterpret_cast<u32x4 *>(a.y + ((tokbase + tok) * H + h) * kP + 8 * c8) = v;
            }
            __builtin_amdgcn_wave_barrier();
        }

        // ---- state update, 32 tokens at a time: wave w owns states n in [32w, 32w+32) ----
        float m_prev = 0.0f;
        for (int sb = 0; sb < kNBlk; ++sb) {
            if (sb * kBlk >= nv) break;  // the padded steps are identity steps
            const float m = s_cum[sb * kBlk + kBlk - 1];
            const float gdec = __expf(m - m_prev);
            m_prev = m;
#pragma unroll
            for (int pt = 0; pt < 2; ++pt)
#pragma unroll
                for (int r = 0; r < 16; ++r) st[pt][r] *= gdec;
#pragma unroll
            for (int ks = 0; ks < 2; ++ks) {
                const int col = sb * kBlk + 16 * ks + 8 * hb;
                const u32x2 w = *reinterpret_cast<const u32x2 *>(s_bt + (32 * wave + l32) * kBtStride + col);
                const f16x8 bf = i8x8_to_f16(w[0], w[1]);
#pragma unroll
                for (int pt = 0; pt < 2; ++pt) {
                    const f16x8 xb = *reinterpret_cast<const f16x8 *>(s_xs + (pt * 32 + l32) * kXsStride + col);
                    st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, xb, st[pt], 0, 0, 0);
                    if (PRECISE) {
                        const f16x8 xlo = *reinterpret_cast<const f16x8 *>(s_xl + (pt * 32 + l32) * kXsStride + col);
                        st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, xlo, st[pt], 0, 0, 0);
                    }
                }
            }
        }
        __syncthreads();
    }

    if (a.state) {
#pragma unroll
        for (int pt = 0; pt < 2; ++pt) {
            const int p = pt * 32 + l32;
            const float sc = s_sx[p] * sB;
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int n0 = 32 * wave + 8 * rg + 4 * hb;
                f32x4 v;
#pragma unroll
                for (int i = 0; i < 4; ++i) v[i] = st[pt][4 * rg + i] * sc;
                *reinterpret_cast<f32x4 *>(a.state + ((size_t)bh * kP + p) * kN + n0) = v;
            }
        }
    }
}

}  // namespace

bool prefill_mfma_supports(const quamba_ssd_shape_t &s)
{
    return s.headdim == kP && s.d_state == kN && s.chunk == kQ;
}

hipError_t launch_prefill_mfma(const SsdArgs &a, hipStream_t stream)
{
    const bool precise = a.state != nullptr || (a.s.flags & QUAMBA_FLAG_PRECISE_STATE);
    const dim3 grid((unsigned)(a.s.batch * a.s.nheads));
    if (precise) {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(prefill_mfma_kernel<true>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsPrecise);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(prefill_mfma_kernel<true>, grid, dim3(kThreads), kLdsPrecise, stream, a);
    } else {
        hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(prefill_mfma_kernel<false>),
                                           hipFuncAttributeMaxDynamicSharedMemorySize, kLdsFast);
        if (e != hipSuccess) return e;
        hipLaunchKernelGGL(prefill_mfma_kernel<false>, grid, dim3(kThreads), kLdsFast, stream, a);
    }
    return hipGetLastError();
}

}  // namespace quamba
