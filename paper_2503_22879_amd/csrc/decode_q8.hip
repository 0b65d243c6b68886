// Single-token decode on an 8-bit cached state (Appendix E, "Quantizing cached SSM states"), in place, and the
// quantizer that turns an fp32 state into that cache.
//
// The cached state is int8 codes; the scale of code (h, p, n) belongs to the (head cluster, channel range) cell of
// (h, p) -- the m x n cells of x (Section 4.1) -- and to the state n.  A step reads a code, de-quantizes it (inverse of
// Eq. 1), applies Eq. 2, adds the element to y, and writes the re-quantized code (Eq. 1) back: 1 B read + 1 B written
// per state element instead of 4 B + 4 B, with about 8 vector instructions per element, which puts the kernel near
// the point where the vector ALU and HBM take the same time.  One workgroup per (sequence, head); a lane owns 16
// consecutive states of a row (one 16-byte load), the head's scale rows and their reciprocals sit in LDS.
//
// The new code is an integer decided by fp32 arithmetic, so every operation that leads to it is rounded on its own, in
// a fixed order (the header states it); the compiler must not contract multiplies and adds, and the exponential of
// the decay is a fixed sequence of such operations instead of a library call.
#include <algorithm>
#include <atomic>

#include "quamba_internal.h"

// no fused multiply-add unless written as one: the quantization decision depends on the individual roundings
#pragma clang fp contract(off)

namespace quamba {
namespace {

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / 64;
constexpr int kMaxSeqs = 16;  // sequences of one head a workgroup of the vector kernel may own
constexpr size_t kLdsLimit = 160 * 1024;
typedef float f32x4 __attribute__((ext_vector_type(4)));
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

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

// Four values -> four codes in one dword: clamp, then the rounding add writes its low byte (the code) straight into
// byte k of the result through the sub-dword destination select, so rounding and packing cost one instruction per code.
__device__ __forceinline__ uint32_t codes4(float r0, float r1, float r2, float r3)
{
    // the median of (r, -127, 127) is r clamped to the code range, in one instruction
    const float c0 = __builtin_amdgcn_fmed3f(r0, -127.0f, 127.0f);
    const float c1 = __builtin_amdgcn_fmed3f(r1, -127.0f, 127.0f);
    const float c2 = __builtin_amdgcn_fmed3f(r2, -127.0f, 127.0f);
    const float c3 = __builtin_amdgcn_fmed3f(r3, -127.0f, 127.0f);
    const float magic = 12582912.0f;  // 1.5 * 2^23
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

__device__ __forceinline__ float code_to_float(uint32_t w, int e) { return (float)(int)(int8_t)(w >> (8 * e)); }

// LDS of a workgroup: xv[P] de-quantized x (or, without x, the scale s_x of every row), cl[P] channel range of every row, s_tab[n][N] the head's scale rows,
// inv_tab[n][N] their reciprocals (correctly rounded divisions, done once per workgroup).
// floats in front of the scale tables: xv and cl, rounded up so that the tables' rows can be read 16 bytes at a time
__host__ __device__ inline size_t table_offset(int P) { return ((size_t)2 * P + 3) & ~(size_t)3; }

// Rows of N floats that lanes read 16 bytes at a time, lane j of a row at floats 16 j ...: with 4-byte banks lanes j and
// j + 4 would meet in the same banks, and rows of different cells start N floats apart, in the same bank again.  The
// vector kernel therefore keeps such rows padded: 4 floats after every 64, element e at e + 4 (e / 64), rows
// padded_row(N) apart (136 floats for N = 128: a shift of 8 banks from row to row).
__host__ __device__ constexpr int padded_row(int N) { return N + 4 * ((N + 63) / 64); }
__host__ __device__ constexpr int padded_pos(int e) { return e + 4 * (e >> 6); }

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
        t.xv[p] = with_x ? a.x_scales[cell] * (float)a.x[(size_t)bh * P + p] : a.x_scales[cell];
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
//
// A workgroup owns one head and every gridDim.y-th slice of the batch; the grid is sized so that all workgroups are
// resident at once (no tail of partly filled rounds).  Everything but the codes goes through LDS: once per workgroup
// the head's scale rows, their reciprocals and the cell of every row; once per slice dt, the decay, the decayed scale
// rows, x as fp32 codes, s_B B and C as fp32 codes.  The loop over the sequences of a slice then issues nothing but
// the 16-byte code loads (one sequence ahead) and stores, so that the dependent look-ups, divisions and conversions
// are paid once per workgroup or slice instead of once per 8 KB of state.  Four workgroups of four waves share a
// compute unit (one wave of each per SIMD), which needs at most 128 vector registers per lane: hence the second
// launch bound.
template <int N, int ROWS, bool FULL>
__global__ __launch_bounds__(kThreads, 4) void decode_q8_vec_kernel(SsdArgs a, const float *state_scales,
                                                                    int8_t *state_q, int seqs_per_block)
{
    constexpr int LPR = N / 16, RPI = 64 / LPR;
    constexpr int NP = padded_row(N);
    extern __shared__ float lds[];
    const int P = a.s.headdim, H = a.s.nheads, G = a.s.ngroups;
    const int h = blockIdx.x, g = h / (H / G);
    const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
    const int j = lane % LPR, sub = lane / LPR;

    // per-sequence arrays behind the head's tables
    float *s_dt = lds + table_offset(P) + 2 * (size_t)a.s.n_chan_clusters * N;
    float *s_dA = s_dt + kMaxSeqs;
    float *s_xf = s_dA + kMaxSeqs;                     // [nb][P]  x codes as fp32
    // the arrays below hold padded rows (padded_row, padded_pos)
    float *s_Bv = s_xf + (((size_t)seqs_per_block * P + 3) & ~(size_t)3);  // [nb][NP]  s_B * B code (one rounding)
    float *s_Cf = s_Bv + (size_t)seqs_per_block * NP;  // [nb][NP]  C codes as fp32 (s_C is applied to the sum)
    float *s_sd = s_Cf + (size_t)seqs_per_block * NP;  // [nb][n cells][NP]  decay * scale: the decayed scale rows
    const int nc = a.s.n_chan_clusters;
    float *s_inv = s_sd + (size_t)seqs_per_block * nc * NP;  // [n cells][NP]  reciprocal scale rows
    const float sB = a.B_scales[g], sC = a.C_scales[g];
    const float Dh = a.D ? a.D[h] : 0.0f;
    // The side inputs of a slice (step sizes, x, B and C codes) are requested one slice ahead and wait in registers
    // while the slice in front of them is computed: under full streaming load a trip to memory takes about as long as
    // two sequences' worth of the main loop, and a slice would otherwise start with such a trip.  Thread t holds 4
    // states of B and C of the slice's sequence t / (N/4) (the host keeps seqs_per_block within kThreads / (N/4)), the
    // step size of sequence t, and, when headdim is a multiple of 4, dword t of the slice's x codes.
    constexpr int kQuads = N / 4;
    static_assert(kThreads % kQuads == 0, "whole rows of B per round of threads");
    struct Side {
        float dt;
        uint32_t bw, cw, xw[1];
    };
    const bool x_quads = (P & 3) == 0;
    auto request_side = [&](int slice, Side &sd) {
        // a thread index the compiler cannot carry across slices: what is derived from it is recomputed here instead
        // of occupying registers throughout the main loop
        int tix = (int)threadIdx.x;
        asm volatile("" : "+v"(tix));
        const int side_bb = tix / kQuads, side_q = tix % kQuads;
        const int bb0 = slice * seqs_per_block, nbs = min(seqs_per_block, a.s.batch - bb0);
        if (tix < nbs) sd.dt = a.dt[(size_t)(bb0 + tix) * H + h];
        if (side_bb < nbs) {
            const size_t bg = (size_t)(bb0 + side_bb) * G + g;
            sd.bw = *reinterpret_cast<const uint32_t *>(a.B + bg * N + 4 * side_q);
            sd.cw = *reinterpret_cast<const uint32_t *>(a.C + bg * N + 4 * side_q);
        }
        if (x_quads) {
            const int xq = P >> 2;
#pragma unroll
            for (int k = 0; k < 1; ++k) {
                const int e = tix + k * kThreads;
                if (e < nbs * xq) {
                    const int bb = e / xq, pq = e - bb * xq;
                    sd.xw[k] = *reinterpret_cast<const uint32_t *>(a.x + ((size_t)(bb0 + bb) * H + h) * P + 4 * pq);
                }
            }
        }
    };
    auto stage_side = [&](int b_begin, int nb, const Side &sd) {
        // a thread index the compiler cannot carry across slices: what is derived from it is recomputed here instead
        // of occupying registers throughout the main loop
        int tix = (int)threadIdx.x;
        asm volatile("" : "+v"(tix));
        const int side_bb = tix / kQuads, side_q = tix % kQuads;
        if (tix < nb) {  // one decay per thread: the exponential is a long dependent chain
            s_dt[tix] = sd.dt;
            s_dA[tix] = exp_steps(sd.dt * a.A[h]);
        }
        if (side_bb < nb) {
            f32x4 bv, cv;
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                bv[k] = sB * code_to_float(sd.bw, k);
                cv[k] = code_to_float(sd.cw, k);
            }
            *reinterpret_cast<f32x4 *>(s_Bv + side_bb * NP + padded_pos(4 * side_q)) = bv;
            *reinterpret_cast<f32x4 *>(s_Cf + side_bb * NP + padded_pos(4 * side_q)) = cv;
        }
        if (x_quads) {
            const int xq = P >> 2;
#pragma unroll
            for (int k = 0; k < 1; ++k) {
                const int e = tix + k * kThreads;
                if (e < nb * xq) {
                    f32x4 xv4;
#pragma unroll
                    for (int i = 0; i < 4; ++i) xv4[i] = code_to_float(sd.xw[k], i);
                    *reinterpret_cast<f32x4 *>(s_xf + 4 * e) = xv4;
                }
            }
            // what one dword per thread does not cover (headdim * sequences above 4 * kThreads) is read here
            for (int e = tix + kThreads; e < nb * xq; e += kThreads) {
                const int bb = e / xq, pq = e - bb * xq;
                const uint32_t w = *reinterpret_cast<const uint32_t *>(a.x + ((size_t)(b_begin + bb) * H + h) * P + 4 * pq);
#pragma unroll
                for (int i = 0; i < 4; ++i) s_xf[4 * e + i] = code_to_float(w, i);
            }
        } else {
            for (int e = tix; e < nb * P; e += kThreads) {
                const int bb = e / P, p = e - bb * P;
                s_xf[e] = (float)a.x[((size_t)(b_begin + bb) * H + h) * P + p];
            }
        }
    };
    Side side = {};
    request_side((int)blockIdx.y, side);  // the grid has at most one row of workgroups per slice

    const Tables t = stage_tables(a, state_scales, 0, h, lds, false);  // xv holds s_x of every row; ends in a barrier
    for (int i = threadIdx.x; i < nc * N; i += kThreads) {
        const int c = i / N, n = i - c * N;
        s_inv[c * NP + padded_pos(n)] = t.inv_tab[i];
    }

    // the workgroup's slices of the batch: slice s covers sequences [s seqs_per_block, (s + 1) seqs_per_block)
    const int nslices = (a.s.batch + seqs_per_block - 1) / seqs_per_block;
    for (int slice = blockIdx.y; slice < nslices; slice += gridDim.y) {
    const int b_begin = slice * seqs_per_block, b_end = min(b_begin + seqs_per_block, a.s.batch);
    const int nb = b_end - b_begin;
    stage_side(b_begin, nb, side);
    __syncthreads();
    for (int bb = 0; bb < nb; ++bb) {
        const float dA = s_dA[bb];
        for (int i = threadIdx.x; i < nc * N; i += kThreads) {
            const int c = i / N, n = i - c * N;
            s_sd[(bb * nc + c) * NP + padded_pos(n)] = dA * t.s_tab[i];
        }
    }
    __syncthreads();
    if (slice + (int)gridDim.y < nslices) request_side(slice + (int)gridDim.y, side);

    for (int p0 = wave * RPI * ROWS; p0 < P; p0 += kWaves * RPI * ROWS) {
        // per row of this trip: its scale rows and its x scale (the same for every sequence)
        int prow[ROWS];
        const float *srow[ROWS], *irow[ROWS];
        float sx[ROWS];
#pragma unroll
        for (int i = 0; i < ROWS; ++i) {
            prow[i] = FULL ? p0 + i * RPI + sub : min(p0 + i * RPI + sub, P - 1);
            srow[i] = s_sd + t.cl[prow[i]] * NP + padded_pos(16 * j);  // of the slice's first sequence; the others nc * NP apart
            irow[i] = s_inv + t.cl[prow[i]] * NP + padded_pos(16 * j);
            sx[i] = t.xv[prow[i]];
        }
        auto load = [&](int b, u32x4(&w)[ROWS]) {
#pragma unroll
            for (int i = 0; i < ROWS; ++i)
                w[i] = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(
                    state_q + (((size_t)b * H + h) * P + prow[i]) * N + 16 * j));
        };
        // The codes of the next sequence are requested while one is computed, and the results of a sequence (codes
        // and outputs) are stored at the start of the next step, right behind that request: the wait for the requested
        // codes at the top of a step then meets only loads and stores that were issued a whole step earlier.  Stored
        // at the end of their own step, the results would be a step's worth of fresh stores in front of that wait
        // (loads and stores complete in the order they were issued).
        u32x4 nxt[ROWS], out[ROWS];
        uint16_t yout[ROWS];
        auto store_results = [&](int bb) {
            const size_t bh = (size_t)(b_begin + bb) * H + h;
#pragma unroll
            for (int i = 0; i < ROWS; ++i)
                if (FULL || p0 + i * RPI + sub < P)
                    __builtin_nontemporal_store(out[i],
                                                reinterpret_cast<u32x4 *>(state_q + (bh * P + prow[i]) * N + 16 * j));
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                const int p = p0 + i * RPI + sub;
                if (j == 0 && (FULL || p < P)) a.y[bh * P + p] = yout[i];
            }
        };
        load(b_begin, nxt);
        for (int bb = 0; bb < nb; ++bb) {
            const int b = b_begin + bb;
            u32x4 cur[ROWS];
#pragma unroll
            for (int i = 0; i < ROWS; ++i) cur[i] = nxt[i];
            if (bb + 1 < nb) load(b + 1, nxt);
            if (bb > 0) store_results(bb - 1);
            const float dt = s_dt[bb];
            const size_t bh = (size_t)b * H + h;
            float acc[ROWS], xv[ROWS], dtx[ROWS];
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                xv[i] = sx[i] * s_xf[bb * P + prow[i]];
                dtx[i] = dt * xv[i];
                acc[i] = 0.0f;
            }
#pragma unroll
            for (int q4 = 0; q4 < 4; ++q4) {
                const f32x4 B4 = *reinterpret_cast<const f32x4 *>(s_Bv + bb * NP + padded_pos(16 * j) + 4 * q4);
                const f32x4 C4 = *reinterpret_cast<const f32x4 *>(s_Cf + bb * NP + padded_pos(16 * j) + 4 * q4);
#pragma unroll
                for (int i = 0; i < ROWS; ++i) {
                    const f32x4 s4 = *reinterpret_cast<const f32x4 *>(srow[i] + (size_t)bb * nc * NP + 4 * q4);
                    const f32x4 i4 = *reinterpret_cast<const f32x4 *>(irow[i] + 4 * q4);
                    float r[4];
#pragma unroll
                    for (int k = 0; k < 4; ++k) {
                        const float d = s4[k] * code_to_float(cur[i][q4], k);  // decayed scale * code: Eq. 2's decay
                        const float u = dtx[i] * B4[k];                         // ... plus B-dot x
                        const float hn = d + u;
                        acc[i] = __builtin_fmaf(C4[k], hn, acc[i]);             // y from the updated state
                        r[k] = hn * i4[k];                                      // Eq. 1
                    }
                    out[i][q4] = codes4(r[0], r[1], r[2], r[3]);
                }
            }
#pragma unroll
            for (int i = 0; i < ROWS; ++i) acc[i] = group_sum<LPR>(acc[i]);
#pragma unroll
            for (int i = 0; i < ROWS; ++i) {
                const int p = p0 + i * RPI + sub;
                if (j == 0 && (FULL || p < P))
                {
                    const float gate = a.z ? silu_of_code(a.z_scale, a.z[bh * P + p]) : 1.0f;  // y * SiLU(z)
                    yout[i] = f32_to_f16_bits(__builtin_fmaf(Dh, xv[i], sC * acc[i]) * gate);
                }
            }
        }
        store_results(nb - 1);
    }
    __syncthreads();  // every wave is done with the slice's arrays before the next slice overwrites them
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
            const float d = (dA * srow[n]) * (float)row[n];
            const float u = dtx * (sB * (float)Bq[n]);
            const float hn = d + u;
            acc = __builtin_fmaf(sC * (float)Cq[n], hn, acc);
            row[n] = (int8_t)(code_bits(hn * irow[n]) & 0xffu);
        }
        acc = group_sum<64>(acc);
        if (lane == 0) {
            const float gate = a.z ? silu_of_code(a.z_scale, a.z[(size_t)bh * P + p]) : 1.0f;  // y * SiLU(z)
            a.y[(size_t)bh * P + p] = f32_to_f16_bits(__builtin_fmaf(Dh, t.xv[p], acc) * gate);
        }
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

template <typename K, typename... Extra>
hipError_t launch(K kernel, dim3 grid, const SsdArgs &a, const float *ss, int8_t *q, size_t lds, hipStream_t stream,
                  Extra... extra)
{
    if (lds > 48 * 1024) {
        const hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(kernel),
                                                 hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
        if (e != hipSuccess) return e;
    }
    hipLaunchKernelGGL(kernel, grid, dim3(kThreads), lds, stream, a, ss, q, extra...);
    return hipGetLastError();
}

// Compute units of the current device (cached per device id).
int compute_units()
{
    static std::atomic<int> cached[64];  // zero-initialised; concurrent first calls store the same value
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
    int n = cached[dev].load(std::memory_order_relaxed);
    if (n == 0) {
        if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0) n = 256;
        cached[dev].store(n, std::memory_order_relaxed);
    }
    return n;
}

// Sequences per workgroup of the vector kernel: enough workgroups to fill the chip several times over (>= 4096 when
// the batch allows), at most kMaxSeqs, the per-sequence arrays within 64 KB of LDS, a grid y dimension <= 65535.
// Returns 0 when no choice fits (the caller then takes the any-shape kernel).
size_t vec_lds_bytes(const quamba_ssd_shape_t &s, int seqs);
int seqs_per_block(const quamba_ssd_shape_t &s)
{
    const int64_t pairs = (int64_t)s.batch * s.nheads;
    int n = (int)std::min<int64_t>(kMaxSeqs, std::max<int64_t>(1, pairs / 4096));
    if (s.d_state >= 4) n = std::min(n, std::max(1, kThreads / (s.d_state / 4)));  // one round of threads covers the slice's B rows
    while (n > 1 && vec_lds_bytes(s, n) > 64 * 1024) --n;
    if (vec_lds_bytes(s, n) > kLdsLimit || (s.batch + n - 1) / n > 65535) return 0;
    return n;
}

template <int N>
hipError_t launch_vec(const SsdArgs &a, const float *ss, int8_t *q, int spb, hipStream_t stream)
{
    constexpr int RPI = 64 / (N / 16);
    const int P = a.s.headdim;
    const size_t lds = vec_lds_bytes(a.s, spb);
    // all workgroups resident at once: 4 waves of up to 128 registers each allow 4 workgroups per compute unit
    // (one wave of each per SIMD), the LDS footprint may allow fewer
    const int nslices = (a.s.batch + spb - 1) / spb;
    const int per_cu = (int)std::max<size_t>(1, std::min<size_t>(4, kLdsLimit / lds));
    const int want_y = (compute_units() * per_cu + a.s.nheads - 1) / a.s.nheads;
    const dim3 grid((unsigned)a.s.nheads, (unsigned)std::max(1, std::min(nslices, want_y)));
    if (P % (kWaves * RPI * 2) == 0) return launch(decode_q8_vec_kernel<N, 2, true>, grid, a, ss, q, lds, stream, spb);
    if (P % (kWaves * RPI) == 0) return launch(decode_q8_vec_kernel<N, 1, true>, grid, a, ss, q, lds, stream, spb);
    return launch(decode_q8_vec_kernel<N, 1, false>, grid, a, ss, q, lds, stream, spb);
}

}  // namespace

size_t decode_q8_lds_bytes(const quamba_ssd_shape_t &s)
{
    return sizeof(float) * (table_offset(s.headdim) + 2 * (size_t)s.n_chan_clusters * s.d_state);
}

namespace {

// LDS of the vector kernel with `seqs` sequences per workgroup: the head's tables plus the per-sequence arrays.
size_t vec_lds_bytes(const quamba_ssd_shape_t &s, int seqs)
{
    const size_t xf = ((size_t)seqs * s.headdim + 3) & ~(size_t)3;
    const size_t np = (size_t)padded_row(s.d_state);
    return decode_q8_lds_bytes(s) +
           sizeof(float) * (2 * kMaxSeqs + xf + (2 + (size_t)s.n_chan_clusters) * seqs * np + s.n_chan_clusters * np);
}

}  // namespace

hipError_t launch_decode_q8(const SsdArgs &a, const float *state_scales, int8_t *state_q, hipStream_t stream)
{
    // the vector kernel reads the codes 16 bytes at a time and x, B and C 4 bytes at a time
    const bool al = reinterpret_cast<uintptr_t>(state_q) % 16 == 0 && reinterpret_cast<uintptr_t>(a.x) % 4 == 0 &&
                    reinterpret_cast<uintptr_t>(a.B) % 4 == 0 && reinterpret_cast<uintptr_t>(a.C) % 4 == 0;
    const int spb = seqs_per_block(a.s);
    if (al && spb > 0) {
        switch (a.s.d_state) {
            case 16: return launch_vec<16>(a, state_scales, state_q, spb, stream);
            case 32: return launch_vec<32>(a, state_scales, state_q, spb, stream);
            case 64: return launch_vec<64>(a, state_scales, state_q, spb, stream);
            case 128: return launch_vec<128>(a, state_scales, state_q, spb, stream);
            case 256: return launch_vec<256>(a, state_scales, state_q, spb, stream);
            default: break;
        }
    }
    return launch(decode_q8_any_kernel, dim3((unsigned)(a.s.batch * a.s.nheads)), a, state_scales, state_q,
                  decode_q8_lds_bytes(a.s), stream);
}

hipError_t launch_quantize_state(const SsdArgs &a, const float *state_scales, int8_t *state_q, hipStream_t stream)
{
    const size_t lds = decode_q8_lds_bytes(a.s);
    const bool vec = a.s.d_state % 4 == 0 && reinterpret_cast<uintptr_t>(a.state) % 16 == 0 &&
                     reinterpret_cast<uintptr_t>(state_q) % 4 == 0;
    const dim3 grid((unsigned)(a.s.batch * a.s.nheads));
    return vec ? launch(quantize_state_kernel<true>, grid, a, state_scales, state_q, lds, stream)
               : launch(quantize_state_kernel<false>, grid, a, state_scales, state_q, lds, stream);
}

}  // namespace quamba
