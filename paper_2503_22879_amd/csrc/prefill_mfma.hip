// Chunked prefill of the 8-bit SSD on the gfx950 matrix cores.
//
// One workgroup (8 waves) owns one (sequence, head), or half of a head's channels when the batch is too small to
// fill the chip, and walks it in chunks of kQ = 128 tokens; the head's state never leaves the chip.  The waves split
// into two roles that run side by side between the two barriers of a chunk: waves 0..3 produce the outputs (each owns
// one 32-token block of the chunk), waves 4..7 own the state (each a quarter of its columns): they stage the chunk into
// LDS, compute the token weights, and update the state while the output waves work.  The LDS footprint (< 80 KB) and
// the register budget (128 per lane) let two workgroups share a compute unit, so that each SIMD holds four waves (two
// of each role) whose matrix-core, vector-ALU and memory phases overlap.  Per chunk, with a_t = dt_t A_h, cum_t
// its inclusive prefix sum inside the chunk, 32-token blocks tb / sb, and m_sb = cum at the last token of block
// sb (so cum_t <= m_sb <= cum_s whenever s lies in block sb and t in a later block: every exponent is <= 0):
//
//   G^T[s,t]   = sum_n Bq[s,n] Cq[t,n]                                   int8 MFMA 32x32x32, int32 (exact)
//   off-diagonal block pair (sb < tb):  Y^T[p,t] += xq^T[p,s] * (G^T[s,t] exp(cum_t - m_sb) * exp(m_sb - cum_s) dt_s)
//   diagonal block (sb = tb):           Y^T[p,t] += xq^T[p,s] * (G^T[s,t] exp(cum_t - cum_s) dt_s [s <= t])
//   carried state:                      Y^T[p,t] += sum_n H[p,n] (exp(cum_t) Cq[t,n])               fp16 MFMA
//   state:   H <- exp(cum_last) H + sum_s xq[s,:]^T (exp(cum_last - cum_s) dt_s Bq[s,:])            fp16 MFMA
//   y[t,p]     = s_x(h,p) * (s_B s_C * Y[t,p] + D_h xq[t,p])             fp32 epilogue, fp16 store
//
// x is staged once per chunk as exact fp16 codes; every token weight sits on the other operand of its product: on the
// columns of the narrowed score tiles (the row factor exp(cum_t - m_sb) is applied in fp32 before narrowing), and on
// the rows of B in the state update.  When the final state is returned it has to meet 1e-4 of its maximum, which one
// product rounded to fp16 cannot: the state then decays block by block in fp32, H <- exp(m_sb - m_{sb-1}) H + ..., and
// the token weight w_s = exp(m_sb - cum_s) dt_s is split as wq_s (1 + d_s), wq_s = w_s rounded to 4 significant bits,
// so that Bq wq_s is exact in fp16 (7 + 4 bits); the update takes two products, xq^T (wq_s Bq) and xq^T (d_s wq_s Bq),
// the first exact, the second (|d_s| <= 1/16) rounded at 2^-16 of the total.
//
// Every exponent that spans a stretch of tokens is formed from sums of dt A over that stretch (the block's own prefix
// and suffix sums, the blocks' totals), not from differences of the chunk's prefix sums, which carry rounding of the
// size of whatever decay lies in front of the stretch; a block pair, a carried-state product or a block's share of the chunk state
// whose decay factor is below 2^-32 is left out unless QUAMBA_FLAG_NO_DECAY_SKIP is set.  The chunk's closing barrier
// sits in front of the output epilogue, which reads registers and constant tables only.
//
// Batches with fewer (sequence, head) pairs than compute units are also cut along the sequence: a first kernel
// (segment_state_kernel) walks all but the last segment without outputs and leaves every segment's end state (from a
// zero start) and decay total in the workspace, then this kernel (SEG instantiations) gives every segment its own
// workgroups, which start from the combination of the earlier segments' states (Eq. 2 is linear in the state).
//
// All of this is Eq. 2 with A-dot = exp(dt A), B-dot = dt B (Section 3.2) regrouped; the quantization scales of
// Section 4.1 enter only in the epilogue because x enters linearly and channel-wise and B, C have one scale per
// state group.  The result does not depend on the chunk length, so the caller's `chunk` is not used here.
// int8 codes are exact in fp16; G (|G| <= 2^21) is scaled by 2^-7 in fp32 before it is narrowed.
// The MFMA output layout (a lane holds one column and 16 rows) equals the operand layout (a lane holds one
// row/column and 8 or 16 consecutive k) up to a fixed permutation of k, so G^T tiles feed the next MFMA straight
// from registers.  x and B sit in LDS token-major, exactly as they arrive (no transposes on the vector ALU); the
// operands that need the token index as k (x^T, B^T) are fetched with the transposing LDS loads
// (ds_read_b64_tr_b8 / _tr_b16), whose source lanes address whole token rows; the rows are stored with bits 2 and 3
// of the token index swapped so that the 8 tokens of one k group are 8 consecutive rows.
#include <algorithm>
#include <climits>
#include <atomic>

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

constexpr int kP = 64, kN = 128, kQ = 128, kBlk = 32, kNBlk = kQ / kBlk;
constexpr int kThreads = 512;
constexpr int kHsStride = 136;  // halves per row of H [p][n]
constexpr int kBqStride = 144;  // bytes per row of Bq [token][n]
constexpr float kNarrow = 1.0f / 128.0f;  // applied to G and H before narrowing to fp16; undone in the epilogue
// Scales that keep every fp16 operand in the normal range.  x is staged as fp16 codes times kXs; the output
// accumulators hold the output in code units times 2^-7 kAcc; the state accumulators the state times 2^-7 (kNarrow).
// Hence the token weights on the score columns carry kAcc / kXs = 1/4 (score tiles, up to 2^14 after their own 2^-7,
// times dt / 4 stay finite for dt up to 16), those on the rows of B carry kNarrow / kXs = 1/8 (dt / 8 times the decay
// is far from the subnormals), and the C operand of the carried-state product carries kAcc.
constexpr float kXs = 1.0f / 16.0f;
constexpr float kAcc = 1.0f / 64.0f;
// A product whose operands are separated by a decay factor below 2^-kDead (prefix sums are in log2 units) is left out
// unless the caller asks for it: it is below 2.4e-10 of the term's own undecayed size.
constexpr float kDead = 32.0f;

// LDS map (bytes) for PT 32-channel tiles per workgroup.  Row pitches: with 4-byte banks, the 8 token rows x 16 bytes
// a group of 16 lanes fetches from Bq fall into distinct banks (pitch of 36 banks), and so do the 4 token rows x 32
// bytes that each of the two 16-lane groups of a half-wave fetches from x in the same cycle (pitch of 48 banks: rows
// at banks 0, 48, 32, 16, the second group 8 banks further; the pitch of 40 banks used before put the second group's
// last row on the first group's first and showed as a third of the LDS time in the bank-conflict counter).
template <int PT>
struct Lds {
    static constexpr int kPw = 32 * PT;                      // channels of the workgroup
    static constexpr int kXsStride = PT == 2 ? 96 : 48;      // halves per row of x [token][p]
    static constexpr int kOffCum = 0;                        // float[128]  prefix sums (log2 units)
    static constexpr int kOffDt = kOffCum + 4 * kQ;          // float[128]  dt 2^-7 / kXs
    static constexpr int kOffW2 = kOffDt + 4 * kQ;           // float[128]  column weights of the diagonal blocks
    static constexpr int kOffWe = kOffW2 + 4 * kQ;           // fp16[128]   token weights of the off-diagonal blocks
    static constexpr int kOffWs = kOffWe + 2 * kQ;           // fp16[128]   token weights of the state update
    static constexpr int kOffWd = kOffWs + 2 * kQ;           // fp16[128]   their residuals (two-term path)
    static constexpr int kOffSx = kOffWd + 2 * kQ;           // float[64]
    static constexpr int kOffLoc = kOffSx + 4 * kP;          // float[128]  prefix sums inside each 32-token block
    static constexpr int kOffTot = kOffLoc + 4 * kQ;         // float[4]    the blocks' totals
    static constexpr int kOffGap = kOffTot + 4 * kNBlk;      // float[4][4] [tb][sb]: sum of the totals of blocks sb+1..tb-1
    static constexpr int kOffBq = kOffGap + 4 * kNBlk * kNBlk + 48;  // int8 [128][144]
    static constexpr int kOffHs = kOffBq + kQ * kBqStride;   // fp16 [kPw][136]
    static constexpr int kOffXs = kOffHs + 2 * kPw * kHsStride;  // fp16 [128][kXsStride]
    static constexpr int kBytes = kOffXs + 2 * kQ * kXsStride;
    // gated variant only: the chunk's gate codes, int8 [128][kZsStride], plain token order
    static constexpr int kZsStride = 32 * PT + 8;
    static constexpr int kOffZs = kBytes;
    static constexpr int kOffSilu = kOffZs + kQ * kZsStride;  // float[256]: SiLU of every possible gate code
    static constexpr int kBytesGated = kOffSilu + 4 * 256;
    static_assert(kOffBq % 16 == 0 && kOffHs % 16 == 0 && kOffXs % 16 == 0, "LDS arrays must be 16-byte aligned");
};
static_assert(Lds<2>::kBytesGated <= 80 * 1024, "two workgroups must fit the 160 KB LDS of a gfx950 compute unit");

// 2^x by the hardware instruction (prefix sums are carried in log2 units, so no multiply by log2 e is needed).
__device__ __forceinline__ float exp2_fast(float x) { return __builtin_amdgcn_exp2f(x); }

// LDS row of token s of the chunk: bits 2 and 3 swapped (see file comment).
// Lane index recomputed where it is called: the mask passes through an empty asm statement, so the compiler can neither
// hoist the result out of a loop nor keep it in a register across one.
__device__ __forceinline__ int fresh_lane() {
    unsigned m = ~0u;
    asm volatile("" : "+s"(m));
    return (int)__builtin_amdgcn_mbcnt_hi(m, __builtin_amdgcn_mbcnt_lo(m, 0u));
}
__device__ __forceinline__ int tok_pos(int s) { return (s & ~12) | ((s & 4) << 1) | ((s & 8) >> 1); }

// Transposing LDS loads.  Inside each group of 16 lanes, result byte j of lane i comes from the 8 bytes addressed by
// lane 2j + (i >> 3), byte i & 7 (8-bit form); result half j of lane i from the 8 bytes addressed by lane
// 4j + (i >> 2), half i & 3 (16-bit form).  With source lane 2j + q pointing at (token row j, 8 columns starting at
// 8q), resp. 4j + q at (token row j, 4 columns starting at 4q), lane i receives column i of 8 (resp. 4) token rows:
// the layout of an MFMA operand whose k index is the token.
typedef int v2i_lds __attribute__((ext_vector_type(2)));
__device__ __forceinline__ u32x2 lds_read_tr8(const unsigned char *p)
{
    return __builtin_bit_cast(
        u32x2, __builtin_amdgcn_ds_read_tr8_b64_v2i32((__attribute__((address_space(3))) v2i_lds *)(p)));
}
__device__ __forceinline__ f16x4 lds_read_tr16(const unsigned char *p)
{
    typedef short v4s_lds __attribute__((ext_vector_type(4)));
    return __builtin_bit_cast(
        f16x4, __builtin_amdgcn_ds_read_tr16_b64_v4i16((__attribute__((address_space(3))) v4s_lds *)(p)));
}
// 8 tokens x one column of fp16 x (two 4-token transposing loads, token rows r .. r+7 of the lane group)
template <int PITCH_HALVES>
__device__ __forceinline__ f16x8 lds_read_tr16x8(const unsigned char *p)
{
    const f16x4 lo = lds_read_tr16(p), hi = lds_read_tr16(p + 4 * 2 * PITCH_HALVES);
    return __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
}

// 8 int8 codes (two dwords, lowest address first) -> 8 exact fp16 values, one conversion per code: the source byte is
// picked and sign-extended by the instruction's sub-dword source select, the result written to the low or high half of
// the destination by its destination select (the high half keeps the low one).
__device__ __forceinline__ uint32_t i8x2_to_f16_lo_hi(uint32_t w, int first_byte)
{
    uint32_t r;
    if (first_byte == 0) {
        asm("v_cvt_f16_i16_sdwa %0, sext(%1) dst_sel:WORD_0 dst_unused:UNUSED_PAD src0_sel:BYTE_0" : "=v"(r) : "v"(w));
        asm("v_cvt_f16_i16_sdwa %0, sext(%1) dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_1" : "+v"(r) : "v"(w));
    } else {
        asm("v_cvt_f16_i16_sdwa %0, sext(%1) dst_sel:WORD_0 dst_unused:UNUSED_PAD src0_sel:BYTE_2" : "=v"(r) : "v"(w));
        asm("v_cvt_f16_i16_sdwa %0, sext(%1) dst_sel:WORD_1 dst_unused:UNUSED_PRESERVE src0_sel:BYTE_3" : "+v"(r) : "v"(w));
    }
    return r;
}
__device__ __forceinline__ f16x8 i8x8_to_f16(uint32_t w0, uint32_t w1)
{
    const u32x4 r = {i8x2_to_f16_lo_hi(w0, 0), i8x2_to_f16_lo_hi(w0, 2), i8x2_to_f16_lo_hi(w1, 0),
                     i8x2_to_f16_lo_hi(w1, 2)};
    return __builtin_bit_cast(f16x8, r);
}

// 4 int8 codes (one dword) -> fp16 values kXs * code, exact: byte^0x80 placed under the fp16 pattern of 64 (whose
// last mantissa bit weighs 1/16) gives 64 + (code + 128) / 16; subtract 72.
__device__ __forceinline__ f16x4 i8x4_to_f16_xs(uint32_t w)
{
    static_assert(kXs == 1.0f / 16.0f, "the bit pattern below encodes a step of 1/16");
    const f16x2 bias = {(_Float16)72.0f, (_Float16)72.0f};
    w ^= 0x80808080u;
    union { f16x4 v; f16x2 h[2]; } r;
    r.h[0] = __builtin_bit_cast(f16x2, __builtin_amdgcn_perm(0x54545454u, w, 0x04010400u)) - bias;
    r.h[1] = __builtin_bit_cast(f16x2, __builtin_amdgcn_perm(0x54545454u, w, 0x04030402u)) - bias;
    return r.v;
}

template <int CTRL, int ROW_MASK, bool BOUND>
__device__ __forceinline__ float dpp_f32(float v)
{
    return __builtin_bit_cast(
        float, __builtin_amdgcn_update_dpp(0, __builtin_bit_cast(int, v), CTRL, ROW_MASK, 0xf, BOUND));
}

// Inclusive prefix sum over the 64 lanes of a wave with data-parallel-primitive moves only (no LDS round trips):
// shifts by 1, 2, 4, 8 inside each row of 16 lanes (zero fill), then the last lane of row 0/2 is added to row 1/3
// and the last lane of row 1 to rows 2 and 3.
// `row` receives the scan inside the lane's row of 16 lanes alone (the first four steps).
__device__ __forceinline__ float wave_inclusive_scan(float v, float &row)
{
    v += dpp_f32<0x111, 0xf, true>(v);   // row_shr:1
    v += dpp_f32<0x112, 0xf, true>(v);   // row_shr:2
    v += dpp_f32<0x114, 0xf, true>(v);   // row_shr:4
    v += dpp_f32<0x118, 0xf, true>(v);   // row_shr:8
    row = v;
    v += dpp_f32<0x142, 0xa, false>(v);  // row_bcast:15 into rows 1 and 3
    v += dpp_f32<0x143, 0xc, false>(v);  // row_bcast:31 into rows 2 and 3
    return v;
}

// Sum of the values of the lanes behind this one inside its row of 16 lanes (0 for the row's last lane): row shifts
// towards lower lanes with zero fill.  Unlike the difference of two prefix sums it carries no rounding error of the
// size of the sums in front of the lane.
__device__ __forceinline__ float row_suffix_sum_exclusive(float v)
{
    float s = dpp_f32<0x101, 0xf, true>(v);  // row_shl:1
    s += dpp_f32<0x101, 0xf, true>(s);
    s += dpp_f32<0x102, 0xf, true>(s);       // row_shl:2
    s += dpp_f32<0x104, 0xf, true>(s);       // row_shl:4
    s += dpp_f32<0x108, 0xf, true>(s);       // row_shl:8
    return s;
}

__device__ __forceinline__ f16x8 pack_f16x8(const float v[8])
{
    f16x8 r;
#pragma unroll
    for (int j = 0; j < 8; ++j) r[j] = (_Float16)v[j];
    return r;
}

// Workgroup -> (sequence, head).  Hardware hands consecutive workgroup ids to the 8 XCDs round-robin, each XCD with
// its own L2.  When the number of (sequence, state group) units is a multiple of 8, all heads of a unit are put on
// one XCD, so that the B and C rows they share are fetched into one L2 instead of eight.
__device__ __forceinline__ int block_to_bh(const SsdArgs &a, int i)
{
    const int H = a.s.nheads, G = a.s.ngroups, hpg = H / G;
    const int units = a.s.batch * G;
    if (units % 8 != 0) return i;
    const int x = i & 7, slot = i >> 3;
    const int u = x + 8 * (slot / hpg), hl = slot % hpg;
    const int b = u / G, g = u - b * G;
    return b * H + g * hpg + hl;
}

// PT: 32-channel tiles per workgroup.  2: one workgroup per (sequence, head).  1: two workgroups per head, each with
// half of the channels, its own half of the state and its own copy of the G^T work; chosen when there are fewer
// heads in the batch than compute units, so that the whole chip works on short batches.
// GATED: the output is multiplied by SiLU(z) of the caller's int8 gate codes (Section 3.2) in the epilogue.
// SEG: the launch belongs to a sequence split (see SsdArgs); the instantiations without it carry none of its code.
template <bool PRECISE, int PT, bool GATED, bool SEG>
__global__ __launch_bounds__(kThreads, 4) void prefill_mfma_kernel(SsdArgs a)
{
    typedef Lds<PT> LY;
    constexpr int kPw = LY::kPw;  // channels of this workgroup
    constexpr int kXsStride = LY::kXsStride;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *s_cum = reinterpret_cast<float *>(smem + LY::kOffCum);
    float *s_dt = reinterpret_cast<float *>(smem + LY::kOffDt);
    float *s_w2 = reinterpret_cast<float *>(smem + LY::kOffW2);
    _Float16 *s_we = reinterpret_cast<_Float16 *>(smem + LY::kOffWe);
    _Float16 *s_ws = reinterpret_cast<_Float16 *>(smem + LY::kOffWs);
    _Float16 *s_wd = reinterpret_cast<_Float16 *>(smem + LY::kOffWd);  // PRECISE only
    float *s_sx = reinterpret_cast<float *>(smem + LY::kOffSx);
    float *s_loc = reinterpret_cast<float *>(smem + LY::kOffLoc);
    float *s_tot = reinterpret_cast<float *>(smem + LY::kOffTot);
    float *s_gap = reinterpret_cast<float *>(smem + LY::kOffGap);
    unsigned char *s_bq = smem + LY::kOffBq;
    _Float16 *s_hs = reinterpret_cast<_Float16 *>(smem + LY::kOffHs);
    unsigned char *s_xs = smem + LY::kOffXs;  // fp16 rows, addressed in bytes
    unsigned char *s_zs = smem + LY::kOffZs;  // gate codes (GATED only)
    float *s_silu = reinterpret_cast<float *>(smem + LY::kOffSilu);  // SiLU(z_scale * code), indexed by the code's byte
    constexpr int kZsStride = LY::kZsStride;

    const int L = a.s.seqlen, H = a.s.nheads, G = a.s.ngroups;
    // Sequence split: the workgroups of segment `seg` walk the chunks [c_begin, c_end) of their sequence; without a
    // split that is the whole sequence.  Everything below is uniform over the workgroup.
    const int wgs_per_seg = a.s.batch * H * (2 / PT);
    const int seg = SEG ? (int)blockIdx.x / wgs_per_seg : 0;
    const int nchunks = (L + kQ - 1) / kQ;
    const int c_begin = SEG ? seg * a.seg_chunks : 0;
    const int c_end = (SEG && seg + 1 < a.nseg) ? c_begin + a.seg_chunks : nchunks;
    const bool convert_init = a.init_state && (!SEG || seg == 0);  // the caller's initial state belongs to segment 0
    // with two workgroups per head, ids i and i + 8 (same XCD, and the same compute unit when two workgroups fit one)
    // take the two halves of a head
    const int bid = SEG ? (int)blockIdx.x - seg * wgs_per_seg : (int)blockIdx.x;
    int pair = bid, half = 0;  // index of the (sequence, head) pair before the XCD mapping; channel half
    if (PT == 1) {
        // complete groups of 8 pairs take 16 consecutive ids (8 first halves, 8 second halves); the last, incomplete
        // group of r pairs takes the remaining 2 r ids (r first halves, r second halves)
        const int npairs = a.s.batch * H, full = npairs >> 3;
        if (bid < 16 * full) {
            pair = (bid & 7) | ((bid >> 4) << 3);
            half = (bid >> 3) & 1;
        } else {
            const int t = bid - 16 * full, r = npairs - 8 * full;
            pair = 8 * full + t % r;
            half = t / r;
        }
    }
    const int p_base = 32 * half;
    const int bh = block_to_bh(a, pair);
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int tid = threadIdx.x, lane = tid & 63;
    // wave-uniform: keeps block indices in scalar registers
    const int wave8 = __builtin_amdgcn_readfirstlane(tid >> 6);
    const bool out_role = wave8 < 4;  // waves 0..3: outputs; waves 4..7: staging, token weights, state
    const int wave = wave8 & 3;       // index inside the role (waves w and w + 4 share a SIMD)
    const int tid4 = tid & 255;       // thread index inside the role
    const int l32 = lane & 31, hb = lane >> 5;
    // The causal work of an output wave grows with its block index, and a wave's block rotates with the chunk index;
    // every other group of 8 workgroup ids (one id per XCD) walks the blocks in the opposite order, so that the long
    // and the short blocks of different workgroups are spread over the SIMDs.
    const int rot_flip = ((bid >> 3) & 1) ? (kNBlk - 1) : 0;
    // Two workgroups share a compute unit, and its SIMDs favour the waves of the one dispatched first: that one would
    // finish well before the other, which then runs alone at less than the unit's paired throughput.  Workgroups are
    // dispatched in id order, one per compute unit and round; when the host asks for it (a launch of at most two
    // rounds, all resident at once), those of the second round (ids from pace_first on) raise their priority in every
    // other chunk, which lets the pair advance at about the same pace.
    auto set_chunk_priority = [&](int c) {
        if ((int)blockIdx.x >= a.pace_first) {  // never without pacing: pace_first is then INT_MAX
            if (c & 1) __builtin_amdgcn_s_setprio(1);
            else __builtin_amdgcn_s_setprio(0);
        }
    };

    const float Ah = a.A[h] * 1.44269504088896340736f;  // log2(e): prefix sums are kept in log2 units (exp2 below)
    const float Dh = a.D ? a.D[h] : 0.0f;
    const float sB = a.B_scales[g], sC = a.C_scales[g];
    const float y_scale = sB * sC * (1.0f / (kNarrow * kAcc));  // output accumulator -> s_B s_C (x-code units)
    // Skip term D x[t,p]: the diagonal block multiplies exact x codes by L[t,s], so adding D/y_scale to L[t,t]
    // (in fp32, before L is narrowed to fp16 like every other entry) makes the matrix core add D x for free.
    // When D/y_scale would leave the fp16 range (extreme scales), the term is added in the epilogue from LDS instead.
    const float d_acc = Dh / (y_scale * kXs);  // it multiplies x codes staged times kXs
    const bool d_by_mfma = fabsf(d_acc) < 3.0e4f;
    const float d_sel = d_by_mfma ? d_acc : 0.0f;

    // The channel scales (three dependent look-ups in global memory) and the SiLU table are written by the output waves
    // after they have requested their first C rows, so that the look-ups do not stand in front of the first chunk's
    // loads; their first readers sit behind the first chunk's staging barrier.  Only an initial state needs the scales
    // earlier (the state waves convert it with them), which costs one more barrier.
    auto fill_tables = [&]() {
        if (tid < kPw) s_sx[tid] = x_scale_lookup(a, h, p_base + tid) * (d_by_mfma ? y_scale : 1.0f);
        // a gate code has 256 values: their SiLU is tabulated once (exp and reciprocal are quarter-rate instructions)
        if (GATED && tid < 256) s_silu[tid] = silu_of_code(a.z_scale, (int8_t)tid);
    };
    // decay below which a 32-token block's product is left out; +inf keeps everything
    const float dead = (a.s.flags & QUAMBA_FLAG_NO_DECAY_SKIP) ? __builtin_inff() : kDead;
    constexpr float kStScale = kNarrow;
    const uint32_t x_row = (uint32_t)H * kP, b_row = (uint32_t)G * kN, dt_row = (uint32_t)H * 4u;
    typedef uint32_t xvec __attribute__((ext_vector_type(PT)));

    if (out_role) {
        // ================= output waves: wave w produces the outputs of one 32-token block per chunk =================
        // C rows of the wave's block of chunk c (operand of G^T, and, as fp16, of the carried-state product), loaded a
        // chunk ahead.  k-step kk of the G^T product covers states 32 kk + 16 hb + [0,16): the two half-waves read
        // adjacent 16-byte pieces of a C row.  Rows past the end of the sequence are read from the last valid row and
        // zeroed where they are consumed.
        i32x4 ct[4];
        auto issue_c_rows = [&](int c) {
            const int t0 = c * kQ;
            const int nv = min(kQ, L - t0);
            const int8_t *cbase = a.C + (((size_t)b * L + t0) * G + g) * kN;
            const int ln = fresh_lane();
            const uint32_t row = (uint32_t)min((((wave + c) & (kNBlk - 1)) ^ rot_flip) * kBlk + (ln & 31), nv - 1);
#pragma unroll
            for (int kk = 0; kk < 4; ++kk)
                ct[kk] = *reinterpret_cast<const i32x4 *>(cbase + (row * b_row + 16u * (ln >> 5)) + 32 * kk);
        };
        issue_c_rows(c_begin);
        fill_tables();
        if (convert_init) __syncthreads();  // the state waves wait for the scales
        for (int c = c_begin; c < c_end; ++c) {
            set_chunk_priority(c);
            const int t0 = c * kQ;
            const int nv = min(kQ, L - t0);
            const size_t tokbase = (size_t)b * L + t0;
            // this wave's output block rotates with the chunk index so that the causal work (tb + 1 block pairs)
            // evens out over four chunks
            const int tb = ((wave + c) & (kNBlk - 1)) ^ rot_flip;
            const int tl = tb * kBlk + l32;  // this lane's token inside the chunk
            if (nv < kQ) {
#pragma unroll
                for (int kk = 0; kk < 4; ++kk) ct[kk] = tl < nv ? ct[kk] : (i32x4){0, 0, 0, 0};
            }
            // the C rows must have arrived here (the empty asm pins the wait to this point): a wait placed after the
            // next chunk's loads are issued would wait for those as well
#pragma unroll
            for (int kk = 0; kk < 4; ++kk) asm volatile("" : "+v"(ct[kk]));
            __syncthreads();  // the state waves have staged the chunk: x, B, the token weights, the fp16 state
            // ---- outputs of block tb ----
            if (tb * kBlk < nv) {
                // LDS addresses of this phase are rebuilt from a lane index the compiler must treat as new in every
                // chunk: kept in registers across the whole chunk loop they would push other values into scratch memory
                int lane_a = fresh_lane();
                asm volatile("" : "+v"(lane_a));
                const int l32a = lane_a & 31, hba = lane_a >> 5;
                // source-lane roles of the transposing loads (see lds_read_tr8 / lds_read_tr16): token row of the lane
                // inside a k group of 8 tokens, and its first column inside the 32 columns of the operand
                const int i16 = lane_a & 15, c16 = (lane_a >> 4) & 1;
                const unsigned char *xs_src =
                    s_xs + ((8 * hba + (i16 >> 2)) * kXsStride + 16 * c16 + 4 * (i16 & 3)) * 2;
                const float cum_t = s_cum[tb * kBlk + l32a];
                const float loc_t = s_loc[tb * kBlk + l32a];  // the same sum from the start of the token's own block

                // B rows of block sb as the A operand of G^T
                auto load_bq = [&](int sb, i32x4(&bq)[4]) {
                    const unsigned char *row = s_bq + (sb * kBlk + tok_pos(l32a)) * kBqStride + hba * 16;
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk) bq[kk] = *reinterpret_cast<const i32x4 *>(row + 32 * kk);
                };
                auto gemm_g = [&](const i32x4(&bq)[4]) {
                    i32x16 gi;
#pragma unroll
                    for (int r = 0; r < 16; ++r) gi[r] = 0;
#pragma unroll
                    for (int kk = 0; kk < 4; ++kk)
                        gi = __builtin_amdgcn_mfma_i32_32x32x32_i8(bq[kk], ct[kk], gi, 0, 0, 0);
                    return gi;
                };
                // Prefix sums never rise (dt >= 0, A <= 0), so the blocks whose decay towards this block has died are
                // the first ones: sb0 is the first block still alive (tb itself if none is), and the carried state is
                // dead when the prefix sum in front of the block is.  Wave-uniform.
                const float r_tb = tb > 0 ? s_cum[tb * kBlk - 1] : 0.0f;
                int sb0 = 0;
                while (sb0 < tb && __builtin_amdgcn_readfirstlane(r_tb - s_cum[sb0 * kBlk + kBlk - 1] < -dead)) ++sb0;
                const bool carry_alive = !__builtin_amdgcn_readfirstlane(r_tb < -dead);
                i32x4 bq[4];
                load_bq(sb0, bq);
                i32x16 gi = gemm_g(bq);

                // carried-state term: Y^T[p,t] = sum_n H[p,n] (exp(cum_t) Cq[t,n])
                f32x16 acc[PT];
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) acc[pt][r] = 0.0f;
                // per lane (token t); folded into the C operand
                const _Float16 e_t = (_Float16)(exp2_fast(cum_t) * kAcc);
#pragma unroll
                for (int k2 = 0; k2 < 4; ++k2) {  // batches of two k-steps: all LDS reads of a batch are issued first
                    if (!carry_alive) break;
                    f16x8 hf[2][PT];
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk)
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            hf[kk][pt] = *reinterpret_cast<const f16x8 *>(s_hs + (pt * 32 + l32a) * kHsStride +
                                                                         32 * k2 +
                                                                         16 * hba + 8 * kk);
                    // keep the LDS reads above in flight: nothing may be moved across
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int kk = 0; kk < 2; ++kk) {
                        const int k8 = 2 * k2 + kk;
                        const i32x4 c4 = ct[k8 >> 1];
                        const f16x8 cf = i8x8_to_f16((uint32_t)c4[2 * (k8 & 1)], (uint32_t)c4[2 * (k8 & 1) + 1]) * e_t;
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            acc[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(hf[kk][pt], cf, acc[pt], 0, 0, 0);
                    }
                }

                // intra-chunk term, block pairs (sb <= tb); the G^T tile of the next pair is issued before this one is
                // scaled and narrowed so that the matrix core and the vector ALU overlap inside the wave
                for (int sb = sb0; sb < tb; ++sb) {  // strictly lower block pairs that are alive
                    load_bq(sb + 1, bq);
                    f16x8 xa[2][PT];
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            xa[ks][pt] = lds_read_tr16x8<kXsStride>(
                                xs_src + ((sb * kBlk + 16 * ks) * kXsStride + 32 * pt) * 2);
                    // cum_t - m_sb, formed from the block's own prefix sum and the totals of the blocks in between
                    // (the difference of two chunk-wide sums would carry their rounding)
                    const float gap_sb = s_gap[tb * kNBlk + sb];
                    f16x4 wq4[4];  // weights of tokens 8 rg + 4 hb + [0,4) of block sb
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg)
                        wq4[rg] = *reinterpret_cast<const f16x4 *>(s_we + sb * kBlk + 8 * rg + 4 * hba);
                    __builtin_amdgcn_sched_barrier(0);
                    // the current tile is narrowed before the next one is issued, so that both can share registers (the
                    // other wave of the SIMD fills the matrix core meanwhile)
                    const float rowf = exp2_fast(loc_t + gap_sb) * kNarrow;
                    float lv[16];
#pragma unroll
                    for (int r = 0; r < 16; ++r) lv[r] = (float)gi[r] * rowf;
                    // narrowed, then times the weights of the lane's 16 tokens of block sb (x is staged without them)
                    const f16x8 l0 = pack_f16x8(lv) * __builtin_shufflevector(wq4[0], wq4[1], 0, 1, 2, 3, 4, 5, 6, 7);
                    const f16x8 l1 =
                        pack_f16x8(lv + 8) * __builtin_shufflevector(wq4[2], wq4[3], 0, 1, 2, 3, 4, 5, 6, 7);
                    __builtin_amdgcn_sched_barrier(0);
                    const i32x16 gn = gemm_g(bq);
                    // the next tile first: its conversion then overlaps the products below
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            acc[pt] =
                                __builtin_amdgcn_mfma_f32_32x32x16_f16(xa[ks][pt], ks ? l1 : l0, acc[pt], 0, 0, 0);
                    gi = gn;
                }
                __builtin_amdgcn_sched_barrier(0);
                if (c + 1 < c_end) issue_c_rows(c + 1);
                __builtin_amdgcn_sched_barrier(0);
                {  // diagonal block pair: per-element decay, causal mask, plain x codes
                    f16x8 xd[2][PT];
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            xd[ks][pt] = lds_read_tr16x8<kXsStride>(
                                xs_src + ((tb * kBlk + 16 * ks) * kXsStride + 32 * pt) * 2);
                    // When the decay across the block (its total of dt*A) stays
                    // below 2^64 the weight exp2(cum_t - cum_s) dt_s is the product of a row factor and the staged
                    // column weights (both inside the fp32 range); otherwise every element takes its own exponential.
                    const bool factored = __builtin_amdgcn_readfirstlane(-s_tot[tb] < 64.0f);
                    // the skip coefficient is made new per chunk for the compiler: the 16 selects below then stay here
                    // (lane masks in scalar registers) instead of 16 loop-invariant vector registers
                    float d_sel_c = d_sel;
                    asm volatile("" : "+v"(d_sel_c));
                    // four tokens s at a time, narrowed at once: the scheduling barriers keep the register groups apart
                    // so that at most one group's temporaries are live
                    f16x4 lq[4];
                    if (factored) {
                        const float e_row = exp2_fast(loc_t);
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg) {
                            const int s0 = 8 * rg + 4 * hb;
                            const f32x4 w4 = *reinterpret_cast<const f32x4 *>(s_w2 + tb * kBlk + 8 * rg + 4 * hba);
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                const float wgt = (s0 + i <= l32) ? e_row * w4[i] : 0.0f;  // causal mask
                                const float dd = (s0 + i == l32) ? d_sel_c : 0.0f;        // skip term on the diagonal
                                lq[rg][i] = (_Float16)fmaf((float)gi[4 * rg + i], wgt, dd);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    } else {
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg) {  // four consecutive tokens of the block per register group
                            const int s0 = 8 * rg + 4 * hb;
                            const f32x4 cs4 = *reinterpret_cast<const f32x4 *>(s_loc + tb * kBlk + 8 * rg + 4 * hba);
                            const f32x4 ds4 = *reinterpret_cast<const f32x4 *>(s_dt + tb * kBlk + 8 * rg + 4 * hba);
#pragma unroll
                            for (int i = 0; i < 4; ++i) {
                                // exponent forced to a huge negative value above the diagonal: weight exactly 0, no
                                // branch cum is non-increasing (dt >= 0, A <= 0): the exponent is <= 0 on and below the
                                // diagonal
                                const float arg = (s0 + i <= l32) ? loc_t - cs4[i] : -1.0e30f;
                                const float dd = (s0 + i == l32) ? d_sel_c : 0.0f;  // skip term on the diagonal
                                lq[rg][i] = (_Float16)fmaf((float)gi[4 * rg + i], exp2_fast(arg) * ds4[i], dd);
                            }
                            __builtin_amdgcn_sched_barrier(0);
                        }
                    }
                    const f16x8 l0 = __builtin_shufflevector(lq[0], lq[1], 0, 1, 2, 3, 4, 5, 6, 7);
                    const f16x8 l1 = __builtin_shufflevector(lq[2], lq[3], 0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            acc[pt] =
                                __builtin_amdgcn_mfma_f32_32x32x16_f16(xd[ks][pt], ks ? l1 : l0, acc[pt], 0, 0, 0);
                }

                // epilogue: scales and skip term in fp32, narrowing to fp16; a lane holds 4 consecutive channels of
                // token t per register group, and one exchange with the lane 32 positions away (same token) turns two
                // such groups into 8 consecutive channels, so that every lane stores 16 bytes and a token row gets 32
                uint16_t *yrow = a.y + ((tokbase + min(tl, nv - 1)) * H + h) * kP + p_base;
                // gate codes of the lane's outputs (staged by the state waves): 4 consecutive channels, one dword,
                // per register group
                uint32_t zq[PT][4];
                if (GATED) {
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg)
                            zq[pt][rg] =
                                *reinterpret_cast<const uint32_t *>(s_zs + tl * kZsStride + pt * 32 + 8 * rg + 4 * hb);
                }
                if (d_by_mfma) {
                    // the chunk's LDS arrays are not read past this point (the scale and SiLU tables stay as they are):
                    // the state waves restage them for the next chunk while this wave scales and stores its outputs
                    __syncthreads();
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt) {
                        f32x4 k4[4];  // s_x(h,p) * y_scale of the lane's 16 channels of this p tile
#pragma unroll
                        for (int rg = 0; rg < 4; ++rg)
                            k4[rg] = *reinterpret_cast<const f32x4 *>(s_sx + pt * 32 + 8 * rg + 4 * hba);
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            uint32_t w[2][2];  // [register group 2j, 2j+1][dword]
#pragma unroll
                            for (int e = 0; e < 2; ++e) {
                                const int rg = 2 * j + e;
                                f16x4 o;
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    float v = k4[rg][i] * acc[pt][4 * rg + i];
                                    if (GATED) v *= s_silu[(zq[pt][rg] >> (8 * i)) & 0xffu];
                                    o[i] = (_Float16)v;
                                }
                                const u32x2 ow = __builtin_bit_cast(u32x2, o);
                                w[e][0] = ow[0];
                                w[e][1] = ow[1];
                            }
                            // lanes 0..31 end up with group 2j of both half-waves (channels 16j .. 16j+7 of this p
                            // tile), lanes 32..63 with group 2j+1 (channels 16j+8 .. 16j+15)
                            const auto s0 = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                            const auto s1 = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                            const u32x4 v = {s0[0], s1[0], s0[1], s1[1]};
                            if (tl < nv) *reinterpret_cast<u32x4 *>(yrow + pt * 32 + 16 * j + 8 * hb) = v;
                        }
                    }
                } else {
                    const int tq = tok_pos(tl);
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                        for (int j = 0; j < 2; ++j) {
                            uint32_t w[2][2];
#pragma unroll
                            for (int e = 0; e < 2; ++e) {
                                const int rg = 2 * j + e;
                                f16x4 o;
#pragma unroll
                                for (int i = 0; i < 4; ++i) {
                                    const int p = pt * 32 + 8 * rg + 4 * hb + i;
                                    const _Float16 *xrow = reinterpret_cast<const _Float16 *>(s_xs) + tq * kXsStride;
                                    const float xc = (float)xrow[p] * (1.0f / kXs);
                                    float v = s_sx[p] * fmaf(y_scale, acc[pt][4 * rg + i], Dh * xc);
                                    if (GATED) v *= s_silu[(zq[pt][rg] >> (8 * i)) & 0xffu];
                                    o[i] = (_Float16)v;
                                }
                                const u32x2 ow = __builtin_bit_cast(u32x2, o);
                                w[e][0] = ow[0];
                                w[e][1] = ow[1];
                            }
                            const auto s0 = __builtin_amdgcn_permlane32_swap(w[0][0], w[1][0], false, false);
                            const auto s1 = __builtin_amdgcn_permlane32_swap(w[0][1], w[1][1], false, false);
                            const u32x4 v = {s0[0], s1[0], s0[1], s1[1]};
                            if (tl < nv) *reinterpret_cast<u32x4 *>(yrow + pt * 32 + 16 * j + 8 * hb) = v;
                        }
                    __syncthreads();  // this epilogue reads the staged x: the chunk's LDS arrays are free only now
                }
            } else {
                if (c + 1 < c_end) issue_c_rows(c + 1);
                __syncthreads();  // both roles are done with the chunk's LDS arrays
            }
        }
    } else {
        // ================= state waves: staging, token weights, state update ================= Carried state in x-code
        // * B-code units times kStScale (true state = s_x(p) s_B * st / kStScale): the state is carried already
        // narrowed by 2^-7, so that its fp16 copy for the C.H product needs no multiply (the factor rides on the token
        // weights of the B operand instead).  Wave w owns states n in [32w, 32w+32); st[pt][r]: p = 32 pt + l32, n = 32
        // w + 8 (r/4) + 4 hb + r%4.
        f32x16 st[PT];
#pragma unroll
        for (int pt = 0; pt < PT; ++pt)
#pragma unroll
            for (int r = 0; r < 16; ++r) st[pt][r] = 0.0f;
        // Registers that carry one chunk's global loads from the point of issue (the start of the previous chunk's
        // state update) to the staging phase: x codes (4 tokens x 4 PT channels), B codes (4 tokens x 16 states), and
        // dt of tokens 2 lane, 2 lane + 1 (first wave only: it computes every weight of the chunk).  Rows past the end
        // of the sequence are read from the last valid row and zeroed where they are consumed.  Vector-memory results
        // return in issue order, hence the loads are issued in the order they are consumed.
        xvec xr[4];
        u32x4 br[4];
        xvec zr[4];  // gate codes, same rows and columns as xr (GATED only)
        float dt0 = 0.0f, dt1 = 0.0f;
        // Staging lane maps: a thread takes 4 consecutive tokens and 4 PT channels of x (8 lanes cover a row of this
        // workgroup's channels), resp. 16 states of B (8 lanes cover a 128-byte row).
        const int xs4 = tid4 >> 3, xp8 = tid4 & 7;
        const int bs4 = tid4 >> 3, bn16 = tid4 & 7;
        auto issue_loads = [&](int c) {
            const int t0 = c * kQ;
            const int nv = min(kQ, L - t0);
            const size_t tokbase = (size_t)b * L + t0;
            const int8_t *xbase = a.x + (tokbase * H + h) * kP + p_base;
            const int8_t *bbase = a.B + (tokbase * G + g) * kN;
            const char *dbase = reinterpret_cast<const char *>(a.dt + tokbase * H + h);
            if (wave == 0) {
                if (a.dt_q) {  // codes of the pre-activation: kept as they arrive, turned into dt where they are used
                    const int8_t *qbase = a.dt_q + tokbase * H + h;
                    dt0 = __builtin_bit_cast(float, (int)qbase[(uint32_t)min(2 * lane, nv - 1) * (uint32_t)H]);
                    dt1 = __builtin_bit_cast(float, (int)qbase[(uint32_t)min(2 * lane + 1, nv - 1) * (uint32_t)H]);
                } else {
                    dt0 = *reinterpret_cast<const float *>(dbase + (uint32_t)min(2 * lane, nv - 1) * dt_row);
                    dt1 = *reinterpret_cast<const float *>(dbase + (uint32_t)min(2 * lane + 1, nv - 1) * dt_row);
                }
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t row = (uint32_t)min(4 * xs4 + k, nv - 1);
                xr[k] = *reinterpret_cast<const xvec *>(xbase + (row * x_row + (uint32_t)(4 * PT) * xp8));
                if (GATED)
                    zr[k] = *reinterpret_cast<const xvec *>(a.z + (tokbase * H + h) * kP + p_base +
                                                            (row * x_row + (uint32_t)(4 * PT) * xp8));
            }
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const uint32_t row = (uint32_t)min(4 * bs4 + k, nv - 1);
                br[k] = *reinterpret_cast<const u32x4 *>(bbase + (row * b_row + 16u * bn16));
            }
        };
        issue_loads(c_begin);
        if (SEG && seg > 0) {
            // Start state of segment seg from the state pass: with local_j the state segment j ends with when started
            // from zero (segment 0: from the caller's initial state) and d_j the sum of dt*A*log2(e) over its tokens,
            //   H = local_{seg-1} + 2^{d_{seg-1}} local_{seg-2} + 2^{d_{seg-1} + d_{seg-2}} local_{seg-3} + ...
            // (accumulator units: no scales involved)
            const size_t pairs = (size_t)a.s.batch * H;
            float dsum = 0.0f;
            for (int j = seg - 1; j >= 0; --j) {
                const float w = exp2_fast(dsum);
                const float *src = a.seg_state + ((size_t)j * pairs + bh) * kP * kN;
#pragma unroll
                for (int pt = 0; pt < PT; ++pt) {
                    const int p = pt * 32 + l32;
#pragma unroll
                    for (int rg = 0; rg < 4; ++rg) {
                        const int n0 = 32 * wave + 8 * rg + 4 * hb;
                        const f32x4 v = *reinterpret_cast<const f32x4 *>(src + (size_t)(p_base + p) * kN + n0);
#pragma unroll
                        for (int i = 0; i < 4; ++i) st[pt][4 * rg + i] = fmaf(w, v[i], st[pt][4 * rg + i]);
                    }
                }
                dsum += a.seg_decay[(size_t)j * pairs + bh];
            }
        }
        if (convert_init) {
            __syncthreads();  // the scales are in LDS
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const int p = pt * 32 + l32;
                const float inv = kStScale * (d_by_mfma ? y_scale : 1.0f) / (s_sx[p] * sB);
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int n0 = 32 * wave + 8 * rg + 4 * hb;
                    const f32x4 v =
                        *reinterpret_cast<const f32x4 *>(a.init_state + ((size_t)bh * kP + p_base + p) * kN + n0);
#pragma unroll
                    for (int i = 0; i < 4; ++i) st[pt][4 * rg + i] = v[i] * inv;
                }
            }
        }
        for (int c = c_begin; c < c_end; ++c) {
            set_chunk_priority(c);
            const int t0 = c * kQ;
            const int nv = min(kQ, L - t0);
            // ---- the first wave turns dt into everything the chunk needs of it: the inclusive prefix sum of dt*A
            // (two tokens per lane, data-parallel-primitive moves only) and, per token s, the weights that stand
            // between the x codes and their uses.  With m the prefix sum at the last token of the token's 32-token
            // block, R the one in front of the block, cum_last the one at the end of the chunk:
            //   we = dt exp2(m - cum_s) kAcc / kXs          off-diagonal blocks (row factor exp2(cum_t - m) 2^-7)
            //   w2 = dt exp2(R - cum_s) 2^-7 kAcc / kXs     diagonal block (row factor exp2(cum_t - R))
            //   ws = dt exp2(cum_last - cum_s) 2^-7 / kXs   state update of the single-term path
            //   two-term path: the state decays block by block in fp32, its token weight dt exp2(m - cum_s) 2^-7 /
            //   kXs is wq (1 + wd) with wq rounded to 4 significant bits, so that B codes (7 bits) times wq are exact
            //   in fp16: ws = wq, wd
            // All exponents are <= 0 except in w2, which may overflow under extreme decay (it is not used then). ----
            if (wave == 0) {
                if (a.dt_q) {  // step size = softplus(s_dt * code + bias) (Section 3.2)
                    const float bias = a.dt_bias ? a.dt_bias[h] : 0.0f;
                    const float v0 = a.dt_scale * (float)__builtin_bit_cast(int, dt0) + bias;
                    const float v1 = a.dt_scale * (float)__builtin_bit_cast(int, dt1) + bias;
                    dt0 = fmaxf(v0, 0.0f) + log1pf(expf(-fabsf(v0)));
                    dt1 = fmaxf(v1, 0.0f) + log1pf(expf(-fabsf(v1)));
                }
                if (2 * lane >= nv) dt0 = 0.0f;  // padded steps: dt = 0
                if (2 * lane + 1 >= nv) dt1 = 0.0f;
                const float a0 = dt0 * Ah, a1 = dt1 * Ah;
                // A row of 16 lanes is one 32-token block: the weights inside a block are formed from the block's own
                // sums, not from differences of the chunk's prefix sums, which lose ulp(|prefix sum|) when the decay
                // is extreme.  With m and R the chunk's prefix sums at the block's end and in front of it:
                // m - cum_s is the sum of dt*A over the block's tokens behind s, taken as that sum (a difference of
                // two prefix sums would be off by their rounding, 1e-4 of the weight of the last token of a block that
                // decays by 2^-2000), and R - cum_s = -loc_s with loc the block's own prefix sum.
                float loc1;
                const float cum1 = wave_inclusive_scan(a0 + a1, loc1), cum0 = cum1 - a1;
                const float loc0 = loc1 - a1;
                const float suf1 = row_suffix_sum_exclusive(a0 + a1), suf0 = suf1 + a1;  // behind tokens 2l+1, 2l
                // weights towards the output accumulators
                const float d0 = dt0 * (kAcc / kXs), d1 = dt1 * (kAcc / kXs);
                // weights towards the state accumulators
                const float q0 = dt0 * (kNarrow / kXs), q1 = dt1 * (kNarrow / kXs);
                const float e0 = exp2_fast(suf0), e1 = exp2_fast(suf1);
                const float we0 = e0 * d0, we1 = e1 * d1;
                *reinterpret_cast<float2 *>(s_cum + 2 * lane) = make_float2(cum0, cum1);
                // Every exponent that spans a stretch of tokens is formed from sums over that stretch: the block's own
                // prefix sums, the blocks' totals (the row scan's value in the last lane of a row) and the sums of the
                // totals in between, never from differences of the chunk's prefix sums, which carry rounding of the
                // size of what lies in front of the stretch.
                *reinterpret_cast<float2 *>(s_loc + 2 * lane) = make_float2(loc0, loc1);
                const float T1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, loc1), 31));
                const float T2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, loc1), 47));
                const float T3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, loc1), 63));
                if ((lane & 15) == 15) s_tot[lane >> 4] = loc1;
                if (lane < kNBlk * kNBlk)  // [tb][sb]: lane 8 = (2,0): T1, lane 12 = (3,0): T1 + T2, lane 13 = (3,1): T2
                    s_gap[lane] = lane == 8 ? T1 : lane == 12 ? T1 + T2 : lane == 13 ? T2 : 0.0f;
                *reinterpret_cast<float2 *>(s_dt + 2 * lane) = make_float2(d0 * kNarrow, d1 * kNarrow);
                *reinterpret_cast<float2 *>(s_w2 + 2 * lane) =
                    make_float2(exp2_fast(-loc0) * d0 * kNarrow, exp2_fast(-loc1) * d1 * kNarrow);
                *reinterpret_cast<f16x2 *>(s_we + 2 * lane) = (f16x2){(_Float16)we0, (_Float16)we1};
                if (!PRECISE) {
                    // cum_last - cum_s: what lies behind s in its block plus the totals of the later blocks
                    const int row = lane >> 4;
                    const float later = row == 0 ? T1 + (T2 + T3) : row == 1 ? T2 + T3 : row == 2 ? T3 : 0.0f;
                    *reinterpret_cast<f16x2 *>(s_ws + 2 * lane) = (f16x2){(_Float16)(exp2_fast(suf0 + later) * q0),
                                                                          (_Float16)(exp2_fast(suf1 + later) * q1)};
                } else {
                    f16x2 wq, wd;
                    const float w[2] = {e0 * q0, e1 * q1};
#pragma unroll
                    for (int i = 0; i < 2; ++i) {
                        const float q =
                            __builtin_bit_cast(float, (__builtin_bit_cast(uint32_t, w[i]) + 0x00080000u) & 0xfff00000u);
                        wq[i] = (_Float16)q;
                        wd[i] = (_Float16)(q > 0.0f ? (w[i] - q) / q : 0.0f);
                    }
                    *reinterpret_cast<f16x2 *>(s_ws + 2 * lane) = wq;
                    *reinterpret_cast<f16x2 *>(s_wd + 2 * lane) = wd;
                }
            }

            // carried state -> LDS as fp16 (operand of the C.H product of this chunk)
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    f16x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = (_Float16)st[pt][4 * rg + i];
                    *reinterpret_cast<f16x4 *>(s_hs + (pt * 32 + l32) * kHsStride + 32 * wave + 8 * rg + 4 * hb) = v;
                }

            // ---- x (fp16 codes times kXs) and B codes into LDS, token-major, token rows permuted ----
            {
                const int s0 = 4 * xs4, row0 = tok_pos(s0);
#pragma unroll
                for (int k = 0; k < 4; ++k) {
                    xvec w = xr[k];
                    if (nv < kQ) {  // partial last chunk: rows past the end are zero
                        if (s0 + k >= nv) w = (xvec)(0u);
                    }
                    unsigned char *xs_row = s_xs + ((row0 + k) * kXsStride + 4 * PT * xp8) * 2;
#pragma unroll
                    for (int q = 0; q < PT; ++q) *reinterpret_cast<f16x4 *>(xs_row + 8 * q) = i8x4_to_f16_xs(w[q]);
                    if (GATED) *reinterpret_cast<xvec *>(s_zs + (s0 + k) * kZsStride + 4 * PT * xp8) = zr[k];
                }
            }
            {
                const int row0 = tok_pos(4 * bs4);
                if (nv < kQ) {
#pragma unroll
                    for (int k = 0; k < 4; ++k)
                        if (4 * bs4 + k >= nv) br[k] = (u32x4){0u, 0u, 0u, 0u};
                }
#pragma unroll
                for (int k = 0; k < 4; ++k)
                    *reinterpret_cast<u32x4 *>(s_bq + (row0 + k) * kBqStride + 16 * bn16) = br[k];
            }
            __syncthreads();  // the chunk is staged: the output waves start on it
            if (c + 1 < c_end) issue_loads(c + 1);  // the next chunk's global loads fly while this chunk is computed
            // ---- state update: wave w owns states n in [32w, 32w+32) ----
            // source-lane roles of the transposing loads, rebuilt per chunk like the addresses of the output phase
            int lane_s = fresh_lane();
            asm volatile("" : "+v"(lane_s));
            const int i16s = lane_s & 15, c16s = (lane_s >> 4) & 1, hbs = lane_s >> 5;
            const unsigned char *bq_src =
                s_bq + (8 * hbs + (i16s >> 1)) * kBqStride + 32 * wave + 16 * c16s + 8 * (i16s & 1);
            const int xs_off = ((8 * hbs + (i16s >> 2)) * kXsStride + 16 * c16s + 4 * (i16s & 3)) * 2;
            if (PRECISE) {
                for (int sb = 0; sb < kNBlk; ++sb) {
                    if (sb * kBlk >= nv) break;  // the padded steps are identity steps
                    const float m = s_cum[sb * kBlk + kBlk - 1];
                    const float gdec = exp2_fast(s_tot[sb]);  // the block's own total, not m - m_prev
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) st[pt][r] *= gdec;
                    // what this block adds decays by exp2(cum_last - m) before the chunk ends: dead blocks only decay
                    if (__builtin_amdgcn_readfirstlane(s_cum[kQ - 1] - m < -dead)) continue;
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const int row = sb * kBlk + 16 * ks;
                        const u32x2 w = lds_read_tr8(bq_src + row * kBqStride);
                        // weights of the 8 tokens of this k group: tokens row + 4 hb + [0,4) and row + 8 + 4 hb + [0,4)
                        const f16x4 *ws4 = reinterpret_cast<const f16x4 *>(s_ws + row + 4 * hbs);
                        const f16x4 *wd4 = reinterpret_cast<const f16x4 *>(s_wd + row + 4 * hbs);
                        const f16x8 wq = __builtin_shufflevector(ws4[0], ws4[2], 0, 1, 2, 3, 4, 5, 6, 7);
                        const f16x8 wd = __builtin_shufflevector(wd4[0], wd4[2], 0, 1, 2, 3, 4, 5, 6, 7);
                        const f16x8 bf = i8x8_to_f16(w[0], w[1]) * wq;  // exact: 7 bits times 4 bits
                        const f16x8 bfd = bf * wd;                      // the small term, rounded
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt) {
                            const int off = xs_off + (row * kXsStride + 32 * pt) * 2;
                            const f16x8 xb = lds_read_tr16x8<kXsStride>(s_xs + off);
                            st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, xb, st[pt], 0, 0, 0);
                            st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bfd, xb, st[pt], 0, 0, 0);
                        }
                    }
                }
            } else {
                {
                    // padded steps leave cum flat: cum at the last valid token
                    const float gdec = exp2_fast(s_cum[kQ - 1]);
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                        for (int r = 0; r < 16; ++r) st[pt][r] *= gdec;
                }
#pragma unroll
                // blocks past the end hold zero weights (dt = 0): they add nothing
                for (int sb = 0; sb < kNBlk; ++sb) {
                    // the block's largest weight is that of its last token, exp2(cum_last - m_sb) dt
                    if (__builtin_amdgcn_readfirstlane(s_cum[kQ - 1] - s_cum[sb * kBlk + kBlk - 1] < -dead)) continue;
                    u32x2 bw[2];
                    f16x8 xb[2][PT], wv[2];
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const int row = sb * kBlk + 16 * ks;
                        bw[ks] = lds_read_tr8(bq_src + row * kBqStride);
                        // weights of the 8 tokens of this k group: tokens row + 4 hb + [0,4) and row + 8 + 4 hb + [0,4)
                        wv[ks] = __builtin_shufflevector(*reinterpret_cast<const f16x4 *>(s_ws + row + 4 * hbs),
                                                         *reinterpret_cast<const f16x4 *>(s_ws + row + 8 + 4 * hbs),
                                                         0, 1, 2, 3, 4, 5, 6, 7);
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            xb[ks][pt] = lds_read_tr16x8<kXsStride>(s_xs + xs_off + (row * kXsStride + 32 * pt) * 2);
                    }
                    // all LDS reads of the block are in flight before the first conversion
                    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                    for (int ks = 0; ks < 2; ++ks) {
                        const f16x8 bf = i8x8_to_f16(bw[ks][0], bw[ks][1]) * wv[ks];
#pragma unroll
                        for (int pt = 0; pt < PT; ++pt)
                            st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, xb[ks][pt], st[pt], 0, 0, 0);
                    }
                }
            }
            __syncthreads();  // the output waves are done with x, B, the weights and the fp16 state of this chunk
        }

        if (a.state && (!SEG || seg + 1 == a.nseg)) {
#pragma unroll
            for (int pt = 0; pt < PT; ++pt) {
                const int p = pt * 32 + l32;
                const float sc = s_sx[p] * sB / ((d_by_mfma ? y_scale : 1.0f) * kStScale);
#pragma unroll
                for (int rg = 0; rg < 4; ++rg) {
                    const int n0 = 32 * wave + 8 * rg + 4 * hb;
                    f32x4 v;
#pragma unroll
                    for (int i = 0; i < 4; ++i) v[i] = st[pt][4 * rg + i] * sc;
                    *reinterpret_cast<f32x4 *>(a.state + ((size_t)bh * kP + p_base + p) * kN + n0) = v;
                }
            }
        }
    }
}


// ---- State pass of the sequence split ----
// One workgroup of four waves carries the state of one (sequence, head) (or channel half) through the chunks of one
// segment, from zero (segment 0: from the caller's initial state), and leaves it in the workspace as it stands in the
// accumulators, with the segment's decay total.  Staging, token weights and the state update are those of the state
// waves of prefill_mfma_kernel (same operations in the same order on the same values).  There are no outputs and a
// launch has one or two workgroups per compute unit, so nothing hides latency but the wave itself: the global loads
// of kStateDepth chunks are in flight, each chunk's in a register set of its own, and the LDS operands of a group of
// 16 tokens are requested one group ahead of their use.  Measured per chunk and workgroup (cycles): staging 640,
// barrier 260, issuing the next loads 640, state update 2090, barrier 160; a lone wave issues a vector instruction
// every 8 cycles and an LDS instruction every 12, which is what these phases add up to.  Eight waves that split a
// chunk's tokens between two copies of the state were not faster (the phases are serial between the barriers and
// the two waves of a SIMD share its LDS and memory paths).
constexpr int kStateThreads = 256;
constexpr int kStateDepth = 2;

template <int PT>
struct StateLds {
    static constexpr int kXsStride = Lds<PT>::kXsStride;
    static constexpr int kOffCum = 0;                       // float[128]
    static constexpr int kOffWs = kOffCum + 4 * kQ;         // fp16[128]
    static constexpr int kOffWd = kOffWs + 2 * kQ;          // fp16[128]
    static constexpr int kOffTot = kOffWd + 2 * kQ;         // float[4]  the blocks' totals
    static constexpr int kOffBq = kOffTot + 4 * kNBlk + 48; // int8 [128][144]
    static constexpr int kOffXs = kOffBq + kQ * kBqStride;  // fp16 [128][kXsStride]
    static constexpr int kBytes = kOffXs + 2 * kQ * kXsStride;
    static_assert(kOffBq % 16 == 0 && kOffXs % 16 == 0, "LDS arrays must be 16-byte aligned");
};

template <bool PRECISE, int PT>
__global__ __launch_bounds__(kStateThreads, 2) void segment_state_kernel(SsdArgs a)
{
    typedef StateLds<PT> LY;
    constexpr int kXsStride = LY::kXsStride;
    extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
    float *s_cum = reinterpret_cast<float *>(smem + LY::kOffCum);
    _Float16 *s_ws = reinterpret_cast<_Float16 *>(smem + LY::kOffWs);
    _Float16 *s_wd = reinterpret_cast<_Float16 *>(smem + LY::kOffWd);
    float *s_tot = reinterpret_cast<float *>(smem + LY::kOffTot);
    unsigned char *s_bq = smem + LY::kOffBq;
    unsigned char *s_xs = smem + LY::kOffXs;

    const int L = a.s.seqlen, H = a.s.nheads, G = a.s.ngroups;
    const int wgs_per_seg = a.s.batch * H * (2 / PT);
    const int seg = (int)blockIdx.x / wgs_per_seg;  // 0 .. nseg-2
    const int c_begin = seg * a.seg_chunks, c_end = c_begin + a.seg_chunks;
    const int bid = (int)blockIdx.x - seg * wgs_per_seg;
    int pair = bid, half = 0;  // as in prefill_mfma_kernel
    if (PT == 1) {
        const int npairs = a.s.batch * H, full = npairs >> 3;
        if (bid < 16 * full) {
            pair = (bid & 7) | ((bid >> 4) << 3);
            half = (bid >> 3) & 1;
        } else {
            const int t = bid - 16 * full, r = npairs - 8 * full;
            pair = 8 * full + t % r;
            half = t / r;
        }
    }
    const int p_base = 32 * half;
    const int bh = block_to_bh(a, pair);
    const int b = bh / H, h = bh - b * H, g = h / (H / G);
    const int tid = threadIdx.x, lane = tid & 63;
    const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
    const int l32 = lane & 31, hb = lane >> 5;
    const float Ah = a.A[h] * 1.44269504088896340736f;
    const float dead = (a.s.flags & QUAMBA_FLAG_NO_DECAY_SKIP) ? __builtin_inff() : kDead;
    const uint32_t x_row = (uint32_t)H * kP, b_row = (uint32_t)G * kN, dt_row = (uint32_t)H * 4u;
    typedef uint32_t xvec __attribute__((ext_vector_type(PT)));

    f32x16 st[PT];
#pragma unroll
    for (int pt = 0; pt < PT; ++pt)
#pragma unroll
        for (int r = 0; r < 16; ++r) st[pt][r] = 0.0f;

    struct LoadSet {
        xvec xr[4];
        u32x4 br[4];
        float dt0, dt1;
    };
    LoadSet sets[kStateDepth];
    const int xs4 = tid >> 3, xp8 = tid & 7;
    const int bs4 = tid >> 3, bn16 = tid & 7;
    // Every chunk of the state pass is complete (only the last segment, which this kernel does not walk, can end in a
    // partial chunk), so a thread's rows sit at fixed offsets from the chunk's first token.
    uint32_t x_off[4], b_off[4];
#pragma unroll
    for (int k = 0; k < 4; ++k) {
        x_off[k] = (uint32_t)(4 * xs4 + k) * x_row + (uint32_t)(4 * PT) * xp8;
        b_off[k] = (uint32_t)(4 * bs4 + k) * b_row + 16u * bn16;
    }
    const uint32_t dt_off = (uint32_t)(2 * lane) * dt_row, dq_off = (uint32_t)(2 * lane) * (uint32_t)H;
    auto issue_loads = [&](int c, LoadSet &ls) {
        const size_t tokbase = (size_t)b * L + (size_t)c * kQ;
        const int8_t *xbase = a.x + (tokbase * H + h) * kP + p_base;
        const int8_t *bbase = a.B + (tokbase * G + g) * kN;
        // every wave issues the same loads (only the first uses dt): a wait for one set's registers is then an exact
        // count of the younger loads, and leaves those of the other sets in flight
        ls.dt0 = ls.dt1 = 0.0f;
        if (wave == 0) {
            if (a.dt_q) {
                const int8_t *qbase = a.dt_q + tokbase * H + h;
                ls.dt0 = __builtin_bit_cast(float, (int)qbase[dq_off]);
                ls.dt1 = __builtin_bit_cast(float, (int)qbase[dq_off + (uint32_t)H]);
            } else {
                const char *dbase = reinterpret_cast<const char *>(a.dt + tokbase * H + h);
                ls.dt0 = *reinterpret_cast<const float *>(dbase + dt_off);
                ls.dt1 = *reinterpret_cast<const float *>(dbase + dt_off + dt_row);
            }
        }
#pragma unroll
        for (int k = 0; k < 4; ++k) ls.xr[k] = *reinterpret_cast<const xvec *>(xbase + x_off[k]);
#pragma unroll
        for (int k = 0; k < 4; ++k) ls.br[k] = *reinterpret_cast<const u32x4 *>(bbase + b_off[k]);
    };
    // Loads are issued unconditionally (past the segment's end: its last chunk once more, unused), for the same reason.
#pragma unroll
    for (int k = 0; k < kStateDepth; ++k) issue_loads(min(c_begin + k, c_end - 1), sets[k]);

    if (a.init_state && seg == 0) {
        // the caller's initial state in accumulator units: the same arithmetic as in prefill_mfma_kernel
        const float sB = a.B_scales[g], sC = a.C_scales[g];
        const float y_scale = sB * sC * (1.0f / (kNarrow * kAcc));
        const float Dh = a.D ? a.D[h] : 0.0f;
        const float d_acc = Dh / (y_scale * kXs);
        const bool d_by_mfma = fabsf(d_acc) < 3.0e4f;
#pragma unroll
        for (int pt = 0; pt < PT; ++pt) {
            const int p = pt * 32 + l32;
            const float sx = x_scale_lookup(a, h, p_base + p) * (d_by_mfma ? y_scale : 1.0f);
            const float inv = kNarrow * (d_by_mfma ? y_scale : 1.0f) / (sx * sB);
#pragma unroll
            for (int rg = 0; rg < 4; ++rg) {
                const int n0 = 32 * wave + 8 * rg + 4 * hb;
                const f32x4 v = *reinterpret_cast<const f32x4 *>(a.init_state + ((size_t)bh * kP + p_base + p) * kN + n0);
#pragma unroll
                for (int i = 0; i < 4; ++i) st[pt][4 * rg + i] = v[i] * inv;
            }
        }
    }

    float seg_cum = 0.0f;  // sum of the chunks' dt*A*log2(e) totals (first wave)
    auto stage = [&](LoadSet &ls) {
        if (wave == 0) {
            float dt0 = ls.dt0, dt1 = ls.dt1;
            if (a.dt_q) {  // step size = softplus(s_dt * code + bias) (Section 3.2)
                const float bias = a.dt_bias ? a.dt_bias[h] : 0.0f;
                const float v0 = a.dt_scale * (float)__builtin_bit_cast(int, dt0) + bias;
                const float v1 = a.dt_scale * (float)__builtin_bit_cast(int, dt1) + bias;
                dt0 = fmaxf(v0, 0.0f) + log1pf(expf(-fabsf(v0)));
                dt1 = fmaxf(v1, 0.0f) + log1pf(expf(-fabsf(v1)));
            }
            const float a0 = dt0 * Ah, a1 = dt1 * Ah;
            float loc1;
            const float cum1 = wave_inclusive_scan(a0 + a1, loc1), cum0 = cum1 - a1;
            const float cum_last = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, cum1), 63));
            seg_cum += cum_last;
            const float q0 = dt0 * (kNarrow / kXs), q1 = dt1 * (kNarrow / kXs);
            *reinterpret_cast<float2 *>(s_cum + 2 * lane) = make_float2(cum0, cum1);
            // exponents from sums over their own stretch of tokens, as in prefill_mfma_kernel
            const float suf1 = row_suffix_sum_exclusive(a0 + a1), suf0 = suf1 + a1;
            if ((lane & 15) == 15) s_tot[lane >> 4] = loc1;
            if (!PRECISE) {
                const float T1 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, loc1), 31));
                const float T2 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, loc1), 47));
                const float T3 = __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, loc1), 63));
                const int row = lane >> 4;
                const float later = row == 0 ? T1 + (T2 + T3) : row == 1 ? T2 + T3 : row == 2 ? T3 : 0.0f;
                *reinterpret_cast<f16x2 *>(s_ws + 2 * lane) =
                    (f16x2){(_Float16)(exp2_fast(suf0 + later) * q0), (_Float16)(exp2_fast(suf1 + later) * q1)};
            } else {
                const float e0 = exp2_fast(suf0), e1 = exp2_fast(suf1);
                const float w[2] = {e0 * q0, e1 * q1};
                f16x2 wq, wd;
#pragma unroll
                for (int i = 0; i < 2; ++i) {
                    const float q =
                        __builtin_bit_cast(float, (__builtin_bit_cast(uint32_t, w[i]) + 0x00080000u) & 0xfff00000u);
                    wq[i] = (_Float16)q;
                    wd[i] = (_Float16)(q > 0.0f ? (w[i] - q) / q : 0.0f);
                }
                *reinterpret_cast<f16x2 *>(s_ws + 2 * lane) = wq;
                *reinterpret_cast<f16x2 *>(s_wd + 2 * lane) = wd;
            }
        }
        {
            const int s0 = 4 * xs4, row0 = tok_pos(s0);
#pragma unroll
            for (int k = 0; k < 4; ++k) {
                const xvec w = ls.xr[k];
                unsigned char *xs_row = s_xs + ((row0 + k) * kXsStride + 4 * PT * xp8) * 2;
#pragma unroll
                for (int q = 0; q < PT; ++q) *reinterpret_cast<f16x4 *>(xs_row + 8 * q) = i8x4_to_f16_xs(w[q]);
            }
        }
        {
            const int row0 = tok_pos(4 * bs4);
#pragma unroll
            for (int k = 0; k < 4; ++k)
                *reinterpret_cast<u32x4 *>(s_bq + (row0 + k) * kBqStride + 16 * bn16) = ls.br[k];
        }
    };
    // The LDS operands of the next group of 16 tokens are requested before the current group is converted and
    // multiplied: the workgroup has one wave per SIMD, so nothing else hides the LDS latency.
    struct StepOps {
        u32x2 bw;
        f16x8 wv, wd, xb[PT];
    };
    const int i16s = lane & 15, c16s = (lane >> 4) & 1;
    const unsigned char *bq_src = s_bq + (8 * hb + (i16s >> 1)) * kBqStride + 32 * wave + 16 * c16s + 8 * (i16s & 1);
    const int xs_off = ((8 * hb + (i16s >> 2)) * kXsStride + 16 * c16s + 4 * (i16s & 3)) * 2;
    auto update = [&]() {
        auto fetch = [&](int step, StepOps &o) {  // step = 2 sb + ks: tokens 16 step .. 16 step + 15
            const int row = 16 * step;
            o.bw = lds_read_tr8(bq_src + row * kBqStride);
            // weights of the 8 tokens of this k group: tokens row + 4 hb + [0,4) and row + 8 + 4 hb + [0,4)
            o.wv = __builtin_shufflevector(*reinterpret_cast<const f16x4 *>(s_ws + row + 4 * hb),
                                           *reinterpret_cast<const f16x4 *>(s_ws + row + 8 + 4 * hb), 0, 1, 2, 3, 4, 5, 6,
                                           7);
            if (PRECISE)
                o.wd = __builtin_shufflevector(*reinterpret_cast<const f16x4 *>(s_wd + row + 4 * hb),
                                               *reinterpret_cast<const f16x4 *>(s_wd + row + 8 + 4 * hb), 0, 1, 2, 3, 4,
                                               5, 6, 7);
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
                o.xb[pt] = lds_read_tr16x8<kXsStride>(s_xs + xs_off + (row * kXsStride + 32 * pt) * 2);
        };
        StepOps ops[2];
        fetch(0, ops[0]);
        const float cum_last = s_cum[kQ - 1];
        if (!PRECISE) {
            const float gdec = exp2_fast(cum_last);
#pragma unroll
            for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                for (int r = 0; r < 16; ++r) st[pt][r] *= gdec;
        }
#pragma unroll
        for (int step = 0; step < 2 * kNBlk; ++step) {
            const int sb = step >> 1;
            if (step + 1 < 2 * kNBlk) fetch(step + 1, ops[(step + 1) & 1]);
            const StepOps &o = ops[step & 1];
            const float m = s_cum[sb * kBlk + kBlk - 1];
            if (PRECISE && (step & 1) == 0) {
                const float gdec = exp2_fast(s_tot[sb]);  // the block's own total
#pragma unroll
                for (int pt = 0; pt < PT; ++pt)
#pragma unroll
                    for (int r = 0; r < 16; ++r) st[pt][r] *= gdec;
            }
            // what this block adds decays by exp2(cum_last - m) before the chunk ends: dead blocks only decay
            const bool skip = __builtin_amdgcn_readfirstlane(cum_last - m < -dead);
            if (!skip) {
                const f16x8 bf = i8x8_to_f16(o.bw[0], o.bw[1]) * o.wv;  // two-term path: exact (7 bits times 4 bits)
                if (PRECISE) {
                    const f16x8 bfd = bf * o.wd;  // the small term, rounded
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt) {
                        st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, o.xb[pt], st[pt], 0, 0, 0);
                        st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bfd, o.xb[pt], st[pt], 0, 0, 0);
                    }
                } else {
#pragma unroll
                    for (int pt = 0; pt < PT; ++pt)
                        st[pt] = __builtin_amdgcn_mfma_f32_32x32x16_f16(bf, o.xb[pt], st[pt], 0, 0, 0);
                }
            }
        }
    };

    int c = c_begin;
    for (; c + kStateDepth <= c_end; c += kStateDepth) {
#pragma unroll
        for (int k = 0; k < kStateDepth; ++k) {
            stage(sets[k]);
            __syncthreads();  // the chunk is staged
            issue_loads(min(c + k + kStateDepth, c_end - 1), sets[k]);
            update();
            __syncthreads();  // every wave is done with the staged chunk
        }
    }
    // the remaining chunks (fewer than kStateDepth) are in flight already
#pragma unroll
    for (int k = 0; k + 1 < kStateDepth; ++k) {
        if (c + k < c_end) {  // uniform over the workgroup
            stage(sets[k]);
            __syncthreads();
            update();
            __syncthreads();
        }
    }

    const size_t pairs = (size_t)a.s.batch * H;
    float *dst = a.seg_state + ((size_t)seg * pairs + bh) * kP * kN;
#pragma unroll
    for (int pt = 0; pt < PT; ++pt) {
        const int p = pt * 32 + l32;
#pragma unroll
        for (int rg = 0; rg < 4; ++rg) {
            const int n0 = 32 * wave + 8 * rg + 4 * hb;
            f32x4 v;
#pragma unroll
            for (int i = 0; i < 4; ++i) v[i] = st[pt][4 * rg + i];
            *reinterpret_cast<f32x4 *>(dst + (size_t)(p_base + p) * kN + n0) = v;
        }
    }
    if (wave == 0 && lane == 0 && half == 0) a.seg_decay[(size_t)seg * pairs + bh] = seg_cum;
}

}  // namespace

bool prefill_mfma_supports(const quamba_ssd_shape_t &s) { return s.headdim == kP && s.d_state == kN; }

namespace {

template <bool PRECISE, int PT, bool GATED, bool SEG>
hipError_t launch_scan_seg(const SsdArgs &a, hipStream_t stream)
{
    constexpr int lds = GATED ? Lds<PT>::kBytesGated : Lds<PT>::kBytes;
    const int segs = a.nseg > 1 ? a.nseg : 1;  // one set of workgroups per segment
    const dim3 grid((unsigned)(a.s.batch * a.s.nheads * (2 / PT) * segs));
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void *>(prefill_mfma_kernel<PRECISE, PT, GATED, SEG>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, lds);
    if (e != hipSuccess) return e;
    hipLaunchKernelGGL((prefill_mfma_kernel<PRECISE, PT, GATED, SEG>), grid, dim3(kThreads), lds, stream, a);
    return hipGetLastError();
}

template <bool PRECISE, int PT, bool GATED>
hipError_t launch_scan_gated(const SsdArgs &a, hipStream_t stream)
{
    return a.nseg > 1 ? launch_scan_seg<PRECISE, PT, GATED, true>(a, stream)
                      : launch_scan_seg<PRECISE, PT, GATED, false>(a, stream);
}

template <bool PRECISE, int PT>
hipError_t launch_scan(const SsdArgs &a, hipStream_t stream)
{
    return a.z ? launch_scan_gated<PRECISE, PT, true>(a, stream) : launch_scan_gated<PRECISE, PT, false>(a, stream);
}

// The state pass of a sequence split: segments 0 .. nseg-2, one workgroup per (segment, sequence, head or channel half).
template <bool PRECISE, int PT>
hipError_t launch_segment_state(const SsdArgs &a, hipStream_t stream)
{
    constexpr int lds = StateLds<PT>::kBytes;
    const dim3 grid((unsigned)(a.s.batch * a.s.nheads * (2 / PT) * (a.nseg - 1)));
    hipLaunchKernelGGL((segment_state_kernel<PRECISE, PT>), grid, dim3(kStateThreads), lds, stream, a);
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

}  // namespace

// Few (sequence, head) pairs leave compute units idle, and a workgroup walks its sequence chunk by chunk.  Such
// batches are cut along the sequence: with `pairs` workgroups per segment (twice that with the channel split) the
// plan aims at two workgroups per compute unit, at least two chunks per segment and at most kMaxSegments segments.
constexpr int kMaxSegments = 8;
PrefillPlan prefill_mfma_plan(const quamba_ssd_shape_t &s)
{
    const int64_t pairs = (int64_t)s.batch * s.nheads;
    const int cus = compute_units();
    PrefillPlan plan;
    // fewer (sequence, head) pairs than compute units: give every head two workgroups (half of the channels each)
    plan.channel_split = !(s.flags & QUAMBA_FLAG_NO_CHANNEL_SPLIT) && pairs <= (int64_t)cus;
    plan.nseg = 1;
    plan.seg_chunks = 0;
    const int nchunks = (s.seqlen + kQ - 1) / kQ;
    // The split costs a second launch and a pass over all but the last segment that only carries the state (about a
    // third of the work of those tokens).  Measured on MI355X it pays from 8 chunks on where the unsplit launch leaves
    // compute units empty, and from 16 chunks on where it already has a workgroup on every compute unit (the split
    // then only buys the second workgroup per unit).
    const int64_t unsplit_wgs = pairs * (plan.channel_split ? 2 : 1);
    const int min_chunks = unsplit_wgs >= (int64_t)cus ? 16 : 8;
    if ((s.flags & QUAMBA_FLAG_NO_SEQ_SPLIT) || !prefill_mfma_supports(s) || nchunks < min_chunks ||
        pairs > (int64_t)cus)
        return plan;
    // Whole heads (one workgroup per pair and segment) compute the score tiles once instead of twice, so the channel
    // split is kept only where even kMaxSegments segments of whole heads would not fill the compute units.
    const int seg_cap = (int)std::min<int64_t>(kMaxSegments, nchunks / 2);
    int nseg;
    if (!plan.channel_split || pairs * seg_cap >= (int64_t)cus) {
        plan.channel_split = false;
        nseg = (int)std::min<int64_t>(seg_cap, (2 * (int64_t)cus) / pairs);
    } else {
        nseg = (int)std::min<int64_t>(seg_cap, (int64_t)cus / pairs);
    }
    if (nseg < 2) return plan;
    plan.seg_chunks = (nchunks + nseg - 1) / nseg;
    plan.nseg = (nchunks + plan.seg_chunks - 1) / plan.seg_chunks;  // every segment holds at least one chunk
    if (plan.nseg < 2) {
        plan.nseg = 1;
        plan.seg_chunks = 0;
    }
    return plan;
}

size_t prefill_mfma_workspace_bytes(const quamba_ssd_shape_t &s)
{
    const PrefillPlan plan = prefill_mfma_plan(s);
    if (plan.nseg < 2) return 0;
    const size_t pairs = (size_t)s.batch * s.nheads;
    return sizeof(float) * (size_t)(plan.nseg - 1) * pairs * ((size_t)kP * kN + 1);
}

hipError_t launch_prefill_mfma(const SsdArgs &a_in, void *workspace, hipStream_t stream)
{
    SsdArgs a = a_in;
    const bool precise = a.state != nullptr || (a.s.flags & QUAMBA_FLAG_PRECISE_STATE);
    PrefillPlan plan = prefill_mfma_plan(a.s);
    // A final state that overlaps the initial state (allowed: an update in place) rules the split out: the last
    // segment's workgroups write the final state while those of the first segment may still have to read the initial one.
    const size_t state_bytes = sizeof(float) * (size_t)a.s.batch * a.s.nheads * kP * kN;
    const uintptr_t i0 = reinterpret_cast<uintptr_t>(a.init_state), f0 = reinterpret_cast<uintptr_t>(a.state);
    const bool in_place = a.init_state && a.state && i0 < f0 + state_bytes && f0 < i0 + state_bytes;
    if (plan.nseg > 1 && (in_place || !workspace || reinterpret_cast<uintptr_t>(workspace) % 16 != 0)) {
        // also without a usable workspace (the entry point passes NULL when the caller's is missing or too small)
        const int64_t pairs = (int64_t)a.s.batch * a.s.nheads;
        plan.nseg = 1;
        plan.channel_split = !(a.s.flags & QUAMBA_FLAG_NO_CHANNEL_SPLIT) && pairs <= (int64_t)compute_units();
    }
    auto launch = [&](const SsdArgs &args) {
        if (precise) return plan.channel_split ? launch_scan<true, 1>(args, stream) : launch_scan<true, 2>(args, stream);
        return plan.channel_split ? launch_scan<false, 1>(args, stream) : launch_scan<false, 2>(args, stream);
    };
    a.nseg = 1;
    a.seg_chunks = 0;
    a.seg_state = nullptr;
    a.seg_decay = nullptr;
    // Pacing of the two workgroups of a compute unit (see the kernel) pays when the whole launch is resident at once and
    // most compute units hold two workgroups that each walk many chunks; with more workgroups than that, the early finish
    // of the first arrivals is what lets the rest start, and pacing costs time (measured on 640 pairs).
    const int cus = compute_units();
    auto pace = [&](int segs, int chunks_per_wg) {
        const int64_t wgs = (int64_t)a.s.batch * a.s.nheads * (plan.channel_split ? 2 : 1) * segs;
        return (wgs > cus + cus / 2 && wgs <= 2 * (int64_t)cus && chunks_per_wg >= 8) ? cus : INT_MAX;
    };
    const int nchunks = (a.s.seqlen + kQ - 1) / kQ;
    a.pace_first = pace(1, nchunks);
    if (plan.nseg < 2) return launch(a);

    const size_t pairs = (size_t)a.s.batch * a.s.nheads;
    a.nseg = plan.nseg;
    a.seg_chunks = plan.seg_chunks;
    a.seg_state = static_cast<float *>(workspace);
    a.seg_decay = a.seg_state + (size_t)(plan.nseg - 1) * pairs * kP * kN;
    a.pace_first = pace(plan.nseg, plan.seg_chunks);
    // first kernel: the states at the ends of segments 0 .. nseg-2 (it reads x, B, dt, A and the initial state only)
    hipError_t e;
    if (precise)
        e = plan.channel_split ? launch_segment_state<true, 1>(a, stream) : launch_segment_state<true, 2>(a, stream);
    else
        e = plan.channel_split ? launch_segment_state<false, 1>(a, stream) : launch_segment_state<false, 2>(a, stream);
    if (e != hipSuccess) return e;
    // then every segment with its own workgroups
    return launch(a);
}

}  // namespace quamba
