// The C-ABI layer: argument validation (before anything is enqueued) and kernel dispatch.
#include <atomic>
#include <cmath>

#include "quamba_internal.h"

namespace {

constexpr size_t kMaxLdsBytes = 160 * 1024;  // LDS of one gfx950 compute unit

int check_shape(const quamba_ssd_shape_t *s, bool prefill)
{
    if (s->batch <= 0 || s->nheads <= 0 || s->headdim <= 0 || s->d_state <= 0 || s->ngroups <= 0 ||
        s->n_head_clusters <= 0 || s->n_chan_clusters <= 0)
        return QUAMBA_ESHAPE;
    if (s->nheads % s->ngroups) return QUAMBA_ESHAPE;
    if (s->flags & ~(QUAMBA_FLAG_GENERIC_KERNEL | QUAMBA_FLAG_PRECISE_STATE | QUAMBA_FLAG_NO_CHANNEL_SPLIT |
                     QUAMBA_FLAG_NO_DECAY_SKIP | QUAMBA_FLAG_NO_SEQ_SPLIT))
        return QUAMBA_EINVAL;
    if ((int64_t)s->batch * s->nheads > 0x7fffffffLL) return QUAMBA_ESHAPE;
    if (prefill) {
        if (s->seqlen <= 0 || s->chunk <= 0) return QUAMBA_ESHAPE;
    } else if (s->headdim > 16384) {
        return QUAMBA_ESHAPE;
    }
    return QUAMBA_OK;
}

int check_scales(const quamba_ssd_scales_t *sc)
{
    if (!sc || !sc->x_scales || !sc->head_cluster_end || !sc->chan_cluster_end || !sc->B_scales || !sc->C_scales)
        return QUAMBA_ENULL;
    return QUAMBA_OK;
}

quamba::SsdArgs pack(const quamba_ssd_shape_t *s, const quamba_ssd_scales_t *sc, const int8_t *x, const int8_t *B,
                     const int8_t *C, const float *dt, const float *A, const float *D, const float *init,
                     float *state, uint16_t *y)
{
    quamba::SsdArgs a;
    a.s = *s;
    a.x_scales = sc->x_scales;
    a.head_cluster_end = sc->head_cluster_end;
    a.chan_cluster_end = sc->chan_cluster_end;
    a.B_scales = sc->B_scales;
    a.C_scales = sc->C_scales;
    a.x = x; a.B = B; a.C = C; a.dt = dt; a.A = A; a.D = D;
    a.init_state = init;
    a.state = state;
    a.y = y;
    a.z = nullptr; a.z_scale = 0.0f; a.dt_q = nullptr; a.dt_scale = 0.0f; a.dt_bias = nullptr;
    a.nseg = 1; a.seg_chunks = 0; a.seg_state = nullptr; a.seg_decay = nullptr; a.pace_first = 0x7fffffff;
    return a;
}

// Validates the optional side inputs and copies them into the launch arguments.  `dt` may be NULL only when the
// step size comes as codes.
int apply_gate(const quamba_ssd_gate_t *gate, const float *dt, quamba::SsdArgs *a)
{
    if (!gate || !gate->dt_q) {
        if (!dt) return QUAMBA_ENULL;
    } else {
        if (!(gate->dt_scale > 0.0f) || !std::isfinite(gate->dt_scale)) return QUAMBA_EINVAL;
        a->dt_q = gate->dt_q; a->dt_scale = gate->dt_scale; a->dt_bias = gate->dt_bias;
    }
    if (gate && gate->z) {
        if (!(gate->z_scale > 0.0f) || !std::isfinite(gate->z_scale)) return QUAMBA_EINVAL;
        a->z = gate->z; a->z_scale = gate->z_scale;
    }
    return QUAMBA_OK;
}

bool aligned16(const void *p) { return reinterpret_cast<uintptr_t>(p) % 16 == 0; }

// The chunked MFMA kernel moves 16-byte vectors; tensors a caller sliced to an odd offset take the generic kernel.
bool use_mfma(const quamba_ssd_shape_t *s, const void *x, const void *B, const void *C, const void *y,
              const void *init, const void *fin)
{
    return !(s->flags & QUAMBA_FLAG_GENERIC_KERNEL) && quamba::prefill_mfma_supports(*s) && aligned16(x) &&
           aligned16(B) && aligned16(C) && aligned16(y) && aligned16(init) && aligned16(fin);
}

}  // namespace

extern "C" size_t quamba_ssd_prefill_workspace_size(const quamba_ssd_shape_t *shape)
{
    if (!shape || check_shape(shape, true) != QUAMBA_OK) return 0;
    // the generic kernel keeps every intermediate on chip; the matrix-core kernel needs the segment states of a
    // sequence split (short batches only)
    if ((shape->flags & QUAMBA_FLAG_GENERIC_KERNEL) || !quamba::prefill_mfma_supports(*shape)) return 0;
    return quamba::prefill_mfma_workspace_bytes(*shape);
}

extern "C" int quamba_ssd_prefill(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                  const int8_t *x, const int8_t *B, const int8_t *C, const float *dt, const float *A,
                                  const float *D, const float *init_state, uint16_t *y, float *final_state,
                                  void *workspace, size_t workspace_bytes, void *hip_stream)
{
    return quamba_ssd_prefill_gated(shape, scales, nullptr, x, B, C, dt, A, D, init_state, y, final_state, workspace,
                                    workspace_bytes, hip_stream);
}

extern "C" int quamba_ssd_prefill_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                        const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B,
                                        const int8_t *C, const float *dt, const float *A, const float *D,
                                        const float *init_state, uint16_t *y, float *final_state, void *workspace,
                                        size_t workspace_bytes, void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!x || !B || !C || !A || !y) return QUAMBA_ENULL;
    rc = check_shape(shape, true);
    if (rc != QUAMBA_OK) return rc;
    // a workspace that is missing or too small selects the launch that needs none
    const size_t need = quamba_ssd_prefill_workspace_size(shape);
    if (!workspace || workspace_bytes < need) workspace = nullptr;
    const bool mfma = use_mfma(shape, x, B, C, y, init_state, final_state) && (!gate || aligned16(gate->z));
    if (!mfma && quamba::prefill_generic_lds_bytes(*shape) > kMaxLdsBytes) return QUAMBA_ESHAPE;

    quamba::SsdArgs a = pack(shape, scales, x, B, C, dt, A, D, init_state, final_state, y);
    rc = apply_gate(gate, dt, &a);
    if (rc != QUAMBA_OK) return rc;
    hipStream_t stream = static_cast<hipStream_t>(hip_stream);
    const hipError_t e = mfma ? quamba::launch_prefill_mfma(a, workspace, stream)
                              : quamba::launch_prefill_generic(a, stream);
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

namespace {

// Scratch area of quamba_ssd_prefill_noalloc: device memory that belongs to the library's code object, one copy per
// GPU, held until the process ends.  16 MiB covers the sequence split of every shape the matrix-core kernel takes
// (at most 7 * 64 (sequence, head) pairs * (64 * 128 + 1) floats).  In host code the array's name is only a handle:
// the address kernels can use comes from hipGetSymbolAddress, once per device.
constexpr size_t kScratchBytes = (size_t)16 << 20;
static __device__ __align__(256) unsigned char scratch[kScratchBytes];
constexpr int kMaxDevices = 64;
std::atomic<unsigned char *> scratch_address[kMaxDevices];  // zero-initialised; concurrent first calls store the same value

int scratch_of_current_device(unsigned char **out)
{
    int dev = 0;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return QUAMBA_EHIP;
    unsigned char *p = scratch_address[dev].load(std::memory_order_acquire);
    if (!p) {
        void *sym = nullptr;
        if (hipGetSymbolAddress(&sym, HIP_SYMBOL(scratch)) != hipSuccess || !sym) return QUAMBA_EHIP;
        p = static_cast<unsigned char *>(sym);
        scratch_address[dev].store(p, std::memory_order_release);
    }
    *out = p;
    return QUAMBA_OK;
}

}  // namespace

extern "C" int quamba_ssd_prefill_noalloc(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                          const int8_t *x, const int8_t *B, const int8_t *C, const float *dt,
                                          const float *A, const float *D, const float *init_state, uint16_t *y,
                                          float *final_state, void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!x || !B || !C || !dt || !A || !y) return QUAMBA_ENULL;
    rc = check_shape(shape, true);
    if (rc != QUAMBA_OK) return rc;
    const size_t need = quamba_ssd_prefill_workspace_size(shape);
    if (need > kScratchBytes) return QUAMBA_EWORKSPACE;
    unsigned char *ws = nullptr;
    if (need) {
        rc = scratch_of_current_device(&ws);
        if (rc != QUAMBA_OK) return rc;
    }
    return quamba_ssd_prefill_gated(shape, scales, nullptr, x, B, C, dt, A, D, init_state, y, final_state, ws,
                                    need ? kScratchBytes : 0, hip_stream);
}

extern "C" int quamba_ssd_decode_step(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                      const int8_t *x, const int8_t *B, const int8_t *C, const float *dt,
                                      const float *A, const float *D, float *state, uint16_t *y, void *hip_stream)
{
    return quamba_ssd_decode_step_gated(shape, scales, nullptr, x, B, C, dt, A, D, state, y, hip_stream);
}

extern "C" int quamba_ssd_decode_step_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                            const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B,
                                            const int8_t *C, const float *dt, const float *A, const float *D,
                                            float *state, uint16_t *y, void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!x || !B || !C || !A || !state || !y) return QUAMBA_ENULL;
    rc = check_shape(shape, false);
    if (rc != QUAMBA_OK) return rc;
    quamba::SsdArgs a = pack(shape, scales, x, B, C, dt, A, D, nullptr, state, y);
    rc = apply_gate(gate, dt, &a);
    if (rc != QUAMBA_OK) return rc;
    const hipError_t e = quamba::launch_decode(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_ssd_decode_step_q8(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                         const float *state_scales, const int8_t *x, const int8_t *B,
                                         const int8_t *C, const float *dt, const float *A, const float *D,
                                         int8_t *state_q, uint16_t *y, void *hip_stream)
{
    return quamba_ssd_decode_step_q8_gated(shape, scales, nullptr, state_scales, x, B, C, dt, A, D, state_q, y,
                                           hip_stream);
}

extern "C" int quamba_ssd_decode_step_q8_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                               const quamba_ssd_gate_t *gate, const float *state_scales,
                                               const int8_t *x, const int8_t *B, const int8_t *C, const float *dt,
                                               const float *A, const float *D, int8_t *state_q, uint16_t *y,
                                               void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    if (gate && gate->dt_q) return QUAMBA_EINVAL;  // the re-quantization decision is defined on the fp32 dt
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!state_scales || !x || !B || !C || !dt || !A || !state_q || !y) return QUAMBA_ENULL;
    rc = check_shape(shape, false);
    if (rc != QUAMBA_OK) return rc;
    if (quamba::decode_q8_lds_bytes(*shape) > kMaxLdsBytes) return QUAMBA_ESHAPE;
    quamba::SsdArgs a = pack(shape, scales, x, B, C, dt, A, D, nullptr, nullptr, y);
    rc = apply_gate(gate, dt, &a);
    if (rc != QUAMBA_OK) return rc;
    const hipError_t e = quamba::launch_decode_q8(a, state_scales, state_q, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_ssd_quantize_state(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                         const float *state_scales, const float *state, int8_t *state_q,
                                         void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!state_scales || !state || !state_q) return QUAMBA_ENULL;
    rc = check_shape(shape, false);
    if (rc != QUAMBA_OK) return rc;
    if (quamba::decode_q8_lds_bytes(*shape) > kMaxLdsBytes) return QUAMBA_ESHAPE;
    const quamba::SsdArgs a = pack(shape, scales, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                   const_cast<float *>(state), nullptr);
    const hipError_t e = quamba::launch_quantize_state(a, state_scales, state_q, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

namespace {
int check_mamba1(const quamba_ssd_shape_t *s, bool scan)
{
    const int rc = check_shape(s, scan);
    if (rc != QUAMBA_OK) return rc;
    if (s->nheads != 1 || s->ngroups != 1 || s->n_head_clusters != 1) return QUAMBA_ESHAPE;
    if ((int64_t)s->batch * s->headdim > 0x7fffffffLL || s->batch > 65535) return QUAMBA_ESHAPE;
    return QUAMBA_OK;
}
}  // namespace

extern "C" int quamba_mamba1_scan(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *x,
                                  const int8_t *B, const int8_t *C, const float *dt, const float *A, const float *D,
                                  const float *init_state, uint16_t *y, float *final_state, void *hip_stream)
{
    return quamba_mamba1_scan_gated(shape, scales, nullptr, x, B, C, dt, A, D, init_state, y, final_state, hip_stream);
}

extern "C" int quamba_mamba1_scan_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                        const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B,
                                        const int8_t *C, const float *dt, const float *A, const float *D,
                                        const float *init_state, uint16_t *y, float *final_state, void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!x || !B || !C || !A || !y) return QUAMBA_ENULL;
    rc = check_mamba1(shape, true);
    if (rc != QUAMBA_OK) return rc;
    if (shape->flags & ~QUAMBA_FLAG_GENERIC_KERNEL) return QUAMBA_EINVAL;
    if (!quamba::mamba1_scan_supports_any(*shape)) return QUAMBA_ESHAPE;  // d_state <= 64
    quamba::SsdArgs a = pack(shape, scales, x, B, C, dt, nullptr, D, nullptr, nullptr, y);
    rc = apply_gate(gate, dt, &a);
    if (rc != QUAMBA_OK) return rc;
    const hipError_t e = quamba::launch_mamba1_scan(a, A, init_state, final_state, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_mamba1_decode_step(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                         const int8_t *x, const int8_t *B, const int8_t *C, const float *dt,
                                         const float *A, const float *D, float *state, uint16_t *y, void *hip_stream)
{
    return quamba_mamba1_decode_step_gated(shape, scales, nullptr, x, B, C, dt, A, D, state, y, hip_stream);
}

extern "C" int quamba_mamba1_decode_step_gated(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales,
                                               const quamba_ssd_gate_t *gate, const int8_t *x, const int8_t *B,
                                               const int8_t *C, const float *dt, const float *A, const float *D,
                                               float *state, uint16_t *y, void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!x || !B || !C || !A || !state || !y) return QUAMBA_ENULL;
    rc = check_mamba1(shape, false);
    if (rc != QUAMBA_OK) return rc;
    if (shape->flags) return QUAMBA_EINVAL;
    quamba::SsdArgs a = pack(shape, scales, x, B, C, dt, nullptr, D, nullptr, state, y);
    rc = apply_gate(gate, dt, &a);
    if (rc != QUAMBA_OK) return rc;
    const hipError_t e = quamba::launch_mamba1_decode(a, A, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_conv1d_q8(const quamba_ssd_shape_t *shape, const quamba_ssd_scales_t *scales, const int8_t *in,
                                const int8_t *weight, const float *bias, float in_w_scale,
                                const int8_t *conv_state_in, int8_t *x_out, int8_t *B_out, int8_t *C_out,
                                int8_t *conv_state_out, void *hip_stream)
{
    if (!shape) return QUAMBA_ENULL;
    int rc = check_scales(scales);
    if (rc != QUAMBA_OK) return rc;
    if (!in || !weight || !x_out || !B_out || !C_out) return QUAMBA_ENULL;
    rc = check_shape(shape, true);
    if (rc != QUAMBA_OK) return rc;
    const int64_t Ct = (int64_t)shape->nheads * shape->headdim + 2LL * shape->ngroups * shape->d_state;
    if (Ct > 0x7fffffffLL / 4 || shape->batch > 65535 || quamba::conv1d_segments(*shape) > 65535) return QUAMBA_ESHAPE;
    if (!(in_w_scale > 0.0f) || !std::isfinite(in_w_scale)) return QUAMBA_EINVAL;
    if (conv_state_in && conv_state_in == conv_state_out && shape->seqlen > 16) return QUAMBA_EINVAL;
    quamba::ConvArgs a;
    a.s = *shape;
    a.x_scales = scales->x_scales; a.head_cluster_end = scales->head_cluster_end;
    a.chan_cluster_end = scales->chan_cluster_end; a.B_scales = scales->B_scales; a.C_scales = scales->C_scales;
    a.in = in; a.weight = weight; a.bias = bias; a.in_w_scale = in_w_scale;
    a.state_in = conv_state_in; a.state_out = conv_state_out;
    a.x_out = x_out; a.B_out = B_out; a.C_out = C_out; a.seg = 0;
    const hipError_t e = quamba::launch_conv1d_q8(a, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" int quamba_hadamard_quantize(const uint16_t *y, int64_t rows, int32_t n, float s_y, int8_t *out,
                                        void *hip_stream)
{
    if (!y || !out) return QUAMBA_ENULL;
    if (!quamba::hadamard_order_supported(n) || rows < 0 || rows > 0x7fffffffLL) return QUAMBA_ESHAPE;
    if (!(s_y > 0.0f) || !std::isfinite(s_y)) return QUAMBA_EINVAL;
    const hipError_t e = quamba::launch_hadamard_quantize(y, rows, n, s_y, out, static_cast<hipStream_t>(hip_stream));
    return e == hipSuccess ? QUAMBA_OK : QUAMBA_EHIP;
}

extern "C" const char *quamba_strerror(int status)
{
    switch (status) {
        case QUAMBA_OK: return "ok";
        case QUAMBA_ENULL: return "a required pointer is NULL";
        case QUAMBA_ESHAPE: return "a dimension is non-positive, inconsistent or unsupported";
        case QUAMBA_EWORKSPACE: return "workspace too small";
        case QUAMBA_EHIP: return "the HIP runtime refused the launch";
        case QUAMBA_EINVAL: return "invalid argument value";
        default: return "unknown status";
    }
}
