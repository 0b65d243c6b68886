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
};

// Scale of channel position p of head h from the cluster boundary tables (Section 4.1: m x n scales per group).
// The cluster index is the number of boundaries at or below the position, so all boundary loads are independent
// (three dependent memory round trips in total instead of one per boundary).
__device__ __forceinline__ float x_scale_lookup(const SsdArgs &a, int h, int p)
{
    const int hpg = a.s.nheads / a.s.ngroups;
    const int g = h / hpg, hl = h - g * hpg;
    const int m = a.s.n_head_clusters, n = a.s.n_chan_clusters;
    int i = 0;
    for (int k = 0; k < m - 1; ++k) i += hl >= a.head_cluster_end[g * m + k] ? 1 : 0;
    const int base = (g * m + i) * n;
    int j = 0;
    for (int k = 0; k < n - 1; ++k) j += p >= a.chan_cluster_end[base + k] ? 1 : 0;
    return a.x_scales[base + j];
}

hipError_t launch_decode(const SsdArgs &a, hipStream_t stream);
hipError_t launch_prefill_generic(const SsdArgs &a, hipStream_t stream);
bool prefill_mfma_supports(const quamba_ssd_shape_t &s);
hipError_t launch_prefill_mfma(const SsdArgs &a, hipStream_t stream);
size_t prefill_generic_lds_bytes(const quamba_ssd_shape_t &s);

}  // namespace quamba
