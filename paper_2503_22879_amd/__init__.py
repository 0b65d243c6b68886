"""MI355X-native 8-bit Mamba2 selective scan (the SSD hot path of Quamba2, arXiv 2503.22879).

A thin ctypes binding over libquamba_ssd.so (C ABI in include/quamba_ssd.h).  Every step of the path runs in the
library's HIP kernels; this package only marshals arguments.  There is no CPU fallback: calls raise if the
library has not been built.
"""
from .binding import (QuambaError, Shape, HostScales, DeviceScales, Gate, load_library, library_path,
                      quamba_ssd_prefill, quamba_ssd_prefill_noalloc, quamba_ssd_prefill_workspace_size,
                      quamba_ssd_decode_step,
                      quamba_ssd_decode_step_q8, quamba_ssd_quantize_state, quamba_state_scales,
                      quamba_hadamard_quantize, quamba_conv1d_q8, quamba_mamba1_scan, quamba_mamba1_decode_step,
                      quamba_reorder_params, quamba_gather_rows, quamba_quantize_x, quamba_quantize_groups,
                      quamba_strerror, FLAG_GENERIC_KERNEL, FLAG_PRECISE_STATE, FLAG_NO_CHANNEL_SPLIT, FLAG_NO_DECAY_SKIP,
                      FLAG_NO_SEQ_SPLIT,
                      EXPORTED_SYMBOLS, quamba_probe_mfma, quamba_probe_stream_rmw, quamba_probe_stream_read,
                      quamba_probe_clock, quamba_probe_clock_xcd)

__all__ = ["QuambaError", "Shape", "HostScales", "DeviceScales", "Gate", "load_library", "library_path",
           "quamba_ssd_prefill", "quamba_ssd_prefill_noalloc", "quamba_ssd_prefill_workspace_size",
           "quamba_ssd_decode_step",
           "quamba_ssd_decode_step_q8", "quamba_ssd_quantize_state", "quamba_state_scales",
           "quamba_hadamard_quantize", "quamba_conv1d_q8", "quamba_mamba1_scan", "quamba_mamba1_decode_step",
           "quamba_reorder_params", "quamba_gather_rows", "quamba_quantize_x", "quamba_quantize_groups",
           "quamba_strerror", "FLAG_GENERIC_KERNEL", "FLAG_PRECISE_STATE", "FLAG_NO_CHANNEL_SPLIT", "FLAG_NO_DECAY_SKIP",
           "FLAG_NO_SEQ_SPLIT",
           "EXPORTED_SYMBOLS", "quamba_probe_mfma", "quamba_probe_stream_rmw", "quamba_probe_stream_read",
           "quamba_probe_clock", "quamba_probe_clock_xcd"]
