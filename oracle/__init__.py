"""TEST INFRASTRUCTURE: the CPU oracle (fp64 sequential scan in C, utilities in numpy).

Only tests, the smoke check and the benchmark's CPU-baseline leg import this package.  It never
imports the HIP package, and the HIP package never imports it.
"""
from .ssd import (Scales, ref_prefill, ref_decode_step, build_oracle, x_scale_table)
from .snc import quantize, sort_and_cluster, group_scales
from .gate import dt_from_codes, silu_gate
from .hadamard import fwht_f32, hadamard_quantize, hadamard_f32, paley_hadamard
from .conv1d import conv1d_silu_f64, ref_conv1d_q8, output_scales
from .mamba1 import ref_mamba1_scan, channel_scales
from .state_q8 import (exp_f32, cell_index_table, state_scales_from_absmax, quantize_state, ref_decode_step_q8)

__all__ = ["Scales", "ref_prefill", "ref_decode_step", "build_oracle", "x_scale_table",
           "quantize", "sort_and_cluster", "group_scales",
           "dt_from_codes", "silu_gate", "fwht_f32", "hadamard_quantize", "hadamard_f32", "paley_hadamard",
           "conv1d_silu_f64", "ref_conv1d_q8", "output_scales", "ref_mamba1_scan", "channel_scales",
           "exp_f32", "cell_index_table", "state_scales_from_absmax", "quantize_state", "ref_decode_step_q8"]
