"""Seeded synthetic Mamba2-shaped SSD inputs (random draws and index gathers only).

This package holds none of the method's arithmetic: no quantizer, no scan, no
clustering.  Both the CPU oracle's tests and the HIP path's harness draw their
raw floating-point tensors from here and then quantize them with their own code.
"""
from .synth import (CONFIGS, LayerShape, draw_layer, draw_decode_step, draw_state,
                    draw_calibration, apply_reorder, draw_cached_state, draw_cached_state_calibration,
                    reorder_state, draw_gate, draw_ssd_output, draw_conv, draw_mamba1,
                    draw_mamba1_gate)

__all__ = ["CONFIGS", "LayerShape", "draw_layer", "draw_decode_step", "draw_state",
           "draw_calibration", "apply_reorder", "draw_cached_state", "draw_cached_state_calibration",
           "reorder_state", "draw_gate", "draw_ssd_output", "draw_conv", "draw_mamba1",
           "draw_mamba1_gate"]
