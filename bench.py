#!/usr/bin/env python3
"""Benchmark of the 8-bit SSD hot path on one MI355X.

    python bench.py [--gpus 1] [--steps K] [--warmup W] [--workload m2_8b_b4] [--no-cpu]

A "step" is one pass of the hot path over one batch of synthetic input: one chunked prefill of the
Mamba2-8B-shaped layer (batch 4 x 4096 tokens, 128 heads x 64, d_state 128, 8 state groups, chunk 256).  The
decode state update (batch 256, 1 GiB fp32 state) is timed in the same run, K steps as well, and reported in the
"decode" object.  Inputs are seeded synthetic tensors, resident in HBM before the timed regions; the offline
sort-and-cluster and the quantizer run through the library's own host entry points.  The fp64 CPU oracle is
timed on a bounded sample of the same workload for the "cpu_baseline" object (and doubles as a parity spot check).

Prints ONE JSON line.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

import workloads as W  # noqa: E402

HBM_PEAK_GBS = 8000.0        # MI355X HBM3E
MFMA_F16_PEAK_TFLOPS = 2500.0  # dense fp16/bf16
MFMA_I8_PEAK_TOPS = 5000.0     # dense int8
KERNEL_CHUNK = 128             # tokens per chunk of prefill_mfma_kernel (the caller's `chunk` does not change the result)

# HBM traffic per launch measured with rocprofv3 --pmc (FETCH_SIZE, WRITE_SIZE, each scaled by its reading for a plain
# 256 MiB device copy in the same run: factors 1.9998 and 1.0000).  These are constants taken from the committed
# profile summaries, not measurements of this run: `traffic_source` in every roofline object names the file.
# None for workloads that were not profiled.
MEASURED_TRAFFIC_BYTES = {"m2_8b_b4": 496.4e6, "m2_8b_decode": 2162.3e6, "m2_8b_decode_q8": 550.9e6,
                          "m2_8b_b4_hadamard": 402.7e6, "m2_8b_b4_conv1d": 352.1e6,
                          "mamba1_2p8b_scan": 599.1e6, "mamba1_2p8b_decode": 178.8e6}
TRAFFIC_SOURCE = {
    "m2_8b_b4": "profiles/hbm_traffic_prefill_m2_8b_b4_and_decode_m2_8b.txt",
    "m2_8b_decode": "profiles/hbm_traffic_prefill_m2_8b_b4_and_decode_m2_8b.txt",
    "m2_8b_decode_q8": "profiles/hbm_traffic_prefill_m2_8b_b4_and_decode_m2_8b.txt",
    "m2_8b_b4_hadamard": "profiles/hbm_traffic_hadamard_conv1d_m2_8b_b4_and_mamba1_2p8b.txt",
    "m2_8b_b4_conv1d": "profiles/hbm_traffic_hadamard_conv1d_m2_8b_b4_and_mamba1_2p8b.txt",
    "mamba1_2p8b_scan": "profiles/hbm_traffic_hadamard_conv1d_m2_8b_b4_and_mamba1_2p8b.txt",
    "mamba1_2p8b_decode": "profiles/hbm_traffic_hadamard_conv1d_m2_8b_b4_and_mamba1_2p8b.txt"}


def traffic_fields(key):
    """`traffic` (bytes per launch from the committed rocprofv3 counter summary, a constant of that earlier run on
    another box) and where it comes from; both None when the workload was not profiled."""
    return {"traffic": MEASURED_TRAFFIC_BYTES.get(key),
            "traffic_source": (TRAFFIC_SOURCE[key] + " (rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE of an earlier run of "
                               "the same command, not measured in this run)") if key in TRAFFIC_SOURCE else None}


def prefill_algorithmic(s: W.LayerShape, chunk=None):
    """Algorithmic work per token per layer: causal lower triangle only, nothing for padding or recomputation.
    chunk: the chunk length the intra-chunk products are priced at (default: the workload's own)."""
    H, P, N, G = s.nheads, s.headdim, s.d_state, s.ngroups
    Q = s.chunk if chunk is None else chunk
    f16_macs = H * ((Q + 1) / 2 * P + 2 * N * P)
    i8_macs = G * (Q + 1) / 2 * N
    nbytes = H * P + 2 * G * N + 4 * H + 2 * H * P
    return f16_macs, i8_macs, nbytes


def prefill_executed(s: W.LayerShape):
    """Multiply-adds per token per layer that prefill_mfma_kernel issues to the matrix cores: 128-token chunks of four
    32-token blocks, whole 32 x 32 tiles on and below the diagonal (10 per chunk, the masked half of the 4 diagonal
    ones included), the score tiles recomputed per head.  Agrees with SQ_INSTS_VALU_MFMA_MOPS_F16 / _I8 of the
    committed counter profile (9.02e10 flop and 4.29e10 op per launch of the 8B-shaped batch of 4)."""
    H, P, N = s.nheads, s.headdim, s.d_state
    tiles_per_token = 10.0 / KERNEL_CHUNK
    f16_macs = H * (tiles_per_token * 32 * 32 * P + 2 * N * P)
    i8_macs = H * tiles_per_token * 32 * 32 * N
    return f16_macs, i8_macs


# Arithmetic the 8-bit-state step must do per state element, one vector operation each: code -> float, times the
# decayed scale, B-dot times x, add, times C into y (one fused multiply-add), times 1/scale, clamp, round-and-pack: 8.
Q8_OPS_PER_ELEMENT = 8
ALU_PEAK_TOPS = 256 * 4 * 16 * 2.4e9 / 1e12   # 39.3: fp32 vector issue slots per second x 64 lanes, unpacked, unfused

# Vector issue slots the METHOD needs per element (what `roofline` with bound "alu" prices; a transcendental takes a
# quarter-rate instruction = 4 slots), from the definitions, not from what the kernels execute:
#   Mamba1 scan, per (token, channel, state), Eq. 2 with the Mamba1 parameterisation of Section 3.2: dt * A (1),
#   its exponential (4), (dt x) * B (1; dt x is shared by the states), h = a h + u (1 fused), y += C h (1 fused).
MAMBA1_MIN_SLOTS = 8.0
#   W8A8 convolution + SiLU + Eq. 1, per output element: the 4-tap window (1 byte permute) and its exact integer dot
#   product (1), to float (1), times the scale plus bias (1 fused), exp (4), 1 + e (1), reciprocal (4), v * sigmoid (1),
#   times 1 / s_out (1), clamp (1), round and pack (1).
CONV_MIN_SLOTS = 17.0
# Executed vector instructions per element by the counters (rocprofv3 SQ_INSTS_VALU x 64 / elements), for information:
MAMBA1_EXECUTED_PER_ELEMENT = 8.9   # of which 1.06 quarter-rate exponentials
CONV_EXECUTED_PER_ELEMENT = 19.6    # 18.3 in the main loop (two quarter-rate), set-up and the exact-sequence reruns
SPIN_UP_MS = float(os.environ.get("QUAMBA_BENCH_SPIN_UP_MS", "80"))   # untimed device work in front of every timed region, after the W warm-up launches (see time_region)


def HADAMARD_OPS_PER_VALUE(n: int) -> int:
    """fp32 vector operations per value of the quantized Hadamard transform: one add or subtract per butterfly stage,
    then the scale, the clamp and the rounding add of Eq. 1."""
    return n.bit_length() - 1 + 3


def decode_bytes(s: W.LayerShape, state_bytes: int = 4) -> float:
    b, H, P, N, G = s.batch, s.nheads, s.headdim, s.d_state, s.ngroups
    return float(2 * state_bytes * b * H * P * N + b * H * P + 2 * b * G * N + 4 * b * H + 2 * b * H * P)


def build_problem(q, s: W.LayerShape, seed: int):
    """Quantized inputs in sorted/clustered order, made with the library's own offline entry points."""
    xmax, bmax, cmax = W.draw_calibration(s, seed, tokens=2048)
    head_perm, chan_perm, hs = q.quamba_reorder_params(s.nheads, s.headdim, s.ngroups, s.m, s.n, s.d_state,
                                                       xmax, bmax, cmax)
    shape = q.Shape(batch=s.batch, seqlen=s.seqlen, nheads=s.nheads, headdim=s.headdim, d_state=s.d_state,
                    ngroups=s.ngroups, chunk=s.chunk, n_head_clusters=s.m, n_chan_clusters=s.n, flags=0)
    return shape, hs, head_perm, chan_perm


def quantize_layer(q, shape, hs, raw):
    return {"x": q.quamba_quantize_x(shape, hs, raw["x"]),
            "B": q.quamba_quantize_groups(raw["B"], hs.B_scales),
            "C": q.quamba_quantize_groups(raw["C"], hs.C_scales),
            "dt": np.ascontiguousarray(raw["dt"], np.float32)}


# After the prefill leg's timed region (with --power: after every leg's) the same call is repeated for POWER_SECONDS
# and the board power sensor (hwmon power1_input, microwatts; a slow average, hence the long run) is sampled over the
# second half; --no-power skips it.  A kernel that sits on the board's power cap runs as fast as its energy allows.
POWER_SECONDS = 2.0
POWER_ALL_LEGS = False   # by default only the prefill leg (the headline kernel) is sampled
BOARD_POWER_W = {}


def _hwmon(name):
    import glob
    for path in sorted(glob.glob("/sys/class/drm/card*/device/hwmon/hwmon*/" + name)):
        try:
            with open(path) as f:
                return float(f.read().strip()) * 1e-6
        except (OSError, ValueError):
            continue
    return None


def sample_board_power(torch, fn, key):
    """Mean and maximum board power (W) while fn runs back to back, or None when the sensor cannot be read."""
    if _hwmon("power1_input") is None:
        BOARD_POWER_W[key] = None
        return
    t0 = time.perf_counter()
    vals = []
    while time.perf_counter() - t0 < POWER_SECONDS:
        for _ in range(50):
            fn()
        torch.cuda.synchronize()
        if time.perf_counter() - t0 > 0.5 * POWER_SECONDS:
            vals.append(_hwmon("power1_input"))
    vals = [v for v in vals if v is not None]
    # the same call timed at the end of these POWER_SECONDS of uninterrupted launches: the sustained figure
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    ev0.record()
    for _ in range(100):
        fn()
    ev1.record()
    torch.cuda.synchronize()
    BOARD_POWER_W[key] = {"mean": sum(vals) / len(vals), "max": max(vals),
                          "sustained_ms_per_call": ev0.elapsed_time(ev1) / 100,
                          "note": "sustained_ms_per_call: 100 calls timed after %.0f s of uninterrupted launches"
                                  % POWER_SECONDS} if vals else None


def time_region(torch, fn, steps, warmup, min_warm_ms=0.0, power_key=None, after=None):
    """Mean ms per call over `steps` calls on torch's current stream (the stream the kernels are launched on),
    bracketed by device synchronisation; HIP events give the device-side duration.  With min_warm_ms the untimed
    warm-up is continued until that much wall time has gone by: after seconds of host-side preparation the first tens
    of milliseconds of device work run up to 1.5x slower (measured on the decode legs), which a handful of warm-up
    launches does not cover.  `after` is called right behind the last timed launch, after the closing event (the clock
    probe goes there)."""
    for _ in range(warmup):
        fn()
    torch.cuda.synchronize()
    t_w = time.perf_counter()
    while (time.perf_counter() - t_w) * 1e3 < min_warm_ms:
        for _ in range(8):
            fn()
        torch.cuda.synchronize()
    ev0 = torch.cuda.Event(enable_timing=True)
    ev1 = torch.cuda.Event(enable_timing=True)
    t0 = time.perf_counter()
    ev0.record()
    for _ in range(steps):
        fn()
    ev1.record()
    if after is not None:
        after()
    torch.cuda.synchronize()
    wall_ms = (time.perf_counter() - t0) * 1e3
    if POWER_SECONDS > 0 and power_key and (POWER_ALL_LEGS or power_key == "prefill"):
        sample_board_power(torch, fn, power_key)
    return ev0.elapsed_time(ev1) / steps, wall_ms / steps


def measure_attainable(q, torch, dev, big):
    """What this machine sustains for the resources the rooflines are priced against, measured in this run with the
    library's probe kernels (include/quamba_probe.h): a register-resident matrix-core loop in fp16 and int8, and an
    in-place read-modify-write stream over `big` (a device buffer of >= 256 MiB that the legs overwrite later)."""
    sink = torch.zeros(4, dtype=torch.int32, device=dev)
    res = {}
    for kind, uniform, key, unit in ((0, False, "mfma_f16", "TFLOP/s"), (1, False, "mfma_i8", "TOP/s"),
                                     (0, True, "mfma_f16_uniform_operands", "TFLOP/s"),
                                     (1, True, "mfma_i8_uniform_operands", "TOP/s")):
        ops = [0.0]

        def run(kind=kind, uniform=uniform, ops=ops):
            ops[0] = q.quamba_probe_mfma(kind, 4000, sink, uniform_operands=uniform)
        ms, _ = time_region(torch, run, 10, 2, min_warm_ms=40.0)
        res[key] = {"value": ops[0] / (ms * 1e-3) / 1e12, "unit": unit, "ms_per_launch": ms,
                    "shader_clock_mhz": shader_clock_under_load(q, torch, dev, run, launches=12)}
    moved = [0]

    def rmw():
        moved[0] = q.quamba_probe_stream_rmw(big)
    ms, _ = time_region(torch, rmw, 10, 2, min_warm_ms=40.0)
    res["hbm_stream_rmw"] = {"value": moved[0] / (ms * 1e-3) / 1e9, "unit": "GB/s", "bytes_per_launch": moved[0],
                             "ms_per_launch": ms}
    def rd():
        moved[0] = q.quamba_probe_stream_read(big, sink)
    ms, _ = time_region(torch, rd, 10, 2, min_warm_ms=40.0)
    res["hbm_stream_read"] = {"value": moved[0] / (ms * 1e-3) / 1e9, "unit": "GB/s", "bytes_per_launch": moved[0],
                              "ms_per_launch": ms,
                              "note": "reads alone: the ceiling of a kernel that reads more than it writes (the Hadamard "
                                      "transform reads 2 bytes per byte it writes)"}
    res["note"] = ("measured in this run by small kernels of the same library: 4 independent 32x32 MFMA chains per wave, "
                   "2 waves per SIMD, operands in registers -- with operands that differ from lane to lane (mfma_f16, "
                   "mfma_i8: what a real contraction can sustain; the board reaches its power cap and lowers the clock) "
                   "and with the same operand values in every lane (*_uniform_operands: little switching, full clock, "
                   "near the published peak); one in-place pass of 16-byte non-temporal loads and stores over %d MiB"
                   % (big.numel() * big.element_size() >> 20))
    return res


def shader_clock_under_load(q, torch, dev, fn, launches=60):
    """Shader clock in MHz while fn runs back to back: `launches` calls are enqueued on the current stream and the
    library's clock probe (one wave spinning for about 200 us between two readings of the shader-clock counter and of
    the constant 100 MHz counter) on a second stream of the same priority; it takes a wave slot as soon as one opens
    and so samples the clock the power management holds the chip at under this load.  A probe that runs alone behind
    the launches would read the idle clock again: the clock recovers within microseconds."""
    out = torch.zeros(2, dtype=torch.int64, device=dev)
    side = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    for _ in range(launches // 3):
        fn()
    with torch.cuda.stream(side):
        q.quamba_probe_clock(out, 100000, stream=side)
    for _ in range(launches - launches // 3):
        fn()
    torch.cuda.synchronize()
    v = out.cpu().numpy()
    return float(v[0]) / float(v[1]) * 100.0 if v[1] > 0 else None


def xcd_clocks_under_load(q, torch, dev, fn, launches=60):
    """Shader clock per XCD in MHz while fn runs back to back (see shader_clock_under_load): eight one-wave workgroups,
    which the hardware deals out to the eight XCDs in turn.  Returns a list indexed by the XCD id each wave read back,
    or None where a wave did not report."""
    out = torch.full((8, 3), -1, dtype=torch.int64, device=dev)
    side = torch.cuda.Stream(device=dev)
    torch.cuda.synchronize()
    for _ in range(launches // 3):
        fn()
    with torch.cuda.stream(side):
        q.quamba_probe_clock_xcd(out, 100000, stream=side)
    for _ in range(launches - launches // 3):
        fn()
    torch.cuda.synchronize()
    v = out.cpu().numpy()
    res = [None] * 8
    for cyc, ticks, xcd in v:
        if ticks > 0 and 0 <= xcd < 8:
            res[int(xcd)] = round(float(cyc) / float(ticks) * 100.0, 1)
    return res


def prefill_leg(q, torch, dev, s, seed, steps, warmup, args, headline):
    """One prefill workload: inputs made with the library's offline entry points, K timed launches on rotating input
    and output sets (the second set is the first rolled by one sequence, or by 1024 tokens for a single sequence, so
    that consecutive launches touch different memory and the sets together exceed the 256 MB last-level cache), the
    rooflines, and -- for the headline workload -- the untimed-spin-up protocol's cold figure, the default-skip leg
    and the shader clock.  Returns (result dict, context for the later legs)."""
    shape, hs, head_perm, chan_perm = build_problem(q, s, seed)
    raw = W.apply_reorder(W.draw_layer(s, seed), head_perm, chan_perm)
    prob = quantize_layer(q, shape, hs, raw)
    A_np, D_np = raw["A"], raw["D"]
    del raw
    dsc = q.DeviceScales(hs, dev)
    t0 = {k: torch.from_numpy(v).to(dev) for k, v in prob.items()}
    roll = (1, 0) if s.batch > 1 else (1024, 1)
    sets = [t0, {k: torch.roll(v, roll[0], roll[1]).contiguous() for k, v in t0.items()}]
    A = torch.from_numpy(A_np).to(dev)
    D = torch.from_numpy(D_np).to(dev)
    ys = [torch.empty((s.batch, s.seqlen, s.nheads, s.headdim), dtype=torch.float16, device=dev) for _ in sets]
    fin = torch.empty((s.batch, s.nheads, s.headdim, s.d_state), device=dev) if args.precise_state else None
    ws_need = q.quamba_ssd_prefill_workspace_size(shape)
    ws = torch.empty(max(16, ws_need), dtype=torch.uint8, device=dev)

    gate = None
    if args.gated and headline:  # side inputs quantized with the library's host Eq. 1 entry point, one static scale per tensor
        rawg = W.draw_gate(s, seed)
        zr = np.take(rawg["z"], head_perm, axis=-2)
        zr = np.take_along_axis(zr, np.broadcast_to(chan_perm, zr.shape), axis=-1)
        zs = np.float32(np.abs(zr).max() / 127.0)
        ds = np.float32(np.abs(rawg["dt_pre"]).max() / 127.0)
        zq = q.quamba_quantize_groups(zr.reshape(-1, 1, s.nheads * s.headdim), np.array([zs], np.float32))
        dq = q.quamba_quantize_groups(np.take(rawg["dt_pre"], head_perm, axis=-1).reshape(-1, 1, s.nheads),
                                      np.array([ds], np.float32))
        gate = q.Gate(z=torch.from_numpy(zq.reshape(zr.shape)).to(dev), z_scale=float(zs),
                      dt_q=torch.from_numpy(dq.reshape(s.batch, s.seqlen, s.nheads)).to(dev), dt_scale=float(ds),
                      dt_bias=torch.from_numpy(np.ascontiguousarray(rawg["dt_bias"][head_perm])).to(dev))
        del rawg, zr, zq, dq

    # The headline figure is timed with QUAMBA_FLAG_NO_DECAY_SKIP: every product of the scan is computed.  The
    # library's default leaves out 32-token blocks whose decay factor is below 2^-32; that launch is timed right after
    # and reported beside it (`prefill_decay_skip`), never as `value`.
    shape_dense = q.Shape.from_buffer_copy(shape)
    shape_dense.flags |= q.FLAG_NO_DECAY_SKIP
    counter = [0]

    def launch(sh):
        i = counter[0] % len(sets) if gate is None else 0   # the side inputs exist for the first set only
        counter[0] += 1
        t = sets[i]
        q.quamba_ssd_prefill(sh, dsc, t["x"], t["B"], t["C"], t["dt"], A, D, None, ys[i], fin, ws, gate=gate)

    def prefill():
        launch(shape_dense)

    def prefill_skip():
        launch(shape)

    side_legs = headline and not args.lean
    cold_ms = None
    if side_legs:   # the timed region without the spin-up: W warm-up launches, then K timed ones, right after the host-side preparation
        cold_ms, _ = time_region(torch, prefill, steps, warmup)
    ms, wall_ms = time_region(torch, prefill, steps, warmup, min_warm_ms=SPIN_UP_MS,
                              power_key="prefill" if headline else None)
    clock_mhz = shader_clock_under_load(q, torch, dev, prefill) if side_legs else None
    xcd_mhz = xcd_clocks_under_load(q, torch, dev, prefill) if side_legs else None
    ms_skip = None
    if side_legs and not args.no_decay_skip_leg:
        ms_skip, _ = time_region(torch, prefill_skip, steps, warmup, min_warm_ms=SPIN_UP_MS)
    # The same launches with every x, B and C code zero: the instruction stream, the addresses and the bytes moved are
    # the same (nothing in the kernel branches on a code), only the operand bits stop toggling.  A duration that follows
    # the operand values shows a kernel held by the board's power limit, not by an execution unit.
    zero_codes = None
    if side_legs and gate is None:
        kept = [{k: t[k] for k in ("x", "B", "C")} for t in sets]
        for t in sets:
            for k in ("x", "B", "C"):
                t[k] = torch.zeros_like(t[k])
        ms_zero, _ = time_region(torch, prefill, steps, warmup, min_warm_ms=SPIN_UP_MS)
        zero_codes = {"ms_per_step": ms_zero, "shader_clock_mhz": shader_clock_under_load(q, torch, dev, prefill),
                      "note": "same launches on all-zero x, B and C codes: identical instructions, addresses and "
                              "traffic; the duration differs through the power the operands' bit changes draw"}
        for t, k3 in zip(sets, kept):
            t.update(k3)
    tokens = s.batch * s.seqlen
    f16_macs, i8_macs, bytes_tok = prefill_algorithmic(s)
    k16, k8, _ = prefill_algorithmic(s, KERNEL_CHUNK)
    x16, x8 = prefill_executed(s)
    w8 = MFMA_F16_PEAK_TFLOPS / MFMA_I8_PEAK_TOPS

    def tfl(m16, m8):
        return tokens * (2 * m16 + 2 * m8 * w8) / (ms * 1e-3) / 1e12
    tflops = tfl(f16_macs, i8_macs)
    gbs = tokens * bytes_tok / (ms * 1e-3) / 1e9
    key = s.name
    res = {
        "ms_per_step": ms, "wall_ms_per_step": wall_ms, "value": tokens / (ms * 1e-3), "unit": "tokens/s",
        "input_sets": len(sets) if gate is None else 1,
        "bytes_per_input_and_output_set": int(sum(v.numel() * v.element_size() for v in t0.values()) +
                                              ys[0].numel() * 2),
        "shader_clock_mhz": clock_mhz,
        "shader_clock_mhz_per_xcd": xcd_mhz,
        # batches too short to fill the chip are cut along the sequence (two launches: a state pass over all but the last
        # segment, then one set of workgroups per segment); the workspace holds the segment states
        "sequence_split": {"workspace_bytes": int(ws_need),
                           "segments": int(ws_need // (4 * s.batch * s.nheads * (s.headdim * s.d_state + 1))) + 1},
        "roofline": dict({"kernel": "prefill_mfma_kernel", "bound": "mfma", "achieved": tflops,
                          "peak": MFMA_F16_PEAK_TFLOPS, "unit": "TFLOP/s", "frac": tflops / MFMA_F16_PEAK_TFLOPS,
                          "frac_at_kernel_chunk": tfl(k16, k8) / MFMA_F16_PEAK_TFLOPS,
                          "executed": {"fp16_flop": 2 * x16 * tokens, "int8_op": 2 * x8 * tokens,
                                       "frac_of_peak": tfl(x16, x8) / MFMA_F16_PEAK_TFLOPS,
                                       "note": "what the kernel issues: 128-token chunks, whole diagonal tiles, score "
                                               "tiles per head (matches the MFMA op counters of the committed profile)"},
                          "algorithmic": {"fp16_flop": 2 * f16_macs * tokens, "int8_op": 2 * i8_macs * tokens,
                                          "chunk": s.chunk, "bytes": tokens * bytes_tok},
                          "note": "frac prices the algorithmic causal MACs at the workload's chunk (%d); "
                                  "frac_at_kernel_chunk the same formula at the kernel's own chunk of %d tokens (fewer "
                                  "intra-chunk products); int8 MACs weighted by the fp16/int8 peak ratio"
                                  % (s.chunk, KERNEL_CHUNK)}, **traffic_fields(key)),
        "roofline_hbm": dict({"kernel": "prefill_mfma_kernel", "bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS,
                              "unit": "GB/s", "frac": gbs / HBM_PEAK_GBS}, **traffic_fields(key)),
    }
    if cold_ms is not None:
        res["cold_ms_per_step"] = cold_ms
    if zero_codes is not None:
        res["zero_codes"] = zero_codes
    if headline:
        res["prefill_decay_skip"] = None if ms_skip is None else {
            "ms_per_step": ms_skip, "value": tokens / (ms_skip * 1e-3), "unit": "tokens/s",
            "note": "library default: blocks whose decay factor is below 2^-32 are left out; the headline value "
                    "computes them all"}
    ctx = dict(shape=shape, hs=hs, head_perm=head_perm, chan_perm=chan_perm, prob=prob, A_np=A_np, D_np=D_np,
               dsc=dsc, sets=sets, ys=ys, A=A, D=D, fin=fin, ws=ws, shape_dense=shape_dense)
    return res, ctx


def main() -> int:
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=100)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--workload", default="m2_8b_b4", choices=["m2_8b_b4", "m2_8b_b1", "m2_2p7b", "m2_130m"])
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU-oracle baseline leg")
    ap.add_argument("--no-decode", action="store_true", help="skip the decode leg")
    ap.add_argument("--no-mamba1", action="store_true", help="skip the Mamba1 selective scan and its decode step")
    ap.add_argument("--no-conv", action="store_true", help="skip the W8A8 causal convolution in front of the scan")
    ap.add_argument("--no-hadamard", action="store_true",
                    help="skip the quantized Hadamard transform of the prefill output")
    ap.add_argument("--power", action="store_true",
                    help="report the board power (hwmon sensor, 2 more seconds of launches) of every leg, not only of "
                         "the prefill")
    ap.add_argument("--no-power", action="store_true", help="do not sample the board power at all")
    ap.add_argument("--lean", action="store_true",
                    help="time the headline prefill alone: no cold figure, no default-skip leg, no zero-code leg, no "
                         "clock probe (for runs under a profiler, whose kernel statistics then cover these launches only)")
    ap.add_argument("--no-attainable", action="store_true", help="skip the probe kernels that measure attainable peaks")
    ap.add_argument("--no-other-configs", action="store_true",
                    help="skip the legs of the other prefill configurations (8B at batch 1, 2.7B, 130M)")
    ap.add_argument("--no-decay-skip-leg", action="store_true",
                    help="skip the second prefill region (the library's default with the dead-block skip); counter "
                         "profiles use it so that every prefill launch of the run is the headline one")
    ap.add_argument("--precise-state", action="store_true", help="also return the final fp32 state (two-term state path)")
    ap.add_argument("--gated", action="store_true",
                    help="prefill through quamba_ssd_prefill_gated: int8 gate z and int8 step-size codes (not the "
                         "headline configuration; config.side_inputs says so)")
    ap.add_argument("--copy-calibration", action="store_true",
                    help="also run a plain device copy of 256 MiB three times (read 256 MiB + write 256 MiB each): the "
                         "known-size kernel that scales rocprofv3's FETCH_SIZE / WRITE_SIZE readings")
    args = ap.parse_args()
    if args.gpus != 1:
        print("bench.py: this build runs on ONE GPU; --gpus %d is not supported (the path shards by sequence or by "
              "state group with no exchange between devices)" % args.gpus, file=sys.stderr)
        return 2

    global POWER_SECONDS, POWER_ALL_LEGS
    POWER_ALL_LEGS = args.power
    if args.no_power:
        POWER_SECONDS = 0.0
    import torch
    import paper_2503_22879_amd as q
    q.load_library()
    assert torch.cuda.is_available(), "bench.py needs the GPU"
    dev = torch.device("cuda:0")
    seed = 3
    # The decode legs' state buffers are allocated first, while the process's device address space is still empty: the
    # same kernels ran up to 1.5x (fp32 state) and 3x (int8 state) slower on buffers allocated after the other legs had
    # allocated and freed theirs (the allocation's physical backing, not the kernel, differs).
    sd0 = W.CONFIGS["m2_8b_decode"]
    state_buf = qstate_buf = None
    if not args.no_decode:
        state_buf = torch.empty((sd0.batch, sd0.nheads, sd0.headdim, sd0.d_state), device=dev)
        qstate_buf = torch.empty((sd0.batch, sd0.nheads, sd0.headdim, sd0.d_state), dtype=torch.int8, device=dev)

    # ------------------------------------------------------------------ what the machine attains (probes)
    attainable = None
    if not args.no_attainable:
        big = state_buf if state_buf is not None else torch.empty(256 << 20, dtype=torch.uint8, device=dev)
        attainable = measure_attainable(q, torch, dev, big)
        if state_buf is None:
            del big

    # ------------------------------------------------------------------ prefill
    s = W.CONFIGS[args.workload]
    pre, ctx = prefill_leg(q, torch, dev, s, seed, args.steps, args.warmup, args, headline=True)
    shape, hs, prob, A_np, D_np, dsc = ctx["shape"], ctx["hs"], ctx["prob"], ctx["A_np"], ctx["D_np"], ctx["dsc"]
    y, t = ctx["ys"][0], ctx["sets"][0]
    # the checks and the later legs read the first set's output: one more launch of it, every product computed
    q.quamba_ssd_prefill(ctx["shape_dense"], dsc, t["x"], t["B"], t["C"], t["dt"], ctx["A"], ctx["D"], None, y,
                         ctx["fin"], ctx["ws"])
    torch.cuda.synchronize()
    ms = pre["ms_per_step"]
    tokens = s.batch * s.seqlen

    out = {
        "metric": "int8 SSD prefill tokens/s/layer", "value": pre["value"], "unit": "tokens/s",
        "n_gpus": 1, "steps": args.steps, "warmup": args.warmup, "spin_up_ms": SPIN_UP_MS, "ms_per_step": ms,
        "wall_ms_per_step": pre["wall_ms_per_step"], "cold_ms_per_step": pre.get("cold_ms_per_step"),
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None, "dtype": "int8 x/B/C, fp16 MFMA, fp32 acc",
        "data": "synthetic",
        "config": {"workload": f"{s.name}: Mamba2-8B-shaped SSD layer prefill" if "8b" in s.name else s.name,
                   "batch": s.batch, "seqlen": s.seqlen, "nheads": s.nheads, "headdim": s.headdim,
                   "d_state": s.d_state, "ngroups": s.ngroups, "chunk": s.chunk, "clusters": f"{s.m}x{s.n} per group",
                   "final_state": bool(args.precise_state),
                   "side_inputs": "int8 gate z and int8 step-size codes" if args.gated else "none",
                   "input_sets": pre["input_sets"],
                   "bytes_per_input_and_output_set": pre["bytes_per_input_and_output_set"]},
        "timing_protocol": "W warm-up launches, K timed launches (cold_ms_per_step), then %g ms of untimed launches and K "
                           "timed launches again (ms_per_step, value); HIP events on the launch stream; consecutive "
                           "launches rotate over the input/output sets" % SPIN_UP_MS,
        "shader_clock_mhz": pre["shader_clock_mhz"],
        "shader_clock_mhz_per_xcd": pre.get("shader_clock_mhz_per_xcd"),
        "sustained_ms_per_step": (BOARD_POWER_W.get("prefill") or {}).get("sustained_ms_per_call"),
        "prefill_decay_skip": pre.get("prefill_decay_skip"),
        "prefill_zero_codes": pre.get("zero_codes"),
        "roofline": pre["roofline"], "roofline_hbm": pre["roofline_hbm"],
    }
    if attainable is not None:
        out["attainable"] = attainable
        att16 = attainable["mfma_f16"]["value"]
        out["roofline"]["frac_of_attainable"] = out["roofline"]["achieved"] / att16
        out["roofline"]["attainable"] = att16
        out["roofline_hbm"]["frac_of_attainable"] = out["roofline_hbm"]["achieved"] / attainable["hbm_stream_rmw"]["value"]
        out["roofline_hbm"]["attainable"] = attainable["hbm_stream_rmw"]["value"]
    if pre["shader_clock_mhz"]:
        out["roofline"]["frac_at_measured_clock"] = out["roofline"]["frac"] * 2400.0 / pre["shader_clock_mhz"]
        out["roofline"]["clock_note"] = ("the published peak is priced at 2400 MHz; a probe wave that ran beside the "
                                         "back-to-back launches read %.0f MHz (the board holds its power cap by "
                                         "lowering the clock)" % pre["shader_clock_mhz"])

    # ------------------------------------------------------------------ the other prefill configurations
    if not args.no_other_configs and args.workload == "m2_8b_b4":
        out["other_configs"] = {}
        for name in ("m2_8b_b1", "m2_2p7b", "m2_130m"):
            so = W.CONFIGS[name]
            ro, co = prefill_leg(q, torch, dev, so, seed, args.steps, args.warmup, args, headline=False)
            ro["config"] = {"workload": name, "batch": so.batch, "seqlen": so.seqlen, "nheads": so.nheads,
                            "headdim": so.headdim, "d_state": so.d_state, "ngroups": so.ngroups, "chunk": so.chunk}
            if name == "m2_130m":
                ro["note"] = ("one sequence of 24 heads: cut into 8 segments (two launches), 384 workgroups; about half "
                              "of the time is the two launches' ramp")
            out["other_configs"][name] = ro
            del co
            torch.cuda.empty_cache()

    # ------------------------------------------------------------------ CPU oracle on a bounded sample
    if not args.no_cpu:
        import oracle
        sc = oracle.Scales(s.m, s.n, hs.x_scales, hs.head_cluster_end, hs.chan_cluster_end, hs.B_scales, hs.C_scales)
        nseq = s.batch
        pairs = [(b, h) for b in range(nseq) for h in range(s.nheads)]
        # the whole prefill workload, repeated until about 10 s of wall time have gone by (at least twice: the first
        # pass also pages the inputs in); the rate is that of the passes after the first
        cpu_times = []
        while len(cpu_times) < 2 or (sum(cpu_times) < 10.0 and len(cpu_times) < 40):
            t0 = time.perf_counter()
            yref, _, threads = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], A_np, D_np,
                                                  pairs=pairs, want_state=False)
            cpu_times.append(time.perf_counter() - t0)
        cpu_s = sum(cpu_times[1:]) / (len(cpu_times) - 1)
        yg = y[:nseq].float().cpu().numpy().transpose(0, 2, 1, 3).reshape(len(pairs), s.seqlen, s.headdim)
        ymax = float(np.abs(yref).max())
        err = float(np.abs(yg - yref).max() / ymax)
        rel = np.abs(yg - yref) / np.maximum(np.abs(yref), 1e-4 * ymax)
        # cell by cell (Section 4.1): the largest error of a (head cluster, channel range) cell over that cell's largest output
        cells = oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups)
        dmax = np.abs(yg - yref).reshape(nseq, s.nheads, s.seqlen, s.headdim).max(axis=(0, 2))
        rmax = np.abs(yref).reshape(nseq, s.nheads, s.seqlen, s.headdim).max(axis=(0, 2))
        worst_cell = max(float(dmax[cells == c].max() / rmax[cells == c].max()) for c in np.unique(cells))
        out["cpu_baseline"] = {"value": nseq * s.seqlen / cpu_s, "unit": "tokens/s", "cores": int(threads),
                               "kind": "oracle", "seconds": cpu_s, "passes": len(cpu_times),
                               "sample": f"sequences 0..{nseq - 1} of the prefill workload, all {s.nheads} heads "
                                         f"({nseq * s.seqlen} tokens), fp64 sequential scan; mean of the passes "
                                         f"after the first, {sum(cpu_times):.1f} s of CPU wall time in total"}
        out["parity_spot_check"] = {"max_abs_err_over_max_abs_ref": err, "bar": 2e-3, "pairs": len(pairs),
                                    "worst_cell_err_over_cell_max": worst_cell, "cells": int(np.unique(cells).size),
                                    "elementwise_rel_err_floor_1e-4_max": {"max": float(rel.max()),
                                                                           "p99.9": float(np.quantile(rel[::7].ravel(), 0.999))}}
        del yref, yg, rel
        # the same oracle on ONE thread, on 16 (sequence, head) pairs of the same workload
        p1 = pairs[:: max(1, len(pairs) // 16)][:16]
        oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], A_np, D_np, pairs=p1[:2], want_state=False,
                           nthreads=1)
        t0 = time.perf_counter()
        _, _, th1 = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], A_np, D_np, pairs=p1,
                                       want_state=False, nthreads=1)
        one_s = time.perf_counter() - t0
        out["cpu_baseline_1core"] = {"value": len(p1) * s.seqlen / s.nheads / one_s, "unit": "tokens/s", "cores": int(th1),
                                     "kind": "oracle", "seconds": one_s,
                                     "sample": f"{len(p1)} of the {len(pairs)} (sequence, head) pairs, all {s.seqlen} "
                                               f"tokens each; tokens/s/layer = pairs x tokens / heads / seconds"}

    # ------------------------------------------------ quantized Hadamard transform of the prefill output (Section 4.2)
    n_had = s.nheads * s.headdim
    if not args.no_hadamard and n_had & (n_had - 1) == 0:
        rows = s.batch * s.seqlen
        # static scale of the transformed output: 4 standard deviations of a transformed value map to code 127
        # (its variance is n times the mean square of y); the scale is an input of the method, not part of it
        s_y = float(4.0 * (n_had * y.float().pow(2).mean()).sqrt().item() / 127.0)
        yq = torch.empty((s.batch, s.seqlen, n_had), dtype=torch.int8, device=dev)
        yflat = y.view(s.batch, s.seqlen, n_had)

        def hadamard():
            q.quamba_hadamard_quantize(yflat, s_y, yq)

        hms, hwall = time_region(torch, hadamard, args.steps, max(args.warmup, 4), min_warm_ms=SPIN_UP_MS, power_key="hadamard")
        hbytes = 3.0 * rows * n_had
        hgbs = hbytes / (hms * 1e-3) / 1e9
        hops = HADAMARD_OPS_PER_VALUE(n_had) * rows * n_had
        out["hadamard"] = {
            "metric": "quantized Hadamard transform us/call", "value": hms * 1e3, "unit": "us/call", "steps": args.steps,
            "higher_is_better": False, "wall_us_per_call": hwall * 1e3,
            "config": {"workload": "%s output: %d tokens x %d channels, fp16 in, int8 out, the scan's own y as input"
                                   % (s.name, rows, n_had), "s_y": s_y},
            "roofline": {"kernel": "hadamard_quantize_kernel", "bound": "hbm", "achieved": hgbs, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": hgbs / HBM_PEAK_GBS, **traffic_fields(s.name + "_hadamard")},
            "roofline_alu": {"kernel": "hadamard_quantize_kernel", "bound": "alu",
                             "achieved": hops / (hms * 1e-3) / 1e12, "peak": ALU_PEAK_TOPS,
                             "unit": "Top/s (fp32 vector instructions x 64 lanes)",
                             "frac": hops / (hms * 1e-3) / 1e12 / ALU_PEAK_TOPS,
                             "note": "log2(n) butterfly operations + scale, clamp and rounding add per value"},
            "saturated_fraction": float(((yq == 127) | (yq == -128)).float().mean().item()),
        }
        if attainable is not None:
            out["hadamard"]["roofline"]["attainable"] = attainable["hbm_stream_rmw"]["value"]
            out["hadamard"]["roofline"]["frac_of_attainable"] = hgbs / attainable["hbm_stream_rmw"]["value"]
            out["hadamard"]["roofline"]["frac_of_read_stream"] = hgbs / attainable["hbm_stream_read"]["value"]
        if not args.no_cpu:   # spot check against the oracle: 16 rows spread over the launch, codes bit for bit
            import oracle
            pick = torch.arange(0, rows, rows // 16, device=dev)
            ref = oracle.hadamard_quantize(yflat.view(rows, n_had)[pick].cpu().numpy(), s_y)
            out["hadamard"]["parity_spot_check"] = {
                "rows": int(pick.numel()), "codes_differing": int((yq.view(rows, n_had)[pick].cpu().numpy() != ref).sum())}
        del yq, yflat

    # ------------------------------------------------ W8A8 causal convolution in front of the scan (Section 4.2)
    if not args.no_conv:
        Ct = s.nheads * s.headdim + 2 * s.ngroups * s.d_state
        rawc = W.draw_conv(s, seed)
        s_in = np.float32(4.5 / 127.0)
        s_w = np.float32(np.abs(rawc["weight"]).max() / 127.0)
        cin = torch.from_numpy(q.quamba_quantize_groups(rawc["xBC"].reshape(-1, 1, Ct), np.array([s_in], np.float32))
                               .reshape(s.batch, s.seqlen, Ct)).to(dev)
        cw_np = q.quamba_quantize_groups(rawc["weight"].reshape(1, 1, -1), np.array([s_w], np.float32)).reshape(Ct, 4)
        cw = torch.from_numpy(cw_np).to(dev)
        cbias = torch.from_numpy(rawc["bias"]).to(dev)
        in_w_scale = float(np.float32(s_in * s_w))
        cx = torch.empty((s.batch, s.seqlen, s.nheads, s.headdim), dtype=torch.int8, device=dev)
        cB = torch.empty((s.batch, s.seqlen, s.ngroups, s.d_state), dtype=torch.int8, device=dev)
        cC = torch.empty_like(cB)
        cst = torch.empty((s.batch, 3, Ct), dtype=torch.int8, device=dev)

        def conv():
            q.quamba_conv1d_q8(shape, dsc, cin, cw, cbias, in_w_scale, cx, cB, cC, conv_state_out=cst)

        cms, cwall = time_region(torch, conv, args.steps, max(args.warmup, 4), min_warm_ms=SPIN_UP_MS, power_key="conv1d")
        celems = float(s.batch) * s.seqlen * Ct
        cgbs = 2.0 * celems / (cms * 1e-3) / 1e9
        cops = CONV_MIN_SLOTS * celems
        out["conv1d"] = {
            "metric": "W8A8 causal conv1d + SiLU + Eq. 1 us/call", "value": cms * 1e3, "unit": "us/call",
            "steps": args.steps, "higher_is_better": False, "wall_us_per_call": cwall * 1e3,
            "config": {"workload": "%s: %d tokens x %d channels [x|B|C], 4 taps, int8 in, int8 x/B/C out with the "
                                   "scan's cell and group scales" % (s.name, s.batch * s.seqlen, Ct)},
            "roofline": {"kernel": "conv1d_q8_vec_kernel", "bound": "alu", "achieved": cops / (cms * 1e-3) / 1e12,
                         "peak": ALU_PEAK_TOPS, "unit": "Top/s (fp32 vector instructions x 64 lanes)",
                         "frac": cops / (cms * 1e-3) / 1e12 / ALU_PEAK_TOPS,
                         "slots_per_element": CONV_MIN_SLOTS, "executed_per_element": CONV_EXECUTED_PER_ELEMENT,
                         **traffic_fields(s.name + "_conv1d"),
                         "note": "priced on what the method needs per output element, %.0f vector issue slots (window "
                                 "permute, 4-tap integer dot product, to float, scale + bias, exponential and "
                                 "reciprocal at quarter rate, 1 + e, times sigmoid, times 1/s_out, clamp, round and "
                                 "pack), against one slot per lane and cycle; the kernel executes %.1f vector "
                                 "instructions per element by the counters (executed_per_element), so added "
                                 "instructions lower frac" % (CONV_MIN_SLOTS, CONV_EXECUTED_PER_ELEMENT)},
            "roofline_hbm": {"kernel": "conv1d_q8_vec_kernel", "bound": "hbm", "achieved": cgbs,
                             "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": cgbs / HBM_PEAK_GBS,
                             **traffic_fields(s.name + "_conv1d")},
            "saturated_fraction": float((cx == 127).float().mean().item()),
        }
        if not args.no_cpu:   # spot check against the oracle: the last 8 tokens of sequence 0, codes bit for bit
            import oracle
            sc = oracle.Scales(s.m, s.n, hs.x_scales, hs.head_cluster_end, hs.chan_cluster_end, hs.B_scales,
                               hs.C_scales)
            os_ = oracle.output_scales(sc, s.nheads, s.headdim, s.ngroups, s.d_state)
            win = cin[:1, -11:].cpu().numpy()
            ref, _ = oracle.ref_conv1d_q8(win, cw_np, in_w_scale, rawc["bias"], os_)
            got = torch.cat([cx[:1, -8:].reshape(1, 8, -1), cB[:1, -8:].reshape(1, 8, -1),
                             cC[:1, -8:].reshape(1, 8, -1)], dim=2).cpu().numpy()
            out["conv1d"]["parity_spot_check"] = {"tokens": 8, "codes_differing": int((got != ref[:, -8:]).sum())}
        del cin, cw, cx, cB, cC, cst, rawc

    # ------------------------------------------------ 8-bit Mamba1 selective scan (Eq. 2, Mamba1 parameterisation)
    if not args.no_mamba1:
        mb, mD, mN, mL = 4, 5120, 16, 4096          # the Mamba1-2.8B-shaped layer: d_inner 5120, 16 states
        rawm = W.draw_mamba1(mb, mD, mN, mL, seed)
        _, mperm, mhs = q.quamba_reorder_params(1, mD, 1, 1, 4, mN, rawm["x_absmax"], np.abs(rawm["B"]).max((0, 2)),
                                                np.abs(rawm["C"]).max((0, 2)))
        mperm = mperm[0]
        mshape = q.Shape(batch=mb, seqlen=mL, nheads=1, headdim=mD, d_state=mN, ngroups=1, chunk=1,
                         n_head_clusters=1, n_chan_clusters=4, flags=0)
        mdsc = q.DeviceScales(mhs, dev)
        # per-channel scale of the sorted positions, then Eq. 1 by the library's host quantizer (one "group" per channel)
        ends = mhs.chan_cluster_end
        xs_c = np.repeat(mhs.x_scales, np.diff(np.concatenate([[0], ends])))
        mx = torch.from_numpy(q.quamba_quantize_groups(np.ascontiguousarray(rawm["x"][:, mperm]), xs_c)).to(dev)
        mB = torch.from_numpy(q.quamba_quantize_groups(rawm["B"].reshape(mb, 1, -1), mhs.B_scales)
                              .reshape(mb, mN, mL)).to(dev)
        mC = torch.from_numpy(q.quamba_quantize_groups(rawm["C"].reshape(mb, 1, -1), mhs.C_scales)
                              .reshape(mb, mN, mL)).to(dev)
        mdt = torch.from_numpy(np.ascontiguousarray(rawm["dt"][:, mperm])).to(dev)
        mA = torch.from_numpy(np.ascontiguousarray(rawm["A"][mperm])).to(dev)
        mDk = torch.from_numpy(np.ascontiguousarray(rawm["D"][mperm])).to(dev)
        my = torch.empty((mb, mD, mL), dtype=torch.float16, device=dev)
        mfin = torch.empty((mb, mD, mN), device=dev)

        def mamba1():
            q.quamba_mamba1_scan(mshape, mdsc, mx, mB, mC, mdt, mA, mDk, my, final_state=mfin)

        mms, mwall = time_region(torch, mamba1, max(20, args.steps // 2), max(args.warmup // 2, 3), min_warm_ms=SPIN_UP_MS, power_key="mamba1_scan")
        melems = float(mb) * mD * mL * mN
        mbytes = float(mb) * mD * mL * 7 + 2.0 * mb * mN * mL
        out["mamba1_scan"] = {
            "metric": "int8 Mamba1 selective scan tokens/s/layer", "value": mb * mL / (mms * 1e-3), "unit": "tokens/s",
            "us_per_call": mms * 1e3, "wall_us_per_call": mwall * 1e3, "higher_is_better": True,
            "config": {"workload": "Mamba1-2.8B-shaped layer: batch 4 x 4096 tokens, 5120 channels, 16 states, "
                                   "4 channel ranges; int8 x/B/C, fp32 dt, fp16 y, final state returned"},
            "roofline": {"kernel": "mamba1_scan_kernel", "bound": "alu",
                         "achieved": MAMBA1_MIN_SLOTS * melems / (mms * 1e-3) / 1e12, "peak": ALU_PEAK_TOPS,
                         "unit": "Top/s (fp32 vector issue slots x 64 lanes)",
                         "frac": MAMBA1_MIN_SLOTS * melems / (mms * 1e-3) / 1e12 / ALU_PEAK_TOPS,
                         "slots_per_element": MAMBA1_MIN_SLOTS, "executed_per_element": MAMBA1_EXECUTED_PER_ELEMENT,
                         **traffic_fields("mamba1_2p8b_scan"),
                         "note": "priced on what Eq. 2 needs per (token, channel, state) element, %.0f vector issue slots "
                                 "(dt A, its exponential at quarter rate, (dt x) B, the fused state update, the fused "
                                 "C h), against one slot per lane and cycle; the kernel executes %.1f vector "
                                 "instructions per element by the counters (executed_per_element, 1.06 of them "
                                 "quarter-rate), so added instructions lower frac"
                                 % (MAMBA1_MIN_SLOTS, MAMBA1_EXECUTED_PER_ELEMENT)},
            "roofline_hbm": {"kernel": "mamba1_scan_kernel", "bound": "hbm", "achieved": mbytes / (mms * 1e-3) / 1e9,
                             "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": mbytes / (mms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                             **traffic_fields("mamba1_2p8b_scan")},
            "finite": bool(torch.isfinite(my).all().item()),
        }
        if not args.no_cpu:   # spot check against the oracle: 6 channels of sequence 0, all tokens
            import oracle
            pick = np.array([0, 1, mD // 3, mD // 2, mD - 2, mD - 1])
            yref, sref = oracle.ref_mamba1_scan(xs_c[pick], mhs.B_scales[0], mhs.C_scales[0], mx[:1, pick].cpu().numpy(),
                                                mB[:1].cpu().numpy(), mC[:1].cpu().numpy(), mdt[:1, pick].cpu().numpy(),
                                                mA[pick].cpu().numpy(), mDk[pick].cpu().numpy())
            err = float(np.abs(my[:1, pick].float().cpu().numpy() - yref).max() / np.abs(yref).max())
            out["mamba1_scan"]["parity_spot_check"] = {"max_abs_err_over_max_abs_ref": err, "bar": 2e-3,
                                                       "channels": int(pick.size)}
        # one generation step of the same layer at batch 256 on the fp32 state
        db = 256
        dshape1 = q.Shape(batch=db, seqlen=1, nheads=1, headdim=mD, d_state=mN, ngroups=1, chunk=1, n_head_clusters=1,
                          n_chan_clusters=4, flags=0)
        sx1 = mx[0, :, :64].t().contiguous().repeat(4, 1)       # 256 token columns of the prefill inputs as the batch
        sdt1 = mdt[0, :, :64].t().contiguous().repeat(4, 1)
        sB1 = mB[0, :, :64].t().contiguous().repeat(4, 1)
        sC1 = mC[0, :, :64].t().contiguous().repeat(4, 1)
        mstate = mfin[:1].repeat(db, 1, 1).contiguous()
        y1 = torch.empty((db, mD), dtype=torch.float16, device=dev)

        def mamba1_step():
            q.quamba_mamba1_decode_step(dshape1, mdsc, sx1, sB1, sC1, sdt1, mA, mDk, mstate, y1)

        sms, swall = time_region(torch, mamba1_step, args.steps, max(args.warmup, 4), min_warm_ms=SPIN_UP_MS, power_key="mamba1_decode")
        sbytes = 8.0 * db * mD * mN + 7.0 * db * mD + 2.0 * db * mN + 4.0 * mD * mN
        out["mamba1_decode"] = {
            "metric": "Mamba1 decode state update us/step", "value": sms * 1e3, "unit": "us/step",
            "higher_is_better": False, "wall_us_per_step": swall * 1e3,
            "config": {"workload": "Mamba1-2.8B-shaped layer, batch 256: fp32 state [256, 5120, 16] (84 MB) in place"},
            "roofline": {"kernel": "mamba1_decode16_kernel", "bound": "hbm", "achieved": sbytes / (sms * 1e-3) / 1e9,
                         "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": sbytes / (sms * 1e-3) / 1e9 / HBM_PEAK_GBS,
                         **traffic_fields("mamba1_2p8b_decode")},
            "finite": bool(torch.isfinite(mstate).all().item()),
        }
        if attainable is not None:
            out["mamba1_decode"]["roofline"]["attainable"] = attainable["hbm_stream_rmw"]["value"]
            out["mamba1_decode"]["roofline"]["frac_of_attainable"] = (sbytes / (sms * 1e-3) / 1e9 /
                                                                      attainable["hbm_stream_rmw"]["value"])
        del mx, mB, mC, mdt, my, rawm, mstate

    # ------------------------------------------------------------------ decode
    if not args.no_decode:
        del t, y, prob, ctx
        torch.cuda.empty_cache()
        sd = W.CONFIGS["m2_8b_decode"]
        dshape, dhs, dhp, dcp = build_problem(q, sd, seed)
        ddsc = q.DeviceScales(dhs, dev)
        rawp = W.apply_reorder({k: v for k, v in W.draw_layer(sd.with_(batch=1, seqlen=1), seed).items()
                                if k in ("A", "D", "x", "dt")}, dhp, dcp)
        dA = torch.from_numpy(rawp["A"]).to(dev)
        dD = torch.from_numpy(rawp["D"]).to(dev)
        nsets = sd.decode_steps
        steps_in = []
        for k in range(nsets):
            r = W.apply_reorder(W.draw_decode_step(sd, seed, k), dhp, dcp)
            qd = quantize_layer(q, dshape, dhs, r)
            steps_in.append({n: torch.from_numpy(v).to(dev) for n, v in qd.items()})
        state = state_buf
        state.copy_(torch.from_numpy(W.draw_state(sd, seed)))
        yd = torch.empty((sd.batch, sd.nheads, sd.headdim), dtype=torch.float16, device=dev)
        counter = [0]

        def decode():
            i = steps_in[counter[0] % nsets]
            counter[0] += 1
            q.quamba_ssd_decode_step(dshape, ddsc, i["x"], i["B"], i["C"], i["dt"], dA, dD, state, yd)

        dsteps = max(args.steps, sd.decode_steps)
        dms, dwall = time_region(torch, decode, dsteps, max(args.warmup, 4), min_warm_ms=SPIN_UP_MS, power_key="decode")
        dclk = shader_clock_under_load(q, torch, dev, decode, launches=30)
        dgbs = decode_bytes(sd) / (dms * 1e-3) / 1e9
        out["decode"] = {
            "metric": "decode state update us/step", "value": dms * 1e3, "unit": "us/step", "steps": dsteps,
            "higher_is_better": False, "wall_us_per_step": dwall * 1e3,
            "config": {"workload": "m2_8b_decode: batch 256, 128 heads x 64, d_state 128, fp32 state 1 GiB in place"},
            "roofline": {"kernel": "decode_vec_kernel", "bound": "hbm", "achieved": dgbs, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": dgbs / HBM_PEAK_GBS, **traffic_fields("m2_8b_decode")},
            "shader_clock_mhz": dclk,
            "finite": bool(torch.isfinite(state).all().item()),
        }
        if attainable is not None:
            out["decode"]["roofline"]["attainable"] = attainable["hbm_stream_rmw"]["value"]
            out["decode"]["roofline"]["frac_of_attainable"] = dgbs / attainable["hbm_stream_rmw"]["value"]

        # ------------------------------------------------ decode on the 8-bit cached state (Appendix E)
        ncell = sd.ngroups * sd.m * sd.n
        mx = W.reorder_state(W.draw_cached_state_calibration(sd, seed), dhp, dcp)
        ss = q.quamba_state_scales(sd.nheads, sd.headdim, sd.ngroups, sd.m, sd.n, sd.d_state, dhs.head_cluster_end,
                                   dhs.chan_cluster_end, mx)
        assert ss.shape == (ncell, sd.d_state)
        dss = torch.from_numpy(ss).to(dev)
        # cached states of 32 sequences, drawn once and repeated over the batch, quantized by the library itself
        rep = 32
        st32 = torch.from_numpy(W.reorder_state(W.draw_cached_state(sd, seed, batch=rep), dhp, dcp)).to(dev)
        qstate = qstate_buf
        shape32 = q.Shape(**{f: (rep if f == "batch" else getattr(dshape, f)) for f, _ in dshape._fields_})
        q32 = torch.empty((rep, sd.nheads, sd.headdim, sd.d_state), dtype=torch.int8, device=dev)
        q.quamba_ssd_quantize_state(shape32, ddsc, dss, st32, q32)
        for i0 in range(0, sd.batch, rep):
            qstate[i0:i0 + rep].copy_(q32[:min(rep, sd.batch - i0)])
        del st32, q32
        counter[0] = 0

        def decode_q8():
            i = steps_in[counter[0] % nsets]
            counter[0] += 1
            q.quamba_ssd_decode_step_q8(dshape, ddsc, dss, i["x"], i["B"], i["C"], i["dt"], dA, dD, qstate, yd)

        qms, qwall = time_region(torch, decode_q8, dsteps, max(args.warmup, 4), min_warm_ms=SPIN_UP_MS, power_key="decode_q8")
        qclk = shader_clock_under_load(q, torch, dev, decode_q8, launches=60)
        qbytes = decode_bytes(sd, state_bytes=1)
        qgbs = qbytes / (qms * 1e-3) / 1e9
        elems = sd.batch * sd.nheads * sd.headdim * sd.d_state
        qops = Q8_OPS_PER_ELEMENT * elems
        out["decode_q8"] = {
            "metric": "decode state update us/step, 8-bit cached state", "value": qms * 1e3, "unit": "us/step",
            "steps": dsteps, "higher_is_better": False, "wall_us_per_step": qwall * 1e3,
            "config": {"workload": "m2_8b_decode with an int8 cached state: batch 256, 128 heads x 64, d_state 128, "
                                   "256 MiB of codes in place, 4x4 cells x 128 state scales per group"},
            "roofline": {"kernel": "decode_q8_vec_kernel", "bound": "hbm", "achieved": qgbs, "peak": HBM_PEAK_GBS,
                         "unit": "GB/s", "frac": qgbs / HBM_PEAK_GBS, **traffic_fields("m2_8b_decode_q8")},
            "shader_clock_mhz": qclk,
            "roofline_alu": {"kernel": "decode_q8_vec_kernel", "bound": "alu", "achieved": qops / (qms * 1e-3) / 1e12,
                             "peak": ALU_PEAK_TOPS, "unit": "Top/s (fp32 vector instructions x 64 lanes)",
                             "frac": qops / (qms * 1e-3) / 1e12 / ALU_PEAK_TOPS,
                             "note": "%d fp32 vector operations per state element; peak = 256 CUs x 4 SIMDs x 16 "
                                     "lanes x 2.4 GHz, one unfused, unpacked operation per lane and cycle"
                                     % Q8_OPS_PER_ELEMENT},
            "speedup_over_fp32_state": dms / qms,
            "codes_in_range": bool((qstate.abs() <= 127).all().item()),
        }
        if attainable is not None:
            out["decode_q8"]["roofline"]["attainable"] = attainable["hbm_stream_rmw"]["value"]
            out["decode_q8"]["roofline"]["frac_of_attainable"] = qgbs / attainable["hbm_stream_rmw"]["value"]

    if args.copy_calibration:
        src = torch.empty(256 << 20, dtype=torch.uint8, device=dev).random_(0, 255)
        dst = torch.empty_like(src)
        for _ in range(3):
            dst.copy_(src)
        torch.cuda.synchronize()
        out["copy_calibration"] = {"bytes_read": 256 << 20, "bytes_written": 256 << 20, "launches": 3}

    if POWER_SECONDS > 0:
        out["board_power_w"] = dict(BOARD_POWER_W, cap=_hwmon("power1_cap"), seconds_per_leg=POWER_SECONDS)
    print(json.dumps(out))
    return 0


if __name__ == "__main__":
    sys.exit(main())
