"""Shared by the tests: build a quantized problem from a seeded workload with the ORACLE's offline utilities
(numpy sort-and-cluster + Eq. 1), so that no oracle input ever comes from the HIP library."""
from __future__ import annotations

import numpy as np

import oracle
import workloads as W


def make_problem(s: W.LayerShape, seed: int = 0, calib_tokens: int = 1024, with_D: bool = True):
    """Returns (Scales, dict of int8/fp32 numpy arrays in reordered order)."""
    xmax, bmax, cmax = W.draw_calibration(s, seed, tokens=calib_tokens)
    r = oracle.sort_and_cluster(xmax, s.ngroups, s.m, s.n)
    sc = oracle.Scales(s.m, s.n, r["x_scales"], r["head_cluster_end"], r["chan_cluster_end"],
                       oracle.group_scales(bmax), oracle.group_scales(cmax))
    raw = W.apply_reorder(W.draw_layer(s, seed), r["head_perm"], r["chan_perm"])
    tab = oracle.x_scale_table(sc, s.nheads, s.headdim, s.ngroups)
    prob = {
        "x": oracle.quantize(raw["x"], tab),
        "B": oracle.quantize(raw["B"], sc.B_scales[:, None]),
        "C": oracle.quantize(raw["C"], sc.C_scales[:, None]),
        "dt": raw["dt"], "A": raw["A"], "D": raw["D"] if with_D else None,
    }
    return sc, prob, r


def make_decode_inputs(s: W.LayerShape, sc, r, seed: int, step: int, batch=None):
    raw = W.draw_decode_step(s if batch is None else s.with_(batch=batch), seed, step)
    raw = W.apply_reorder(raw, r["head_perm"], r["chan_perm"])
    tab = oracle.x_scale_table(sc, s.nheads, s.headdim, s.ngroups)
    return {"x": oracle.quantize(raw["x"], tab), "B": oracle.quantize(raw["B"], sc.B_scales[:, None]),
            "C": oracle.quantize(raw["C"], sc.C_scales[:, None]), "dt": raw["dt"]}


def to_shape(q, s: W.LayerShape, flags: int = 0, **over):
    d = dict(batch=s.batch, seqlen=s.seqlen, nheads=s.nheads, headdim=s.headdim, d_state=s.d_state,
             ngroups=s.ngroups, chunk=s.chunk, n_head_clusters=s.m, n_chan_clusters=s.n, flags=flags)
    d.update(over)
    return q.Shape(**d)


def host_scales(q, sc):
    return q.HostScales(np.ascontiguousarray(sc.x_scales, np.float32),
                        np.ascontiguousarray(sc.head_cluster_end, np.int32),
                        np.ascontiguousarray(sc.chan_cluster_end, np.int32),
                        np.ascontiguousarray(sc.B_scales, np.float32),
                        np.ascontiguousarray(sc.C_scales, np.float32))


def make_state_cache(s: W.LayerShape, sc, r, seed: int, batch=None, calib_sequences: int = 8):
    """Scales of the 8-bit cached state (oracle's calibration rule on a separate draw) and initial codes (oracle's
    Eq. 1 on a seeded cached-state draw), both in the reordered order.  Returns (state_scales [cells,N], codes)."""
    mx = W.reorder_state(W.draw_cached_state_calibration(s, seed, calib_sequences), r["head_perm"], r["chan_perm"])
    ss = oracle.state_scales_from_absmax(sc, mx, s.ngroups)
    st = W.reorder_state(W.draw_cached_state(s, seed, batch=batch), r["head_perm"], r["chan_perm"])
    return ss, oracle.quantize_state(sc, ss, st, s.ngroups), st


def make_gate_inputs(s: W.LayerShape, r, seed: int, decode: bool = False, step: int = 0):
    """int8 codes of the optional side inputs in the reordered order, quantized with the oracle's Eq. 1 and one static
    scale per tensor (absolute maximum of the draw / 127).  Returns dict(z, z_scale, dt_q, dt_scale, dt_bias)."""
    raw = W.draw_gate(s, seed, decode=decode, step=step)
    hp, cp = r["head_perm"], r["chan_perm"]
    z = np.take(raw["z"], hp, axis=-2)
    z = np.take_along_axis(z, np.broadcast_to(cp, z.shape), axis=-1)
    pre = np.take(raw["dt_pre"], hp, axis=-1)
    bias = raw["dt_bias"][hp]
    zs = np.float32(np.abs(raw["z"]).max() / 127.0)
    ds = np.float32(np.abs(raw["dt_pre"]).max() / 127.0)
    return {"z": oracle.quantize(z, zs), "z_scale": float(zs), "dt_q": oracle.quantize(pre, ds),
            "dt_scale": float(ds), "dt_bias": np.ascontiguousarray(bias, np.float32)}


def make_conv_inputs(s: W.LayerShape, seed: int, batch=None, seqlen=None, stream: int = 50):
    """int8 codes of the convolution's input and filter, quantized with the oracle's Eq. 1 and one static scale per
    tensor (absolute maximum / 127; the input scale is fixed at 4.5 / 127 so that pieces of one sequence share it).
    Returns dict(xBC, weight, bias, in_w_scale)."""
    raw = W.draw_conv(s, seed, batch=batch, seqlen=seqlen, stream=stream)
    s_in = np.float32(4.5 / 127.0)
    s_w = np.float32(np.abs(raw["weight"]).max() / 127.0)
    return {"xBC": oracle.quantize(raw["xBC"], s_in), "weight": oracle.quantize(raw["weight"], s_w),
            "bias": raw["bias"], "in_w_scale": float(np.float32(s_in * s_w))}


def make_mamba1_problem(batch: int, channels: int, d_state: int, seqlen: int, seed: int, nranges: int = 4):
    """A Mamba1-shaped selective-scan problem: channels sorted by their calibrated maximum and clustered into n ranges
    (Section 4.1 for a block without heads), raw tensors gathered into that order, Eq. 1 with the oracle's quantizer.  Returns (Scales, dict of numpy arrays: int8 x [b,D,L], B, C [b,N,L]; fp32 dt, A, D; scale vectors)."""
    raw = W.draw_mamba1(batch, channels, d_state, seqlen, seed)
    # channels sorted by their calibrated maximum; the ranges come from the oracle's clustering of an evenly thinned
    # profile (at most 512 points: its exact 1-D clustering is quadratic in the number of points), scaled back
    perm = np.argsort(raw["x_absmax"], kind="stable")
    smax = raw["x_absmax"][perm]
    step = max(1, channels // 512)
    r = oracle.sort_and_cluster(smax[::step][None, :], 1, 1, nranges)
    ends = np.minimum(r["chan_cluster_end"].astype(np.int64) * step, channels).astype(np.int32)
    ends[-1] = channels
    los = np.concatenate([[0], ends[:-1]])
    xsc = oracle.group_scales(np.array([[smax[lo:hi].max() if hi > lo else 0.0] for lo, hi in zip(los, ends)], np.float32))
    r = {"x_scales": xsc, "head_cluster_end": np.array([1], np.int32), "chan_cluster_end": ends}
    bmax = np.abs(raw["B"]).max()
    cmax = np.abs(raw["C"]).max()
    sc = oracle.Scales(1, nranges, r["x_scales"], r["head_cluster_end"], r["chan_cluster_end"],
                       oracle.group_scales(np.array([[bmax]], np.float32)), oracle.group_scales(np.array([[cmax]], np.float32)))
    xs = oracle.channel_scales(sc.x_scales, sc.chan_cluster_end, channels).astype(np.float32)
    x = raw["x"][:, perm]
    prob = {"x": oracle.quantize(x, xs[None, :, None]), "B": oracle.quantize(raw["B"], sc.B_scales[0]),
            "C": oracle.quantize(raw["C"], sc.C_scales[0]), "dt": np.ascontiguousarray(raw["dt"][:, perm]),
            "A": np.ascontiguousarray(raw["A"][perm]), "D": np.ascontiguousarray(raw["D"][perm]), "xs": xs}
    return sc, prob


def make_mamba1_gate(batch: int, channels: int, seqlen: int, seed: int):
    """int8 codes of the Mamba1 scan's side inputs [b,D,L] (drawn in the sorted channel order), quantized with the
    oracle's Eq. 1 and one static scale per tensor (absolute maximum / 127).  Returns dict(z, z_scale, dt_q, dt_scale,
    dt_bias [D])."""
    raw = W.draw_mamba1_gate(batch, channels, seqlen, seed)
    zs = np.float32(np.abs(raw["z"]).max() / 127.0)
    ds = np.float32(np.abs(raw["dt_pre"]).max() / 127.0)
    return {"z": oracle.quantize(raw["z"], zs), "z_scale": float(zs), "dt_q": oracle.quantize(raw["dt_pre"], ds),
            "dt_scale": float(ds), "dt_bias": raw["dt_bias"]}
