"""Seeded synthetic inputs with the shapes and value structure of the paper's workloads.

The paper calibrates on real activations of trained Mamba2 checkpoints, which are not
available; these draws stand in for them.  What is reproduced is the structure the paper
reports for the SSM input x (per-channel magnitudes that persist over time, a few
large-magnitude outlier channels; Section 4.1 "Sort-and-cluster") and for B and C (only a
few state groups carry large values; Section 4.1 "Per-state-group quantization").

Everything here is a random draw or an index gather.  The quantizer (Eq. 1), the
clustering and the scan are NOT here: callers apply their own.
"""
from __future__ import annotations

from dataclasses import dataclass, replace
import numpy as np


@dataclass(frozen=True)
class LayerShape:
    name: str
    batch: int
    seqlen: int
    nheads: int
    headdim: int
    d_state: int
    ngroups: int
    chunk: int
    m: int                     # head clusters per state group
    n: int                     # channel clusters per head cluster
    outlier_channels: int = 0  # fixed count of channels whose std is multiplied by 20
    outlier_frac: float = 0.0  # fraction of channels multiplied by 20 and drawn Student-t(3)
    decode_steps: int = 0

    def with_(self, **kw) -> "LayerShape":
        return replace(self, **kw)


CONFIGS = {
    "tiny": LayerShape("tiny", 1, 256, 8, 64, 16, 1, 64, 1, 4, outlier_channels=2),
    "m2_130m": LayerShape("m2_130m", 1, 2048, 24, 64, 128, 1, 256, 4, 4),
    "m2_2p7b": LayerShape("m2_2p7b", 8, 2048, 80, 64, 128, 1, 256, 4, 4, outlier_frac=0.01),
    "m2_8b_b1": LayerShape("m2_8b_b1", 1, 4096, 128, 64, 128, 8, 256, 4, 4),
    "m2_8b_b4": LayerShape("m2_8b_b4", 4, 4096, 128, 64, 128, 8, 256, 4, 4),
    "m2_8b_decode": LayerShape("m2_8b_decode", 256, 1, 128, 64, 128, 8, 256, 4, 4,
                               decode_steps=32),
}

_BASE_SEED = 228790


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[(_BASE_SEED + seed) & 0xFFFFFFFFFFFFFFFF,
                                                     stream]))


def _softplus(v: np.ndarray) -> np.ndarray:
    return np.logaddexp(0.0, v)


def _channel_profile(s: LayerShape, seed: int):
    """Per-channel std sigma[h,p] and the mask of heavy-tailed channels (stream 0)."""
    g = _rng(seed, 0)
    sigma = np.exp(g.standard_normal((s.nheads, s.headdim)))
    heavy = np.zeros((s.nheads, s.headdim), dtype=bool)
    flat = s.nheads * s.headdim
    if s.outlier_channels:
        idx = g.choice(flat, size=s.outlier_channels, replace=False)
        sigma.reshape(-1)[idx] *= 20.0
    if s.outlier_frac > 0.0:
        k = max(1, int(round(flat * s.outlier_frac)))
        idx = g.choice(flat, size=k, replace=False)
        sigma.reshape(-1)[idx] *= 20.0
        heavy.reshape(-1)[idx] = True
    return sigma, heavy


def _group_profile(s: LayerShape, seed: int, which: int):
    """Per-state gain for B (which=0) or C (which=1): gain[g]*tau[g,n], largest gain = 1."""
    g = _rng(seed, 1 + which)
    gain = np.exp(g.standard_normal(s.ngroups))
    gain = gain / gain.max()
    tau = np.exp(0.5 * g.standard_normal((s.ngroups, s.d_state)))
    return gain[:, None] * tau


def _draw_x(g: np.random.Generator, tokens_shape, sigma, heavy) -> np.ndarray:
    shape = tuple(tokens_shape) + sigma.shape
    x = g.standard_normal(shape, dtype=np.float32)
    if heavy.any():
        hh, pp = np.nonzero(heavy)
        t3 = g.standard_t(3.0, size=tuple(tokens_shape) + (hh.size,)).astype(np.float32)
        x[..., hh, pp] = t3
    x *= sigma.astype(np.float32)
    return x


def draw_calibration(s: LayerShape, seed: int = 0, tokens: int = 8192):
    """Per-channel |x| maxima [H,P] and per-state |B|,|C| maxima [G,N] over a separate draw
    that plays the role of the paper's calibration set (Appendix C, "Quantization setup")."""
    sigma, heavy = _channel_profile(s, seed)
    g = _rng(seed, 5)
    xmax = np.zeros(sigma.shape, dtype=np.float32)
    step = 1024
    for t0 in range(0, tokens, step):
        nt = min(step, tokens - t0)
        xmax = np.maximum(xmax, np.abs(_draw_x(g, (nt,), sigma, heavy)).max(axis=0))
    out = [xmax]
    for which in (0, 1):
        prof = _group_profile(s, seed, which).astype(np.float32)
        v = g.standard_normal((tokens,) + prof.shape, dtype=np.float32) * prof
        out.append(np.abs(v).max(axis=0))
    return tuple(out)


def draw_layer(s: LayerShape, seed: int = 0) -> dict:
    """Raw floating-point inputs of one prefill, in the model's ORIGINAL head/channel order.

    Returns x [b,L,H,P], B, C [b,L,G,N], dt [b,L,H] (softplus already applied), A [H] (<0),
    D [H], all float32.
    """
    sigma, heavy = _channel_profile(s, seed)
    g = _rng(seed, 10)
    x = _draw_x(g, (s.batch, s.seqlen), sigma, heavy)
    bc = []
    for which in (0, 1):
        prof = _group_profile(s, seed, which).astype(np.float32)
        bc.append(g.standard_normal((s.batch, s.seqlen) + prof.shape, dtype=np.float32) * prof)
    dt = _softplus(g.standard_normal((s.batch, s.seqlen, s.nheads)) - 3.0).astype(np.float32)
    gp = _rng(seed, 11)
    A = (-np.exp(gp.uniform(0.0, np.log(16.0), s.nheads))).astype(np.float32)
    D = gp.standard_normal(s.nheads).astype(np.float32)
    return {"x": x, "B": bc[0], "C": bc[1], "dt": dt, "A": A, "D": D}


def draw_decode_step(s: LayerShape, seed: int, step: int) -> dict:
    """Raw inputs of decode step `step`: x [b,H,P], B, C [b,G,N], dt [b,H] (A, D as in draw_layer)."""
    sigma, heavy = _channel_profile(s, seed)
    g = _rng(seed, 100 + step)
    x = _draw_x(g, (s.batch,), sigma, heavy)
    bc = []
    for which in (0, 1):
        prof = _group_profile(s, seed, which).astype(np.float32)
        bc.append(g.standard_normal((s.batch,) + prof.shape, dtype=np.float32) * prof)
    dt = _softplus(g.standard_normal((s.batch, s.nheads)) - 3.0).astype(np.float32)
    return {"x": x, "B": bc[0], "C": bc[1], "dt": dt}


def draw_state(s: LayerShape, seed: int = 0, batch: int | None = None) -> np.ndarray:
    """Persistent SSM state [b,H,P,N] float32, N(0, std 0.1)."""
    g = _rng(seed, 20)
    b = s.batch if batch is None else batch
    st = g.standard_normal((b, s.nheads, s.headdim, s.d_state), dtype=np.float32)
    st *= np.float32(0.1)
    return st


def draw_gate(s: LayerShape, seed: int = 0, decode: bool = False, step: int = 0) -> dict:
    """Raw floats of the SSD kernel's optional side inputs, in the model's ORIGINAL head/channel order: the gate branch
    z (standard normal times a per-channel magnitude, like x), the step size's pre-activation without its bias
    (N(-3, 1) minus the bias) and the per-head bias (N(0, 0.5)).  decode=True draws one token ([b,H,P] / [b,H])."""
    g = _rng(seed, 30 + (1000 + step if decode else 0))
    gb = _rng(seed, 31)
    tok = (s.batch,) if decode else (s.batch, s.seqlen)
    zsig = np.exp(0.5 * _rng(seed, 32).standard_normal((s.nheads, s.headdim))).astype(np.float32)
    z = g.standard_normal(tok + (s.nheads, s.headdim), dtype=np.float32) * zsig
    bias = (0.5 * gb.standard_normal(s.nheads)).astype(np.float32)
    pre = (g.standard_normal(tok + (s.nheads,), dtype=np.float32) - np.float32(3.0)) - bias
    return {"z": z, "dt_pre": pre.astype(np.float32), "dt_bias": bias}


def draw_ssd_output(rows: int, n: int, seed: int = 0, outlier_frac: float = 0.005):
    """Output of the scan flattened to [rows, n] float16 (n = nheads * headdim) as the input of the quantized Hadamard
    transform: standard normal times a log-normal per-channel magnitude, a fraction of the channels 20 times larger
    (the outlier channels the transform spreads out).  Also returns the per-channel std [n] (float64), from which a
    caller can set a static scale for the transformed values (their std is the root of the sum of squares)."""
    g = _rng(seed, 40)
    sigma = 0.05 * np.exp(0.5 * g.standard_normal(n))
    k = int(round(n * outlier_frac))
    if k:
        sigma[g.choice(n, size=k, replace=False)] *= 20.0
    y = _rng(seed, 41).standard_normal((rows, n), dtype=np.float32) * sigma.astype(np.float32)
    return y.astype(np.float16), sigma


def draw_mamba1(batch: int, channels: int, d_state: int, seqlen: int, seed: int = 0, stream: int = 70) -> dict:
    """Raw floats of a Mamba1-shaped selective-scan layer, channel-major with time last, channels already in sorted
    order: x [b,D,L] = N(0,1) times a per-channel magnitude that rises with the channel index (log-normal values,
    sorted; 1 % of the channels 10x larger), B, C [b,N,L] = N(0,1) times a per-state gain exp(N(0,0.5)), dt [b,D,L] =
    softplus(N(-3,1) + a per-channel offset N(0,0.5)), A [D,N] = -(n+1) exp(N(0,0.2)) (the S4D-real start the Mamba1
    block trains from, perturbed), D [D] ~ N(0,1), and the per-channel maxima of |x| over a separate draw of 256 tokens
    for calibration."""
    g = _rng(seed, stream)
    gp = _rng(seed, 71)
    sigma = np.exp(gp.standard_normal(channels))
    k = max(1, channels // 100)
    sigma[gp.choice(channels, size=k, replace=False)] *= 10.0
    sigma = np.sort(sigma).astype(np.float32)
    gainB = np.exp(0.5 * gp.standard_normal(d_state)).astype(np.float32)
    gainC = np.exp(0.5 * gp.standard_normal(d_state)).astype(np.float32)
    off = (0.5 * gp.standard_normal(channels)).astype(np.float32)
    A = (-(np.arange(1, d_state + 1, dtype=np.float32))[None, :] * np.exp(0.2 * gp.standard_normal((channels, d_state)))).astype(np.float32)
    Dk = gp.standard_normal(channels).astype(np.float32)
    xcal = np.abs(gp.standard_normal((256, channels), dtype=np.float32)).max(0) * sigma
    x = g.standard_normal((batch, channels, seqlen), dtype=np.float32) * sigma[None, :, None]
    B = g.standard_normal((batch, d_state, seqlen), dtype=np.float32) * gainB[None, :, None]
    C = g.standard_normal((batch, d_state, seqlen), dtype=np.float32) * gainC[None, :, None]
    dt = _softplus(g.standard_normal((batch, channels, seqlen), dtype=np.float32) - np.float32(3.0) + off[None, :, None])
    return {"x": x, "B": B, "C": C, "dt": dt.astype(np.float32), "A": A, "D": Dk, "x_absmax": xcal.astype(np.float32)}


def draw_mamba1_gate(batch: int, channels: int, seqlen: int, seed: int = 0, stream: int = 75) -> dict:
    """Raw floats of the Mamba1 scan's optional side inputs, channel-major with time last like draw_mamba1's tensors
    and in the same sorted channel order: the gate branch z [b,D,L] (standard normal times a log-normal per-channel
    magnitude), the step size's pre-activation without its bias [b,D,L] (N(-3, 1) minus the bias) and the per-channel
    bias [D] (N(0, 0.5))."""
    g = _rng(seed, stream)
    gp = _rng(seed, 76)
    zsig = np.exp(0.5 * gp.standard_normal(channels)).astype(np.float32)
    bias = (0.5 * gp.standard_normal(channels)).astype(np.float32)
    z = g.standard_normal((batch, channels, seqlen), dtype=np.float32) * zsig[None, :, None]
    pre = (g.standard_normal((batch, channels, seqlen), dtype=np.float32) - np.float32(3.0)) - bias[None, :, None]
    return {"z": z, "dt_pre": pre.astype(np.float32), "dt_bias": bias}


def draw_conv(s: LayerShape, seed: int = 0, batch: int | None = None, seqlen: int | None = None, stream: int = 50):
    """Raw floats of the causal convolution in front of the scan, channels [x | B | C] (H*P + 2*G*N of them) already in
    the sorted order the offline reordering gives them: the block's pre-convolution activations xBC [b,L,Ct] (standard
    normal times a log-normal per-channel magnitude), the depthwise filter [Ct,4] (normal, a log-normal per-channel
    gain, scaled so that the convolution's output has a standard deviation of about 1.5 per unit gain) and the bias
    [Ct] (N(0, 0.3)).  `stream` separates draws (a later piece of a sequence, a decode step)."""
    b = s.batch if batch is None else batch
    L = s.seqlen if seqlen is None else seqlen
    Ct = s.nheads * s.headdim + 2 * s.ngroups * s.d_state
    gp = _rng(seed, 51)
    in_sigma = np.exp(0.3 * gp.standard_normal(Ct)).astype(np.float32)
    gain = np.exp(0.5 * gp.standard_normal(Ct)).astype(np.float32)
    w = gp.standard_normal((Ct, 4)).astype(np.float32) * (gain / in_sigma * np.float32(0.75))[:, None]
    bias = (0.3 * gp.standard_normal(Ct)).astype(np.float32)
    x = _rng(seed, stream).standard_normal((b, L, Ct), dtype=np.float32) * in_sigma
    return {"xBC": x, "weight": w, "bias": bias}


def draw_cached_state(s: LayerShape, seed: int = 0, batch: int | None = None, stream: int = 21) -> np.ndarray:
    """Cached SSM state [b,H,P,N] float32 with the structure a state built from x and B has: the magnitude of
    element (h,p,n) follows the channel profile of x (rows, in the model's ORIGINAL head/channel order, like x) times
    the per-state profile of B's group, times a standard normal draw and 0.1.  Stands in for the cached states of a
    real checkpoint, whose rows follow the channel magnitudes of x (Appendix E)."""
    g = _rng(seed, stream)
    b = s.batch if batch is None else batch
    sigma, _ = _channel_profile(s, seed)
    prof = _group_profile(s, seed, 0)                                  # [G,N]
    hpg = s.nheads // s.ngroups
    st = g.standard_normal((b, s.nheads, s.headdim, s.d_state), dtype=np.float32)
    st *= (0.1 * sigma).astype(np.float32)[None, :, :, None]
    st *= np.repeat(prof, hpg, axis=0).astype(np.float32)[None, :, None, :]
    return st


def draw_cached_state_calibration(s: LayerShape, seed: int = 0, sequences: int = 8) -> np.ndarray:
    """Per-element |state| maxima [H,P,N] over a separate draw of `sequences` cached states (original order)."""
    return np.abs(draw_cached_state(s, seed + 5, batch=sequences, stream=22)).max(axis=0)


def reorder_state(st: np.ndarray, head_perm: np.ndarray, chan_perm: np.ndarray) -> np.ndarray:
    """Gather the head and channel axes of a [..., H, P, N] array into the sorted/clustered order (index gathers
    only): new head i = old head head_perm[i], its channel position k = old channel chan_perm[i, k]."""
    st = np.take(st, head_perm, axis=-3)
    idx = chan_perm.astype(np.int64)[..., None]
    idx = np.broadcast_to(idx.reshape((1,) * (st.ndim - 3) + idx.shape), st.shape[:-1] + (1,))
    idx = np.broadcast_to(idx, st.shape)
    return np.ascontiguousarray(np.take_along_axis(st, idx, axis=-2))


def apply_reorder(raw: dict, head_perm: np.ndarray, chan_perm: np.ndarray) -> dict:
    """Gather x, dt, A, D into the sorted/clustered order (new index -> old index).

    head_perm [H]; chan_perm [H,P], row i holds the channel order of NEW head i.  This is what
    the offline weight reordering (Section 4.2) makes the projections produce directly.
    """
    out = dict(raw)
    x = raw["x"][..., head_perm, :]
    idx = np.broadcast_to(chan_perm.reshape((1,) * (x.ndim - 2) + chan_perm.shape), x.shape)
    out["x"] = np.ascontiguousarray(np.take_along_axis(x, idx, axis=-1))
    out["dt"] = np.ascontiguousarray(raw["dt"][..., head_perm])
    for k in ("A", "D"):
        if k in raw:
            out[k] = np.ascontiguousarray(raw[k][head_perm])
    return out
