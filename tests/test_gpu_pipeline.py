"""The three steps around one layer chained on the GPU, each feeding the next through the library's own tensors:
W8A8 convolution -> int8 x, B, C -> SSD prefill -> fp16 y -> quantized Hadamard transform -> int8 codes; against
the same chain of oracles."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import make_problem, make_conv_inputs, to_shape, host_scales

pytestmark = pytest.mark.gpu


def test_conv_scan_hadamard_chain(gpu_lib):
    import torch
    q = gpu_lib
    s = W.LayerShape("chain", 2, 300, 16, 64, 128, 2, 256, 2, 4)         # 16 heads x 64 = 1024 channels, 2 state groups
    sc, prob, _ = make_problem(s, seed=21, calib_tokens=512)
    inp = make_conv_inputs(s, seed=21)
    shape = to_shape(q, s)
    dsc = q.DeviceScales(host_scales(q, sc))
    dev = lambda a: torch.from_numpy(np.ascontiguousarray(a)).cuda()
    x = torch.empty((s.batch, s.seqlen, s.nheads, s.headdim), dtype=torch.int8, device="cuda")
    B = torch.empty((s.batch, s.seqlen, s.ngroups, s.d_state), dtype=torch.int8, device="cuda")
    C = torch.empty_like(B)
    y = torch.empty(x.shape, dtype=torch.float16, device="cuda")
    n = s.nheads * s.headdim
    yq = torch.empty((s.batch, s.seqlen, n), dtype=torch.int8, device="cuda")
    q.quamba_conv1d_q8(shape, dsc, dev(inp["xBC"]), dev(inp["weight"]), dev(inp["bias"]), inp["in_w_scale"], x, B, C)
    q.quamba_ssd_prefill(shape, dsc, x, B, C, dev(prob["dt"]), dev(prob["A"]), dev(prob["D"]), None, y, None)
    # the scale of the transformed output from the oracle's y (a calibration, fixed before the GPU result is looked at)
    os_ = oracle.output_scales(sc, s.nheads, s.headdim, s.ngroups, s.d_state)
    cref, _ = oracle.ref_conv1d_q8(inp["xBC"], inp["weight"], inp["in_w_scale"], inp["bias"], os_)
    HP, GN = n, s.ngroups * s.d_state
    xr = cref[:, :, :HP].reshape(x.shape)
    Br = cref[:, :, HP:HP + GN].reshape(B.shape)
    Cr = cref[:, :, HP + GN:].reshape(C.shape)
    yref, _, _ = oracle.ref_prefill(sc, xr, Br, Cr, prob["dt"], prob["A"], prob["D"])
    s_y = float(4.0 * np.sqrt(n * np.mean(yref ** 2)) / 127.0)
    q.quamba_hadamard_quantize(y.view(s.batch, s.seqlen, n), s_y, yq)
    # step 1: codes bit for bit; step 2: y within the scan's bar; step 3: bit for bit on the GPU's own y, and within a
    # code of the oracle chain wherever the fp16 difference of y cannot move the transformed value across a boundary
    assert np.array_equal(x.cpu().numpy(), xr) and np.array_equal(B.cpu().numpy(), Br) and np.array_equal(C.cpu().numpy(), Cr)
    yg = y.cpu().numpy()
    err = np.abs(yg.astype(np.float64) - yref).max() / np.abs(yref).max()
    assert err <= 2e-3, err
    got = yq.cpu().numpy()
    assert np.array_equal(got, oracle.hadamard_quantize(yg.reshape(s.batch, s.seqlen, n), s_y))
    chain = oracle.hadamard_quantize(yref.reshape(s.batch, s.seqlen, n).astype(np.float16), s_y)
    diff = np.abs(got.astype(int) - chain.astype(int))
    assert diff.max() <= 2 and (diff > 0).mean() < 0.2, (diff.max(), (diff > 0).mean())
