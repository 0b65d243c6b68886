"""GPU parity of the quantized Hadamard transform (quamba_hadamard_quantize) against the oracle, through the C ABI:
the int8 codes bit for bit (both sides evaluate the same fp32 butterfly network, stride by stride)."""
import numpy as np
import pytest

import oracle
import workloads as W

pytestmark = pytest.mark.gpu


def _scale(sigma, k=4.0):
    """Static scale: k standard deviations of a transformed value map to code 127 (so a few values saturate)."""
    return float(k * np.sqrt((sigma ** 2).sum()) / 127.0)


def _run(q, y16, s_y):
    import torch
    y = torch.from_numpy(y16).cuda()
    out = torch.full(y.shape, 77, dtype=torch.int8, device="cuda")
    q.quamba_hadamard_quantize(y, s_y, out)
    return out.cpu().numpy()


def _check(got, y16, s_y):
    ref = oracle.hadamard_quantize(y16, s_y)
    bad = np.argwhere(got != ref)
    assert bad.size == 0, f"{len(bad)} codes differ, first at {bad[0]}: {got[tuple(bad[0])]} vs {ref[tuple(bad[0])]}"
    return ref


@pytest.mark.parametrize("n", [2, 4, 64, 256, 512, 1024, 2048, 4096, 8192, 16384])
def test_codes_bit_exact_every_order(gpu_lib, n):
    rows = 37                                   # not a multiple of anything the launch uses
    y16, sigma = W.draw_ssd_output(rows, n, seed=n, outlier_frac=0.01 if n >= 256 else 0.0)
    s_y = _scale(sigma, k=3.0)
    ref = _check(_run(gpu_lib, y16, s_y), y16, s_y)
    if n >= 256:
        assert (np.abs(ref.astype(int)) >= 127).any() and len(np.unique(ref)) > 100     # saturation and spread


@pytest.mark.parametrize("n", [48, 80, 1536, 3072, 5120, 12288, 10240])
def test_codes_bit_exact_paley_orders(gpu_lib, n):
    """Orders 12 * 2^k and 20 * 2^k: the block widths of the Mamba models that are no power of two."""
    y16, sigma = W.draw_ssd_output(29, n, seed=n, outlier_frac=0.01 if n >= 256 else 0.0)
    s_y = _scale(sigma, k=3.0)
    ref = _check(_run(gpu_lib, y16, s_y), y16, s_y)
    if n >= 1536:
        assert (np.abs(ref.astype(int)) >= 127).any() and len(np.unique(ref)) > 100


def test_paley_order_unaligned_output_and_2p7b_rows(gpu_lib):
    import torch
    n = 5120
    y16, sigma = W.draw_ssd_output(2048, n, seed=77)
    s_y = _scale(sigma)
    got = _run(gpu_lib, y16, s_y)
    pick = np.arange(0, 2048, 61)
    assert np.array_equal(got[pick], oracle.hadamard_quantize(y16[pick], s_y))
    buf = torch.zeros(7 * n + 1, dtype=torch.int8, device="cuda")
    out = buf[1:].view(7, n)                                   # 1 byte off: byte stores
    gpu_lib.quamba_hadamard_quantize(torch.from_numpy(y16[:7]).cuda(), s_y, out)
    assert np.array_equal(out.cpu().numpy(), oracle.hadamard_quantize(y16[:7], s_y)) and int(buf[0]) == 0


def test_saturation_and_ties(gpu_lib):
    """Rows built so that the transformed values hit exact half-integers and both clamps: a single non-zero input
    c at position j gives +-c in every output; with s_y = 1 the values c = k + 0.5 are ties of Eq. 1."""
    n = 1024
    cs = np.array([0.5, 1.5, 2.5, -0.5, -1.5, -2.5, 126.5, 127.5, -127.5, -128.5, 300.0, -300.0, 0.0, 127.0, -128.0])
    y = np.zeros((len(cs), n), np.float16)
    for r, c in enumerate(cs):
        y[r, (37 * r + 5) % n] = c
    ref = _check(_run(gpu_lib, y, 1.0), y, 1.0)
    assert ref.max() == 127 and ref.min() == -128
    assert set(np.unique(np.abs(ref[0]))) == {0} and set(np.unique(np.abs(ref[1]))) == {2}     # ties to even


def test_subnormal_and_extreme_fp16_inputs(gpu_lib):
    """fp16 subnormals (below 6.1e-5) and the largest finite fp16 values go through the first butterfly stage, which
    the kernel computes from the packed halves directly; the scale is chosen so that the subnormals decide codes."""
    n = 4096
    g = np.random.default_rng(5)
    bits = g.integers(0, 0x0400, size=(9, n), dtype=np.uint16) | (g.integers(0, 2, size=(9, n), dtype=np.uint16) << 15)
    y = bits.view(np.float16)                                   # every value subnormal or zero
    assert (np.abs(y.astype(np.float64)) < 6.2e-5).all()
    s_y = float(np.abs(oracle.fwht_f32(y.astype(np.float32))).max() / 100.0)
    ref = _check(_run(gpu_lib, y, s_y), y, s_y)
    assert len(np.unique(ref)) > 50
    big = np.where(g.integers(0, 2, size=(4, n)) == 1, 65504.0, -65504.0).astype(np.float16)
    big[:, ::7] = np.float16(0.00390625)
    s_big = float(65504.0 * n / 4 / 127.0)
    _check(_run(gpu_lib, big, s_big), big, s_big)


def test_unaligned_pointers_and_leading_axes(gpu_lib):
    """A view that starts 2 bytes into an allocation takes the path without 16-byte loads; leading axes flatten."""
    import torch
    n = 2048
    y16, sigma = W.draw_ssd_output(3 * 5 + 1, n, seed=3)
    s_y = _scale(sigma)
    flat = torch.from_numpy(y16.reshape(-1)).cuda()
    view = flat[1:1 + 15 * n].view(3, 5, n)
    buf = torch.zeros(15 * n + 3, dtype=torch.int8, device="cuda")
    out = buf[3:].view(3, 5, n)
    gpu_lib.quamba_hadamard_quantize(view, s_y, out)
    ref = oracle.hadamard_quantize(y16.reshape(-1)[1:1 + 15 * n].reshape(3, 5, n), s_y)
    assert (out.cpu().numpy() == ref).all()
    assert (buf[:3] == 0).all()


def test_zero_rows_and_bad_arguments(gpu_lib):
    import torch
    y = torch.zeros((0, 1024), dtype=torch.float16, device="cuda")
    gpu_lib.quamba_hadamard_quantize(y, 1.0, torch.zeros((0, 1024), dtype=torch.int8, device="cuda"))
    y = torch.zeros((2, 36), dtype=torch.float16, device="cuda")
    with pytest.raises(gpu_lib.QuambaError):
        gpu_lib.quamba_hadamard_quantize(y, 1.0, torch.zeros((2, 36), dtype=torch.int8, device="cuda"))
    y = torch.zeros((2, 64), dtype=torch.float16, device="cuda")
    for bad in (0.0, -1.0, float("inf"), float("nan")):
        with pytest.raises(gpu_lib.QuambaError):
            gpu_lib.quamba_hadamard_quantize(y, bad, torch.zeros((2, 64), dtype=torch.int8, device="cuda"))


def test_bench_size_sampled_rows(gpu_lib):
    """The 8B layer's output at the prefill batch the bench times: 16384 tokens x 8192 channels, 96 rows spread over
    the launch (first, last, a stride in between) checked bit for bit."""
    rows, n = 16384, 8192
    y16, sigma = W.draw_ssd_output(rows, n, seed=11)
    s_y = _scale(sigma)
    got = _run(gpu_lib, y16, s_y)
    pick = np.unique(np.concatenate([np.arange(0, rows, 173), [rows - 1]]))
    ref = oracle.hadamard_quantize(y16[pick], s_y)
    assert (got[pick] == ref).all()
    # every row was written: the fill value 77 survives nowhere as a whole row
    assert not (got == 77).all(axis=1).any()
