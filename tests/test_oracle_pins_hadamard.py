"""Pins of oracle/hadamard.py against the Hadamard matrix built by a library (scipy), its algebra, and the
compute-invariance it exists for (Section 4.2).  No GPU."""
import numpy as np
from scipy.linalg import hadamard

import oracle

RNG = np.random.default_rng(8192)


def test_transform_is_the_sylvester_hadamard_matrix():
    for n in (1, 2, 8, 64, 1024):
        H = hadamard(n).astype(np.int64)
        x = RNG.integers(-50, 51, (3, n))                          # small integers: every fp32 operation is exact
        got = oracle.fwht_f32(x)
        assert got.dtype == np.float32
        assert np.array_equal(got.astype(np.int64), x @ H.T)       # row i of the result is H x_i (H is symmetric)
        e = np.zeros(n); e[n // 3] = 1
        assert np.array_equal(oracle.fwht_f32(e), H[:, n // 3])    # column of H from a unit vector: not transposed
    # applied twice: H H = n I, exactly on integers
    x = RNG.integers(-9, 10, (2, 256))
    assert np.array_equal(oracle.fwht_f32(oracle.fwht_f32(x)), 256 * x)


def test_fp32_transform_against_fp64_and_parseval():
    n = 8192
    x = RNG.standard_normal((4, n)).astype(np.float16).astype(np.float64)
    H = hadamard(n).astype(np.float64)
    exact = x @ H
    got = oracle.fwht_f32(x).astype(np.float64)
    # 13 stages, each one rounding of relative size 2^-24 on partial sums that grow like sqrt(2^stage)
    assert np.abs(got - exact).max() <= 13 * 2.0 ** -24 * np.abs(exact).max() * 2
    assert np.allclose((got ** 2).sum(-1), n * (x ** 2).sum(-1), rtol=1e-5)           # Parseval, H^T H = n I


def test_quantizer_and_compute_invariance():
    n = 512
    y = (RNG.standard_normal((6, n)) * np.exp(RNG.standard_normal(n))).astype(np.float16)
    v = oracle.fwht_f32(y.astype(np.float32))
    s = float(np.abs(v).max() / 127.0)
    q = oracle.hadamard_quantize(y, s)
    assert q.dtype == np.int8 and q.shape == y.shape
    r = v.astype(np.float64) / s
    assert np.all(np.abs(q - r) <= 0.5 + 1e-4)                                         # Eq. 1: nearest code
    assert np.abs(q.astype(int)).max() == 127
    # a scale ten times too small saturates at the bounds of Eq. 1
    qs = oracle.hadamard_quantize(y, s / 10)
    assert qs.max() == 127 and qs.min() == -128
    # ties to even: H_2 (1.5, 1) = (2.5, 0.5) with s = 1 -> (2, 0); H_2 (2.5, 1) = (3.5, 1.5) -> (4, 2)
    assert oracle.hadamard_quantize(np.array([1.5, 1.0], np.float16), 1.0).tolist() == [2, 0]
    assert oracle.hadamard_quantize(np.array([2.5, 1.0], np.float16), 1.0).tolist() == [4, 2]
    # the reason for the transform (Section 4.2): W y = (W H^T / n) (H y), so the projection on the de-quantized codes
    # with the offline-fused weight reproduces W y up to the quantization error
    W = RNG.standard_normal((16, n))
    Wh = W @ hadamard(n).astype(np.float64).T / n
    ref = y.astype(np.float64) @ W.T
    got = (q.astype(np.float64) * s) @ Wh.T
    assert np.abs(got - ref).max() <= 0.02 * np.abs(ref).max()
    assert np.allclose(v.astype(np.float64) @ Wh.T, ref, rtol=0, atol=1e-3 * np.abs(ref).max())


def test_paley_factor_and_mixed_orders():
    """Orders 12 * 2^k and 20 * 2^k (the widths 1536, 3072, 5120 of the Mamba blocks): the Paley factor is a Hadamard
    matrix, the transform is the Kronecker product with it on the slow index, exactly on integers."""
    for m in (12, 20):
        H = oracle.paley_hadamard(m)
        assert set(np.unique(H)) == {-1, 1} and np.array_equal(H @ H.T, m * np.eye(m, dtype=np.int64))
        assert np.all(H[0] == 1) and np.array_equal((H - np.eye(m, dtype=np.int64)).T, -(H - np.eye(m, dtype=np.int64)))
    # the order-12 matrix is unique up to equivalence; its first Paley rows from the squares 1 3 4 5 9 mod 11
    H12 = oracle.paley_hadamard(12)
    assert H12[1].tolist() == [-1, 1, -1, 1, -1, -1, -1, 1, 1, 1, -1, 1]
    for n, m in ((48, 12), (1536, 12), (5120, 20), (80, 20)):
        p2 = n // m
        Hn = np.kron(oracle.paley_hadamard(m), hadamard(p2)).astype(np.int64)
        x = RNG.integers(-20, 21, (2, n))
        got = oracle.hadamard_f32(x)
        assert got.dtype == np.float32 and np.array_equal(got.astype(np.int64), x @ Hn.T)
        if n <= 1536:
            assert np.array_equal(Hn @ Hn.T, n * np.eye(n, dtype=np.int64))
        e = np.zeros(n); e[n - 7] = 1
        assert np.array_equal(oracle.hadamard_f32(e), Hn[:, n - 7])        # not transposed (H_12, H_20 are not symmetric)
    # fp32 against fp64 within the rounding bound, Parseval, and the quantizer on top
    n = 5120
    x = RNG.standard_normal((3, n)).astype(np.float16).astype(np.float64)
    Hn = np.kron(oracle.paley_hadamard(20), hadamard(256)).astype(np.float64)
    exact = x @ Hn.T
    got = oracle.hadamard_f32(x).astype(np.float64)
    assert np.abs(got - exact).max() <= (8 + 20) * 2.0 ** -24 * np.abs(exact).max() * 2
    assert np.allclose((got ** 2).sum(-1), n * (x ** 2).sum(-1), rtol=1e-5)
    s = float(np.abs(exact).max() / 127.0)
    q = oracle.hadamard_quantize(x.astype(np.float16), s)
    assert np.all(np.abs(q - exact / s) <= 0.5 + 1e-3) and np.abs(q.astype(int)).max() == 127
    for bad in (24 * 5, 7, 36, 28 * 64):
        try:
            oracle.hadamard_f32(np.zeros(bad))
            assert False, bad
        except ValueError:
            pass
