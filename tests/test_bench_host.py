"""Host-side logic of bench.py (no GPU): the algorithmic work it prices, and that it refuses more than one GPU."""
import os
import subprocess
import sys

import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
sys.path.insert(0, ROOT)
import bench  # noqa: E402


def test_algorithmic_work_of_the_8b_shape():
    """Per token of the Mamba2-8B-shaped layer (H 128, P 64, N 128, G 8, priced chunk 256): the causal half of the
    score products, the carried-state and state-update products, and the bytes of x, B, C, dt and y."""
    s = W.CONFIGS["m2_8b_b4"]
    f16, i8, nbytes = bench.prefill_algorithmic(s)
    assert f16 == 128 * (257 / 2 * 64 + 2 * 128 * 64) == 3149824
    assert i8 == 8 * 257 / 2 * 128 == 131584
    assert nbytes == 128 * 64 + 2 * 8 * 128 + 4 * 128 + 2 * 128 * 64 == 27136
    tokens = s.batch * s.seqlen
    assert tokens == 16384 and abs(2 * f16 * tokens - 103.2e9) < 0.1e9 and abs(nbytes * tokens - 444.6e6) < 0.1e6


def test_pricing_at_the_kernel_chunk_and_executed_work():
    """The same formula at the kernel's 128-token chunks prices fewer intra-chunk products; what the kernel executes
    (whole diagonal tiles, score tiles per head) is the count the committed matrix-core counters show."""
    s = W.CONFIGS["m2_8b_b4"]
    f16, i8, _ = bench.prefill_algorithmic(s)
    k16, k8, _ = bench.prefill_algorithmic(s, bench.KERNEL_CHUNK)
    assert k16 == 128 * (129 / 2 * 64 + 2 * 128 * 64) < f16 and k8 == 8 * 129 / 2 * 128 < i8
    x16, x8 = bench.prefill_executed(s)
    tokens = s.batch * s.seqlen
    assert abs(2 * x16 * tokens - 9.02e10) < 0.01e10 and abs(2 * x8 * tokens - 4.29e10) < 0.01e10
    assert bench.MAMBA1_MIN_SLOTS < bench.MAMBA1_EXECUTED_PER_ELEMENT + 3 * 1.06   # executed slots: 1.06 quarter-rate
    assert bench.CONV_MIN_SLOTS < bench.CONV_EXECUTED_PER_ELEMENT + 3 * 2
    for key, path in bench.TRAFFIC_SOURCE.items():
        assert key in bench.MEASURED_TRAFFIC_BYTES and os.path.exists(os.path.join(ROOT, path))


def test_decode_bytes_of_the_8b_batch():
    s = W.CONFIGS["m2_8b_decode"] if "m2_8b_decode" in W.CONFIGS else W.CONFIGS["m2_8b_b4"].with_(batch=256, seqlen=1)
    b, H, P, N, G = s.batch, s.nheads, s.headdim, s.d_state, s.ngroups
    assert bench.decode_bytes(s) == 2 * 4 * b * H * P * N + b * H * P + 2 * b * G * N + 4 * b * H + 2 * b * H * P
    assert bench.decode_bytes(s, state_bytes=1) < bench.decode_bytes(s) / 3.9
    assert bench.HADAMARD_OPS_PER_VALUE(8192) == 13 + 3


def test_more_than_one_gpu_is_refused():
    r = subprocess.run([sys.executable, os.path.join(ROOT, "bench.py"), "--gpus", "2"], capture_output=True, text=True,
                       timeout=120)
    assert r.returncode == 2 and "ONE GPU" in r.stderr and r.stdout.strip() == ""
