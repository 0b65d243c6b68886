"""GPU checks of the measurement helpers (include/quamba_probe.h): the in-place stream changes every 16-byte piece
exactly as stated, the read-only stream changes nothing, the matrix-core loop reports the work it performs, and the
clock probe reads a plausible shader clock.  They are not steps of the method; bench.py derives the attainable peaks
and the clock under load from them, so their bookkeeping is pinned here."""
import numpy as np
import pytest

pytestmark = pytest.mark.gpu


def test_stream_rmw_adds_one_two_three_four_to_every_piece(gpu_lib):
    import torch
    q = gpu_lib
    for n16 in (1, 255, 256 * 8, 256 * 8 * 3 + 77):        # below one run, whole runs, runs plus a ragged tail
        buf = torch.arange(4 * n16, dtype=torch.int32, device="cuda")
        ref = buf.cpu().numpy().reshape(n16, 4) + np.array([1, 2, 3, 4], np.int32)
        moved = q.quamba_probe_stream_rmw(buf)
        assert moved == 2 * 16 * n16
        assert np.array_equal(buf.cpu().numpy().reshape(n16, 4), ref)


def test_stream_read_leaves_the_buffer_alone(gpu_lib):
    import torch
    q = gpu_lib
    buf = torch.arange(4 * 100001, dtype=torch.int32, device="cuda")
    ref = buf.clone()
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    assert q.quamba_probe_stream_read(buf, sink) == 16 * 100001
    torch.cuda.synchronize()
    assert torch.equal(buf, ref)
    assert int(sink.abs().sum()) == 0


@pytest.mark.parametrize("kind,per_instruction", [(0, 32 * 32 * 16 * 2), (1, 32 * 32 * 32 * 2)])
def test_mfma_probe_reports_its_work(gpu_lib, kind, per_instruction):
    import torch
    q = gpu_lib
    sink = torch.zeros(4, dtype=torch.int32, device="cuda")
    cus = torch.cuda.get_device_properties(0).multi_processor_count
    for uniform in (False, True):
        ops = q.quamba_probe_mfma(kind, 50, sink, waves_per_simd=2, uniform_operands=uniform)
        # grid = compute units x waves_per_simd workgroups of 4 waves; 4 chains per wave; 50 iterations
        waves = cus * 2 * 4
        assert ops % (waves * per_instruction) == 0
        assert ops == waves * per_instruction * 50 * 4
    torch.cuda.synchronize()


def test_clock_probe_reads_a_shader_clock(gpu_lib):
    import torch
    q = gpu_lib
    out = torch.zeros(2, dtype=torch.int64, device="cuda")
    q.quamba_probe_clock(out, 20000)
    torch.cuda.synchronize()
    cycles, ticks = (int(v) for v in out.cpu().numpy())
    assert ticks > 0 and cycles > 0
    mhz = cycles / ticks * 100.0
    assert 500.0 < mhz < 3000.0, mhz


def test_clock_probe_per_xcd(gpu_lib):
    """Eight one-wave workgroups land on eight different XCDs (the hardware deals the ids out in turn) and each
    reads a plausible clock."""
    import torch
    q = gpu_lib
    out = torch.full((8, 3), -1, dtype=torch.int64, device="cuda")
    q.quamba_probe_clock_xcd(out, 20000)
    torch.cuda.synchronize()
    v = out.cpu().numpy()
    assert (v[:, 0] > 0).all() and (v[:, 1] > 0).all()
    mhz = v[:, 0] / v[:, 1] * 100.0
    assert ((mhz > 500.0) & (mhz < 3000.0)).all(), mhz
    assert sorted(int(x) for x in v[:, 2]) == list(range(8)), v[:, 2]
