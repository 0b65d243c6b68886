"""GPU parity of quamba_ssd_prefill against the fp64 oracle (through the C ABI)."""
import numpy as np
import pytest

import oracle
import workloads as W
from helpers import make_problem, to_shape, host_scales

pytestmark = pytest.mark.gpu

Y_TOL = 2e-3      # max|y_gpu - y_ref| <= Y_TOL * max|y_ref|   (fp16 y, fp32 accumulation)
H_TOL = 1e-4      # max|h_gpu - h_ref| <= H_TOL * max|h_ref|   (final fp32 state)
# The same bar inside every (head cluster, channel range) cell of the sort-and-cluster table (Section 4.1): the largest
# error of a cell against the largest reference output OF THAT CELL.  A cell with a small scale is invisible in the
# global norm (outlier channels are 20x larger), so a wrong scale lookup for it would pass there; here it is a 100 %
# error.  The error sources are relative to the outputs they belong to (fp16 rounding of y, of the narrowed scores and
# of the carried state), so the cell-wise ratio obeys the same budget as the global one.
CELL_TOL = 2e-3
REL_FLOOR = 1e-4  # element-wise relative error is reported with |y_ref| floored at REL_FLOOR * max|y_ref| (information)


def run_prefill(q, s, sc, prob, flags=0, init_state=None, want_state=True, chunk=None):
    import torch
    dsc = q.DeviceScales(host_scales(q, sc))
    shape = to_shape(q, s, flags=flags, **({} if chunk is None else {"chunk": chunk}))
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    y = torch.full((s.batch, s.seqlen, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
    fin = torch.full((s.batch, s.nheads, s.headdim, s.d_state), float("nan"), device="cuda") if want_state else None
    init = torch.from_numpy(init_state.astype(np.float32)).cuda() if init_state is not None else None
    ws_bytes = q.quamba_ssd_prefill_workspace_size(shape)
    ws = torch.empty(max(ws_bytes, 1), dtype=torch.uint8, device="cuda")
    q.quamba_ssd_prefill(shape, dsc, t["x"], t["B"], t["C"], t["dt"], t["A"], t["D"], init, y, fin, ws)
    torch.cuda.synchronize()
    return y.cpu().numpy().astype(np.float64), (fin.cpu().numpy().astype(np.float64) if want_state else None)


def cell_errors(yg, yref, cells):
    """Largest |y_gpu - y_ref| of every scale cell over the largest |y_ref| of that cell.  y arrays [..., H, P] (any
    leading axes), cells [H, P] integer cell index of every (head, channel).  Returns (worst ratio, its cell)."""
    H, P = cells.shape
    d = np.abs(yg - yref).reshape(-1, H, P).max(axis=0)
    m = np.abs(yref).reshape(-1, H, P).max(axis=0)
    worst, where = 0.0, -1
    for c in np.unique(cells):
        sel = cells == c
        if m[sel].max() > 0:
            r = d[sel].max() / m[sel].max()
            if r > worst:
                worst, where = float(r), int(c)
    return worst, where


def check(yg, hg, yref, href, what="", cells=None):
    """cells: [H,P] cell index table for y arrays shaped [..., H, P]; adds the cell-wise bar."""
    assert np.isfinite(yg).all(), f"{what}: non-finite y"
    ymax = np.abs(yref).max()
    ey = np.abs(yg - yref).max() / ymax
    assert ymax < 6e4, "workload overflows fp16"
    rel = np.abs(yg - yref) / np.maximum(np.abs(yref), REL_FLOOR * ymax)
    p999 = np.quantile(rel.ravel()[:: max(1, rel.size // 4_000_000)], 0.999)
    msg = (f"{what}: y err {ey:.3e}, element-wise relative (floor {REL_FLOOR:g} max) max {rel.max():.3e} "
           f"99.9% {p999:.3e}")
    del rel
    if cells is not None:
        ec, where = cell_errors(yg, yref, cells)
        msg += f", worst cell {ec:.3e} (cell {where})"
        assert ec <= CELL_TOL, msg
    eh = None
    if hg is not None:
        assert np.isfinite(hg).all(), f"{what}: non-finite state"
        eh = np.abs(hg - href).max() / np.abs(href).max()
        msg += f", state err {eh:.3e}"
    print(msg)
    assert ey <= Y_TOL, msg
    if eh is not None:
        assert eh <= H_TOL, msg
    return ey, eh


GENERIC = 0x1
NO_SPLIT = 0x4    # one workgroup per head even for small batches (the default splits a head's channels over two)


@pytest.mark.parametrize("flags", [0, GENERIC])
def test_tiny_config(gpu_lib, flags):
    """configs[0]: batch 1, seqlen 256, 8 heads x 64, d_state 16, chunk 64, 1x4 clusters, 2 outlier channels."""
    s = W.CONFIGS["tiny"]
    sc, prob, _ = make_problem(s, 0)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    yg, hg = run_prefill(gpu_lib, s, sc, prob, flags)
    check(yg, hg, yref, href, f"tiny flags={flags}", cells=oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups))


@pytest.mark.parametrize("flags", [0, GENERIC, NO_SPLIT])
@pytest.mark.parametrize("with_D", [True, False])
def test_130m_shape(gpu_lib, flags, with_D):
    """configs[1]: Mamba2-130M-shaped layer, seqlen 2048, 24 heads, d_state 128, chunk 256, 4x4 clusters."""
    s = W.CONFIGS["m2_130m"]
    sc, prob, _ = make_problem(s, 1, with_D=with_D)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    yg, hg = run_prefill(gpu_lib, s, sc, prob, flags)
    check(yg, hg, yref, href, f"130m flags={flags} D={with_D}",
          cells=oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups))


@pytest.mark.parametrize("flags", [0, GENERIC, NO_SPLIT])
@pytest.mark.parametrize("L", [1, 5, 63, 257, 300, 777])
def test_ragged_lengths_and_init_state(gpu_lib, flags, L):
    """Sequence lengths that are not multiples of the chunk (several tiles + a ragged tail), with an initial state."""
    s = W.CONFIGS["m2_8b_b1"].with_(batch=2, seqlen=L, nheads=16, ngroups=2)
    sc, prob, _ = make_problem(s, 2, calib_tokens=256)
    h0 = W.draw_state(s, 2).astype(np.float64)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"],
                                       init_state=h0.astype(np.float32).astype(np.float64))
    yg, hg = run_prefill(gpu_lib, s, sc, prob, flags, init_state=h0)
    check(yg, hg, yref, href, f"L={L} flags={flags}", cells=oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups))
    if flags != GENERIC:  # without the final state the matrix-core path takes its single-term state update
        yg, _ = run_prefill(gpu_lib, s, sc, prob, flags, init_state=h0, want_state=False)
        check(yg, None, yref, None, f"L={L} flags={flags}, no final state")


NO_SEQ_SPLIT = 0x10


@pytest.mark.parametrize("H,G,L,flags", [
    (24, 1, 2048, 0),          # 130M shape: 8 segments of 2 chunks, two workgroups per head and segment
    (24, 1, 2333, 0),          # 19 chunks: 7 segments of 3 chunks, the last one a single ragged chunk
    (24, 1, 1100, NO_SPLIT),   # 9 chunks, whole heads: 3 segments of 3 chunks, the last chunk ragged
    (128, 8, 4096, 0),         # 8B shape at batch 1: whole heads, 4 segments
    (80, 1, 1500, 0),          # 12 chunks, 80 heads: 6 segments of whole heads, ragged last chunk
])
def test_sequence_split_against_the_oracle_and_the_unsplit_launch(gpu_lib, H, G, L, flags):
    """Short batches are cut along the sequence (a state pass, then one set of workgroups per segment).  With an
    initial state and the final state: against the oracle, and against the unsplit launch of the same library, whose
    outputs differ only where an fp16 rounding flips (the start states of the segments are combined in another
    order than the chunk-by-chunk walk forms them)."""
    q = gpu_lib
    s = W.CONFIGS["m2_8b_b1"].with_(batch=1, seqlen=L, nheads=H, ngroups=G)
    assert q.quamba_ssd_prefill_workspace_size(to_shape(q, s, flags=flags)) > 0
    assert q.quamba_ssd_prefill_workspace_size(to_shape(q, s, flags=flags | NO_SEQ_SPLIT)) == 0
    sc, prob, _ = make_problem(s, 31, calib_tokens=512)
    h0 = W.draw_state(s, 31).astype(np.float32)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"],
                                       init_state=h0.astype(np.float64))
    cells = oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups)
    for want_state in (True, False):
        yg, hg = run_prefill(q, s, sc, prob, flags, init_state=h0, want_state=want_state)
        check(yg, hg, yref, href if want_state else None, f"split H={H} L={L} flags={flags} state={want_state}", cells=cells)
        yu, hu = run_prefill(q, s, sc, prob, flags | NO_SEQ_SPLIT, init_state=h0, want_state=want_state)
        flipped = np.count_nonzero(yg != yu)
        assert flipped <= 1e-2 * yg.size, f"{flipped} of {yg.size} outputs differ from the unsplit launch"
        assert np.abs(yg - yu).max() <= 2.0 ** -9 * np.abs(yu).max()
        if want_state:
            assert np.abs(hg - hu).max() <= 2e-5 * np.abs(hu).max()


def _random_split_cases(n, seed):
    rng = np.random.default_rng(seed)
    cases = []
    for _ in range(n):
        G = int(rng.choice([1, 2, 4]))
        H = G * int(rng.choice([1, 2, 3, 5]))
        cases.append((int(rng.choice([1, 1, 2, 3])), H, G, int(rng.integers(1024, 3000)),
                      int(rng.choice([0, 0, 0x2, NO_SPLIT, NO_SPLIT | 0x8, 0x8, 0x2 | 0x8])), int(rng.integers(1, 10 ** 6)),
                      bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return cases


@pytest.mark.parametrize("b,H,G,L,flags,seed,want_state,use_init", _random_split_cases(24, 2503))
def test_sequence_split_on_drawn_shapes(gpu_lib, b, H, G, L, flags, seed, want_state, use_init):
    """Drawn small batches of 1024..3000 tokens, all of which the plan cuts along the sequence (state-pass kernel with
    whole heads or channel halves, single- or two-term state update, odd and even chunk counts per segment, ragged
    last chunks), with step sizes spread over e^-3 .. e^3 per head: against the oracle."""
    q = gpu_lib
    s = W.CONFIGS["m2_130m"].with_(batch=b, seqlen=L, nheads=H, ngroups=G)
    assert q.quamba_ssd_prefill_workspace_size(to_shape(q, s, flags=flags)) > 0
    sc, prob, _ = make_problem(s, seed, calib_tokens=128)
    rng = np.random.default_rng(seed)
    prob = dict(prob)
    prob["dt"] = np.minimum(prob["dt"] * np.exp(rng.uniform(-3, 3.0, size=H)).astype(np.float32)[None, None, :],
                            20.0).astype(np.float32)
    h0 = (0.05 * rng.standard_normal((b, H, s.headdim, s.d_state))).astype(np.float32) if use_init else None
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"],
                                       init_state=None if h0 is None else h0.astype(np.float64), want_state=want_state)
    yg, hg = run_prefill(q, s, sc, prob, flags, init_state=h0, want_state=want_state)
    check(yg, hg, yref, href if want_state else None,
          f"drawn split b={b} H={H} G={G} L={L} flags={flags} state={want_state} init={use_init}")


def test_state_updated_in_place_on_a_shape_that_would_be_split(gpu_lib):
    """final_state may be the init_state buffer.  With a sequence split the last segment would write it while the
    first still reads it, so such a call takes the unsplit launch: bit for bit the flagged launch with two buffers."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_130m"]
    sc, prob, _ = make_problem(s, 33, calib_tokens=512)
    dsc = q.DeviceScales(host_scales(q, sc))
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    h0 = torch.from_numpy(W.draw_state(s, 33)).cuda()
    ws = torch.empty(q.quamba_ssd_prefill_workspace_size(to_shape(q, s)), dtype=torch.uint8, device="cuda")

    def run(flags, init, fin):
        y = torch.full((s.batch, s.seqlen, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
        q.quamba_ssd_prefill(to_shape(q, s, flags=flags), dsc, t["x"], t["B"], t["C"], t["dt"], t["A"], t["D"], init, y,
                             fin, ws)
        torch.cuda.synchronize()
        return y.cpu().numpy().view(np.uint16), fin.cpu().numpy()

    y_ref, h_ref = run(NO_SEQ_SPLIT, h0.clone(), torch.empty_like(h0))
    state = h0.clone()
    y_inp, h_inp = run(0, state, state)
    assert np.array_equal(y_inp, y_ref) and np.array_equal(h_inp, h_ref)


def test_sequence_split_without_a_usable_workspace_takes_the_unsplit_launch(gpu_lib):
    """A missing, short or misaligned workspace is not an error: the call runs unsplit, bit for bit like the flag."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_130m"]
    sc, prob, _ = make_problem(s, 32, calib_tokens=512)
    dsc = q.DeviceScales(host_scales(q, sc))
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    need = q.quamba_ssd_prefill_workspace_size(to_shape(q, s))
    assert need > 0

    def run(flags, ws):
        y = torch.full((s.batch, s.seqlen, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
        q.quamba_ssd_prefill(to_shape(q, s, flags=flags), dsc, t["x"], t["B"], t["C"], t["dt"], t["A"], t["D"], None, y,
                             None, ws)
        torch.cuda.synchronize()
        return y.cpu().numpy()

    ref = run(NO_SEQ_SPLIT, None)
    assert np.isfinite(ref.astype(np.float64)).all()
    buf = torch.empty(need + 64, dtype=torch.uint8, device="cuda")
    assert buf.data_ptr() % 16 == 0
    for ws in (None, buf[:need - 16], buf[4:4 + need]):
        assert np.array_equal(run(0, ws).view(np.uint16), ref.view(np.uint16))
    split = run(0, buf[:need])
    assert np.count_nonzero(split.view(np.uint16) != ref.view(np.uint16)) <= 1e-2 * ref.size


@pytest.mark.parametrize("P,N,H,G,Q", [(64, 64, 4, 2, 128), (32, 128, 4, 1, 64), (64, 32, 6, 3, 256), (48, 24, 4, 2, 32),
                                       (16, 8, 2, 1, 16)])
def test_other_shapes(gpu_lib, P, N, H, G, Q):
    s = W.LayerShape("t", 2, 200, H, P, N, G, Q, 2, 3)
    sc, prob, _ = make_problem(s, 3, calib_tokens=256)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    yg, hg = run_prefill(gpu_lib, s, sc, prob)
    check(yg, hg, yref, href, f"P{P} N{N} H{H} G{G} Q{Q}")


@pytest.mark.parametrize("seed", [101, 102, 103, 104, 105, 106, 107, 108])
def test_seeded_random_problems(gpu_lib, seed):
    """Seeded draws of batch, length, heads, groups, clusters, D, initial state, final state and launch shape on the
    matrix-core path (headdim 64, d_state 128): lengths from one token to a dozen chunks with ragged tails."""
    rng = np.random.default_rng(seed)
    G = int(rng.choice([1, 2, 4]))
    H = G * int(rng.choice([1, 2, 3, 6]))
    L = int(rng.integers(1, 1500))
    s = W.LayerShape(f"r{seed}", int(rng.integers(1, 4)), L, H, 64, 128, G, 256, int(rng.choice([1, 2, 4])),
                     int(rng.choice([1, 2, 4])))
    s = s.with_(m=min(s.m, H // G))
    sc, prob, _ = make_problem(s, seed, calib_tokens=256, with_D=bool(rng.integers(0, 2)))
    h0 = W.draw_state(s, seed).astype(np.float64) if rng.integers(0, 2) else None
    want_state = bool(rng.integers(0, 2))
    flags = int(rng.choice([0, NO_SPLIT]))
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"],
                                       init_state=None if h0 is None else h0.astype(np.float32).astype(np.float64),
                                       want_state=want_state)
    yg, hg = run_prefill(gpu_lib, s, sc, prob, flags, init_state=h0, want_state=want_state)
    check(yg, hg, yref, href if want_state else None,
          f"seed {seed}: b={s.batch} L={L} H={H} G={G} m={s.m} n={s.n} state={want_state} flags={flags}",
          cells=oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups))


@pytest.mark.parametrize("batch,H,G,L", [(8, 48, 8, 300), (5, 56, 7, 200), (3, 96, 8, 130)])
def test_more_heads_than_compute_units(gpu_lib, batch, H, G, L):
    """More (sequence, head) pairs than compute units: one workgroup per head, with the XCD-aware workgroup map
    (number of (sequence, group) units a multiple of 8) and without it."""
    s = W.LayerShape("wide", batch, L, H, 64, 128, G, 256, 2, 2)
    sc, prob, _ = make_problem(s, 20 + batch, calib_tokens=256)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    yg, hg = run_prefill(gpu_lib, s, sc, prob)
    check(yg, hg, yref, href, f"b={batch} H={H} G={G} L={L}")
    yg, _ = run_prefill(gpu_lib, s, sc, prob, want_state=False)
    check(yg, None, yref, None, f"b={batch} H={H} G={G} L={L}, no final state")


def test_exact_integer_case(gpu_lib):
    """A = 0, dt = 1, all scales 1, small integers: y is an exact integer (< 2048, exact in fp16) and so is the state."""
    rng = np.random.default_rng(8)
    s = W.LayerShape("int", 1, 512, 16, 64, 128, 2, 256, 1, 1)
    prob = {"x": rng.integers(-1, 2, (1, 512, 16, 64), dtype=np.int8),
            "B": (rng.random((1, 512, 2, 128)) < 0.02).astype(np.int8) * rng.choice([-1, 1], (1, 512, 2, 128)).astype(np.int8),
            "C": (rng.random((1, 512, 2, 128)) < 0.02).astype(np.int8) * rng.choice([-1, 1], (1, 512, 2, 128)).astype(np.int8),
            "dt": np.ones((1, 512, 16), np.float32), "A": np.zeros(16, np.float32),
            "D": rng.integers(-2, 3, 16).astype(np.float32)}
    sc = oracle.Scales.ones(2, 8, 64)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    assert np.abs(yref).max() < 2048 and np.abs(yref).max() > 4
    for flags in (0, GENERIC, NO_SPLIT):
        yg, hg = run_prefill(gpu_lib, s, sc, prob, flags)
        assert np.array_equal(yg, yref) and np.array_equal(hg, href), f"flags={flags}"


def test_dt_zero_and_permutation_invariance(gpu_lib):
    s = W.CONFIGS["m2_130m"].with_(seqlen=512)
    sc, prob, _ = make_problem(s, 5, calib_tokens=256)
    p0 = dict(prob); p0["dt"] = np.zeros_like(prob["dt"])
    yg, hg = run_prefill(gpu_lib, s, sc, p0)
    tab = oracle.x_scale_table(sc, s.nheads, s.headdim, s.ngroups).astype(np.float64)
    want = prob["D"].astype(np.float64)[None, None, :, None] * tab * prob["x"]
    # dt = 0: y = D x.  The MFMA kernel carries D as one fp16 coefficient on the diagonal of its score matrix, so the
    # result is D x to two fp16 roundings (coefficient and output), element by element; the state stays exactly zero.
    assert np.all(np.abs(yg - want) <= 2.0 ** -10 * np.abs(want) + 1e-12) and not hg.any()
    yq, hq = run_prefill(gpu_lib, s, sc, p0, flags=GENERIC)
    assert np.array_equal(yq, want.astype(np.float16).astype(np.float64)) and not hq.any()
    # swap two heads of the same head cluster and reverse the channels of one channel range: y moves with them
    he = sc.head_cluster_end.reshape(s.ngroups, s.m)[0]
    lo = 0
    pair = None
    for e in he:
        if e - lo >= 2:
            pair = (lo, lo + 1); break
        lo = e
    assert pair is not None
    hp = np.arange(s.nheads); hp[list(pair)] = hp[list(pair)][::-1]
    i_cl = int(np.searchsorted(he, pair[0], side="right"))
    c_end = sc.chan_cluster_end.reshape(s.ngroups, s.m, s.n)[0, i_cl]
    cp = np.arange(s.headdim); cp[:c_end[0]] = cp[:c_end[0]][::-1]
    p2 = dict(prob)
    p2["x"] = np.ascontiguousarray(prob["x"][:, :, hp][..., cp]); p2["dt"] = np.ascontiguousarray(prob["dt"][:, :, hp])
    p2["A"] = prob["A"][hp].copy(); p2["D"] = prob["D"][hp].copy()
    y1, h1 = run_prefill(gpu_lib, s, sc, prob)
    y2, h2 = run_prefill(gpu_lib, s, sc, p2)
    assert np.array_equal(y2, y1[:, :, hp][..., cp]) and np.array_equal(h2, h1[:, hp][:, :, cp])


@pytest.mark.parametrize("flags", [0, NO_SPLIT, GENERIC])
def test_dt_zero_checks_every_scale_cell_of_the_8_group_shape(gpu_lib, flags):
    """dt = 0 makes y = D x exactly (Section 3.2: B-dot = dt B vanishes, the state stays zero), element by element, so
    every output is one look-up in the (state group, head cluster, channel range) table times a code: the
    (g m + i) n + j indexing with 8 groups and 4 x 4 cells per group is checked cell by cell, on the matrix-core kernel
    with and without the channel split and on the generic kernel, and on the decode step of both state formats."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_b1"].with_(seqlen=300)
    assert s.ngroups == 8 and s.m == 4 and s.n == 4
    sc, prob, r = make_problem(s, 7, calib_tokens=256)
    assert len(np.unique(sc.x_scales)) > 100          # the 128 cells carry different scales
    p0 = dict(prob); p0["dt"] = np.zeros_like(prob["dt"])
    tab = oracle.x_scale_table(sc, s.nheads, s.headdim, s.ngroups).astype(np.float64)
    want = prob["D"].astype(np.float64)[None, None, :, None] * tab * prob["x"]
    yg, hg = run_prefill(q, s, sc, p0, flags=flags)
    assert not hg.any()
    if flags == GENERIC:
        assert np.array_equal(yg, want.astype(np.float16).astype(np.float64))
    else:   # the skip coefficient is one fp16 factor on the matrix core: two fp16 roundings per output
        assert np.all(np.abs(yg - want) <= 2.0 ** -10 * np.abs(want) + 1e-12)
    cells = oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups)
    ec, _ = cell_errors(yg, want, cells)
    assert ec <= 2.0 ** -10
    if flags != 0:
        return
    # one decode step with dt = 0 on a zero state: y = D x again, fp32 state and 8-bit cached state
    dsc = q.DeviceScales(host_scales(q, sc))
    x1 = torch.from_numpy(np.ascontiguousarray(prob["x"][:, 0])).cuda()
    B1 = torch.from_numpy(np.ascontiguousarray(prob["B"][:, 0])).cuda()
    C1 = torch.from_numpy(np.ascontiguousarray(prob["C"][:, 0])).cuda()
    dt1 = torch.zeros((1, s.nheads), device="cuda")
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    y1 = torch.empty((1, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    st = torch.zeros((1, s.nheads, s.headdim, s.d_state), device="cuda")
    q.quamba_ssd_decode_step(to_shape(q, s), dsc, x1, B1, C1, dt1, A, D, st, y1)
    w1 = want[:, 0]

    def close(y):   # one fp16 rounding of a product formed in fp32
        return np.all(np.abs(y.cpu().numpy().astype(np.float64) - w1) <= 2.0 ** -11 * np.abs(w1) * (1 + 1e-3) + 1e-12)
    assert close(y1) and not st.cpu().numpy().any()
    ss = np.ones((s.ngroups * s.m * s.n, s.d_state), np.float32)
    qs = torch.zeros((1, s.nheads, s.headdim, s.d_state), dtype=torch.int8, device="cuda")
    q.quamba_ssd_decode_step_q8(to_shape(q, s), dsc, torch.from_numpy(ss).cuda(), x1, B1, C1, dt1, A, D, qs, y1)
    assert close(y1) and not qs.cpu().numpy().any()


def test_tiny_scales_take_the_epilogue_skip_term(gpu_lib):
    """With s_B s_C ~ 1e-10 the skip coefficient D / (s_B s_C 128) leaves the fp16 range, so the MFMA kernel must add
    D x in its epilogue instead of through the matrix core; y is then dominated by D x and must still match."""
    s = W.CONFIGS["m2_130m"].with_(seqlen=300)
    sc, prob, _ = make_problem(s, 9, calib_tokens=256)
    sc.B_scales = (sc.B_scales * 0 + 1e-5).astype(np.float32)
    sc.C_scales = (sc.C_scales * 0 + 1e-5).astype(np.float32)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    yg, hg = run_prefill(gpu_lib, s, sc, prob)
    check(yg, hg, yref, href, "tiny B/C scales")
    # and the opposite extreme: large B/C scales, D = 0 (pure SSM output)
    sc.B_scales = (sc.B_scales * 0 + 0.5).astype(np.float32)
    sc.C_scales = (sc.C_scales * 0 + 0.25).astype(np.float32)
    sc.x_scales = (sc.x_scales * 1e-3).astype(np.float32)
    p0 = dict(prob); p0["D"] = None
    yref, href, _ = oracle.ref_prefill(sc, p0["x"], p0["B"], p0["C"], p0["dt"], p0["A"], None)
    yg, hg = run_prefill(gpu_lib, s, sc, p0)
    check(yg, hg, yref, href, "large B/C scales, no D")


def test_extreme_decay_takes_the_per_element_diagonal(gpu_lib):
    """Decay of more than 2^64 across a 32-token block: the row/column factorisation of the diagonal block's weights
    would leave the fp32 range, so the kernel must fall back to one exponential per element.  Heads alternate between
    mild and extreme decay (dt scaled by 40 on odd heads), both with and without the final state."""
    s = W.CONFIGS["m2_130m"].with_(seqlen=600)
    sc, prob, _ = make_problem(s, 12, calib_tokens=256)
    p1 = dict(prob)
    dt = prob["dt"].copy()
    dt[:, :, 1::2] *= 40.0
    p1["dt"] = dt
    a_log2 = -(dt * prob["A"][None, None, :]) * 1.4426950408889634      # decay per token, log2 units
    blk = a_log2[:, :576].reshape(s.batch, 18, 32, s.nheads).sum(axis=2)
    assert blk[:, :, 1::2].min() > 64.0 and blk[:, :, 0::2].max() < 64.0  # both branches are exercised
    for want_state, flags in ((True, 0), (False, 0), (False, NO_SPLIT)):
        yref, href, _ = oracle.ref_prefill(sc, p1["x"], p1["B"], p1["C"], p1["dt"], p1["A"], p1["D"],
                                           want_state=want_state)
        yg, hg = run_prefill(gpu_lib, s, sc, p1, flags=flags, want_state=want_state)
        check(yg, hg, yref, href if want_state else None, f"extreme decay, state={want_state}, flags={flags}")


@pytest.mark.parametrize("L", [700, 668, 2333])
def test_final_state_when_only_the_last_tokens_count(gpu_lib, L):
    """Decay of 2^-50 and more per token on every other head: the final state of such a head is the last token's
    term alone, sitting at the end of a ragged chunk behind a block prefix sum of thousands (log2 units).  Its weight
    is exp2 of the sum of dt*A over the tokens behind it, here exactly 1; formed as a difference of two prefix sums it
    would be off by their rounding (1e-4 of the state, the whole spec allowance).  The bar here is half of the
    allowance; what remains is the rounding of the two-term product (at most 2^-14).  L = 2333 takes the sequence
    split, whose state-pass kernel forms the same weights."""
    s = W.CONFIGS["m2_130m"].with_(seqlen=L, nheads=8)
    sc, prob, _ = make_problem(s, 45, calib_tokens=256)
    p1 = dict(prob)
    dt = prob["dt"].copy()
    dt[:, :, 1::2] = np.clip(dt[:, :, 1::2] * 60.0, 2.5, 15.0)
    p1["dt"] = dt.astype(np.float32)
    p1["A"] = prob["A"].copy()
    p1["A"][1::2] = -13.0
    h0 = W.draw_state(s, 45).astype(np.float32)
    yref, href, _ = oracle.ref_prefill(sc, p1["x"], p1["B"], p1["C"], p1["dt"], p1["A"], p1["D"],
                                       init_state=h0.astype(np.float64))
    for flags in (0, NO_SPLIT):
        yg, hg = run_prefill(gpu_lib, s, sc, p1, flags=flags, init_state=h0)
        check(yg, hg, yref, href, f"last tokens only, L={L}, flags={flags}")
        for h in range(1, s.nheads, 2):
            e = np.abs(hg[:, h] - href[:, h]).max() / np.abs(href[:, h]).max()
            assert e <= 5e-5, f"head {h}: state err {e:.2e}"


@pytest.mark.parametrize("seed", [26, 626, 654, 727])
def test_step_sizes_that_jump_inside_a_chunk(gpu_lib, seed):
    """Step sizes of 4..16 on the first tokens of every chunk and one small step size (0.01..0.3) from a drawn
    position on, A drawn from -0.5 .. -16 per head: the chunk's prefix sums reach thousands to tens of thousands (log2
    units) in front of a stretch whose own decay is mild, so what that stretch carries and adds is what the final
    state consists of.  Every exponent over such a stretch has to come from sums over the stretch itself (the block's
    own prefix sums, the blocks' totals); taken as a difference of the chunk's prefix sums it is off by their rounding.
    The four seeds are the worst of 1500 draws for a build that took those differences (final state off by 1.8e-4 ..
    2.8e-4 of its maximum; the bar is 1e-4)."""
    rng = np.random.default_rng(seed)
    L = int(rng.choice([256, 300, 640]))
    s = W.CONFIGS["m2_130m"].with_(seqlen=L, nheads=4)
    sc, prob, _ = make_problem(s, 7, calib_tokens=128)
    p1 = dict(prob)
    dt = rng.uniform(4.0, 15.9, (1, L, s.nheads))
    dt[:, (np.arange(L) % 128) >= int(rng.integers(40, 127)), :] = rng.uniform(0.01, 0.3)
    p1["dt"] = dt.astype(np.float32)
    p1["A"] = (-rng.uniform(0.5, 16.0, s.nheads)).astype(np.float32)
    yref, href, _ = oracle.ref_prefill(sc, p1["x"], p1["B"], p1["C"], p1["dt"], p1["A"], p1["D"])
    for want_state, flags in ((True, 0), (True, NO_SPLIT), (False, 0)):
        yg, hg = run_prefill(gpu_lib, s, sc, p1, flags=flags, want_state=want_state)
        check(yg, hg, yref, href if want_state else None, f"jumping step sizes, seed={seed}, state={want_state}, flags={flags}")
        if want_state:
            assert np.abs(hg - href).max() <= 5e-5 * np.abs(href).max()


@pytest.mark.parametrize("mode", [0, 1, 2, 3, 4])
@pytest.mark.parametrize("seed", [1, 2, 3])
def test_drawn_step_size_patterns(gpu_lib, mode, seed):
    """Step-size patterns far from the workloads' (which draw every token alike), on drawn lengths, head counts and A:
    0: every token tiny (1e-4..0.1) or huge (2..16) at a drawn rate; 1: the same per 32-token block; 2: huge, then one
    small value from a drawn position of every chunk on; 3: ordinary step sizes scaled by 0.2..30 with stretches of 16
    tokens set to zero, and A = 0 on some heads; 4: 1e-5..2e-3 everywhere (almost no decay over the whole sequence),
    A = 0 on some heads.  Outputs and the final state against the oracle, lengths up to the sequence split."""
    rng = np.random.default_rng(1000 * mode + seed)
    L = int(rng.choice([256, 300, 511, 640, 1100, 1500])); H = int(rng.choice([2, 4, 8]))
    s = W.CONFIGS["m2_130m"].with_(seqlen=L, nheads=H)
    sc, prob, _ = make_problem(s, int(rng.integers(1, 10 ** 6)), calib_tokens=128)
    p1 = dict(prob)
    tiny = lambda: rng.uniform(1e-4, 0.1, (1, L, H))
    huge = lambda: rng.uniform(2.0, 15.9, (1, L, H))
    if mode == 0:
        dt = np.where(rng.random((1, L, H)) < rng.uniform(0.05, 0.95), huge(), tiny())
    elif mode == 1:
        pick = np.repeat(rng.random((1, (L + 31) // 32, H)) < 0.5, 32, axis=1)[:, :L]
        dt = np.where(pick, huge(), tiny())
    elif mode == 2:
        dt = rng.uniform(4.0, 15.9, (1, L, H))
        dt[:, (np.arange(L) % 128) >= int(rng.integers(40, 127)), :] = rng.uniform(0.01, 0.3)
    elif mode == 3:
        dt = prob["dt"].astype(np.float64) * rng.uniform(0.2, 30.0)
        dt = dt * np.repeat(rng.random((1, (L + 15) // 16, H)) < 0.6, 16, axis=1)[:, :L]
    else:
        dt = rng.uniform(1e-5, 2e-3, (1, L, H))
    p1["dt"] = np.minimum(dt, 15.9).astype(np.float32)
    p1["A"] = (-rng.uniform(0.5, 16.0, H)).astype(np.float32)
    if mode >= 3:
        p1["A"][rng.random(H) < 0.3] = 0.0
    yref, href, _ = oracle.ref_prefill(sc, p1["x"], p1["B"], p1["C"], p1["dt"], p1["A"], p1["D"])
    assert np.isfinite(yref).all() and 0 < np.abs(yref).max() < 6e4
    for want_state, flags in ((True, 0), (False, NO_SPLIT)):
        yg, hg = run_prefill(gpu_lib, s, sc, p1, flags=flags, want_state=want_state)
        check(yg, hg, yref, href if want_state else None,
              f"step-size pattern {mode}, seed {seed}, L={L}, H={H}, state={want_state}, flags={flags}")


def test_step_sizes_up_to_the_documented_limit(gpu_lib):
    """The matrix-core kernel documents 0 <= dt <= 16 (the narrowed scores times dt / 4 must stay in fp16).  Step sizes
    scaled up and capped just below the limit on every other head, B scales lowered so that y stays inside fp16: the
    result meets the oracle like any other, with and without the final state, on both launch shapes."""
    s = W.CONFIGS["m2_130m"].with_(seqlen=400)
    sc, prob, _ = make_problem(s, 16, calib_tokens=256)
    p1 = dict(prob)
    dt = prob["dt"].copy()
    dt[:, :, 0::2] = np.minimum(dt[:, :, 0::2] * 300.0, 15.9)
    p1["dt"] = dt.astype(np.float32)
    assert dt.max() > 15.8 and (dt[:, :, 0::2] > 15.0).mean() > 0.2
    sc.B_scales = (sc.B_scales / 200.0).astype(np.float32)
    for want_state, flags in ((True, 0), (False, 0), (False, NO_SPLIT)):
        yref, href, _ = oracle.ref_prefill(sc, p1["x"], p1["B"], p1["C"], p1["dt"], p1["A"], p1["D"],
                                           want_state=want_state)
        assert np.abs(yref).max() < 6e4
        yg, hg = run_prefill(gpu_lib, s, sc, p1, flags=flags, want_state=want_state)
        check(yg, hg, yref, href if want_state else None, f"dt up to 15.9, state={want_state}, flags={flags}",
              cells=oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups))


NO_DECAY_SKIP = 0x8


@pytest.mark.parametrize("want_state", [True, False])
def test_blocks_with_dead_decay_are_left_out_without_a_trace(gpu_lib, want_state):
    """By default 32-token blocks whose decay factor is below 2^-32 are not computed.  Heads range from no decay to
    a decay that kills the carried state within a block (dt scaled per head), so every skip (carried state, far score
    blocks, state blocks) is taken on some heads and none on others; the result must meet the oracle like the full
    computation (QUAMBA_FLAG_NO_DECAY_SKIP) and agree with it up to a few flipped roundings."""
    s = W.CONFIGS["m2_130m"].with_(batch=2, seqlen=700)
    sc, prob, _ = make_problem(s, 14, calib_tokens=256)
    p1 = dict(prob)
    dt = prob["dt"].copy()
    dt *= np.geomspace(0.05, 8.0, s.nheads).astype(np.float32)[None, None, :]
    p1["dt"] = dt
    per_block = -(dt * prob["A"][None, None, :]).astype(np.float64)[:, :672].reshape(2, 21, 32, s.nheads).sum(axis=2) * 1.4426950408889634
    assert per_block.min() < 1.0 and per_block.max() > 64.0     # log2 units: both ends are there
    init = (0.05 * np.random.default_rng(14).standard_normal((2, s.nheads, s.headdim, s.d_state))).astype(np.float32)
    yref, href, _ = oracle.ref_prefill(sc, p1["x"], p1["B"], p1["C"], p1["dt"], p1["A"], p1["D"],
                                       init_state=init.astype(np.float64), want_state=want_state)
    y0, h0 = run_prefill(gpu_lib, s, sc, p1, flags=0, init_state=init, want_state=want_state)
    y1, h1 = run_prefill(gpu_lib, s, sc, p1, flags=NO_DECAY_SKIP, init_state=init, want_state=want_state)
    check(y0, h0, yref, href if want_state else None, "decay skip on")
    check(y1, h1, yref, href if want_state else None, "decay skip off")
    # what is left out is below 2^-32 of a term: it can flip the fp16 rounding of an output that sat on a tie, no more
    assert (y0 != y1).sum() <= 16 and np.abs(y0 - y1).max() <= 2.0 ** -10 * np.abs(yref).max()
    if want_state:
        assert np.abs(h0 - h1).max() <= 1e-6 * np.abs(href).max()


def test_precise_flag_without_final_state(gpu_lib):
    """QUAMBA_FLAG_PRECISE_STATE selects the two-term state path even when no final state is returned."""
    s = W.CONFIGS["m2_130m"].with_(seqlen=700)
    sc, prob, _ = make_problem(s, 10, calib_tokens=256)
    yref, _, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"], want_state=False)
    yg, _ = run_prefill(gpu_lib, s, sc, prob, flags=0x2, want_state=False)
    check(yg, None, yref, None, "precise flag, no state")


def test_prefill_is_deterministic(gpu_lib):
    s = W.CONFIGS["m2_130m"].with_(seqlen=512)
    sc, prob, _ = make_problem(s, 11, calib_tokens=256)
    y1, h1 = run_prefill(gpu_lib, s, sc, prob)
    y2, h2 = run_prefill(gpu_lib, s, sc, prob)
    assert np.array_equal(y1, y2) and np.array_equal(h1, h2)


def test_prefill_then_decode_matches_longer_prefill(gpu_lib):
    """The final state is the resumable object: prefill(L) + k decode steps == prefill(L + k)."""
    import torch
    q = gpu_lib
    s = W.CONFIGS["m2_8b_b1"].with_(seqlen=512 + 4, nheads=32, ngroups=2)
    sc, prob, _ = make_problem(s, 6, calib_tokens=256)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    k = 4
    head = {n: (v[:, :-k].copy() if n in ("x", "B", "C", "dt") else v) for n, v in prob.items()}
    yg, hg = run_prefill(q, s.with_(seqlen=512), sc, head)
    dsc = q.DeviceScales(host_scales(q, sc))
    st = torch.from_numpy(hg.astype(np.float32)).cuda()
    A = torch.from_numpy(prob["A"]).cuda(); D = torch.from_numpy(prob["D"]).cuda()
    y1 = torch.empty((1, s.nheads, s.headdim), dtype=torch.float16, device="cuda")
    scale = np.abs(yref).max()
    assert np.abs(yg - yref[:, :-k]).max() <= Y_TOL * scale
    for i in range(512, 512 + k):
        t = {n: torch.from_numpy(np.ascontiguousarray(prob[n][:, i])).cuda() for n in ("x", "B", "C", "dt")}
        q.quamba_ssd_decode_step(to_shape(q, s), dsc, t["x"], t["B"], t["C"], t["dt"], A, D, st, y1)
        assert np.abs(y1.cpu().numpy().astype(np.float64) - yref[:, i]).max() <= Y_TOL * scale
    assert np.abs(st.cpu().numpy().astype(np.float64) - href).max() <= H_TOL * np.abs(href).max()


def test_2p7b_shape_full(gpu_lib):
    """configs[2] at full size (batch 8, 80 heads, heavy-tailed outlier channels, final states returned): every
    (sequence, head) pair against the oracle, globally and cell by cell."""
    s = W.CONFIGS["m2_2p7b"]
    sc, prob, _ = make_problem(s, 2)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    yg, hg = run_prefill(gpu_lib, s, sc, prob)
    check(yg, hg, yref, href, "2.7B-shaped, all pairs", cells=oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups))


@pytest.mark.parametrize("batch", [1, 4])
def test_8b_shape_full(gpu_lib, batch):
    """configs[3] at full size, in the launch configuration bench.py times (batch 4) and with the channel split
    (batch 1): every (sequence, head) pair against the oracle, globally and in each of the 128 scale cells."""
    s = W.CONFIGS["m2_8b_b4"].with_(batch=batch)
    sc, prob, _ = make_problem(s, 3)
    cells = oracle.cell_index_table(sc, s.nheads, s.headdim, s.ngroups)
    yref, href, _ = oracle.ref_prefill(sc, prob["x"], prob["B"], prob["C"], prob["dt"], prob["A"], prob["D"])
    yg, hg = run_prefill(gpu_lib, s, sc, prob)
    check(yg, hg, yref, href, f"8B-shaped b={batch}, all pairs", cells=cells)
    del yg, hg
    # without the final state the same y must come out (the state output only switches precision of the state path)
    yg2, _ = run_prefill(gpu_lib, s, sc, prob, want_state=False)
    check(yg2, None, yref, None, f"8B-shaped b={batch}, all pairs, no state", cells=cells)
