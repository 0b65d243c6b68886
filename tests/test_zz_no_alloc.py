"""quamba_ssd_prefill_noalloc (the prefill with the library's own fixed scratch area, for callers that cannot
allocate) against quamba_ssd_prefill with a caller's workspace, through the C ABI: the same launches on the same
inputs, so the outputs and the final states must agree bit for bit.  Two calls in a row share the scratch area, the
second on a smaller input; a third shape needs no scratch at all."""
import numpy as np
import pytest

import workloads as W
from helpers import make_problem, to_shape, host_scales

pytestmark = pytest.mark.gpu


def _both(q, s, seed):
    import torch
    shape = to_shape(q, s)
    sc, prob, _ = make_problem(s, seed, calib_tokens=512)
    dsc = q.DeviceScales(host_scales(q, sc))
    t = {k: (torch.from_numpy(v).cuda() if v is not None else None) for k, v in prob.items()}
    init = torch.from_numpy(W.draw_state(s, seed)).cuda()
    need = q.quamba_ssd_prefill_workspace_size(shape)
    ws = torch.empty(max(need, 16), dtype=torch.uint8, device="cuda")
    out = []
    for entry in ("workspace", "noalloc"):
        y = torch.full((s.batch, s.seqlen, s.nheads, s.headdim), float("nan"), dtype=torch.float16, device="cuda")
        fin = torch.full((s.batch, s.nheads, s.headdim, s.d_state), float("nan"), device="cuda")
        if entry == "workspace":
            q.quamba_ssd_prefill(shape, dsc, t["x"], t["B"], t["C"], t["dt"], t["A"], t["D"], init, y, fin, ws)
        else:
            q.quamba_ssd_prefill_noalloc(shape, dsc, t["x"], t["B"], t["C"], t["dt"], t["A"], t["D"], init, y, fin)
        torch.cuda.synchronize()
        out.append((y.cpu().numpy().view(np.uint16), fin.cpu().numpy()))
    (y0, h0), (y1, h1) = out
    assert np.isfinite(h0).all() and np.isfinite(y0.view(np.float16).astype(np.float32)).all()
    assert np.array_equal(y0, y1), f"{np.count_nonzero(y0 != y1)} outputs differ"
    assert np.array_equal(h0, h1)
    return need


def test_noalloc_entry_point_matches_the_workspace_entry_point(gpu_lib):
    q = gpu_lib
    big = W.CONFIGS["m2_8b_b1"]                              # 128 heads x 4096 tokens: 4 segments, 12.6 MB of scratch
    small = W.CONFIGS["m2_130m"]                             # 24 heads x 2048 tokens: 8 segments, 5.5 MB
    none = W.CONFIGS["m2_130m"].with_(seqlen=300)            # too short for a split: no scratch
    n_big = _both(q, big, 41)
    n_small = _both(q, small, 42)
    assert 0 < n_small < n_big <= 16 << 20
    assert _both(q, none, 43) == 0
    # and once more the large one, on top of what the smaller call left in the scratch area
    _both(q, big, 44)
