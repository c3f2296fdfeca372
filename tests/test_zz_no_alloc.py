"""GPU test of vt_round_log_static, the allocation-free variant of vt_round_log: its outputs must equal
vt_round_log's bit for bit (FP32 values, index list, direction bits, count, packed bytes), on two calls
in a row that share the library's static scratch, the second on a smaller input."""
import numpy as np
import pytest

import synth_inputs as si

pytestmark = pytest.mark.gpu


def _u32(t):
    return t.cpu().numpy().view(np.uint32)


def _run(vt, torch, xd, tau, fmt, static, b_r=32):
    n = xd.numel()
    y = torch.full((max(n, 1),), float("nan"), dtype=torch.float32, device="cuda")[:n]
    log = vt.alloc_log(n) if fmt == "sparse" else vt.alloc_dense_log(n)
    log.b_r = b_r
    log.count.fill_(-1)
    if fmt == "sparse":
        log.idx.fill_(-1)
    else:
        log.dense.fill_(0xEE)
    if static:
        vt.vt_round_log_static(xd, tau, y, log)
    else:
        ws = vt.alloc_workspace(vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, n))
        vt.vt_round_log(xd, tau, y, log, ws)
    torch.cuda.synchronize()
    cnt = int(log.count.item())
    out = {"y": _u32(y), "count": cnt}
    if fmt == "sparse":
        out["idx"] = _u32(log.idx)[:cnt].copy()
        out["dir"] = np.unpackbits(_u32(log.dir)[:(cnt + 31) // 32].view(np.uint8), bitorder="little")[:cnt]
    else:
        out["tlog"] = log.dense.cpu().numpy().copy()
    return out


def _same(a, b):
    assert a["count"] == b["count"]
    for k in a:
        if k != "count":
            assert np.array_equal(a[k], b[k]), k


@pytest.mark.parametrize("fmt", ["sparse", "packed"])
def test_static_scratch_matches_workspace_entry_point(fmt):
    import torch
    import paper_2403_09603_amd as vt
    thr = 1 << 20
    tau = thr * 2.0 ** -29
    # first call: 300 tiles and a ragged tail; second call: smaller (the scratch keeps the first call's words)
    n1, n2 = 8192 * 300 + 1234, 8192 * 7 + 55
    x1, _ = si.planted_vector(n1, si.seed_for(5, 40), thr=thr)
    x2, _ = si.planted_vector(n2, si.seed_for(5, 41), thr=thr)
    x1[:64] = si.edge_values()[:64]
    for b_r in (32, 26):
        for x in (x1, x2, x2[:0], x1[:5]):
            xd = torch.from_numpy(np.ascontiguousarray(x)).cuda()
            got = _run(vt, torch, xd, tau, fmt, static=True, b_r=b_r)
            want = _run(vt, torch, xd, tau, fmt, static=False, b_r=b_r)
            _same(got, want)
            if x.size > 1000 and b_r == 32:      # the planted tenth sits at FP32 midpoints
                assert 0.05 * x.size < got["count"] < 0.5 * x.size


def test_static_scratch_limits():
    import torch
    import paper_2403_09603_amd as vt
    x = torch.zeros(64, dtype=torch.float64, device="cuda")
    y = torch.zeros(64, dtype=torch.float32, device="cuda")
    log = vt.alloc_log(64)
    with pytest.raises(vt.VtError, match="unsupported"):        # index-list log: x must be 16-byte aligned
        vt.vt_round_log_static(x[1:], 0.1, y[1:], log)
    dl = vt.alloc_dense_log(63)
    vt.vt_round_log_static(x[1:], 0.1, y[1:], dl)               # the packed log takes any alignment
    torch.cuda.synchronize()
    assert int(dl.count.item()) == 0
