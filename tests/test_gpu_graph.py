"""GPU: every entry point records into a HIP graph and replays to the same bits.

The library allocates nothing, synchronises nothing and clears its counters with small kernels
(no memset nodes), so a caller may capture a stream of calls once and replay it.  The graph is
replayed three times with the outputs overwritten and eager calls of the same entry points in
between; every replay must reproduce the eager run's outputs bit for bit (FP32 values, both log
formats, counts, statistics, digests).  What the eager run produces is held to the oracle by the
other GPU tests; here the first call's FP32 outputs are checked against it once more.
"""
import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

pytestmark = pytest.mark.gpu


def test_captured_stream_of_calls_replays_bit_identically():
    import torch
    import paper_2403_09603_amd as vt
    dev = "cuda"
    g = si.rng(si.seed_for(9, 0))
    up = lambda a: torch.from_numpy(np.ascontiguousarray(a)).to(dev)
    tau = 0.25
    # operands
    M, N, K = 300, 200, 170
    A, B, bias = up(g.standard_normal((M, K))), up(g.standard_normal((K, N))), up(g.standard_normal(N))
    Mw, Nw, Kw = 96, 80, 20000                                     # A transposed, long K: the split-K route
    assert vt.vt_gemm_plan(Mw, Nw, Kw, 1, transA=True)[2] > 1
    Aw, Bw = up(g.standard_normal((Kw, Mw))), up(g.standard_normal((Kw, Nw)))
    xv, _ = si.planted_vector(60000, si.seed_for(9, 1), thr=32)
    x, xa = up(xv), up(si.perturb_steps(xv, si.seed_for(9, 2), 32))
    tau_x = 32 * 2.0 ** -29
    geo = vt.Conv2d(2, 13, 12, 8, 3, 3, 2, 2, 1, 1, 1, 1)
    Cout = 16
    Mc, Nc, Kc = vt.vt_conv2d_gemm_shape(geo, Cout, vt.VT_CONV_FORWARD)
    Md, Nd, Kd = vt.vt_conv2d_gemm_shape(geo, Cout, vt.VT_CONV_DATA_GRAD)
    X = up(np.maximum(g.standard_normal((2, 13, 12, 8)), 0.0))
    Wt = up(g.standard_normal((3, 3, 8, Cout)) * 0.2)
    dY = up(g.standard_normal(Mc * Cout))
    rows, cols = 64, 96
    La = up(g.standard_normal((rows, cols)))
    # outputs
    f32 = lambda n: torch.empty(n, dtype=torch.float32, device=dev)
    o = {"gemm": f32(M * N), "wgrad": f32(Mw * Nw), "rl": f32(x.numel()), "rld": f32(x.numel()), "rp": f32(x.numel()),
         "rpd": f32(x.numel()), "conv": f32(Mc * Nc), "dgrad": f32(Md * Nd), "softmax": f32(rows * cols),
         "lnorm": f32(rows * cols), "bnorm": f32(rows * cols),
         "stats": torch.empty(68, dtype=torch.int64, device=dev), "digest": torch.empty(32, dtype=torch.uint8, device=dev),
         "root": torch.empty(32, dtype=torch.uint8, device=dev)}
    logs = {"gemm": vt.alloc_log(M * N), "wgrad": vt.alloc_dense_log(Mw * Nw), "rl": vt.alloc_log(x.numel()),
            "rld": vt.alloc_dense_log(x.numel()), "conv": vt.alloc_dense_log(Mc * Nc), "dgrad": vt.alloc_log(Md * Nd),
            "softmax": vt.alloc_dense_log(rows * cols), "lnorm": vt.alloc_log(rows * cols),
            "bnorm": vt.alloc_dense_log(rows * cols)}
    wsb = max(vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, 1), vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, Mw, Nw, Kw, 1),
              vt.vt_workspace_bytes(vt.VT_OP_ROUND_LOG, 1, x.numel()), vt.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, Mc, Nc, Kc, 1),
              vt.vt_workspace_bytes(vt.VT_OP_CONV_DGRAD_ROUND_LOG, Md, Nd, Kd, 1),
              vt.vt_workspace_bytes(vt.VT_OP_LAYER_ROUND_LOG, rows, cols, 0, 1),
              vt.vt_workspace_bytes(vt.VT_OP_SHA256_TREE, 1, x.numel() * 8, 1024, 1), vt.vt_workspace_bytes(vt.VT_OP_MERKLE_ROOT, 1, 5, 0, 1))
    ws = vt.alloc_workspace(wsb)
    leaves = up(g.integers(0, 256, 5 * 32, dtype=np.uint8))
    count_rl = [0]

    def calls():
        vt.vt_gemm_f64_round_log(False, False, M, N, K, 0.5, A, K, 0, B, N, 0, bias, 1, o["gemm"], N, 0, None, 0, tau, logs["gemm"], ws)
        vt.vt_gemm_f64_round_log(True, False, Mw, Nw, Kw, 1.0, Aw, Mw, 0, Bw, Nw, 0, None, 1, o["wgrad"], Nw, 0, None, 1, tau,
                                 logs["wgrad"], ws)
        vt.vt_round_log(x, tau_x, o["rl"], logs["rl"], ws)
        vt.vt_round_log(x, tau_x, o["rld"], logs["rld"], ws)
        vt.vt_round_replay(xa, logs["rl"].idx, logs["rl"].dir, count_rl[0], o["rp"])
        vt.vt_round_replay_dense(xa, logs["rld"].dense, o["rpd"])
        vt.vt_threshold_stats(x, xa, o["stats"])
        vt.vt_conv2d_f64_round_log(vt.VT_CONV_FORWARD, geo, Cout, X.view(-1), Wt.view(-1), None, o["conv"], None, 0, tau, logs["conv"], ws)
        vt.vt_conv2d_f64_round_log(vt.VT_CONV_DATA_GRAD, geo, Cout, dY, Wt.view(-1), None, o["dgrad"], None, 0, tau, logs["dgrad"], ws)
        vt.vt_layer_f64_round_log(vt.VT_LAYER_SOFTMAX, La, None, None, None, rows, cols, o["softmax"], None, 0, tau, logs["softmax"], ws,
                                  scale=0.125, causal_period=cols)
        # (rows held in registers, index-list log: a scanner workgroup inside the captured launch; column statistics)
        vt.vt_layer_f64_round_log(vt.VT_LAYER_NORM, La, None, None, None, rows, cols, o["lnorm"], None, 1, tau, logs["lnorm"], ws, eps=1e-5)
        vt.vt_layer_f64_round_log(vt.VT_LAYER_BATCHNORM_RELU, La, None, None, None, rows, cols, o["bnorm"], None, 0, tau, logs["bnorm"], ws,
                                  eps=1e-5)
        vt.vt_sha256_tree(x, 1024, o["digest"], ws)
        vt.vt_merkle_root(leaves, o["root"], ws)

    def snapshot():
        torch.cuda.synchronize()
        snap = {k: v.cpu().numpy().copy() for k, v in o.items()}
        for k, lg in logs.items():
            c = int(lg.count.item())
            snap["count_" + k] = c
            if lg.dense is not None:
                snap["tlog_" + k] = lg.dense.cpu().numpy().copy()
            else:
                snap["idx_" + k] = lg.idx.cpu().numpy()[:c].copy()
                snap["dir_" + k] = np.unpackbits(lg.dir.cpu().numpy().view(np.uint8), bitorder="little")[:c].copy()
        return snap

    def same(a, b):
        assert a.keys() == b.keys()
        for k in a:
            if isinstance(a[k], int):
                assert a[k] == b[k], k
            else:
                assert np.array_equal(a[k].view(np.uint8), b[k].view(np.uint8)), k

    # the replay's entry count is a host value: take it from a first eager trainer call
    vt.vt_round_log(x, tau_x, o["rl"], logs["rl"], ws)
    torch.cuda.synchronize()
    count_rl[0] = int(logs["rl"].count.item())
    assert count_rl[0] > 1000
    calls()
    ref = snapshot()
    yo, io, _, co = vo.round_log(xv, tau_x)                            # the eager run against the oracle, once
    assert co == count_rl[0] and np.array_equal(ref["rl"].view(np.uint32), yo.view(np.uint32))
    assert np.array_equal(ref["idx_rl"].view(np.uint32), io)
    assert np.array_equal(ref["rp"].view(np.uint32), ref["rl"].view(np.uint32))      # replay on the perturbed copy: no mismatch

    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        calls()
    for rep in range(3):
        for v in o.values():
            v.fill_(0) if v.dtype != torch.float32 else v.fill_(float("nan"))
        for lg in logs.values():
            lg.count.fill_(-1)
            (lg.dense if lg.dense is not None else lg.idx).fill_(0x5A if lg.dense is not None else 0x5A5A5A5A)
        torch.cuda.synchronize()
        graph.replay()
        same(snapshot(), ref)
        # eager work of the same entry points between replays (other threshold: other counters, other logs)
        vt.vt_round_log(x, 0.25, o["rl"], logs["rl"], ws)
        vt.vt_gemm_f64_round_log(False, False, M, N, K, 0.5, A, K, 0, B, N, 0, bias, 1, o["gemm"], N, 0, None, 1, 0.01, logs["gemm"], ws)
        torch.cuda.synchronize()
