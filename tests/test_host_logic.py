"""CPU-only checks of the HIP library's host-visible parts: the C ABI loads and exports every
symbol include/vt.h declares, argument validation rejects bad calls before touching a GPU, and
the per-element integer arithmetic the kernels use (compiled here for the host CPU) agrees with
the oracle on hand-built edge values and random bit patterns."""
import ctypes as C
import os
import re
import subprocess

import numpy as np
import pytest

import synth_inputs as si
from oracle import vt_oracle as vo

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HERE = os.path.join(ROOT, "tests")


@pytest.fixture(scope="module")
def hiplib():
    import paper_2403_09603_amd as vt
    if not os.path.exists(vt.library_path()):
        from paper_2403_09603_amd import build
        build.build_lib()
    return vt.load_library()


def test_every_declared_symbol_is_exported(hiplib):
    hdr = open(os.path.join(ROOT, "include", "vt.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = set(re.findall(r"\b(vt_[a-z0-9_]+)\s*\(", hdr))
    assert {"vt_round_log", "vt_round_replay", "vt_gemm_f64_round_log", "vt_threshold_stats",
            "vt_workspace_bytes", "vt_strerror", "vt_thr_from_tau"} <= names
    for n in names:
        assert hasattr(hiplib, n), n


def test_thr_from_tau_matches_oracle(hiplib):
    for tau in (0.0, 0.5, 0.25, 2.0 ** -24, 2.0 ** -29, 2.0 ** -40, 0.195, 0.035, 0.001, 1e-9,
                2.0 ** -29 + 2.0 ** -60, -1.0, 0.51, float("nan")):
        assert hiplib.vt_thr_from_tau(tau) == vo.thr_from_tau(tau)


def test_workspace_bytes_monotone_and_aligned(hiplib):
    prev = 0
    for n in (0, 1, 63, 64, 4096, 4097, 1 << 20, (1 << 28), (1 << 32) - 1):
        b = hiplib.vt_workspace_bytes(0, 1, n, 0, 1)
        assert b % 256 == 0 and b >= prev and b >= n // 4
        prev = b
    assert hiplib.vt_workspace_bytes(2, 8192, 3072, 768, 1) >= 8192 * 3072 // 4
    assert hiplib.vt_workspace_bytes(1, 1, 1 << 20, 0, 1) == 0
    assert hiplib.vt_workspace_bytes(3, 1, 1 << 20, 0, 1) == 0


def test_workspace_covers_the_slices_of_tail_tiles(hiplib):
    """A launch whose last tiles are cut into slices needs tile-sized slabs for them beside the decision planes."""
    import paper_2403_09603_amd as vt
    for M, N, K in ((12544, 256, 2304), (2112, 512, 1024), (4700, 1000, 1024), (50176, 256, 512)):
        tile = vt.vt_gemm_plan(M, N, K, 1, ldc=N + 8)[0]
        tail_tiles, slices = vt.vt_gemm_tail_plan(M, N, K, 1, ldc=N + 8)
        assert tail_tiles > 0 and slices == 4
        assert hiplib.vt_workspace_bytes(2, M, N, K, 1) >= M * N // 4 + tail_tiles * slices * tile * tile * 8
    assert vt.vt_gemm_tail_plan(8192, 3072, 768, 1) == (0, 1)              # 1536 tiles: six whole rounds
    assert vt.vt_gemm_tail_plan(128, 128, 64, 1) == (0, 1)
    assert hiplib.vt_workspace_bytes(2, 128, 128, 64, 1) < 1 << 20


def test_argument_validation_happens_on_the_host(hiplib):
    """None of these calls may reach a kernel launch: they run here without a GPU."""
    import paper_2403_09603_amd.binding as b
    cnt = (C.c_uint64 * 1)()
    log = b._VtLog(None, None, 0, C.addressof(cnt), None, 0)
    fake = C.c_void_p(0x1000)
    INVALID, WORKSPACE = 1, 2
    assert hiplib.vt_round_log(fake, 16, 0.75, fake, C.byref(log), fake, 1 << 20, None) == INVALID   # tau
    assert hiplib.vt_round_log(fake, 1 << 32, 0.1, fake, C.byref(log), fake, 1 << 20, None) == INVALID  # n
    assert hiplib.vt_round_log(None, 16, 0.1, fake, C.byref(log), fake, 1 << 20, None) == INVALID
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, None, fake, 1 << 20, None) == INVALID
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, C.byref(log), None, 0, None) == WORKSPACE
    assert hiplib.vt_round_log(fake, 1 << 20, 0.1, fake, C.byref(log), fake, 1024, None) == WORKSPACE
    badlog = b._VtLog(None, None, 8, C.addressof(cnt), None, 0)
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, C.byref(badlog), fake, 1 << 20, None) == INVALID
    both = b._VtLog(0x1000, 0x1000, 8, C.addressof(cnt), 0x2000, 0)                 # two formats in one call
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, C.byref(both), fake, 1 << 20, None) == INVALID
    odd = b._VtLog(None, None, 0, C.addressof(cnt), 0x2001, 0)                      # misaligned packed log
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, C.byref(odd), fake, 1 << 20, None) == INVALID
    for bad_br in (9, 33, -1):
        bl = b._VtLog(None, None, 0, C.addressof(cnt), None, bad_br)
        assert hiplib.vt_round_log(fake, 16, 0.1, fake, C.byref(bl), fake, 1 << 20, None) == INVALID
        assert hiplib.vt_round_replay_br(fake, 16, None, None, 0, bad_br, fake, None) == INVALID
        assert hiplib.vt_round_replay_dense_br(fake, 16, fake, bad_br, fake, None) == INVALID
        assert hiplib.vt_threshold_stats_br(fake, fake, 16, bad_br, fake, None) == INVALID
    assert hiplib.vt_round_replay_dense(fake, 16, None, fake, None) == INVALID
    assert hiplib.vt_round_replay_dense(fake, 16, C.c_void_p(0x2002), fake, None) == INVALID
    assert hiplib.vt_round_replay(fake, 1 << 32, None, None, 0, fake, None, 0, None) == INVALID
    assert hiplib.vt_round_replay(fake, 16, None, None, 4, fake, None, 0, None) == INVALID
    g = hiplib.vt_gemm_f64_round_log
    ok = dict(tA=0, tB=0, M=128, N=128, K=64, lda=64, ldb=128, ldc=128)
    def call(**kw):
        a = {**ok, **kw}
        return g(a["tA"], a["tB"], a["M"], a["N"], a["K"], 1.0, fake, a["lda"], 0, fake, a["ldb"], 0, None, 1,
                 fake, a["ldc"], 0, None, a.get("variant", 0), a.get("tau", 0.1), C.byref(log),
                 a.get("ws", fake), a.get("wsb", 1 << 20), None)
    assert call(M=-1) == INVALID and call(lda=63) == INVALID and call(ldb=127) == INVALID
    assert call(ldc=127) == INVALID and call(variant=2) == INVALID and call(tau=-0.1) == INVALID
    assert call(tA=2) == INVALID and call(M=1 << 20, N=1 << 12, lda=64, ldc=1 << 12) == INVALID
    assert call(ws=None, wsb=0) == WORKSPACE and call(wsb=16) == WORKSPACE
    for strideC, want in ((128 * 128 - 1, INVALID), (0, INVALID), (-5, INVALID), (64, INVALID), (200, INVALID)):   # batched outputs may not overlap
        assert g(0, 0, 128, 128, 64, 1.0, fake, 64, 0, fake, 128, 0, None, 2, fake, 128, strideC, None, 0, 0.1, C.byref(log),
                 fake, 1 << 24, None) == want
    log26 = b._VtLog(None, None, 0, C.addressof(cnt), None, 26)                  # b_r < 32 needs a dense C
    assert g(0, 0, 128, 128, 64, 1.0, fake, 64, 0, fake, 128, 0, None, 1, fake, 160, 0, None, 0, 0.1, C.byref(log26),
             fake, 1 << 24, None) == 4
    assert hiplib.vt_workspace_bytes(4, 128, 128, 64, 1) > hiplib.vt_workspace_bytes(2, 128, 128, 64, 1)
    assert hiplib.vt_threshold_stats(fake, fake, 16, None, None) == INVALID
    assert hiplib.vt_strerror(INVALID).decode() == "invalid argument"


def test_abandoned_count_is_a_distinct_status():
    """The all-ones count is reported as "pass abandoned", not as a log overflow (host logic only)."""
    import paper_2403_09603_amd as vt
    assert vt.check_count(0) == 0 and vt.check_count(17, cap=17) == 17
    assert vt.check_count(-1 & ((1 << 64) - 1) - 1) == (1 << 64) - 2          # any other value is a count
    with pytest.raises(vt.VtLogAbandoned):
        vt.check_count(-1)                                                     # int64 view of the sentinel
    with pytest.raises(vt.VtLogAbandoned):
        vt.check_count(vt.VT_COUNT_ABANDONED, cap=5)
    with pytest.raises(vt.VtError, match="overflow"):
        vt.check_count(18, cap=17)
    hdr = open(os.path.join(ROOT, "include", "vt.h")).read()
    assert "VT_COUNT_ABANDONED UINT64_MAX" in hdr


def test_static_scratch_entry_point_validates_on_the_host(hiplib):
    """vt_round_log_static refuses sizes beyond its static scratch, and bad arguments, before any GPU call."""
    import paper_2403_09603_amd.binding as b
    cnt = (C.c_uint64 * 1)()
    log = b._VtLog(None, None, 0, C.addressof(cnt), None, 0)
    fake = C.c_void_p(0x1000)
    f = hiplib.vt_round_log_static
    LIMIT = 5
    assert f(fake, (1 << 30) + 1, 0.1, fake, C.byref(log), None) == LIMIT
    assert f(fake, (1 << 32) - 1, 0.1, fake, C.byref(log), None) == LIMIT
    assert f(fake, 16, 0.75, fake, C.byref(log), None) == 1                     # tau
    assert f(None, 16, 0.1, fake, C.byref(log), None) == 1
    assert f(fake, 16, 0.1, fake, None, None) == 1
    assert f(C.c_void_p(0x1008), 16, 0.1, fake, C.byref(log), None) == 4        # index-list log needs 16-byte x
    assert f(fake, 16, 0.1, C.c_void_p(0x1004), C.byref(log), None) == 4        # ... and 8-byte y
    assert b.VT_ROUND_LOG_STATIC_MAX_N == 1 << 30
    assert "static scratch" in hiplib.vt_strerror(LIMIT).decode()


@pytest.mark.parametrize("b", [32, 31, 29, 26, 16, 10])
def test_kernel_arithmetic_for_other_rounding_amounts_on_host(harith, b):
    """decide_k / directed_k (rounding amounts below 32) against the oracle, on the host."""
    k = 32 - b
    g = si.rng(si.seed_for(0, 20 + b))
    rnd_bits = g.integers(0, 1 << 64, 1 << 14, dtype=np.uint64)
    e = g.integers(1023 - 160, 1023 + 130, 1 << 14, dtype=np.uint64)
    band = (rnd_bits & np.uint64(0x800FFFFFFFFFFFFF)) | (e << np.uint64(52))
    base = g.standard_normal(4000).astype(np.float32).view(np.uint32) & np.uint32(~((1 << k) - 1) & 0xFFFFFFFF)
    base = base.view(np.float32).astype(np.float64)
    mid = (base.view(np.uint64).astype(np.int64) + (1 << (28 + k)) + g.integers(-3, 4, base.size)).astype(np.uint64)
    x = np.concatenate([si.edge_values(), band.view(np.float64), mid.view(np.float64), base])
    bits = np.ascontiguousarray(x).view(np.uint64)
    n = bits.size
    y, D, dr = (np.empty(n, np.uint32) for _ in range(3))
    harith.h_decide_k(bits.ctypes.data_as(C.POINTER(C.c_uint64)), C.c_uint64(n), C.c_uint32(k), _u32p(y), _u32p(D), _u32p(dr))
    yo, _, _, _ = vo.round_log(x, 0.0, b_r=b)
    assert np.array_equal(y, yo.view(np.uint32))
    assert np.array_equal(D, np.array([vo.boundary_distance(float(v), b) for v in x], np.uint32))
    for thr in (1, 1 << 12, 1 << 27, 1 << 28):
        codes = np.array([vo.ternary_code(float(v), thr, b) for v in x[::3]])
        assert np.array_equal(np.where(D[::3] < thr, np.where(dr[::3] == 1, 2, 0), 1), codes)
    idx = np.arange(n, dtype=np.uint32)
    for d in (0, 1):
        yd = np.empty(n, np.uint32)
        harith.h_directed_k(bits.ctypes.data_as(C.POINTER(C.c_uint64)), C.c_uint64(n), C.c_uint32(d), C.c_uint32(k), _u32p(yd))
        want = vo.round_replay(x, idx, np.full((n + 31) // 32, 0xFFFFFFFF if d else 0, np.uint32), b_r=b)
        assert np.array_equal(yd, want.view(np.uint32))


def test_conv_geometry_and_validation_on_the_host(hiplib):
    import paper_2403_09603_amd.binding as b
    cnt = (C.c_uint64 * 1)()
    log = b._VtLog(None, None, 0, C.addressof(cnt), None, 0)
    fake = C.c_void_p(0x1000)
    INVALID, WORKSPACE = 1, 2
    # GEMM shapes of the ResNet-50 geometry at batch 64 against the oracle's output size
    for (H, Cin, K, s, p, Cout) in [(224, 3, 7, 2, 3, 64), (56, 64, 3, 1, 1, 64), (56, 256, 1, 2, 0, 512),
                                    (14, 256, 3, 1, 1, 256), (7, 512, 3, 1, 1, 512)]:
        d = b.Conv2d(64, H, H, Cin, K, K, s, s, p, p, 1, 1)
        _, Ho, Wo = vo.conv2d_geometry((64, H, H, Cin), K, K, s, p, 1)
        assert b.vt_conv2d_gemm_shape(d, Cout, b.VT_CONV_FORWARD) == (64 * Ho * Wo, Cout, K * K * Cin)
        assert b.vt_conv2d_gemm_shape(d, Cout, b.VT_CONV_WEIGHT_GRAD) == (K * K * Cin, Cout, 64 * Ho * Wo)
        Md, Nd, Kd = b.vt_conv2d_gemm_shape(d, Cout, b.VT_CONV_DATA_GRAD)
        assert (Md, Nd, Kd) == (64 * H * H, Cin, K * K * Cout)
        plain = hiplib.vt_workspace_bytes(b.VT_OP_GEMM_ROUND_LOG, Md, Nd, Kd, 1)
        assert hiplib.vt_workspace_bytes(b.VT_OP_CONV_DGRAD_ROUND_LOG, Md, Nd, Kd, 1) >= plain + 8 * Kd * Nd
        assert hiplib.vt_workspace_bytes(b.VT_OP_CONV_DGRAD_ROUND_LOG_BR, Md, Nd, Kd, 1) >= \
            hiplib.vt_workspace_bytes(b.VT_OP_GEMM_ROUND_LOG_BR, Md, Nd, Kd, 1) + 8 * Kd * Nd
    f = hiplib.vt_conv2d_f64_round_log
    good = b.Conv2d(2, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1)
    def call(d=good, mode=0, Cout=8, X=fake, bias=None, variant=0, tau=0.1, ws=fake, wsb=1 << 20):
        return f(mode, C.byref(d), Cout, X, fake, bias, fake, None, variant, tau, C.byref(log), ws, wsb, None)
    assert call(mode=3) == INVALID and call(variant=3) == INVALID and call(tau=0.6) == INVALID
    assert call(mode=2, bias=fake) == INVALID and call(mode=2, X=None) == INVALID and call(mode=2, Cout=-1) == INVALID
    assert call(mode=2, ws=None, wsb=0) == WORKSPACE and call(mode=2, wsb=16) == WORKSPACE
    assert call(mode=2, d=b.Conv2d(1 << 10, 1 << 10, 1 << 11, 1, 3, 3, 1, 1, 1, 1, 1, 1), Cout=1) == INVALID   # N H W >= 2^31
    assert call(mode=2, d=b.Conv2d(2, 600, 600, 4, 300, 300, 1, 1, 1, 1, 1, 1)) == INVALID          # KH KW >= 2^16
    assert call(X=None) == INVALID and call(mode=1, bias=fake) == INVALID and call(Cout=-1) == INVALID
    for field, val in (("KH", 0), ("stride_w", 0), ("dil_h", 0), ("pad_w", -1), ("N", -1), ("H", 1 << 24)):
        bad = b.Conv2d(2, 8, 8, 4, 3, 3, 1, 1, 1, 1, 1, 1)
        setattr(bad, field, val)
        assert call(d=bad) == INVALID, field
    assert call(d=b.Conv2d(1 << 12, 1 << 10, 1 << 10, 4, 3, 3, 1, 1, 1, 1, 1, 1)) == INVALID   # image >= 2^31 elements
    assert call(ws=None, wsb=0) == WORKSPACE and call(wsb=16) == WORKSPACE


def test_layer_validation_on_the_host(hiplib):
    import paper_2403_09603_amd.binding as b
    cnt = (C.c_uint64 * 1)()
    log = b._VtLog(None, None, 0, C.addressof(cnt), None, 0)
    INVALID, WORKSPACE = 1, 2
    f = hiplib.vt_layer_f64_round_log
    def call(op=0, a=0x1000, bb=0x1000, rows=8, cols=16, eps=1e-5, period=0, variant=0, tau=0.1, y=0x1000, ws=0x1000, wsb=1 << 20):
        L = b._VtLayer(op, a, bb, None, None, rows, cols, eps, 1.0, period)
        return f(C.byref(L), C.c_void_p(y), None, variant, tau, C.byref(log), C.c_void_p(ws) if ws else None, wsb, None)
    assert call(op=8) == INVALID and call(op=-1) == INVALID and call(rows=-1) == INVALID and call(variant=2) == INVALID
    assert call(a=None) == INVALID and call(a=0x1008) == INVALID and call(bb=None) == INVALID and call(y=0x1004) == INVALID
    assert call(op=4, eps=-1.0) == INVALID and call(op=6, eps=-1.0) == INVALID and call(op=5, period=-3) == INVALID and call(tau=0.7) == INVALID
    assert call(rows=1 << 20, cols=1 << 12) == INVALID                          # 2^32 outputs
    assert call(ws=None, wsb=0) == WORKSPACE and call(wsb=64) == WORKSPACE
    assert hiplib.vt_workspace_bytes(5, 8192, 768, 0, 1) >= 8192 * 16


def test_im2col_index_arithmetic_on_host(harith):
    """The loader's row/tap decomposition (reciprocal multiply + correction) against plain integer
    arithmetic, including rows and taps past the end of the matrix and geometries near the limits."""
    geoms = [(2, 9, 11, 3, 3, 3, 1, 1, 1, 1, 1, 1), (1, 12, 10, 2, 7, 7, 2, 2, 3, 3, 1, 1), (3, 8, 7, 4, 1, 1, 2, 2, 0, 0, 1, 1),
             (1, 10, 13, 3, 3, 2, 2, 1, 1, 0, 1, 2), (1, 9, 9, 2, 3, 3, 1, 1, 2, 2, 2, 2), (64, 224, 224, 3, 7, 7, 2, 2, 3, 3, 1, 1),
             (5, 1 << 12, 1 << 12, 25, 3, 3, 1, 1, 1, 1, 1, 1)]
    for geo in geoms:
        N, H, W, Cin, KH, KW, sh, sw, ph, pw, dh, dw = geo
        Ho = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
        Wo = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
        rows, taps = N * Ho * Wo, KH * KW * Cin
        arr = np.array(list(geo) + [Ho, Wo], np.int64)
        # the first rows/taps and the last ones (plus some past the end of the matrix)
        for row0, tap0 in ((0, 0), (max(rows - 300, 0), max(taps - 150, 0))):
            nr, nt = min(rows - row0 + 40, 400), min(taps - tap0 + 20, 200)
            out = np.empty((nr, nt), np.int64)
            harith.h_im2col_offsets(arr.ctypes.data_as(C.POINTER(C.c_int64)), C.c_uint32(row0), C.c_uint32(nr),
                                    C.c_uint32(tap0), C.c_uint32(nt), out.ctypes.data_as(C.POINTER(C.c_int64)))
            m, k = np.meshgrid(row0 + np.arange(nr), tap0 + np.arange(nt), indexing="ij")
            n_, ho, wo = m // (Ho * Wo), (m // Wo) % Ho, m % Wo
            kh, kw, ci = k // (KW * Cin), (k // Cin) % KW, k % Cin
            h, w = ho * sh - ph + kh * dh, wo * sw - pw + kw * dw
            ok = (m < rows) & (k < taps) & (h >= 0) & (h < H) & (w >= 0) & (w < W)
            want = np.where(ok, ((n_ * H + h) * W + w) * Cin + ci, -1)
            assert np.array_equal(out, want), (geo, row0, tap0)


def test_input_gradient_index_arithmetic_on_host(harith):
    """The loader's view of dY for the input gradient (stride remainders of row and tap must agree)
    against plain integer arithmetic, past the ends of the matrix too."""
    geoms = [(2, 9, 11, 3, 3, 3, 1, 1, 1, 1, 1, 1), (1, 12, 10, 2, 7, 7, 2, 2, 3, 3, 1, 1), (3, 8, 7, 4, 1, 1, 2, 2, 0, 0, 1, 1),
             (1, 10, 13, 3, 3, 2, 2, 1, 1, 0, 1, 2), (1, 9, 9, 2, 3, 3, 1, 1, 2, 2, 2, 2), (1, 23, 17, 5, 5, 3, 3, 2, 2, 1, 2, 3),
             (64, 56, 56, 128, 3, 3, 2, 2, 1, 1, 1, 1), (3, 1 << 11, 1 << 11, 25, 3, 3, 2, 2, 1, 1, 1, 1)]
    for geo in geoms:
        N, H, W, Cout, KH, KW, sh, sw, ph, pw, dh, dw = geo
        Ho = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
        Wo = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
        rows, cols = N * H * W, KH * KW * Cout
        arr = np.array(list(geo) + [Ho, Wo], np.int64)
        for row0, col0 in ((0, 0), (max(rows - 300, 0), max(cols - 150, 0)), (rows // 2, cols // 3)):
            nr, nt = min(rows - row0 + 40, 400), min(cols - col0 + 20, 200)
            out = np.empty((nr, nt), np.int64)
            harith.h_dgrad_offsets(arr.ctypes.data_as(C.POINTER(C.c_int64)), C.c_uint32(row0), C.c_uint32(nr),
                                   C.c_uint32(col0), C.c_uint32(nt), out.ctypes.data_as(C.POINTER(C.c_int64)))
            m, k = np.meshgrid(row0 + np.arange(nr), col0 + np.arange(nt), indexing="ij")
            n_, h, w = m // (H * W), (m // W) % H, m % W
            kh, kw, co = k // (KW * Cout), (k // Cout) % KW, k % Cout
            hs, ws = h + ph - kh * dh, w + pw - kw * dw
            ok = (m < rows) & (k < cols) & (hs >= 0) & (ws >= 0) & (hs % sh == 0) & (ws % sw == 0) & (hs // sh < Ho) & (ws // sw < Wo)
            want = np.where(ok, ((n_ * Ho + hs // sh) * Wo + ws // sw) * Cout + co, -1)
            assert np.array_equal(out, want), (geo, row0, col0)


def test_integer_only_index_split_on_host(harith):
    """The multiply-high form of x / d (used where a whole wave shares the filter position): exact
    against numpy for random and extreme (x, d), and the loader's offsets are the same with either
    form for every tap of forward and input-gradient geometries (channel counts that are multiples
    of 16 among them: the only ones the kernels use it for)."""
    g = np.random.default_rng(20240309)
    x = np.concatenate([g.integers(0, 1 << 32, 200000, dtype=np.uint64), [0, 1, (1 << 32) - 1, (1 << 32) - 2, 1 << 31]]).astype(np.uint32)
    d = np.concatenate([g.integers(1, 1 << 32, 100000, dtype=np.uint64), g.integers(1, 5000, 100000, dtype=np.uint64),
                        [1, 1, (1 << 32) - 1, 1, 3]]).astype(np.uint32)
    q, r = np.empty_like(x), np.empty_like(x)
    u32 = C.POINTER(C.c_uint32)
    harith.h_divmod_magic(x.ctypes.data_as(u32), d.ctypes.data_as(u32), C.c_uint64(x.size), q.ctypes.data_as(u32), r.ctypes.data_as(u32))
    assert np.array_equal(q, x // d) and np.array_equal(r, x % d)
    for dv in (1, 2, 3, 7, 16, 48, 147, 65535, 65536, (1 << 31) + 1):                 # every x near multiples of d
        k = np.arange(0, ((1 << 32) - 1) // dv + 1, max(1, (1 << 32) // dv // 50000), dtype=np.uint64) * dv
        xs = np.unique(np.clip(np.concatenate([k, k + dv - 1, k[k > 0] - 1]), 0, (1 << 32) - 1)).astype(np.uint32)
        ds = np.full_like(xs, dv)
        q, r = np.empty_like(xs), np.empty_like(xs)
        harith.h_divmod_magic(xs.ctypes.data_as(u32), ds.ctypes.data_as(u32), C.c_uint64(xs.size), q.ctypes.data_as(u32), r.ctypes.data_as(u32))
        assert np.array_equal(q, xs // ds) and np.array_equal(r, xs % ds), dv
    harith.h_tap_split_mismatches.restype = C.c_uint64
    geoms = [(2, 9, 11, 16, 3, 3, 1, 1, 1, 1, 1, 1), (1, 12, 10, 32, 7, 7, 2, 2, 3, 3, 1, 1), (3, 8, 7, 48, 1, 1, 2, 2, 0, 0, 1, 1),
             (1, 10, 13, 3, 3, 2, 2, 1, 1, 0, 1, 2), (1, 9, 9, 64, 3, 3, 1, 1, 2, 2, 2, 2), (1, 23, 17, 80, 5, 3, 3, 2, 2, 1, 2, 3),
             (64, 56, 56, 128, 3, 3, 2, 2, 1, 1, 1, 1), (64, 14, 14, 256, 3, 3, 1, 1, 1, 1, 1, 1), (64, 7, 7, 512, 3, 3, 1, 1, 1, 1, 1, 1)]
    for geo in geoms:
        N, H, W, Cc, KH, KW, sh, sw, ph, pw, dh, dw = geo
        Ho = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
        Wo = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
        arr = np.array(list(geo) + [Ho, Wo], np.int64)
        for dgrad in (0, 1):
            rows = N * H * W if dgrad else N * Ho * Wo
            for row0 in (0, max(rows - 20, 0)):
                bad = harith.h_tap_split_mismatches(arr.ctypes.data_as(C.POINTER(C.c_int64)), C.c_int(dgrad), C.c_uint32(row0), C.c_uint32(24))
                assert bad == 0, (geo, dgrad, row0)


def test_weight_gradient_row_walk_on_host(harith):
    """Rows of the image matrix walked 16 at a time, up and down, against the direct split of the row
    index: outputs narrower and shorter than the step (several carries' worth in one digit), one
    output position per image, walks that run off either end of the matrix."""
    harith.h_row_walk_mismatches.restype = C.c_uint64
    geoms = [(2, 9, 11, 3, 3, 3, 1, 1, 1, 1, 1, 1), (40, 12, 10, 2, 7, 7, 2, 2, 3, 3, 1, 1), (70, 8, 7, 4, 1, 1, 2, 2, 0, 0, 1, 1),
             (9, 10, 13, 3, 3, 2, 2, 1, 1, 0, 1, 2), (300, 3, 3, 2, 3, 3, 1, 1, 0, 0, 1, 1), (50, 1, 40, 2, 1, 3, 1, 1, 0, 1, 1, 1),
             (50, 40, 1, 2, 3, 1, 1, 1, 1, 0, 1, 1), (64, 56, 56, 128, 3, 3, 2, 2, 1, 1, 1, 1), (64, 7, 7, 512, 3, 3, 1, 1, 1, 1, 1, 1),
             (64, 224, 224, 3, 7, 7, 2, 2, 3, 3, 1, 1), (4, 16, 16, 2, 1, 1, 1, 1, 0, 0, 1, 1), (3, 17, 15, 2, 2, 2, 1, 1, 0, 0, 1, 1)]
    for geo in geoms:
        N, H, W, Cc, KH, KW, sh, sw, ph, pw, dh, dw = geo
        Ho = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
        Wo = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
        rows = N * Ho * Wo
        arr = np.array(list(geo) + [Ho, Wo], np.int64)
        ptr = arr.ctypes.data_as(C.POINTER(C.c_int64))
        steps = min(rows // 16 + 6, 3000)
        for m0 in (0, 5, 15, Wo, Ho * Wo - 1):
            assert harith.h_row_walk_mismatches(ptr, C.c_uint32(m0), C.c_uint32(steps), C.c_int(0)) == 0, (geo, m0, "up")
        for m0 in (rows - 1, rows - 16, rows + 13, max(rows - Wo - 3, 0), min(rows - 1, 16 * 2000 + 7)):
            assert harith.h_row_walk_mismatches(ptr, C.c_uint32(m0), C.c_uint32(steps), C.c_int(1)) == 0, (geo, m0, "down")


def test_input_gradient_stride_phases_on_host(harith):
    """The split of a strided layer's input gradient into one stride-1 problem per phase: the phases
    partition the input positions and the filter taps, and every (row, column) of a phase's GEMM reads
    the element of dY that the definition names (or nothing)."""
    geoms = [(2, 9, 11, 4, 3, 3, 2, 2, 1, 1, 1, 1), (1, 12, 10, 2, 7, 7, 2, 2, 3, 3, 1, 1), (3, 8, 7, 4, 1, 1, 2, 2, 0, 0, 1, 1),
             (1, 10, 13, 2, 3, 2, 2, 1, 1, 0, 1, 2), (1, 9, 9, 2, 3, 3, 2, 2, 2, 2, 2, 2), (1, 23, 17, 6, 5, 3, 3, 2, 2, 1, 2, 3),
             (2, 7, 8, 2, 4, 5, 4, 3, 0, 5, 3, 2), (1, 5, 6, 2, 2, 2, 2, 2, 3, 3, 1, 1), (4, 56, 56, 8, 3, 3, 2, 2, 1, 1, 1, 1)]
    for geo in geoms:
        N, H, W, Cout, KH, KW, sh, sw, ph, pw, dh, dw = geo
        Ho = (H + 2 * ph - dh * (KH - 1) - 1) // sh + 1
        Wo = (W + 2 * pw - dw * (KW - 1) - 1) // sw + 1
        arr = np.array(list(geo) + [Ho, Wo], np.int64)
        seen_pos, seen_taps = np.zeros((H, W), int), np.zeros((KH, KW), int)
        for a in range(sh):
            for b in range(sw):
                info = np.zeros(14, np.int64)
                probe = np.empty((1, 1), np.int64)
                harith.h_dgrad_phase_offsets(arr.ctypes.data_as(C.POINTER(C.c_int64)), C.c_int64(a), C.c_int64(b), C.c_uint32(0),
                                             C.c_uint32(1), C.c_uint32(0), C.c_uint32(1), info.ctypes.data_as(C.POINTER(C.c_int64)),
                                             probe.ctypes.data_as(C.POINTER(C.c_int64)))
                q0h, Ha, kh0, sth, nkh, _, _, q0w, Wb, kw0, stw, nkw, _, _ = (int(v) for v in info)
                hs = [sh * (q0h + i) + a - ph for i in range(Ha)]
                ws_ = [sw * (q0w + j) + b - pw for j in range(Wb)]
                khs = [kh0 + sth * t for t in range(nkh)]
                kws = [kw0 + stw * t for t in range(nkw)]
                assert hs == [h for h in range(H) if (h + ph) % sh == a] and ws_ == [w for w in range(W) if (w + pw) % sw == b]
                assert khs == [k for k in range(KH) if (k * dh) % sh == a] and kws == [k for k in range(KW) if (k * dw) % sw == b]
                for h in hs:
                    for w in ws_:
                        seen_pos[h, w] += 1
                for kh in khs:
                    for kw in kws:
                        seen_taps[kh, kw] += 1
                rows, cols = N * Ha * Wb, nkh * nkw * Cout
                if rows == 0 or cols == 0:
                    continue
                for row0, col0 in ((0, 0), (max(rows - 200, 0), max(cols - 100, 0))):
                    nr, nt = min(rows - row0 + 20, 260), min(cols - col0 + 10, 130)
                    out = np.empty((nr, nt), np.int64)
                    harith.h_dgrad_phase_offsets(arr.ctypes.data_as(C.POINTER(C.c_int64)), C.c_int64(a), C.c_int64(b),
                                                 C.c_uint32(row0), C.c_uint32(nr), C.c_uint32(col0), C.c_uint32(nt),
                                                 info.ctypes.data_as(C.POINTER(C.c_int64)), out.ctypes.data_as(C.POINTER(C.c_int64)))
                    m, k = np.meshgrid(row0 + np.arange(nr), col0 + np.arange(nt), indexing="ij")
                    inside = (m < rows) & (k < cols)
                    mm, kk = np.minimum(m, rows - 1), np.minimum(k, cols - 1)
                    n_, i, j = mm // (Ha * Wb), (mm // Wb) % Ha, mm % Wb
                    th, tw, co = kk // (nkw * Cout), (kk // Cout) % nkw, kk % Cout
                    h, w = np.array(hs)[i], np.array(ws_)[j]
                    kh, kw = np.array(khs)[th], np.array(kws)[tw]
                    hsrc, wsrc = h + ph - kh * dh, w + pw - kw * dw
                    assert ((hsrc % sh == 0) & (wsrc % sw == 0)).all()          # inside a phase nothing is a structural zero
                    ok = inside & (hsrc >= 0) & (wsrc >= 0) & (hsrc // sh < Ho) & (wsrc // sw < Wo)
                    want = np.where(ok, ((n_ * Ho + hsrc // sh) * Wo + wsrc // sw) * Cout + co, -1)
                    assert np.array_equal(out, want), (geo, a, b, row0, col0)
        assert (seen_pos == 1).all() and (seen_taps == 1).all()


def test_missing_library_fails_loudly(monkeypatch, tmp_path):
    import paper_2403_09603_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_PATH", str(tmp_path / "nope.so"))
    with pytest.raises(b.VtError):
        b.load_library()


@pytest.fixture(scope="module")
def harith():
    so = os.path.join(HERE, "_host_arith.so")
    subprocess.check_call(["/opt/rocm/bin/hipcc", "-O1", "--offload-arch=gfx950", "-shared", "-fPIC", "-o", so,
                           os.path.join(HERE, "host_arith_check.hip")], stderr=subprocess.DEVNULL)
    return C.CDLL(so)


def _u32p(a):
    return a.ctypes.data_as(C.POINTER(C.c_uint32))


def test_kernel_integer_arithmetic_matches_oracle_on_host(harith):
    g = si.rng(si.seed_for(0, 9))
    rnd_bits = g.integers(0, 1 << 64, 1 << 16, dtype=np.uint64)
    e = g.integers(1023 - 160, 1023 + 130, 1 << 16, dtype=np.uint64)
    band = (rnd_bits & np.uint64(0x800FFFFFFFFFFFFF)) | (e << np.uint64(52))
    x = np.concatenate([si.edge_values(), rnd_bits.view(np.float64), band.view(np.float64),
                        si.planted_vector(1 << 14, si.seed_for(0, 10), thr=64)[0]])
    bits = np.ascontiguousarray(x).view(np.uint64)
    n = bits.size
    y, D, dr = (np.empty(n, np.uint32) for _ in range(3))
    harith.h_decide(bits.ctypes.data_as(C.POINTER(C.c_uint64)), C.c_uint64(n), _u32p(y), _u32p(D), _u32p(dr))
    yo, _, _, _ = vo.round_log(x, 0.0)
    assert np.array_equal(y, yo.view(np.uint32))
    Do = np.array([vo.boundary_distance(float(v)) for v in x], np.uint32)
    assert np.array_equal(D, Do)
    for thr in (1, 64, 1 << 27, 1 << 28):
        codes = np.array([vo.ternary_code(float(v), thr) for v in x[:30000]])
        mine = np.where(D[:30000] < thr, np.where(dr[:30000] == 1, 2, 0), 1)
        assert np.array_equal(mine, codes)
    idx = np.arange(n, dtype=np.uint32)
    for d in (0, 1):
        yd = np.empty(n, np.uint32)
        harith.h_directed(bits.ctypes.data_as(C.POINTER(C.c_uint64)), C.c_uint64(n), C.c_uint32(d), _u32p(yd))
        want = vo.round_replay(x, idx, np.full((n + 31) // 32, 0xFFFFFFFF if d else 0, np.uint32))
        assert np.array_equal(yd, want.view(np.uint32))


def test_sha256_lane_routines_on_host(harith):
    """The per-lane SHA-256 the hash kernels are built from, compiled for the host: every message length
    around the block and padding boundaries, and long random strings, against hashlib."""
    import hashlib
    rng = np.random.default_rng(0x2403096030F4)
    harith.h_sha256.argtypes = [C.c_char_p, C.c_uint64, C.c_char_p]
    lengths = list(range(0, 200)) + [255, 256, 257, 4095, 4096, 4097, 65536 + 55, 65536 + 56, 1 << 20]
    for n in lengths:
        data = rng.integers(0, 256, n, dtype=np.uint8).tobytes()
        out = C.create_string_buffer(32)
        harith.h_sha256(data, n, out)
        assert out.raw == hashlib.sha256(data).digest(), n
    out = C.create_string_buffer(32)
    harith.h_sha256(b"abc", 3, out)
    assert out.raw.hex() == "ba7816bf8f01cfea414140de5dae2223b00361a396177a9cb410ff61f20015ad"   # the standard's example


def test_hash_entry_points_validate_on_the_host(hiplib):
    L = hiplib
    vp, u64 = C.c_void_p, C.c_uint64
    L.vt_sha256_tree.restype = C.c_int
    L.vt_sha256_tree.argtypes = [vp, u64, u64, vp, vp, C.c_size_t, vp]
    L.vt_merkle_root.restype = C.c_int
    L.vt_merkle_root.argtypes = [vp, u64, vp, vp, C.c_size_t, vp]
    L.vt_workspace_bytes.restype = C.c_size_t
    L.vt_workspace_bytes.argtypes = [C.c_int, C.c_int64, C.c_int64, C.c_int64, C.c_int64]
    fake = 0x10000
    assert L.vt_sha256_tree(fake, 1024, 100, fake, fake, 1 << 20, None) == 1      # chunk not a multiple of 64
    assert L.vt_sha256_tree(fake + 8, 1024, 64, fake, fake, 1 << 20, None) == 1   # data not 16-byte aligned
    assert L.vt_sha256_tree(fake, 1024, 64, None, fake, 1 << 20, None) == 1
    assert L.vt_sha256_tree(fake, (1 << 26) + 1, 0, fake, fake, 1 << 20, None) == 4   # sequential form: size limit
    assert L.vt_sha256_tree(fake, 1 << 20, 64, fake, fake, 256, None) == 2        # workspace too small
    assert L.vt_merkle_root(fake, 0, fake, fake, 1 << 20, None) == 1
    assert L.vt_merkle_root(fake, 1000, fake, fake, 256, None) == 2
    # workspace: two ping-pong digest buffers, 32 bytes per chunk at the first level
    n, chunk = 100 << 20, 4096
    need = L.vt_workspace_bytes(6, 1, n, chunk, 1)
    assert 32 * (n // chunk) <= need <= 32 * (n // chunk) * 1.02 + 1024
    assert L.vt_workspace_bytes(6, 1, 100, 4096, 1) == 256
    assert L.vt_workspace_bytes(7, 1, 1001, 0, 1) >= 2 * 32 * 501


def test_nested_batch_validation_on_the_host(hiplib):
    L = hiplib
    vp, i64, dbl, cint = C.c_void_p, C.c_int64, C.c_double, C.c_int
    from paper_2403_09603_amd.binding import _VtLog
    L.vt_gemm_f64_round_log_nested.restype = cint
    L.vt_gemm_f64_round_log_nested.argtypes = [cint, cint, i64, i64, i64, dbl, vp, i64, i64, i64, vp, i64, i64, i64, vp,
                                               i64, i64, vp, i64, i64, vp, cint, dbl, C.POINTER(_VtLog), vp,
                                               C.c_size_t, vp]
    fake = 0x10000
    log = _VtLog(fake, fake, 1 << 20, fake, None, 32)

    def call(inner=4, outer=3, sAo=1000, sBo=1000, M=16, N=16, K=8):
        return L.vt_gemm_f64_round_log_nested(0, 0, M, N, K, 1.0, fake, K, 64, sAo, fake, N, 64, sBo, None, inner, outer,
                                              fake, N, M * N, None, 0, 0.1, C.byref(log), None, 0, None)
    assert call(inner=-1) == 1
    assert call(outer=-1) == 1
    assert call(sAo=-5) == 1
    assert call(sBo=-5) == 1
    assert call(inner=1 << 20, outer=1 << 20) == 1          # more than 2^32 matrices
    assert call() == 2                                       # valid arguments reach the workspace check


def test_threshold_window_form_equals_the_distance_test(harith):
    """The fused epilogue tests D(x) < thr as one subtraction and one unsigned compare on the dropped bits;
    against |r - 2^28| < thr for every threshold size class and every r near the edges of the window."""
    half = 1 << 28
    rng = np.random.default_rng(12)
    for thr in [0, 1, 2, 3, 31, 32, 33, 1 << 20, (1 << 28) - 1, 1 << 28]:
        near = np.array([half + s * (thr + d) for s in (-1, 1) for d in range(-3, 4)] + [0, 1, half - 1, half, half + 1,
                        (1 << 29) - 1], dtype=np.int64)
        r = np.concatenate([near[(near >= 0) & (near < (1 << 29))], rng.integers(0, 1 << 29, 20000)]).astype(np.uint32)
        out = np.zeros(r.size, np.uint8)
        harith.h_window_test(_u32p(r), C.c_uint64(r.size), C.c_uint32(thr), out.ctypes.data_as(C.POINTER(C.c_uint8)))
        expect = np.abs(r.astype(np.int64) - half) < thr
        assert np.array_equal(out.astype(bool), expect), thr
        # the shifted form takes whole low words: the same dropped bits under every pattern of the upper three
        for top in (0, 1, 5, 7):
            lo = (r | np.uint32(top << 29)).astype(np.uint32)
            harith.h_window_key_test(_u32p(lo), C.c_uint64(lo.size), C.c_uint32(thr), out.ctypes.data_as(C.POINTER(C.c_uint8)))
            assert np.array_equal(out.astype(bool), expect), (thr, top)


def test_gemm_plan_is_a_pure_host_function_of_the_shape(hiplib):
    """The plan (tile, split factor) depends on the shape, the A layout and the density of C alone: same
    answer every time, splits only for dense outputs and long K, at least eight k steps per slice, and a
    workspace that covers the largest split factor of any layout."""
    import paper_2403_09603_amd as vt
    INVALID = 1
    tm, tn, sp = (C.c_int(), C.c_int(), C.c_int())
    f = hiplib.vt_gemm_plan
    assert f(2, 64, 64, 64, 1, 64, 4096, C.byref(tm), C.byref(tn), C.byref(sp)) == INVALID          # no such layout
    assert f(0, -1, 64, 64, 1, 64, 4096, C.byref(tm), C.byref(tn), C.byref(sp)) == INVALID
    assert f(0, 64, 64, 64, 1, 64, 4096, None, C.byref(tn), C.byref(sp)) == INVALID
    g = np.random.default_rng(7)
    for _ in range(300):
        M, N, K = (int(v) for v in (g.integers(1, 5000), g.integers(1, 3000), g.integers(1, 200000)))
        batch = int(g.choice([1, 1, 3]))
        for layout in (vt.VT_A_ROW_MAJOR, vt.VT_A_TRANSPOSED, vt.VT_A_IM2COL_T):
            p = vt.vt_gemm_plan(M, N, K, batch, transA=layout)
            assert p == vt.vt_gemm_plan(M, N, K, batch, transA=layout)
            assert p[:2] in ((128, 128), (64, 64)) and 1 <= p[2] <= 256
            if p[2] > 1:
                assert ((K + 15) // 16) // p[2] >= 8
                need = hiplib.vt_workspace_bytes(vt.VT_OP_GEMM_ROUND_LOG, M, N, K, batch)
                assert need >= 8 * M * N * batch * p[2]                          # room for every slab
            assert vt.vt_gemm_plan(M, N, K, batch, ldc=N + 1, transA=layout)[2] == 1   # padded rows: never split
