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


def test_argument_validation_happens_on_the_host(hiplib):
    """None of these calls may reach a kernel launch: they run here without a GPU."""
    import paper_2403_09603_amd.binding as b
    cnt = (C.c_uint64 * 1)()
    log = b._VtLog(None, None, 0, C.addressof(cnt))
    fake = C.c_void_p(0x1000)
    INVALID, WORKSPACE = 1, 2
    assert hiplib.vt_round_log(fake, 16, 0.75, fake, C.byref(log), fake, 1 << 20, None) == INVALID   # tau
    assert hiplib.vt_round_log(fake, 1 << 32, 0.1, fake, C.byref(log), fake, 1 << 20, None) == INVALID  # n
    assert hiplib.vt_round_log(None, 16, 0.1, fake, C.byref(log), fake, 1 << 20, None) == INVALID
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, None, fake, 1 << 20, None) == INVALID
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, C.byref(log), None, 0, None) == WORKSPACE
    assert hiplib.vt_round_log(fake, 1 << 20, 0.1, fake, C.byref(log), fake, 1024, None) == WORKSPACE
    badlog = b._VtLog(None, None, 8, C.addressof(cnt))
    assert hiplib.vt_round_log(fake, 16, 0.1, fake, C.byref(badlog), fake, 1 << 20, None) == INVALID
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
    assert hiplib.vt_threshold_stats(fake, fake, 16, None, None) == INVALID
    assert hiplib.vt_strerror(INVALID).decode() == "invalid argument"


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
