"""The C-ABI library without a GPU: it loads, exports what include/zipvl.h
declares, and rejects bad arguments on the host before touching the device."""
import ctypes as C
import os
import re

import pytest

import paper_2410_08584_amd as z
from paper_2410_08584_amd.binding import Dims

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(z.library_path()):
        from paper_2410_08584_amd.build import build_library
        build_library(verbose=False)
    return z.load_library()


def _dims(B=1, Hq=4, Hkv=4, n=128, d=64, dtype=0, strides=None):
    dm = Dims()
    dm.B, dm.Hq, dm.Hkv, dm.n, dm.d, dm.dtype = B, Hq, Hkv, n, d, dtype
    s = strides or (Hq * n * d, n * d, d)
    dm.q_strides = (C.c_int64 * 3)(*s)
    dm.k_strides = (C.c_int64 * 3)(Hkv * n * d, n * d, d)
    dm.v_strides = (C.c_int64 * 3)(Hkv * n * d, n * d, d)
    return dm


def test_every_declared_symbol_is_exported(lib):
    inc = os.path.join(ROOT, "include")
    header = "".join(open(os.path.join(inc, f)).read() for f in sorted(os.listdir(inc)) if f.endswith(".h"))
    declared = set(re.findall(r"\b(zipvl_[a-z_0-9]+)\s*\(", header))
    assert declared == set(z.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name
    assert z.zipvl_version() >= 100


def test_workspace_sizes(lib):
    dm = _dims(B=1, Hq=28, Hkv=4, n=18432, d=128, dtype=1)
    assert z.workspace_bytes(z.OP_SPARSE_PREFILL, dm) == 2 * 4 * 18432 * 128 * 2
    assert z.workspace_bytes(z.OP_SELECT, dm) == 4 * 4096 * 12      # per unit: 4096 packed 64-bit slots and 4096 counts
    assert z.workspace_bytes(z.OP_SCORE, dm, 64) > 0
    assert z.workspace_bytes(z.OP_DECODE, dm) > 0
    # the fused decode step adds one 256-byte-rounded block of per-unit arrival counters in front of the partial states
    assert z.workspace_bytes(z.OP_DECODE_STEP, dm) == z.workspace_bytes(z.OP_DECODE, dm) + 256
    assert z.workspace_bytes(99, dm) == 0 and "unknown op" in z.zipvl_last_error()


FAKE = C.c_void_p(0x1000)          # aligned, never dereferenced: every call below is rejected first


def _score(lib, dm, probes, scale=0.125, Q=FAKE, K=FAKE, mass=FAKE, ws=FAKE, ws_bytes=1 << 30, flags=0):
    arr = (C.c_int32 * max(1, len(probes)))(*probes)
    return lib.zipvl_score(Q, K, C.byref(dm), arr, len(probes), C.c_float(scale), flags, mass, FAKE, ws, ws_bytes, None)


def test_score_rejects_bad_arguments(lib):
    ok = list(range(64, 128))
    assert _score(lib, _dims(Hq=4, Hkv=3), ok) == -2 and "multiple" in z.zipvl_last_error()
    assert _score(lib, _dims(d=96), ok) == -2
    assert _score(lib, _dims(dtype=7), ok) == -5
    assert _score(lib, _dims(n=0), ok) == -1
    assert _score(lib, _dims(), ok, Q=None) == -1
    assert _score(lib, _dims(), ok, Q=C.c_void_p(0x1004)) == -3
    assert _score(lib, _dims(strides=(4 * 128 * 64, 128 * 64, 66)), ok) == -3
    assert _score(lib, _dims(), [5, 5, 6]) == -1 and "ascending" in z.zipvl_last_error()
    assert _score(lib, _dims(), [5, 128]) == -1
    assert _score(lib, _dims(), []) == -1
    assert _score(lib, _dims(n=256), list(range(129))) == -2
    assert _score(lib, _dims(), ok, scale=0.0) == -1
    assert _score(lib, _dims(), ok, ws=None) == -4
    assert _score(lib, _dims(), ok, ws_bytes=16) == -4 and "workspace" in z.zipvl_last_error()
    assert _score(lib, _dims(), ok, flags=2) == -5 and "flags" in z.zipvl_last_error()


def test_select_rejects_bad_arguments(lib):
    f = lib.zipvl_select
    assert f(None, None, 1, 8, C.c_double(0.9), FAKE, FAKE, None, None, 0, None) == -1
    assert f(FAKE, None, 0, 8, C.c_double(0.9), FAKE, FAKE, None, None, 0, None) == -1
    assert f(FAKE, None, 1, 8, C.c_double(0.0), FAKE, FAKE, None, None, 0, None) == -1
    assert f(FAKE, None, 1, 8, C.c_double(1.5), FAKE, FAKE, None, None, 0, None) == -1
    assert f(FAKE, None, 1, 8, C.c_double(float("nan")), FAKE, FAKE, None, None, 0, None) == -1
    assert f(C.c_void_p(0x1002), None, 1, 8, C.c_double(0.9), FAKE, FAKE, None, None, 0, None) == -3
    assert f(FAKE, None, 1, 8, C.c_double(0.9), FAKE, FAKE, C.c_void_p(0x1002), None, 0, None) == -3          # status word misaligned
    assert f(FAKE, None, 1, 8, C.c_double(0.9), FAKE, FAKE, None, FAKE, 64, None) == -4 and "workspace" in z.zipvl_last_error()


def test_prefill_compact_decode_reject_bad_arguments(lib):
    dm = _dims()
    sp = lib.zipvl_sparse_prefill
    assert sp(FAKE, FAKE, FAKE, C.byref(dm), FAKE, None, C.c_float(0.1), 0, FAKE, FAKE, 1 << 30, None) == -1
    assert sp(FAKE, FAKE, FAKE, C.byref(dm), None, None, C.c_float(0.1), 16, FAKE, FAKE, 1 << 30, None) == -5
    assert sp(FAKE, FAKE, FAKE, C.byref(dm), None, None, C.c_float(0.1), 0, FAKE, FAKE, 8, None) == -4
    assert sp(FAKE, FAKE, FAKE, C.byref(dm), None, None, C.c_float(0.1), 0, FAKE, C.c_void_p(0x1010), 1 << 30, None) == -3
    ck = lib.zipvl_compact_kv
    assert ck(FAKE, FAKE, C.byref(dm), None, None, FAKE, FAKE, 0, FAKE, 0, None) == -1
    assert ck(FAKE, FAKE, C.byref(dm), FAKE, None, FAKE, FAKE, 16, FAKE, 0, None) == -1
    assert ck(FAKE, FAKE, C.byref(dm), None, None, FAKE, FAKE, 16, None, 0, None) == -1
    assert ck(FAKE, FAKE, C.byref(dm), None, None, FAKE, FAKE, 16, FAKE, 3, None) == -5
    sh = lib.zipvl_share_scores
    assert sh(None, None, 1, 4, 8, FAKE, None, None) == -1
    assert sh(FAKE, FAKE, 1, 4, 8, FAKE, None, None) == -1
    assert sh(FAKE, None, 1, 0, 8, FAKE, None, None) == -1
    assert sh(C.c_void_p(0x1002), None, 1, 4, 8, FAKE, None, None) == -3
    dc = lib.zipvl_decode_attn
    assert dc(FAKE, FAKE, FAKE, None, 16, C.byref(dm), C.c_float(0.1), FAKE, FAKE, 1 << 30, None) == -1
    assert dc(FAKE, FAKE, FAKE, FAKE, 16, C.byref(dm), C.c_float(0.1), FAKE, FAKE, 4, None) == -4
    ap = lib.zipvl_kv_append
    assert ap(FAKE, FAKE, None, 16, FAKE, FAKE, C.byref(dm), None) == -1
    assert ap(FAKE, FAKE, FAKE, 0, FAKE, FAKE, C.byref(dm), None) == -1


def test_decode_attn_static_rejects_dims_beyond_its_scratch(lib):
    dm = _dims(B=256, Hq=128, Hkv=128, n=4096, d=128, dtype=1)     # 32768 heads x 520 bytes of partial state
    assert z.workspace_bytes(z.OP_DECODE, dm) > (8 << 20)
    rc = lib.zipvl_decode_attn_static(FAKE, FAKE, FAKE, FAKE, 4096, C.byref(dm), C.c_float(0.1), FAKE, None)
    assert rc == -2 and "scratch" in z.zipvl_last_error()
    assert lib.zipvl_decode_attn_static(FAKE, FAKE, FAKE, None, 4096, C.byref(_dims()), C.c_float(0.1), FAKE, None) == -1


def test_missing_library_fails_loudly(monkeypatch):
    import paper_2410_08584_amd.binding as b
    monkeypatch.setattr(b, "_lib", None)
    monkeypatch.setattr(b, "_LIB_NAME", "libzipvl_not_built.so")
    with pytest.raises(z.ZipvlError):
        b.load_library()


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU: any other count ends with a message and a non-zero status, before any GPU work."""
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    r = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"], capture_output=True, text=True, timeout=120)
    assert r.returncode != 0
    assert "one GPU" in r.stderr
    assert r.stdout.strip() == ""
