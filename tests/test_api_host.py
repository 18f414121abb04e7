"""Host-side logic of the C ABI: exports, layout arithmetic, argument validation.

No compute call is made here: every call below either fails its argument check
(detected before anything is enqueued) or has nothing to do (T = 0), so the fake
pointers are never dereferenced and the tests run without a GPU.
"""
import ctypes
import os
import re

import pytest

import paper_2411_07942_amd as tpq
from refmath import payload_bits, wire_bytes_per_row

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "tpq.h")).read()
    declared = set(re.findall(r"\b(tpq_[a-z_]+)\s*\(", header))
    assert declared == set(tpq.EXPORTS)
    lib = tpq._load()
    for name in declared:
        assert hasattr(lib, name), name


@pytest.mark.parametrize("E,k,G,W,pb,wb", [
    (512, 8, 128, 284, 4.1875, 4.4375),
    (5120, 80, 128, 2840, 4.1875, 4.4375),
    (4608, 72, 128, 2556, 4.1875, 4.4375),
    (8192, 128, 128, 4540, 4.1875, 4.43359375),
    (8192, 128, 64, 4792, 4.1875, 4.6796875),
    (8192, 341, 128, 4856, None, 4.7421875),
    (8192, 341, 64, 5100, None, 4.98046875),
])
def test_layout_closed_forms(E, k, G, W, pb, wb):
    """Bits per value: 4 + 12k/E (paper abstract / Sec. 4); wire adds scale + zero."""
    L = tpq.layout_init(E, k, G)
    assert (L.r, L.ng, L.code_bytes) == (E - k, -(-(E - k) // G), (E - k + 1) // 2)
    assert L.wire_bytes_per_row == W == wire_bytes_per_row(E, k, G)
    assert tpq.payload_bits(L) == payload_bits(E, k) == 4 + 12 * k / E
    if pb is not None:
        assert tpq.payload_bits(L) == pb < 4.2
    assert tpq.wire_bits(L) == wb == 8 * W / E
    for p in (L.pitch_codes, L.pitch_meta, L.pitch_outl):
        assert p % 16 == 0
    assert L.pitch_codes >= L.code_bytes and L.pitch_meta >= 2 * L.ng and L.pitch_outl >= 2 * k
    assert tpq.plan_bytes(L) >= 64 + 4 * k + 2 * (E - k)


@pytest.mark.parametrize("b", [2, 3, 4, 5, 6, 8])
@pytest.mark.parametrize("E,k,G", [(512, 8, 128), (5120, 80, 128), (1032, 1, 64), (64, 64, 32)])
def test_layout_other_widths(E, k, G, b):
    """b bits for the quantised features (Sec. 4, Fig. 3): b + (16 - b) k / E per value."""
    L = tpq.layout_init(E, k, G, b)
    r = E - k
    assert (L.bits, L.r, L.ng, L.code_bytes) == (b, r, -(-r // G), (r * b + 7) // 8)
    assert tpq.payload_bits(L) == b + (16 - b) * k / E
    assert L.wire_bytes_per_row == 2 * k + L.code_bytes + 4 * L.ng
    assert L.pitch_codes % 16 == 0 and L.pitch_codes >= L.code_bytes
    if b != 4 and r > 0:     # whole chunks are stored, 8 bytes are read from the start of each
        assert L.pitch_codes >= -(-r // 8) * b + 8


def test_k_floor_E_over_64_is_under_4p2_bits():
    for E in (512, 4096, 4608, 5120, 8192, 16384):
        assert tpq.payload_bits(tpq.layout_init(E, E // 64, 128)) < 4.2


@pytest.mark.parametrize("args,code", [
    ((512, 8, 128, 7), tpq.ERR_UNSUPPORTED),
    ((512, 8, 128, 1), tpq.ERR_UNSUPPORTED),
    ((512, 8, 128, 16), tpq.ERR_UNSUPPORTED),
    ((512, 8, 100, 4), tpq.ERR_UNSUPPORTED),
    ((512, 8, 16, 4), tpq.ERR_UNSUPPORTED),
    ((500, 8, 128, 4), tpq.ERR_SHAPE),
    ((0, 0, 128, 4), tpq.ERR_SHAPE),
    ((512, 513, 128, 4), tpq.ERR_SHAPE),
    ((512, -1, 128, 4), tpq.ERR_SHAPE),
    ((tpq.MAX_E + 8, 0, 128, 4), tpq.ERR_SHAPE),
])
def test_layout_init_rejects(args, code):
    with pytest.raises(tpq.TpqError) as e:
        tpq.layout_init(*args)
    assert e.value.code == code


def _fake(addr=0x10000):
    return ctypes.c_void_p(addr)


def _ptrs(n, addr=0x10000):
    arr = (ctypes.c_void_p * n)()
    for i in range(n):
        arr[i] = addr + 0x1000 * i
    return arr


def test_encode_argument_errors():
    lib = tpq._load()
    L = tpq.layout_init(512, 8, 128)
    LP = ctypes.byref(L)
    ok = dict(plan=_fake(), Y=_ptrs(2), ldY=512, n=2, T=4, c=_ptrs(2), s=_ptrs(2), z=_ptrs(2), o=_ptrs(2))

    def call(**kw):
        a = dict(ok, **kw)
        return lib.tpq_encode(a.get("L", LP), a["plan"], a["Y"], a["ldY"], a["n"], a["T"], a["c"],
                              a["s"], a["z"], a["o"], None)
    assert call(L=None) == tpq.ERR_NULL
    assert call(plan=None) == tpq.ERR_NULL
    assert call(Y=None) == tpq.ERR_NULL
    assert call(c=None) == tpq.ERR_NULL
    assert call(o=None) == tpq.ERR_NULL
    assert call(n=0) == tpq.ERR_SHAPE
    assert call(n=tpq.MAX_RANKS + 1) == tpq.ERR_SHAPE
    assert call(T=-1) == tpq.ERR_SHAPE
    assert call(ldY=504) == tpq.ERR_SHAPE
    assert call(ldY=516) == tpq.ERR_ALIGN
    assert call(plan=_fake(0x10008)) == tpq.ERR_ALIGN
    assert call(Y=_ptrs(2, 0x10002)) == tpq.ERR_ALIGN
    hole = _ptrs(2)
    hole[1] = None
    assert call(z=hole) == tpq.ERR_NULL
    assert call(T=0) == tpq.OK                      # nothing to do, nothing enqueued
    # a layout whose derived fields were tampered with is refused
    bad = tpq.layout_init(512, 8, 128)
    bad.ng = 3
    assert call(L=ctypes.byref(bad)) == tpq.ERR_SHAPE
    bad = tpq.layout_init(512, 8, 128)
    bad.pitch_codes = 250
    assert call(L=ctypes.byref(bad)) == tpq.ERR_ALIGN
    bad.pitch_codes = 240
    assert call(L=ctypes.byref(bad)) == tpq.ERR_SHAPE


def test_decode_argument_errors():
    lib = tpq._load()
    L = tpq.layout_init(512, 8, 128)
    LP = ctypes.byref(L)
    ok = dict(plan=_fake(), n=2, T=4, c=_ptrs(2), s=_ptrs(2), z=_ptrs(2), o=_ptrs(2), acc=0, od=0,
              out=_fake(0x90000), ld=512)

    def call(**kw):
        a = dict(ok, **kw)
        return lib.tpq_decode_reduce(LP, a["plan"], a["n"], a["T"], a["c"], a["s"], a["z"], a["o"],
                                     a["acc"], a["od"], a["out"], a["ld"], None)
    assert call(acc=3) == tpq.ERR_UNSUPPORTED  # 0, 1, 2 are the modes
    assert call(od=3) == tpq.ERR_UNSUPPORTED
    assert call(out=None) == tpq.ERR_NULL
    assert call(out=_fake(0x90004)) == tpq.ERR_ALIGN
    assert call(ld=500) == tpq.ERR_SHAPE
    assert call(ld=516) == tpq.ERR_ALIGN
    assert call(ld=518, od=1) == tpq.ERR_ALIGN      # fp32 rows: multiples of 4 elements
    assert call(n=65) == tpq.ERR_SHAPE
    assert call(s=None) == tpq.ERR_NULL
    assert call(T=0) == tpq.OK


def test_calibrate_and_plan_argument_errors():
    lib = tpq._load()
    f = _fake
    assert tpq.calibrate_workspace_bytes(16384, 4608) > 0
    assert tpq.calibrate_workspace_bytes(16384, 4609) == 0
    ws = tpq.calibrate_workspace_bytes(64, 512)
    call = lib.tpq_calibrate
    assert call(None, 64, 512, 512, 0, 4, 0, 0.01, f(), f(), f(), ws, None) == tpq.ERR_NULL
    assert call(f(), 64, 512, 512, 4, 4, 0, 0.01, f(), f(), f(), ws, None) == tpq.ERR_SHAPE
    assert call(f(), 64, 512, 512, 0, 4, -1, 0.01, f(), f(), f(), ws, None) == tpq.ERR_SHAPE
    assert call(f(), 64, 512, 512, 0, 4, 0, 1.5, f(), f(), f(), ws, None) == tpq.ERR_SHAPE
    assert call(f(), 64, 500, 512, 0, 4, 0, 0.01, f(), f(), f(), ws, None) == tpq.ERR_SHAPE
    assert call(f(), 64, 520, 512, 0, 4, 0, 0.01, f(), f(), f(), ws - 1, None) == tpq.ERR_WORKSPACE
    assert call(f(0x10002), 64, 512, 512, 0, 4, 0, 0.01, f(), f(), f(), ws, None) == tpq.ERR_ALIGN
    assert call(f(), 0, 512, 512, 0, 4, 0, 0.01, f(), f(), f(), ws, None) == tpq.OK
    fin = lib.tpq_calibrate_finalize
    wsf = tpq.calibrate_finalize_workspace_bytes(512)
    assert fin(f(), f(), 4, 512, 513, None, f(), f(), None, f(), wsf, None) == tpq.ERR_SHAPE
    assert fin(f(), f(), 4, 512, 8, None, None, f(), None, f(), wsf, None) == tpq.ERR_NULL
    assert fin(f(), f(), 4, 512, 8, None, f(), f(), None, f(), wsf - 1, None) == tpq.ERR_WORKSPACE
    L = tpq.layout_init(512, 8, 128)
    assert lib.tpq_plan_build(ctypes.byref(L), f(), f(), tpq.plan_bytes(L) - 1, None) == tpq.ERR_WORKSPACE
    assert lib.tpq_plan_build(ctypes.byref(L), None, f(), tpq.plan_bytes(L), None) == tpq.ERR_NULL
    assert lib.tpq_plan_build(ctypes.byref(L), f(), f(0x10004), tpq.plan_bytes(L), None) == tpq.ERR_ALIGN


def test_strerror_covers_every_code():
    lib = tpq._load()
    seen = set()
    for code in range(0, -8, -1):
        s = lib.tpq_strerror(code).decode()
        assert s and s != "unknown error"
        seen.add(s)
    assert len(seen) == 8
    assert lib.tpq_strerror(-99).decode() == "unknown error"


def test_bench_refuses_more_than_one_gpu():
    """bench.py measures one GPU; asking for more ends with a message, before anything runs."""
    import os
    import subprocess
    import sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    p = subprocess.run([sys.executable, os.path.join(root, "bench.py"), "--gpus", "2"],
                       capture_output=True, text=True, timeout=120)
    assert p.returncode != 0
    assert "one GPU" in (p.stdout + p.stderr)
