"""The oracle under AddressSanitizer and UndefinedBehaviorSanitizer (host code, CPU only): a
stand-alone driver (oracle/sanitize_driver.c, which includes the oracle's source) is built with
-fsanitize=address,undefined, run on the Tiny configuration and on a ragged shape, and its
results are compared byte for byte with the ordinary build's.  A memory error or undefined
operation anywhere in the oracle ends the driver with a sanitizer report."""
import os
import subprocess

import numpy as np
import pytest

import oracle
import workloads as wl

HERE = os.path.dirname(os.path.abspath(__file__))
SRC = os.path.join(os.path.dirname(HERE), "oracle", "sanitize_driver.c")


@pytest.fixture(scope="module")
def driver(tmp_path_factory):
    exe = str(tmp_path_factory.mktemp("san") / "orc_san")
    cmd = ["gcc", "-O1", "-g", "-std=c11", "-ffp-contract=off", "-fno-fast-math",
           "-fsanitize=address,undefined", "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer",
           "-static-libasan", "-static-libubsan", "-Wno-unknown-pragmas", "-o", exe, SRC, "-lm"]
    r = subprocess.run(cmd, capture_output=True, text=True)
    if r.returncode != 0:
        pytest.skip("sanitizer build not available here: " + r.stderr[-300:])
    return exe


def _expected(Ys, idx, E, G):
    """What the driver writes, from the ordinary build through the Python wrapper."""
    N, T = len(Ys), Ys[0].shape[0]
    k = idx.size
    parts = []
    for bits in (4, 3):
        msgs = [oracle.encode(Y, idx, G, bits=bits) for Y in Ys]
        for mg in msgs:
            parts += [mg.outl, mg.codes, mg.scale, mg.zero]
        parts.append(oracle.decode_reduce(msgs, idx, E, G, oracle.ACC_FP32, out_fp32=True, bits=bits))
        parts.append(oracle.decode_reduce(msgs, idx, E, G, oracle.ACC_BF16, out_fp32=False, bits=bits))
        if bits == 4:
            bias = Ys[1 if N > 1 else 0][0]
            parts.append(oracle.decode_reduce_fused(msgs, idx, E, G, addend=Ys[0], bias=bias,
                                                    accum=oracle.ACC_BF16, out_fp32=False))
    m = np.zeros((N, E), np.float32)
    M = np.zeros((N, E), np.float32)
    for i in range(N):
        for s in range(N):
            oracle.calibrate_update(Ys[(i + s) % N], m[i], M[i], first=(s == 0), gamma=0.25)
    R, Rbar, idx_s, idx_r = oracle.calibrate_finalize(m, M, k)
    parts += [m.copy(), M.copy(), R, Rbar, idx_s.astype(np.int32), idx_r.astype(np.int32)]
    step, inv = oracle.static_params(m, M)
    parts += [step, inv]
    smsgs = [oracle.encode_static(Ys[i], idx, inv[i]) for i in range(N)]
    for mg in smsgs:
        parts += [mg.outl, mg.codes]
    parts.append(oracle.decode_reduce_static(smsgs, idx, step, oracle.ACC_BF16, out_fp32=False))
    if N >= 2:   # the linear layer: device 0's tensor times the first rows of device 1's
        Yl, mag = oracle.linear(Ys[0], Ys[1][: min(T, 7)], with_magnitude=True)
        parts += [Yl, mag]
    return b"".join(np.ascontiguousarray(p).tobytes() for p in parts)


def _run(driver, tmp_path, Ys, idx, E, G):
    N, T = len(Ys), Ys[0].shape[0]
    fin, fout = str(tmp_path / "in.bin"), str(tmp_path / "out.bin")
    with open(fin, "wb") as f:
        f.write(np.array([N, T, E, idx.size, G], np.int32).tobytes())
        f.write(idx.astype(np.int32).tobytes())
        for Y in Ys:
            f.write(np.ascontiguousarray(Y, dtype=np.uint16).tobytes())
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    r = subprocess.run([driver, fin, fout], capture_output=True, text=True, timeout=300, env=env)
    assert r.returncode == 0, "driver failed (%d):\n%s" % (r.returncode, r.stderr[-2000:])
    assert "runtime error" not in r.stderr and "AddressSanitizer" not in r.stderr, r.stderr[-2000:]
    with open(fout, "rb") as f:
        return f.read()


def test_tiny_configuration_under_sanitizers(driver, tmp_path):
    w = wl.TINY
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w)]
    cols, _ = wl.outlier_columns(w)
    idx = np.sort(cols.numpy()).astype(np.int32)
    assert _run(driver, tmp_path, Ys, idx, w.E, w.G) == _expected(Ys, idx, w.E, w.G)


@pytest.mark.parametrize("E,k,G,T,N", [(1032, 1, 128, 3, 2),    # odd r: the pad nibble, a ragged last group
                                        (64, 0, 32, 2, 1),       # nothing selected, one device
                                        (96, 95, 32, 2, 2),      # a single quantised feature
                                        (40, 40, 32, 2, 2)])     # everything selected
def test_ragged_shapes_under_sanitizers(driver, tmp_path, E, k, G, T, N):
    rng = np.random.default_rng(E + k)
    Ys = []
    for i in range(N):
        x = (rng.standard_normal((T, E)) * 3).astype(np.float32)
        x[:, ::7] *= 30
        x[0, : E // 2] = 0.0
        Ys.append((x.view(np.uint32) >> 16).astype(np.uint16))      # truncation is fine: any bf16 pattern will do
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    assert _run(driver, tmp_path, Ys, idx, E, G) == _expected(Ys, idx, E, G)
