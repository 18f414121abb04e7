"""Pins for the oracle's encode / decode_reduce.

What the paper and the mathematics fix (Sec. 1: summed quantisation errors follow
the Irwin-Hall law; Sec. 1 and 4: 16 -> 4 + 12k/E bits per value, k = floor(E/64)
gives 4.1875 < 4.2; Fig. 2 and Sec. 3: selected features travel in BF16, i.e.
verbatim; Sec. 2: the devices' outputs are summed) is checked here against
definitions written independently of the oracle: a float64 search over all 16
codes, closed forms, torch's own bf16 conversion, numpy sums.
"""
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from refmath import (bits_to_f32, compaction, f32_to_bf16_bits_lib, f32_vals_to_bits,
                     group_expand, payload_bits, unpack_codes, wire_bytes_per_row)

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "codec_worked_example.txt")


def _tiny_inputs():
    w = wl.TINY
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w)]
    cols, _ = wl.outlier_columns(w)
    idx = np.sort(cols.numpy()).astype(np.int32)
    assert idx.size == w.k
    return w, Ys, idx


def test_worked_example():
    spec = {}
    for line in open(GOLDEN):
        line = line.strip()
        if line and not line.startswith("#"):
            key, *rest = line.split()
            spec[key] = rest
    E, G = int(spec["E"][0]), int(spec["G"][0])
    idx = np.array([int(v) for v in spec["idx"]], np.int32)
    Y = f32_vals_to_bits(np.array([[float(v) for v in spec["row"]]], np.float32))
    msg = oracle.encode(Y, idx, G)
    assert bits_to_f32(msg.outl)[0].tolist() == [float(v) for v in spec["expect_outl"]]
    assert msg.codes[0].tolist() == [int(v, 16) for v in spec["expect_codes"]]
    assert bits_to_f32(msg.scale)[0].tolist() == [float(v) for v in spec["expect_scale"]]
    assert bits_to_f32(msg.zero)[0].tolist() == [float(v) for v in spec["expect_zero"]]
    xh = oracle.dequantize(msg, idx, E, G)
    assert xh[0].tolist() == [float(v) for v in spec["expect_dequant"]]
    for accum in (oracle.ACC_FP32, oracle.ACC_BF16):
        s2 = oracle.decode_reduce([msg, msg], idx, E, G, accum, out_fp32=False)
        assert bits_to_f32(s2)[0].tolist() == [float(v) for v in spec["expect_sum2"]]


def _check_message_against_definitions(Y, idx, G, msg):
    """zero = group min, scale = bf16((max-min)/15), code = nearest of 16 levels."""
    T, E = Y.shape
    k = idx.size
    r = E - k
    comp = compaction(idx, E)
    x = bits_to_f32(Y)
    # (1) selected features are copied verbatim
    assert np.array_equal(msg.outl, Y[:, idx])
    if r == 0:
        return
    xc = x[:, comp].astype(np.float64)
    ng = (r + G - 1) // G
    pad = ng * G - r
    xp = np.pad(xc, ((0, 0), (0, pad)), mode="edge").reshape(T, ng, G)
    if pad:  # the padded tail repeats the last real value: harmless for min/max
        pass
    mn, mx = xp.min(2), xp.max(2)
    # (2) zero is the group minimum (+0 for a zero), stored exactly
    zero = bits_to_f32(msg.zero).astype(np.float64)
    assert np.array_equal(zero, mn + 0.0)
    assert not np.any(msg.zero == 0x8000)
    # (3) scale is (max-min)/15 rounded to bf16 by the library conversion
    s32 = ((mx - mn).astype(np.float32) / np.float32(15.0)).astype(np.float32)
    s_lib = f32_to_bf16_bits_lib(s32)
    degenerate = bits_to_f32(s_lib) < 1e-30
    assert np.array_equal(msg.scale, np.where(degenerate, 0, s_lib).astype(np.uint16))
    # (4) brute force: the chosen code minimises |x - (zero + q*scale)| over q = 0..15
    codes, padnib = unpack_codes(msg.codes, r)
    assert np.all(padnib == 0)
    s_el = group_expand(bits_to_f32(msg.scale).astype(np.float64), G, r)
    z_el = group_expand(zero, G, r)
    levels = z_el[..., None] + np.arange(16)[None, None, :] * s_el[..., None]
    dist = np.abs(xc[..., None] - levels)
    best = dist.min(-1)
    chosen = np.take_along_axis(dist, codes[..., None].astype(np.int64), -1)[..., 0]
    # a tie region of 2^-16 steps: the encoder multiplies by a rounded reciprocal
    assert np.all(chosen <= best + s_el * 2.0 ** -16)
    deg_el = group_expand(degenerate, G, r)
    assert np.all(codes[deg_el] == 0)
    # (5) error bound: half a step (fp32 dequantisation), group minimum exact
    xh = z_el + codes * s_el
    err = np.abs(xh - xc)
    assert np.all(err <= 0.5 * s_el * (1 + 2.0 ** -18) + 15e-30)
    # the group maximum lands on code 15; its error is the bf16 rounding of the
    # step (relative 2^-8 at most) times 15, far below half a step
    is_max = xc == group_expand(mx, G, r)
    assert np.all(codes[is_max & ~deg_el] == 15)
    assert np.all(err[is_max] <= 15 * s_el[is_max] * 2.0 ** -8 * (1 + 2.0 ** -12) + 15e-30)
    is_min = xc == z_el
    assert np.all(err[is_min] == 0)


def test_tiny_brute_force_all_ranks():
    w, Ys, idx = _tiny_inputs()
    for Y in Ys:
        msg = oracle.encode(Y, idx, w.G)
        _check_message_against_definitions(Y, idx, w.G, msg)


@pytest.mark.parametrize("E,k,G,T", [(96, 0, 32, 5), (96, 3, 32, 4), (104, 7, 32, 3),
                                     (256, 11, 64, 6), (520, 9, 128, 3), (64, 64, 32, 2),
                                     (40, 1, 8, 9), (16, 15, 4, 3)])
def test_brute_force_shapes(E, k, G, T):
    """Ragged last group, odd r (pad nibble), k = 0, k = E, single-element groups."""
    rng = np.random.default_rng(E * 1000 + k)
    x = rng.standard_normal((T, E)).astype(np.float32)
    x[:, ::7] *= 40
    x[0, :] = 0.0                    # constant row: every group degenerate
    if T > 1:
        x[1, : E // 2] = -3.25       # constant half
    Y = f32_to_bf16_bits_lib(x)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    msg = oracle.encode(Y, idx, G)
    _check_message_against_definitions(Y, idx, G, msg)


def test_round_trip_single_device_and_grid_inputs():
    """N = 1: outlier columns bit-identical; inputs on the code grid come back exactly."""
    rng = np.random.default_rng(7)
    T, E, k, G = 8, 256, 4, 64
    idx = np.array([3, 64, 65, 255], np.int32)
    q = rng.integers(0, 16, (T, E))
    q[:, 0] = 0
    q[:, 1] = 15                       # every group of the compacted row spans 0..15
    q[:, 70] = 0
    q[:, 71] = 15
    q[:, 130:132] = [0, 15]
    q[:, 200:202] = [0, 15]
    x = (q * 0.5 - 2.0).astype(np.float32)   # scale 0.5, zero -2: exact in bf16
    Y = f32_vals_to_bits(x)
    msg = oracle.encode(Y, idx, G)
    out = oracle.decode_reduce([msg], idx, E, G, oracle.ACC_FP32, out_fp32=False)
    comp = compaction(idx, E)
    # groups that contain both a 0 and a 15 code reproduce the grid exactly
    codes, _ = unpack_codes(msg.codes, E - k)
    assert np.array_equal(out[:, idx], Y[:, idx])
    assert np.array_equal(bits_to_f32(out)[:, comp], x[:, comp])
    assert np.array_equal(codes, q[:, comp])
    out_b = oracle.decode_reduce([msg], idx, E, G, oracle.ACC_BF16, out_fp32=False)
    assert np.array_equal(out_b, out)


def test_k_equals_E_is_plain_sum():
    """Everything in BF16: decode_reduce is the textbook sum of N bf16 tensors."""
    rng = np.random.default_rng(8)
    N, T, E = 5, 7, 48
    idx = np.arange(E, dtype=np.int32)
    Ys = [f32_to_bf16_bits_lib(rng.standard_normal((T, E)).astype(np.float32) * 3) for _ in range(N)]
    msgs = [oracle.encode(Y, idx, 32) for Y in Ys]
    out = oracle.decode_reduce(msgs, idx, E, 32, oracle.ACC_FP32, out_fp32=True)
    ref = np.zeros((T, E), np.float64)
    for Y in Ys:
        ref += bits_to_f32(Y)
    assert np.allclose(out, ref, rtol=1e-6, atol=1e-6)
    # sequential fp32 sum in ascending device order, exactly
    acc = bits_to_f32(Ys[0]).copy()
    for Y in Ys[1:]:
        acc = (acc + bits_to_f32(Y)).astype(np.float32)
    assert np.array_equal(out, acc)
    out_b = oracle.decode_reduce(msgs, idx, E, 32, oracle.ACC_FP32, out_fp32=False)
    assert np.array_equal(out_b, f32_to_bf16_bits_lib(acc))
    # literal bf16 chain against torch's bf16 adds
    import torch
    t = wl.from_bits(Ys[0]).clone()
    for Y in Ys[1:]:
        t = t + wl.from_bits(Y)          # bf16 + bf16 -> rounded bf16
    out_c = oracle.decode_reduce(msgs, idx, E, 32, oracle.ACC_BF16, out_fp32=False)
    assert np.array_equal(out_c, wl.to_bits(t))


def test_decode_reduce_matches_independent_dequant_sum():
    """Rebuild the sum from the message bytes with numpy only."""
    w, Ys, idx = _tiny_inputs()
    msgs = [oracle.encode(Y, idx, w.G) for Y in Ys]
    comp = compaction(idx, w.E)
    acc = None
    for mg in msgs:
        codes, _ = unpack_codes(mg.codes, w.r)
        s = group_expand(bits_to_f32(mg.scale), w.G, w.r)
        z = group_expand(bits_to_f32(mg.zero), w.G, w.r)
        xh = np.empty((w.T, w.E), np.float32)
        xh[:, comp] = (codes.astype(np.float32) * s + z).astype(np.float32)
        xh[:, idx] = bits_to_f32(mg.outl)
        acc = xh if acc is None else (acc + xh).astype(np.float32)
    out = oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_FP32, out_fp32=True)
    assert np.array_equal(out, acc)
    out16 = oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_FP32, out_fp32=False)
    assert np.array_equal(out16, f32_to_bf16_bits_lib(acc))
    # the bf16 chain, rebuilt exactly: every term and every partial sum through the library's
    # bf16 conversion (the term is the fp32 value code * scale + zero rounded once)
    chain = None
    for mg in msgs:
        codes, _ = unpack_codes(mg.codes, w.r)
        s = group_expand(bits_to_f32(mg.scale), w.G, w.r)
        z = group_expand(bits_to_f32(mg.zero), w.G, w.r)
        xh = np.empty((w.T, w.E), np.float32)
        xh[:, comp] = (codes.astype(np.float32) * s + z).astype(np.float32)
        xh[:, idx] = bits_to_f32(mg.outl)
        term = bits_to_f32(f32_to_bf16_bits_lib(xh))
        chain = term if chain is None else bits_to_f32(f32_to_bf16_bits_lib((chain + term).astype(np.float32)))
    outb_bits = oracle.decode_reduce(msgs, idx, w.E, w.G, oracle.ACC_BF16)
    assert np.array_equal(bits_to_f32(outb_bits), chain)
    # ... and it stays within bf16 rounding of the fp32 result
    outb = bits_to_f32(outb_bits)
    scale = np.zeros_like(acc)
    for mg in msgs:
        scale += np.abs(bits_to_f32(oracle.decode_reduce([mg], idx, w.E, w.G, oracle.ACC_FP32)))
    assert np.all(np.abs(outb - acc) <= 1e-2 * scale + 1e-30)


def test_bits_per_value_closed_form():
    """4 + 12k/E payload bits; k = floor(E/64) gives 4.1875 (< 4.2)."""
    for E, G in ((512, 128), (5120, 128), (4608, 128), (8192, 128), (8192, 64)):
        k = E // 64
        assert payload_bits(E, k) == 4.1875 < 4.2
        Y = np.zeros((3, E), np.uint16)
        idx = np.arange(0, 64 * k, 64, dtype=np.int32)
        msg = oracle.encode(Y, idx, G)
        r = E - k
        assert msg.outl.nbytes * 8 + 4 * r * 3 == payload_bits(E, k) * 3 * E
        written = msg.outl.nbytes + msg.codes.nbytes + msg.scale.nbytes + msg.zero.nbytes
        assert written == 3 * wire_bytes_per_row(E, k, G)
    assert wire_bytes_per_row(5120, 80, 128) == 2840
    assert wire_bytes_per_row(512, 8, 128) == 284
    assert wire_bytes_per_row(8192, 341, 64) == 5100
    assert abs(payload_bits(8192, 341) - 4.4995) < 1e-4


@pytest.mark.parametrize("N", [4, 8])
def test_irwin_hall_error_statistics(N):
    """Sum of N independent uniform quantisation errors: mean 0, variance
    sum_i step_i^2 / 12, excess kurtosis -1.2/N (Irwin-Hall, paper Sec. 1)."""
    import dataclasses
    w = dataclasses.replace(wl.LLAMA_PREFILL, N=N)
    T = 48
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w, T=T)]
    # keep the planted outlier columns and fill up to k with other columns
    cols, _ = wl.outlier_columns(w)
    rest = np.setdiff1d(np.arange(w.E), cols.numpy())[: w.k - cols.numel()]
    idx = np.sort(np.concatenate([cols.numpy(), rest])).astype(np.int32)
    comp = compaction(idx, w.E)
    e = np.zeros((T, w.r))
    v = np.zeros((T, w.r))
    interior = np.ones((T, w.r), bool)
    for Y in Ys:
        msg = oracle.encode(Y, idx, w.G)
        xh = oracle.dequantize(msg, idx, w.E, w.G).astype(np.float64)
        x = bits_to_f32(Y).astype(np.float64)
        e += (xh - x)[:, comp]
        s = group_expand(bits_to_f32(msg.scale).astype(np.float64), w.G, w.r)
        v += s * s / 12.0
        codes, _ = unpack_codes(msg.codes, w.r)
        interior &= (codes > 0) & (codes < 15)
    z = e / np.sqrt(v)
    n = z.size
    # all elements: the two group extremes per device carry (almost) no error
    assert abs(np.mean(z * z) - (w.G - 2) / w.G) < 0.05
    assert abs(np.mean(z)) < 4 / np.sqrt(n)
    # elements that are interior on every device: the clean Irwin-Hall case
    zi = z[interior]
    assert zi.size > 0.5 * n
    assert abs(np.var(zi) - 1.0) < 0.03
    kurt = np.mean(zi ** 4) / np.mean(zi ** 2) ** 2 - 3.0
    assert abs(kurt - (-1.2 / N)) < 0.05
    assert np.max(np.abs(zi)) <= np.sqrt(3.0 * N) * (1 + 1e-3)   # support of the sum


def test_heavy_tail_variance_upper_bound():
    """t(3) base: errors are no longer uniform, but the variance bound holds."""
    import dataclasses
    w = dataclasses.replace(wl.LARGE_PREFILL, N=4, E=1024, k=16)
    T = 32
    Ys = [wl.to_bits(y) for y in wl.partial_sums(w, T=T)]
    cols, _ = wl.outlier_columns(w)
    rest = np.setdiff1d(np.arange(w.E), cols.numpy())[: w.k - cols.numel()]
    idx = np.sort(np.concatenate([cols.numpy(), rest])).astype(np.int32)
    comp = compaction(idx, w.E)
    e = np.zeros((T, w.r))
    v = np.zeros((T, w.r))
    for Y in Ys:
        msg = oracle.encode(Y, idx, w.G)
        _check_message_against_definitions(Y[:4], idx, w.G, oracle.encode(Y[:4], idx, w.G))
        xh = oracle.dequantize(msg, idx, w.E, w.G).astype(np.float64)
        e += (xh - bits_to_f32(Y).astype(np.float64))[:, comp]
        s = group_expand(bits_to_f32(msg.scale).astype(np.float64), w.G, w.r)
        v += s * s / 12.0
    assert np.mean(e * e / v) <= 1.02


def test_bad_arguments_are_rejected():
    Y = np.zeros((2, 16), np.uint16)
    for bad in ([3, 3], [5, 2], [16], [-1]):
        with pytest.raises(ValueError):
            oracle.encode(Y, np.array(bad, np.int32), 8)


def test_division_by_15_shortcut_is_exact(tmp_path):
    """(max - min) / 15, the quantiser's scale (Sec. 2): the GPU kernels multiply by fl(1/15)
    and correct once with a fused multiply-add; the oracle divides.  Equal for every mantissa
    (checked here at exponents across the range, including the smallest normal ones)."""
    import os
    import subprocess
    src = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "div15_check.c")
    exe = str(tmp_path / "div15_check")
    subprocess.run(["gcc", "-O2", "-ffp-contract=off", "-o", exe, src, "-lm"], check=True)
    r = subprocess.run([exe, "1", "2", "5", "27", "100", "127", "128", "200", "253", "254"],
                       capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and r.stdout.strip() == "0", r.stdout + r.stderr
