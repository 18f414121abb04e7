"""GPU parity of the code widths other than 4 bits (Sec. 4 / Fig. 3: the experiment that
varies the bits of the quantised features; b in 2, 3, 5, 6, 8) against the CPU oracle.

Bars as for 4 bits: codes, scales, zeros, outlier values bit-exact; sums within 1e-5 (fp32
accumulate) / 1e-2 (bf16 accumulate) of the summation's natural scale, and bit-identical.
All calls go through the C ABI (ctypes binding).
"""
import numpy as np
import pytest
import torch

import oracle
import paper_2411_07942_amd as tpq
import workloads as wl
from gpu_common import CANARY, bits_to_f32, gpu_plan, idx_for

pytestmark = pytest.mark.gpu
WIDTHS = (2, 3, 5, 6, 8)


def _case(E, G, b, Ys, idx, rows=None, ld_out=None):
    N, T = len(Ys), Ys[0].shape[0]
    k = int(idx.size)
    r = E - k
    L = tpq.layout_init(E, k, G, b)
    assert L.bits == b
    plan = gpu_plan(L, idx)
    msgs = [tpq.Message(L, T, "cuda", fill=CANARY) for _ in Ys]
    tpq.encode(L, plan, Ys, msgs)
    torch.cuda.synchronize()
    refs = []
    for i, y in enumerate(Ys):
        Y = wl.to_bits(y if rows is None else y[torch.as_tensor(rows, device=y.device)])
        ref = oracle.encode(Y, idx, G, threads=8, bits=b)
        outl, codes, scale, zero = msgs[i].to_dense(L)
        if rows is not None:
            outl, codes, scale, zero = outl[rows], codes[rows], scale[rows], zero[rows]
        assert np.array_equal(outl, ref.outl), "outlier values differ"
        assert np.array_equal(zero, ref.zero), "zeros differ"
        assert np.array_equal(scale, ref.scale), "scales differ"
        assert np.array_equal(codes, ref.codes), "packed codes differ"
        if r > 0:   # whole chunks are written (zero past the last code), nothing beyond them
            a = msgs[i].codes.cpu().numpy()[: L.pitch_codes * T].reshape(T, L.pitch_codes)
            whole = -(-r // 8) * b
            assert np.all(a[:, L.code_bytes:whole] == 0) and np.all(a[:, whole:] == CANARY)
        for t_, pitch, used in ((msgs[i].scale, L.pitch_meta, 2 * L.ng), (msgs[i].zero, L.pitch_meta, 2 * L.ng),
                                (msgs[i].outl, L.pitch_outl, 2 * k)):
            if pitch:
                a = t_.cpu().numpy()[: pitch * T].reshape(T, pitch)
                assert np.all(a[:, used:] == CANARY)
        refs.append(ref)
    for accum, out_fp32 in ((tpq.ACC_FP32, False), (tpq.ACC_FP32, True), (tpq.ACC_BF16, False)):
        ld = E if ld_out is None else ld_out
        dtype = torch.float32 if out_fp32 else torch.bfloat16
        buf = torch.full((T, ld), 777.0, dtype=dtype, device="cuda")
        out = buf[:, :E] if ld != E else buf
        tpq.decode_reduce(L, plan, msgs, out, accum)
        torch.cuda.synchronize()
        if ld != E:
            assert bool((buf[:, E:] == 777.0).all().item()), "decode wrote outside its rows"
        got = out.cpu().numpy().copy() if out_fp32 else wl.to_bits(out.contiguous())
        if rows is not None:
            got = got[rows]
        want = oracle.decode_reduce(refs, idx, E, G, accum, out_fp32=out_fp32, threads=8, bits=b)
        mag = np.zeros(want.shape, np.float64)
        for ref in refs:
            mag += np.abs(oracle.dequantize(ref, idx, E, G, bits=b).astype(np.float64))
        g = got.astype(np.float64) if out_fp32 else bits_to_f32(got).astype(np.float64)
        w_ = want.astype(np.float64) if out_fp32 else bits_to_f32(want).astype(np.float64)
        rel = 1e-2 if accum == tpq.ACC_BF16 else 1e-5
        slack = 0.0 if out_fp32 else np.abs(w_) * 2.0 ** -8
        assert np.all(np.abs(g - w_) <= rel * mag + slack + 1e-30)
        assert np.array_equal(got, want), "sums within tolerance but not bit-identical"
    return L


def _inputs(E, T, N, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    Ys = []
    for i in range(N):
        x = torch.randn((T, E), generator=g, device="cuda")
        x[:, ::11] *= 37.0
        x[0, : E // 2] = 0.0
        if T > 1:
            x[1] = -1.5
        if T > 2:
            x[2, ::2] = 0.0
            x[2, 1::2] = -0.0
        Ys.append(x.to(torch.bfloat16))
    return Ys


@pytest.mark.parametrize("b", WIDTHS)
def test_tiny_config(b):
    w = wl.TINY
    _case(w.E, w.G, b, wl.partial_sums(w, device="cuda"), idx_for(w))


@pytest.mark.parametrize("b", WIDTHS)
@pytest.mark.parametrize("E,k,G,T,N", [
    (512, 8, 128, 16, 4),
    (1032, 1, 128, 5, 3),      # odd r: a ragged last chunk
    (1024, 0, 64, 7, 2),       # k = 0
    (64, 64, 32, 3, 2),        # k = E
    (96, 95, 32, 4, 2),        # a single quantised feature
    (5120, 80, 128, 6, 8),     # Llama width
    (8192, 341, 64, 4, 9),     # odd r, a partial batch of ranks
    (2048, 600, 64, 5, 2),     # many selected features
    (8, 3, 32, 4, 2),          # the narrowest row
    (2048, 32, 32, 5, 3),      # 4 lanes per group
    (8192, 128, 256, 3, 2),    # 32 lanes per group
])
def test_shapes_random_indices(E, k, G, T, N, b):
    Ys = _inputs(E, T, N, E * 31 + k + b)
    rng = np.random.default_rng(E + k)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    _case(E, G, b, Ys, idx, ld_out=E + 16)


@pytest.mark.parametrize("b", (3, 8))
def test_widest_row(b):
    E, k, G = 32768, 512, 128
    Ys = _inputs(E, 2, 2, 5 + b)
    idx = np.sort(np.random.default_rng(2).choice(E, k, replace=False)).astype(np.int32)
    _case(E, G, b, Ys, idx)


@pytest.mark.parametrize("b", WIDTHS)
def test_llama_prefill_full_size(b):
    """Full size, every row against the oracle."""
    w = wl.LLAMA_PREFILL
    Ys = wl.partial_sums(w, device="cuda")
    L = _case(w.E, w.G, b, Ys, idx_for(w))
    assert tpq.payload_bits(L) == b + (16 - b) * w.k / w.E
