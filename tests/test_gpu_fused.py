"""GPU parity of tpq_decode_reduce_fused (Sec. 2: the sum over the devices plus the bias; an
addend row for a residual or the device's own unquantised partial sum) against the CPU oracle.

Bars: sums within 1e-5 (fp32 accumulate) / 1e-2 (bf16 accumulate) of the summation's natural
scale, and bit-identical (the kernel adds the terms in the oracle's order and precision).
"""
import ctypes

import numpy as np
import pytest
import torch

import oracle
import paper_2411_07942_amd as tpq
import workloads as wl
from gpu_common import bits_to_f32, gpu_encode, gpu_plan, idx_for

pytestmark = pytest.mark.gpu


def _case(E, G, Ys, idx, addend, bias, rows=None, ld_out=None, n_msgs=None):
    T = Ys[0].shape[0]
    L = tpq.layout_init(E, int(idx.size), G)
    plan = gpu_plan(L, idx)
    msgs = gpu_encode(L, plan, Ys)
    if n_msgs is not None:
        msgs = msgs[:n_msgs]
    sel = (lambda a: a) if rows is None else (lambda a: a[rows])
    refs = []
    for i, m in enumerate(msgs):
        outl, codes, scale, zero = m.to_dense(L)
        refs.append(oracle.Message(sel(outl), sel(codes), sel(scale), sel(zero)))
    add_np = None if addend is None else sel(wl.to_bits(addend.contiguous()))
    bias_np = None if bias is None else wl.to_bits(bias.reshape(1, -1))[0]
    for accum, out_fp32 in ((tpq.ACC_FP32, False), (tpq.ACC_FP32, True), (tpq.ACC_BF16, False), (tpq.ACC_BF16, True)):
        ld = E if ld_out is None else ld_out
        dtype = torch.float32 if out_fp32 else torch.bfloat16
        buf = torch.full((T, ld), 777.0, dtype=dtype, device="cuda")
        out = buf[:, :E] if ld != E else buf
        tpq.decode_reduce_fused(L, plan, msgs, out, addend, bias, accum)
        torch.cuda.synchronize()
        if ld != E:
            assert bool((buf[:, E:] == 777.0).all().item()), "decode wrote outside its rows"
        got = sel(out.cpu().numpy().copy() if out_fp32 else wl.to_bits(out.contiguous()))
        want = oracle.decode_reduce_fused(refs, idx, E, G, add_np, bias_np, accum, out_fp32, threads=8)
        mag = np.zeros(want.shape, np.float64)
        for ref in refs:
            mag += np.abs(oracle.dequantize(ref, idx, E, G).astype(np.float64))
        if add_np is not None:
            mag += np.abs(bits_to_f32(add_np))
        if bias_np is not None:
            mag += np.abs(bits_to_f32(bias_np))[None, :]
        g = got.astype(np.float64) if out_fp32 else bits_to_f32(got).astype(np.float64)
        w_ = want.astype(np.float64) if out_fp32 else bits_to_f32(want).astype(np.float64)
        rel = 1e-2 if accum == tpq.ACC_BF16 else 1e-5
        slack = 0.0 if out_fp32 else np.abs(w_) * 2.0 ** -8
        assert np.all(np.abs(g - w_) <= rel * mag + slack + 1e-30)
        assert np.array_equal(got, want), "sums within tolerance but not bit-identical"
    return L, plan, msgs


def _inputs(E, T, N, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    Ys = [(torch.randn((T, E), generator=g, device="cuda") * (1 + 20 * (i % 2))).to(torch.bfloat16) for i in range(N)]
    addend = (torch.randn((T, E), generator=g, device="cuda") * 4).to(torch.bfloat16)
    bias = (torch.randn((E,), generator=g, device="cuda") * 2).to(torch.bfloat16)
    return Ys, addend, bias


@pytest.mark.parametrize("which", ["both", "addend", "bias", "none"])
def test_tiny_config(which):
    w = wl.TINY
    Ys = wl.partial_sums(w, device="cuda")
    _, addend, bias = _inputs(w.E, w.T, 1, 3)
    _case(w.E, w.G, Ys, idx_for(w), addend if which in ("both", "addend") else None,
          bias if which in ("both", "bias") else None)


@pytest.mark.parametrize("E,k,G,T,N", [
    (512, 8, 128, 16, 4),
    (1032, 1, 128, 5, 3),      # odd r
    (1024, 0, 64, 7, 2),       # k = 0
    (64, 64, 32, 3, 2),        # k = E: only selected features
    (5120, 80, 128, 6, 8),     # Llama width
    (8192, 341, 64, 4, 9),     # a partial batch of ranks
    (2048, 600, 64, 5, 2),     # many selected features, short runs (narrow entries)
    (8, 3, 32, 4, 2),
    (2048, 32, 32, 5, 3),
])
def test_shapes_random_indices(E, k, G, T, N):
    Ys, addend, bias = _inputs(E, T, N, E + k)
    rng = np.random.default_rng(E + k)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    # the addend as a view with a row stride of its own
    wide = torch.zeros((T, E + 24), dtype=torch.bfloat16, device="cuda")
    wide[:, 3:E + 3] = addend
    _case(E, G, Ys, idx, wide[:, 3:E + 3], bias, ld_out=E + 16)


def test_own_partial_sum_unquantised():
    """Device 1 leaves its own message out and adds its exact partial sum."""
    w = wl.TINY
    Ys = wl.partial_sums(w, device="cuda")
    own = 1
    others = [y for i, y in enumerate(Ys) if i != own]
    _case(w.E, w.G, others, idx_for(w), Ys[own], None)


def test_llama_prefill_full_size():
    w = wl.LLAMA_PREFILL
    Ys = wl.partial_sums(w, device="cuda")
    _, addend, bias = _inputs(w.E, w.T, 1, 11)
    _case(w.E, w.G, Ys, idx_for(w), addend, bias)


def test_argument_errors():
    E, k, G = 512, 8, 128
    idx = np.arange(0, 24, 3).astype(np.int32)
    L6 = tpq.layout_init(E, k, G, 6)
    L = tpq.layout_init(E, k, G)
    plan = gpu_plan(L, idx)
    msgs = [tpq.Message(L, 2, "cuda", fill=0) for _ in range(2)]
    out = torch.full((2, E), 5.0, dtype=torch.bfloat16, device="cuda")
    addend = torch.zeros((2, E), dtype=torch.bfloat16, device="cuda")
    lib = tpq._load()
    n = 2
    p = lambda name: tpq._ptr_array([getattr(m, name) for m in msgs], n)
    call = lambda Lx, ldAdd: lib.tpq_decode_reduce_fused(
        ctypes.byref(Lx), tpq._ptr(plan), n, 2, p("codes"), p("scale"), p("zero"), p("outl"),
        tpq._ptr(addend), ldAdd, None, tpq.ACC_FP32, tpq.OUT_BF16, tpq._ptr(out), E, None)
    assert call(L6, E) == tpq.ERR_UNSUPPORTED
    assert call(L, E - 8) == tpq.ERR_SHAPE
    torch.cuda.synchronize()
    assert bool((out == 5.0).all().item())
