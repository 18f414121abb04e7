"""GPU parity of the static symmetric mode (the paper's own quantiser, Sec. 3:
per device and feature parameters from calibration, symmetric Int4) against the CPU
oracle on the same seeded inputs.

Bars: parameter tables, packed codes and outlier values bit-exact; reduced sums within
1e-5 (fp32 accumulate) / 1e-2 (bf16 accumulate) of the summation's natural scale --
and, as the kernels follow the oracle's evaluation order, bit-identical.
All calls go through the C ABI (ctypes binding).
"""
import dataclasses

import numpy as np
import pytest
import torch

import oracle
import paper_2411_07942_amd as tpq
import workloads as wl
from gpu_common import CANARY, bits_to_f32, gpu_plan, idx_for
from refmath import compaction

pytestmark = pytest.mark.gpu


def _ranges_from(Ys, shrink_every=5, dead_every=17):
    """Calibration-like (m, M) fp32 [N,E] from the data itself: the column range, shrunk on
    some columns (so that values clamp), zero on others (vanishing range), and on a few
    chosen so that the step is a power of two (ties in the rounding)."""
    m = torch.stack([y.float().amin(0) for y in Ys])
    M = torch.stack([y.float().amax(0) for y in Ys])
    E = m.shape[1]
    cols = torch.arange(E, device=m.device)
    shrink = (cols % shrink_every) == 1
    m[:, shrink] *= 0.55
    M[:, shrink] *= 0.55
    dead = (cols % dead_every) == 3
    m[:, dead] = 0.0
    M[:, dead] = 0.0
    pow2 = (cols % 13) == 6
    m[:, pow2] = -0.25
    M[:, pow2] = 0.9375          # R = 1.875, step = 1/8 exactly
    return m.contiguous(), M.contiguous()


def _static_case(E, G, Ys, idx, m, M, rows=None, modes=((tpq.ACC_FP32, False), (tpq.ACC_FP32, True),
                                                        (tpq.ACC_BF16, False)), ld_out=None, bits=4):
    N, T = len(Ys), Ys[0].shape[0]
    k = int(idx.size)
    r = E - k
    L = tpq.layout_init(E, k, G, bits)
    plan = gpu_plan(L, idx)

    # parameter tables: the oracle's (feature order) gathered into compacted order
    step, inv = tpq.static_params(L, plan, m, M)
    torch.cuda.synchronize()
    step_ref, inv_ref = oracle.static_params(m.cpu().numpy(), M.cpu().numpy(), bits=bits)
    comp = compaction(idx, E)
    W = tpq.static_table_floats(L)
    assert W % 512 == 0 and W >= r and (r == 0 or W - r < 512)
    if r > 0:
        step_np, inv_np = step.cpu().numpy(), inv.cpu().numpy()
        assert np.array_equal(step_np[:, :r].view(np.uint32), step_ref[:, comp].view(np.uint32))
        assert np.array_equal(inv_np[:, :r].view(np.uint32), inv_ref[:, comp].view(np.uint32))
        assert not step_np[:, r:W].any() and not inv_np[:, r:W].any()

    # encode
    msgs = [tpq.Message(L, T, "cuda", fill=CANARY) for _ in Ys]
    tpq.encode_static(L, plan, Ys, inv, msgs)
    torch.cuda.synchronize()
    refs = []
    for i, y in enumerate(Ys):
        Y = wl.to_bits(y if rows is None else y[torch.as_tensor(rows, device=y.device)])
        ref = oracle.encode_static(Y, idx, inv_ref[i], threads=8, bits=bits)
        outl, codes, _, _ = msgs[i].to_dense(L)
        if rows is not None:
            outl, codes = outl[rows], codes[rows]
        assert np.array_equal(outl, ref.outl), "outlier values differ"
        assert np.array_equal(codes, ref.codes), "packed codes differ"
        # scale / zero sections do not exist in this mode: never written
        assert bool((msgs[i].scale == CANARY).all().item()) and bool((msgs[i].zero == CANARY).all().item())
        if T > 0 and L.pitch_codes > 0:
            a = msgs[i].codes.cpu().numpy()[: L.pitch_codes * T].reshape(T, L.pitch_codes)
            z = (L.code_bytes + 3) // 4 * 4 if bits == 4 else -(-r // 8) * bits   # written as zero up to here
            assert np.all(a[:, L.code_bytes:z] == 0) and np.all(a[:, z:] == CANARY)
        if T > 0 and L.pitch_outl > 0:
            a = msgs[i].outl.cpu().numpy()[: L.pitch_outl * T].reshape(T, L.pitch_outl)
            assert np.all(a[:, 2 * k:] == CANARY)
        refs.append(ref)

    # decode + reduce
    for accum, out_fp32 in modes:
        ld = E if ld_out is None else ld_out
        dtype = torch.float32 if out_fp32 else torch.bfloat16
        buf = torch.full((max(T, 1), ld), 777.0, dtype=dtype, device="cuda")
        out = buf[:T, :E] if ld != E else buf[:T]
        tpq.decode_reduce_static(L, plan, msgs, step, out, accum)
        torch.cuda.synchronize()
        if ld != E and T > 0:
            assert bool((buf[:T, E:] == 777.0).all().item()), "decode wrote outside its rows"
        got = out.cpu().numpy().copy() if out_fp32 else wl.to_bits(out.contiguous())
        if rows is not None:
            got = got[rows]
        want = oracle.decode_reduce_static(refs, idx, step_ref, accum, out_fp32=out_fp32, threads=8, bits=bits)
        # tolerance of the bar: |gpu - oracle| <= rel * sum_i |x_hat_i| (+ half a bf16 ulp)
        mag = np.zeros(want.shape, np.float64)
        for i, ref in enumerate(refs):
            one = oracle.decode_reduce_static([ref], idx, step_ref[i:i + 1], tpq.ACC_FP32, out_fp32=True, bits=bits)
            mag += np.abs(one.astype(np.float64))
        g = got.astype(np.float64) if out_fp32 else bits_to_f32(got).astype(np.float64)
        w_ = want.astype(np.float64) if out_fp32 else bits_to_f32(want).astype(np.float64)
        rel = 1e-2 if accum == tpq.ACC_BF16 else 1e-5
        slack = 0.0 if out_fp32 else np.abs(w_) * 2.0 ** -8
        assert np.all(np.abs(g - w_) <= rel * mag + slack + 1e-30)
        assert np.array_equal(got, want), "sums within tolerance but not bit-identical"
    return L, plan, msgs, step


def _random_inputs(E, T, N, seed):
    g = torch.Generator(device="cuda")
    g.manual_seed(seed)
    Ys = []
    for i in range(N):
        x = torch.randn((T, E), generator=g, device="cuda")
        x[:, ::11] *= 37.0
        # multiples of 1/16 on the columns whose step is 1/8: exact ties
        q = torch.randint(-9, 17, (T, E), generator=g, device="cuda").float() / 16.0
        tie = (torch.arange(E, device="cuda") % 13) == 6
        x[:, tie] = q[:, tie]
        if T > 1:
            x[1] = -1.5
        if T > 2:
            x[2, ::2] = 0.0
            x[2, 1::2] = -0.0
        Ys.append(x.to(torch.bfloat16))
    return Ys


def test_tiny_config_static():
    w = wl.TINY
    Ys = wl.partial_sums(w, device="cuda")
    m, M = _ranges_from(Ys)
    _static_case(w.E, w.G, Ys, idx_for(w), m, M)


@pytest.mark.parametrize("E,k,G,T,N", [
    (512, 8, 128, 16, 4),
    (1032, 1, 128, 5, 3),      # odd r: pad nibble
    (1024, 0, 64, 7, 2),       # k = 0: plain symmetric Int4
    (64, 64, 32, 3, 2),        # k = E: everything in bf16
    (96, 95, 32, 4, 2),        # a single quantised feature
    (4608, 72, 128, 9, 8),     # Gemma width
    (5120, 80, 128, 6, 8),     # Llama width
    (8192, 341, 64, 4, 16),    # odd r, 16 ranks
    (2048, 600, 64, 5, 3),     # many selected features; a partial batch of ranks
    (32768, 512, 128, 2, 2),   # the widest row the library takes
    (8, 3, 32, 4, 2),          # the narrowest
    (520, 9, 128, 1, 1),       # one row, one rank
    (1024, 16, 128, 3, 7),     # ranks not a multiple of the decode batch
])
def test_shapes_random_indices_static(E, k, G, T, N):
    Ys = _random_inputs(E, T, N, E * 31 + k)
    rng = np.random.default_rng(E + k)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    m, M = _ranges_from(Ys)
    _static_case(E, G, Ys, idx, m, M, ld_out=E + 16)


@pytest.mark.parametrize("name,cols", [
    ("one_odd_shift", [3]),
    ("run_in_the_middle", list(range(100, 121))),
    ("every_other", list(range(200, 264, 2))),
    ("across_pass_boundaries", list(range(505, 521)) + [1033, 1034, 1040, 1551]),
    ("edges", [0, 1, 2046, 2047]),
])
def test_outlier_patterns_static(name, cols):
    E, G, T, N = 2048, 128, 3, 2
    idx = np.array(sorted(set(cols)), np.int32)
    Ys = _random_inputs(E, T, N, len(cols) * 7 + cols[0])
    m, M = _ranges_from(Ys)
    _static_case(E, G, Ys, idx, m, M)


def test_empty_batch_static():
    """T = 0 is accepted and nothing is written."""
    import ctypes
    E, k, G = 512, 8, 128
    idx = np.arange(0, 8 * 3, 3).astype(np.int32)
    L = tpq.layout_init(E, k, G)
    plan = gpu_plan(L, idx)
    m = torch.full((2, E), -1.0, device="cuda")
    M = torch.full((2, E), 1.0, device="cuda")
    step, inv = tpq.static_params(L, plan, m, M)
    Ys = [torch.zeros((1, E), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    msgs = [tpq.Message(L, 1, "cuda", fill=CANARY) for _ in Ys]
    out = torch.full((1, E), 777.0, dtype=torch.bfloat16, device="cuda")
    lib = tpq._load()
    cp = tpq._ptr_array([g.codes for g in msgs], 2)
    op = tpq._ptr_array([g.outl for g in msgs], 2)
    assert lib.tpq_encode_static(ctypes.byref(L), tpq._ptr(plan), tpq._ptr_array(Ys, 2), E, 2, 0,
                                 tpq._ptr(inv), cp, op, None) == tpq.OK
    assert lib.tpq_decode_reduce_static(ctypes.byref(L), tpq._ptr(plan), 2, 0, cp, op, tpq._ptr(step),
                                        tpq.ACC_FP32, tpq.OUT_BF16, tpq._ptr(out), E, None) == tpq.OK
    torch.cuda.synchronize()
    assert all(bool((g.codes == CANARY).all().item()) and bool((g.outl == CANARY).all().item())
               for g in msgs)
    assert bool((out == 777.0).all().item())


def test_static_argument_errors():
    E, k, G = 512, 8, 128
    L = tpq.layout_init(E, k, G)
    idx = np.arange(0, 8 * 3, 3).astype(np.int32)
    plan = gpu_plan(L, idx)
    m = torch.full((2, E), -1.0, device="cuda")
    M = torch.full((2, E), 1.0, device="cuda")
    step, inv = tpq.static_params(L, plan, m, M)
    Ys = [torch.zeros((4, E), dtype=torch.bfloat16, device="cuda") for _ in range(2)]
    msgs = [tpq.Message(L, 4, "cuda", fill=CANARY) for _ in Ys]
    lib = tpq._load()
    import ctypes
    n = 2
    Yp = tpq._ptr_array(Ys, n)
    cp = tpq._ptr_array([g.codes for g in msgs], n)
    op = tpq._ptr_array([g.outl for g in msgs], n)
    rc = lib.tpq_encode_static(ctypes.byref(L), tpq._ptr(plan), Yp, E, n, 4, None, cp, op, None)
    assert rc == tpq.ERR_NULL
    rc = lib.tpq_encode_static(ctypes.byref(L), tpq._ptr(plan), Yp, E, n, 4,
                               ctypes.c_void_p(inv.data_ptr() + 4), cp, op, None)
    assert rc == tpq.ERR_ALIGN
    rc = lib.tpq_encode_static(ctypes.byref(L), tpq._ptr(plan), Yp, E - 8, n, 4, tpq._ptr(inv), cp, op, None)
    assert rc == tpq.ERR_SHAPE
    out = torch.zeros((4, E), dtype=torch.bfloat16, device="cuda")
    rc = lib.tpq_decode_reduce_static(ctypes.byref(L), tpq._ptr(plan), n, 4, cp, op, None,
                                      tpq.ACC_FP32, tpq.OUT_BF16, tpq._ptr(out), E, None)
    assert rc == tpq.ERR_NULL
    rc = lib.tpq_decode_reduce_static(ctypes.byref(L), tpq._ptr(plan), n, 4, cp, op, tpq._ptr(step),
                                      7, tpq.OUT_BF16, tpq._ptr(out), E, None)
    assert rc == tpq.ERR_UNSUPPORTED
    torch.cuda.synchronize()
    for g in msgs:   # nothing was launched
        assert bool((g.codes == CANARY).all().item())


def test_calibrated_static_end_to_end():
    """tpq_calibrate -> tpq_calibrate_finalize -> plan -> static tables -> encode -> decode,
    all on the device, against the oracle's calibration state."""
    w = wl.TINY
    N, E = w.N, w.E
    m = torch.empty((N, E), device="cuda")
    M = torch.empty((N, E), device="cuda")
    S = w.cal_seq
    ws = torch.zeros(tpq.calibrate_workspace_bytes(S, E), dtype=torch.uint8, device="cuda")
    m_ref = np.zeros((N, E), np.float32)
    M_ref = np.zeros((N, E), np.float32)
    for i in range(N):
        for s in range(wl.n_cal_sequences(w)):
            Y = wl.calibration_sequence(w, 0, i, s, device="cuda", S=S)
            tpq.calibrate(Y, i, N, s, 0.01, m, M, ws)
            oracle.calibrate_update(wl.to_bits(Y), m_ref[i], M_ref[i], first=(s == 0), gamma=0.01)
    Rbar = torch.empty(E, device="cuda")
    idx_s = torch.empty(w.k, dtype=torch.int32, device="cuda")
    idx_r = torch.empty(w.k, dtype=torch.int32, device="cuda")
    ws2 = torch.empty(tpq.calibrate_finalize_workspace_bytes(E), dtype=torch.uint8, device="cuda")
    tpq.calibrate_finalize(m, M, w.k, Rbar, idx_s, idx_r, ws2)
    torch.cuda.synchronize()
    assert np.array_equal(m.cpu().numpy(), m_ref) and np.array_equal(M.cpu().numpy(), M_ref)
    idx = idx_s.cpu().numpy().astype(np.int32)
    Ys = wl.partial_sums(w, device="cuda")
    _static_case(E, w.G, Ys, idx, m, M)


def test_llama_prefill_full_size_static():
    """The Llama-2-13B-shaped prefill block at full size, every row against the oracle."""
    w = wl.LLAMA_PREFILL
    Ys = wl.partial_sums(w, device="cuda")
    m, M = _ranges_from(Ys, shrink_every=3, dead_every=1001)
    _static_case(w.E, w.G, Ys, idx_for(w), m, M)


@pytest.mark.parametrize("b", (2, 3, 5, 6, 8))
@pytest.mark.parametrize("E,k,G,T,N", [
    (512, 8, 128, 16, 4),
    (1032, 1, 128, 5, 3),      # odd r: a ragged last chunk
    (1024, 0, 64, 7, 2),       # k = 0
    (64, 64, 32, 3, 2),        # k = E
    (5120, 80, 128, 6, 8),     # Llama width
    (2048, 600, 64, 5, 3),     # many selected features
    (8, 3, 32, 4, 2),
    (1024, 16, 128, 3, 7),     # ranks not a multiple of the decode batch
])
def test_other_code_widths_static(E, k, G, T, N, b):
    """The static quantiser at b bits (Sec. 4 / Fig. 3): step R / (2^b - 1), signed codes."""
    Ys = _random_inputs(E, T, N, E * 31 + k + b)
    rng = np.random.default_rng(E + k)
    idx = np.sort(rng.choice(E, k, replace=False)).astype(np.int32)
    m, M = _ranges_from(Ys)
    _static_case(E, G, Ys, idx, m, M, ld_out=E + 16, bits=b)


@pytest.mark.parametrize("b", (3, 8))
def test_llama_prefill_full_size_static_other_widths(b):
    w = wl.LLAMA_PREFILL
    Ys = wl.partial_sums(w, device="cuda")
    m, M = _ranges_from(Ys, shrink_every=3, dead_every=1001)
    _static_case(w.E, w.G, Ys, idx_for(w), m, M, bits=b)
