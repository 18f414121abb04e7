"""Shared pieces of the GPU parity tests: run the library, run the oracle, compare."""
import numpy as np
import torch

import oracle
import paper_2411_07942_amd as tpq
import workloads as wl

CANARY = 0xA5


def bits_to_f32(a):
    return (np.asarray(a, np.uint16).astype(np.uint32) << 16).view(np.float32)


def gpu_plan(L, idx_np, device="cuda"):
    idx_dev = torch.from_numpy(np.ascontiguousarray(idx_np, dtype=np.int32)).to(device)
    if idx_dev.numel() == 0:
        idx_dev = torch.zeros(4, dtype=torch.int32, device=device)  # never read when k = 0
    plan = tpq.plan_build(L, idx_dev)
    tpq.plan_check(L, plan)
    return plan


def gpu_encode(L, plan, Ys):
    T = Ys[0].shape[0]
    msgs = [tpq.Message(L, T, Ys[0].device, fill=CANARY) for _ in Ys]
    tpq.encode(L, plan, Ys, msgs)
    torch.cuda.synchronize()
    return msgs


def gpu_decode(L, plan, msgs, T, accum, out_fp32, ld=None):
    """Returns (out [T,E] numpy, guard columns untouched?)."""
    E = L.E
    ld = E if ld is None else ld
    dtype = torch.float32 if out_fp32 else torch.bfloat16
    buf = torch.full((max(T, 1), ld), 777.0, dtype=dtype, device="cuda")
    out = buf[:T, :E] if ld != E else buf[:T]
    tpq.decode_reduce(L, plan, msgs, out, accum)
    torch.cuda.synchronize()
    guard_ok = True
    if ld != E and T > 0:
        guard_ok = bool((buf[:T, E:] == 777.0).all().item())
    if out_fp32:
        return out.cpu().numpy().copy(), guard_ok
    return wl.to_bits(out.contiguous()), guard_ok


def check_pad_bytes(L, msg, T):
    """Bytes outside the logical content keep the canary (codes rows: the tail of
    the last 32-bit word is written as zero)."""
    def pads(t, pitch, used, zero_to=None):
        if T == 0 or pitch == 0:
            return
        a = t.cpu().numpy()[: pitch * T].reshape(T, pitch)
        lo = used
        if zero_to is not None:
            assert np.all(a[:, used:zero_to] == 0)
            lo = zero_to
        assert np.all(a[:, lo:] == CANARY), "pad bytes were overwritten"
    pads(msg.codes, L.pitch_codes, L.code_bytes, (L.code_bytes + 3) // 4 * 4)
    pads(msg.scale, L.pitch_meta, 2 * L.ng)
    pads(msg.zero, L.pitch_meta, 2 * L.ng)
    pads(msg.outl, L.pitch_outl, 2 * L.k)


def assert_message_equal(L, gpu_msg, ref: oracle.Message, rows=None):
    outl, codes, scale, zero = gpu_msg.to_dense(L)
    if rows is not None:
        outl, codes, scale, zero = outl[rows], codes[rows], scale[rows], zero[rows]
    assert np.array_equal(outl, ref.outl), "outlier values differ"
    assert np.array_equal(zero, ref.zero), "zeros differ"
    assert np.array_equal(scale, ref.scale), "scales differ"
    assert np.array_equal(codes, ref.codes), "packed codes differ"


def sum_tolerance_ok(gpu_out, ref_out, ref_msgs, idx, E, G, out_fp32, rel):
    """|gpu - oracle| <= rel * sum_i |x_hat_i|  (+ half a bf16 ulp of the oracle value
    when the output itself is rounded to bf16)."""
    mag = np.zeros(ref_out.shape, np.float64)
    for mg in ref_msgs:
        mag += np.abs(oracle.dequantize(mg, idx, E, G).astype(np.float64))
    if out_fp32:
        g, r = gpu_out.astype(np.float64), ref_out.astype(np.float64)
        slack = 0.0
    else:
        g, r = bits_to_f32(gpu_out).astype(np.float64), bits_to_f32(ref_out).astype(np.float64)
        slack = np.abs(r) * 2.0 ** -8
    return bool(np.all(np.abs(g - r) <= rel * mag + slack + 1e-30))


def sum_tolerance_fraction(gpu_out, ref_out, ref_msgs, idx, E, G, out_fp32, rel):
    """Fraction of the elements inside the bar of sum_tolerance_ok, and the worst
    |gpu - oracle| / sum_i |x_hat_i|."""
    mag = np.zeros(ref_out.shape, np.float64)
    for mg in ref_msgs:
        mag += np.abs(oracle.dequantize(mg, idx, E, G).astype(np.float64))
    if out_fp32:
        g, r = gpu_out.astype(np.float64), ref_out.astype(np.float64)
        slack = 0.0
    else:
        g, r = bits_to_f32(gpu_out).astype(np.float64), bits_to_f32(ref_out).astype(np.float64)
        slack = np.abs(r) * 2.0 ** -8
    err = np.abs(g - r)
    inside = err <= rel * mag + slack + 1e-30
    worst = float(np.max((err - slack).clip(min=0) / (mag + 1e-30))) if err.size else 0.0
    return float(np.mean(inside)) if err.size else 1.0, worst


def idx_for(w, block=0):
    """The k selected features of a workload block: the planted outlier columns,
    filled up with the lowest other columns (stands in for a calibration run)."""
    cols, _ = wl.outlier_columns(w, block)
    cols = cols.numpy()
    if cols.size > w.k:
        cols = cols[: w.k]
    rest = np.setdiff1d(np.arange(w.E), cols)[: w.k - cols.size]
    return np.sort(np.concatenate([cols, rest])).astype(np.int32)
