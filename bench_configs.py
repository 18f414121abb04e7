#!/usr/bin/env python3
"""Timings of the codec on the other benchmark configurations (one MI355X).

bench.py measures the headline number (the Llama-2-13B-shaped prefill block, whole path).
This script adds what a deployment asks next, one JSON line per section:

  llama   the same block: encode of all 8 simulated ranks, encode of ONE rank (a device's real
          share), decode_reduce in both accumulate modes, and the per-device-share bandwidth
          (B_enc / N + B_dec) / (t_enc1 + t_dec);
  gemma   the Gemma-2-27B-shaped decode regime: 92 blocks of [64 x 4608], each with its own outlier
          set; per block one tpq_encode of the device's own partial sum and one tpq_decode_reduce
          over 8 messages, (a) launched back to back, (b) the same 184 launches replayed from one
          HIP graph (every replay is checked against the eager result);
  large   the large prefill stress block (16 ranks, [16384 x 8192]) in its four variants, fp32
          accumulate, bf16 and fp32 output;
  bits    the Llama-2-13B-shaped block at the other code widths (2, 3, 5, 6, 8 bits beside 4);
  fused   the Llama-2-13B-shaped block: decode_reduce with the residual and bias added inside the
          kernel, beside decode_reduce followed by two elementwise additions;
  gemm    one device's linear layer at the Llama-2-13B shape with the compression in the GEMM's
          epilogue, beside the library GEMM followed by tpq_encode;
  static  the Llama-2-13B-shaped block in the static symmetric mode (per device and feature steps
          from calibration; only codes and selected features travel): encode of all ranks, of one
          rank, decode_reduce in both accumulate modes.

Inputs are seeded synthetic activations (workloads/), resident in HBM before timing.  The selected
features of each block are its planted outlier columns filled up to k with random other columns (a
stand-in for a calibration run, which bench.py and the tests exercise).
"""
from __future__ import annotations

import argparse
import json
import sys
import time

import numpy as np
import torch

HBM_PEAK_GBS = 8000.0


def idx_for(wl, w, block=0):
    """The block's planted outlier columns, filled up to k with seeded random other columns
    (what a calibration run returns when the remaining ranges are nearly equal)."""
    cols, _ = wl.outlier_columns(w, block)
    cols = cols.numpy()[: w.k]
    others = np.setdiff1d(np.arange(w.E), cols)
    rng = np.random.default_rng(wl.seed_for(w, block, 0, 7))
    rest = rng.choice(others, w.k - cols.size, replace=False)
    return np.sort(np.concatenate([cols, rest])).astype(np.int32)


def timed(calls, reps, sync_every=None):
    """Average microseconds per sweep over `calls`, launched back to back."""
    for c in calls:
        c()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        for c in calls:
            c()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e6 / reps


def section_llama(tpq, wl, args):
    w = wl.LLAMA_PREFILL
    N, T, E = w.N, w.T, w.E
    dev = "cuda"
    L = tpq.layout_init(E, w.k, w.G)
    plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w)).to(dev))
    tpq.plan_check(L, plan)
    sets = []
    for s in range(6):
        Ys = wl.partial_sums(w, block=s, device=dev)
        msgs = [tpq.Message(L, T, dev) for _ in range(N)]
        out = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
        sets.append(dict(enc=tpq.encode_call(L, plan, Ys, msgs),
                         enc1=tpq.encode_call(L, plan, Ys[:1], msgs[:1]),
                         dec_bf16=tpq.decode_reduce_call(L, plan, msgs, out, tpq.ACC_BF16),
                         dec_fp32=tpq.decode_reduce_call(L, plan, msgs, out, tpq.ACC_FP32), keep=(Ys, msgs, out)))
    W = L.wire_bytes_per_row
    B_enc, B_dec = N * T * (2 * E + W), T * (N * W + 2 * E)
    t = {k: timed([s[k] for s in sets], 40) / len(sets) for k in ("enc", "enc1", "dec_bf16", "dec_fp32")}
    share = (B_enc / N + B_dec) / ((t["enc1"] + t["dec_bf16"]) * 1e-6) / 1e9
    return {"section": "llama2_13b_prefill", "us": {k: round(v, 2) for k, v in t.items()},
            "encode_all_ranks_GBps": round(B_enc / t["enc"] / 1e3, 1),
            "encode_one_rank_GBps": round(B_enc / N / t["enc1"] / 1e3, 1),
            "decode_reduce_GBps": {"bf16": round(B_dec / t["dec_bf16"] / 1e3, 1), "fp32": round(B_dec / t["dec_fp32"] / 1e3, 1)},
            "per_device_share_GBps": round(share, 1), "per_device_share_frac_of_peak": round(share / HBM_PEAK_GBS, 4),
            "note": "launches back to back (no events between them), 6 rotating buffer sets"}


def section_gemma(tpq, wl, args):
    w = wl.GEMMA_DECODE
    N, T, E, nb = w.N, w.T, w.E, w.blocks
    dev = "cuda"
    L = tpq.layout_init(E, w.k, w.G)
    blocks = []
    for b in range(nb):
        plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w, b)).to(dev))
        Ys = wl.partial_sums(w, block=b, device=dev)
        msgs = [tpq.Message(L, T, dev) for _ in range(N)]
        tpq.encode(L, plan, Ys, msgs)          # the other ranks' messages, as the all-gather would deliver them
        out = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
        blocks.append(dict(enc1=tpq.encode_call(L, plan, Ys[:1], msgs[:1]),
                           dec=tpq.decode_reduce_call(L, plan, msgs, out, tpq.ACC_BF16), out=out, keep=(plan, Ys, msgs)))
    tpq.plan_check(L, blocks[-1]["keep"][0])
    calls = [c for blk in blocks for c in (blk["enc1"], blk["dec"])]
    eager_us = timed(calls, 20)
    eager = [blk["out"].clone() for blk in blocks]

    # the same launches from one graph
    graph_us, graph_ok = None, None
    try:
        side = torch.cuda.Stream()
        side.wait_stream(torch.cuda.current_stream())
        with torch.cuda.stream(side):
            for c in calls:
                c()
        torch.cuda.current_stream().wait_stream(side)
        torch.cuda.synchronize()
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g):
            for c in calls:
                c()
        graph_ok = True
        for rep in range(3):          # replays with eager work and synchronisation in between
            for blk in blocks:
                blk["out"].zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            graph_ok = graph_ok and all(torch.equal(blk["out"], e) for blk, e in zip(blocks, eager))
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(20):
            g.replay()
        torch.cuda.synchronize()
        graph_us = (time.perf_counter() - t0) * 1e6 / 20
    except Exception as exc:  # graph capture is optional: report why it was not measured
        graph_ok = "not measured: %s" % (str(exc).splitlines()[0] if str(exc) else type(exc).__name__)
    W = L.wire_bytes_per_row
    B_blk = T * (2 * E + W) + T * (N * W + 2 * E)
    res = {"section": "gemma2_27b_decode", "blocks": nb,
           "eager_us_per_block": round(eager_us / nb, 2), "eager_GBps": round(B_blk * nb / eager_us / 1e3, 1),
           "graph_us_per_block": None if graph_us is None else round(graph_us / nb, 2),
           "graph_matches_eager": graph_ok,
           "note": "per block: tpq_encode of one rank + tpq_decode_reduce over 8 messages; launch-latency-bound regime"}
    return res


def section_large(tpq, wl, args):
    dev = "cuda"
    results = []
    for w in wl.large_variants():
        if args.only and args.only not in w.name:
            continue
        N, T, E = w.N, w.T, w.E
        L = tpq.layout_init(E, w.k, w.G)
        plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w)).to(dev))
        tpq.plan_check(L, plan)
        Ys = wl.partial_sums(w, device=dev)
        msgs = [tpq.Message(L, T, dev) for _ in range(N)]
        out16 = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
        out32 = torch.empty((T, E), dtype=torch.float32, device=dev)
        enc = tpq.encode_call(L, plan, Ys, msgs)
        d16 = tpq.decode_reduce_call(L, plan, msgs, out16, tpq.ACC_FP32)
        d32 = tpq.decode_reduce_call(L, plan, msgs, out32, tpq.ACC_FP32)
        W = L.wire_bytes_per_row
        B_enc, B_d16, B_d32 = N * T * (2 * E + W), T * (N * W + 2 * E), T * (N * W + 4 * E)
        t_enc, t_d16, t_d32 = timed([enc], 5), timed([d16], 5), timed([d32], 5)
        results.append({"variant": w.name, "encode_us": round(t_enc, 1), "encode_GBps": round(B_enc / t_enc / 1e3, 1),
                        "decode_bf16_out_us": round(t_d16, 1), "decode_bf16_out_GBps": round(B_d16 / t_d16 / 1e3, 1),
                        "decode_fp32_out_us": round(t_d32, 1), "decode_fp32_out_GBps": round(B_d32 / t_d32 / 1e3, 1),
                        "partials_GBps": round(N * T * E * 2 / (t_enc + t_d16) / 1e3, 1)})
        del Ys, msgs, out16, out32, enc, d16, d32
        torch.cuda.empty_cache()
    return {"section": "large_prefill", "variants": results,
            "note": "16 ranks x [16384 x 8192], fp32 accumulate; one buffer set (5.6 GB, far beyond the caches)"}


def section_bits(tpq, wl, args):
    w = wl.LLAMA_PREFILL
    N, T, E = w.N, w.T, w.E
    dev = "cuda"
    idx = torch.from_numpy(idx_for(wl, w)).to(dev)
    Yss = [wl.partial_sums(w, block=s, device=dev) for s in range(6)]
    out = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
    rows = []
    for b in (2, 3, 4, 5, 6, 8):
        L = tpq.layout_init(E, w.k, w.G, b)
        plan = tpq.plan_build(L, idx)
        tpq.plan_check(L, plan)
        sets = []
        for Ys in Yss:
            msgs = [tpq.Message(L, T, dev) for _ in range(N)]
            sets.append(dict(enc=tpq.encode_call(L, plan, Ys, msgs),
                             dec_bf16=tpq.decode_reduce_call(L, plan, msgs, out, tpq.ACC_BF16),
                             dec_fp32=tpq.decode_reduce_call(L, plan, msgs, out, tpq.ACC_FP32), keep=msgs))
        W = L.wire_bytes_per_row
        B_enc, B_dec = N * T * (2 * E + W), T * (N * W + 2 * E)
        t = {k: timed([s[k] for s in sets], 30) / len(sets) for k in ("enc", "dec_bf16", "dec_fp32")}
        rows.append({"bits": b, "payload_bits": round(tpq.payload_bits(L), 4), "wire_bits": round(tpq.wire_bits(L), 4),
                     "us": {k: round(v, 2) for k, v in t.items()},
                     "encode_GBps": round(B_enc / t["enc"] / 1e3, 1),
                     "decode_reduce_GBps": {"bf16": round(B_dec / t["dec_bf16"] / 1e3, 1),
                                            "fp32": round(B_dec / t["dec_fp32"] / 1e3, 1)}})
        del sets
    return {"section": "llama2_13b_prefill_code_widths", "widths": rows,
            "note": "8 ranks x [2048 x 5120], k = 80, G = 128; launches back to back, 6 rotating buffer sets"}


def section_fused(tpq, wl, args):
    w = wl.LLAMA_PREFILL
    N, T, E = w.N, w.T, w.E
    dev = "cuda"
    L = tpq.layout_init(E, w.k, w.G)
    plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w)).to(dev))
    tpq.plan_check(L, plan)
    bias = torch.randn(E, device=dev).to(torch.bfloat16)
    sets = []
    for s in range(6):
        Ys = wl.partial_sums(w, block=s, device=dev)
        msgs = [tpq.Message(L, T, dev) for _ in range(N)]
        tpq.encode(L, plan, Ys, msgs)
        out = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
        res = torch.randn((T, E), device=dev).to(torch.bfloat16)
        plain = tpq.decode_reduce_call(L, plan, msgs, out, tpq.ACC_BF16)

        def unfused(plain=plain, out=out, res=res):
            plain()
            out.add_(res)
            out.add_(bias)
        sets.append(dict(plain=plain, unfused=unfused,
                         fused_bf16=tpq.decode_reduce_fused_call(L, plan, msgs, out, res, bias, tpq.ACC_BF16),
                         fused_fp32=tpq.decode_reduce_fused_call(L, plan, msgs, out, res, bias, tpq.ACC_FP32),
                         keep=(Ys, msgs, out, res)))
    t = {k: round(timed([s[k] for s in sets], 40) / len(sets), 2)
         for k in ("plain", "unfused", "fused_bf16", "fused_fp32")}
    return {"section": "llama2_13b_prefill_fused_epilogue", "us": t,
            "note": "decode_reduce (bf16 chain) alone; followed by two torch additions (residual, bias); "
                    "tpq_decode_reduce_fused with both, bf16 chain and fp32 accumulate"}


def section_hop(tpq, wl, args):
    """Ring step at the Llama shape: 8 devices side by side in one launch, and one device alone
    (its real share), against the same result from the two existing entry points (decode the one
    message with the partial sum as addend into a bf16 tensor, then encode that tensor)."""
    w = wl.LLAMA_PREFILL
    N, T, E = w.N, w.T, w.E
    dev = "cuda"
    L = tpq.layout_init(E, w.k, w.G)
    plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w)).to(dev))
    tpq.plan_check(L, plan)
    sets = []
    for s in range(6):
        Ys = wl.partial_sums(w, block=s, device=dev)
        got = [tpq.Message(L, T, dev) for _ in range(N)]
        tpq.encode(L, plan, Ys[1:] + Ys[:1], got)       # what each device has received
        out = [tpq.Message(L, T, dev) for _ in range(N)]
        tmp = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
        dec1 = tpq.decode_reduce_fused_call(L, plan, got[:1], tmp, Ys[0], None, tpq.ACC_BF16)
        enc1 = tpq.encode_call(L, plan, [tmp], out[:1])

        def two_calls(dec1=dec1, enc1=enc1):
            dec1()
            enc1()
        sets.append(dict(hop=tpq.hop_call(L, plan, Ys, got, out, tpq.ACC_BF16),
                         hop_fp32=tpq.hop_call(L, plan, Ys, got, out, tpq.ACC_FP32),
                         hop1=tpq.hop_call(L, plan, Ys[:1], got[:1], out[:1], tpq.ACC_BF16),
                         two_calls1=two_calls, keep=(Ys, got, out, tmp)))
    t = {k: round(timed([s[k] for s in sets], 40) / len(sets), 2) for k in ("hop", "hop_fp32", "hop1", "two_calls1")}
    W = L.wire_bytes_per_row
    B = N * T * (2 * E + 2 * W)     # per launch: partial sums and received messages read, messages written
    return {"section": "llama2_13b_prefill_ring_step", "us": t,
            "hop_all_ranks_GBps": round(B / t["hop"] / 1e3, 1), "hop_one_rank_GBps": round(B / N / t["hop1"] / 1e3, 1),
            "algorithmic_bytes": B,
            "note": "tpq_hop for 8 devices in one launch (bf16 chain / fp32), for one device, and one device's step "
                    "through tpq_decode_reduce_fused + tpq_encode with the bf16 sum in memory between them"}


def section_static(tpq, wl, args):
    w = wl.LLAMA_PREFILL
    N, T, E = w.N, w.T, w.E
    dev = "cuda"
    L = tpq.layout_init(E, w.k, w.G)
    plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w)).to(dev))
    tpq.plan_check(L, plan)
    sets = []
    step = inv = None
    for s in range(6):
        Ys = wl.partial_sums(w, block=s, device=dev)
        if step is None:   # ranges of the first block stand in for the calibration state
            m = torch.stack([y.float().amin(0) for y in Ys]).contiguous()
            M = torch.stack([y.float().amax(0) for y in Ys]).contiguous()
            step, inv = tpq.static_params(L, plan, m, M)
        msgs = [tpq.Message(L, T, dev) for _ in range(N)]
        out = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
        sets.append(dict(enc=tpq.encode_static_call(L, plan, Ys, inv, msgs),
                         enc1=tpq.encode_static_call(L, plan, Ys[:1], inv, msgs[:1]),
                         dec_bf16=tpq.decode_reduce_static_call(L, plan, msgs, step, out, tpq.ACC_BF16),
                         dec_fp32=tpq.decode_reduce_static_call(L, plan, msgs, step, out, tpq.ACC_FP32),
                         keep=(Ys, msgs, out)))
    W = L.code_bytes + 2 * L.k          # bytes per row that travel in this mode
    B_enc, B_dec = N * T * (2 * E + W), T * (N * W + 2 * E)
    t = {k: timed([s[k] for s in sets], 40) / len(sets) for k in ("enc", "enc1", "dec_bf16", "dec_fp32")}
    share = (B_enc / N + B_dec) / ((t["enc1"] + t["dec_bf16"]) * 1e-6) / 1e9
    return {"section": "llama2_13b_prefill_static_mode", "bits_per_value": round(8.0 * W / E, 4),
            "us": {k: round(v, 2) for k, v in t.items()},
            "encode_all_ranks_GBps": round(B_enc / t["enc"] / 1e3, 1),
            "encode_one_rank_GBps": round(B_enc / N / t["enc1"] / 1e3, 1),
            "decode_reduce_GBps": {"bf16": round(B_dec / t["dec_bf16"] / 1e3, 1), "fp32": round(B_dec / t["dec_fp32"] / 1e3, 1)},
            "per_device_share_GBps": round(share, 1), "per_device_share_frac_of_peak": round(share / HBM_PEAK_GBS, 4),
            "note": "algorithmic bytes exclude the step tables (160 KB per device, shared by all rows, served by L2)"}


MFMA_BF16_PEAK_TFLOPS = 2500.0


def section_gemm(tpq, wl, args):
    """One device's row-parallel linear layer at the Llama-2-13B shape with the compression in
    the GEMM's epilogue (tpq_gemm_encode), beside the library GEMM (torch.matmul) followed by
    tpq_encode with the bf16 partial sums in memory between them.  K = 13824 / 8 (MLP down
    projection) and 5120 / 8 (attention output projection)."""
    w = wl.LLAMA_PREFILL
    T, E = w.T, w.E
    dev = "cuda"
    L = tpq.layout_init(E, w.k, w.G)
    idx = idx_for(wl, w)
    plan = tpq.plan_build(L, torch.from_numpy(idx).to(dev))
    tpq.plan_check(L, plan)
    shapes = []
    for K in (1728, 640):
        if args.only and args.only != str(K):
            continue
        sets = []
        for s in range(4):
            X, Wt = wl.linear_inputs(T, K, E, idx, 100 + s, device=dev)
            Wp = tpq.gemm_weights(L, plan, Wt)
            msg = tpq.Message(L, T, dev)
            Y = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
            Wk = Wt.t()                                   # [K, E] view: torch.matmul(X, Wk) = X Wt^T
            enc1 = tpq.encode_call(L, plan, [Y], [msg])

            def lib_gemm(X=X, Wk=Wk, Y=Y):
                torch.matmul(X, Wk, out=Y)

            def unfused(lib_gemm=lib_gemm, enc1=enc1):
                lib_gemm()
                enc1()
            sets.append(dict(fused=tpq.gemm_encode_call(L, X, Wp, msg), fused_y=tpq.gemm_encode_call(L, X, Wp, msg, Y),
                             lib_gemm=lib_gemm, unfused=unfused, enc1=enc1, keep=(X, Wt, Wp, msg, Y)))
        t = {k: round(timed([s[k] for s in sets], 40) / len(sets), 2) for k in ("fused", "fused_y", "lib_gemm", "unfused", "enc1")}
        flop = 2.0 * T * K * E
        shapes.append({"K": K, "us": t, "fused_TFLOPs": round(flop / t["fused"] / 1e6, 1),
                       "fused_frac_of_mfma_peak": round(flop / t["fused"] / 1e6 / MFMA_BF16_PEAK_TFLOPS, 4),
                       "lib_gemm_TFLOPs": round(flop / t["lib_gemm"] / 1e6, 1)})
    return {"section": "llama2_13b_prefill_gemm_epilogue", "T": T, "E": E, "shapes": shapes,
            "note": "fused = tpq_gemm_encode (message only); fused_y = the same, also storing the bf16 product; "
                    "lib_gemm = torch.matmul into a bf16 tensor; unfused = lib_gemm then tpq_encode of that tensor; "
                    "enc1 = that tpq_encode alone"}


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--sections", default="llama,gemma,large,static,bits,fused,hop,gemm")
    ap.add_argument("--only", default="", help="large: only the variants whose name contains this; gemm: only this K "
                                               "(so that a kernel trace holds one shape per kernel)")
    args = ap.parse_args()
    if not torch.cuda.is_available():
        sys.exit("bench_configs.py: no GPU visible")
    import paper_2411_07942_amd as tpq
    import workloads as wl
    table = {"llama": section_llama, "gemma": section_gemma, "large": section_large,
             "static": section_static, "bits": section_bits, "fused": section_fused, "hop": section_hop,
             "gemm": section_gemm}
    for name in args.sections.split(","):
        print(json.dumps(table[name](tpq, wl, args)), flush=True)


if __name__ == "__main__":
    main()
