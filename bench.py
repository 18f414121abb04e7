#!/usr/bin/env python3
"""Benchmark of the codec hot path on one MI355X.

A step = one pass of the online hot path over one batch of synthetic partial sums:
tpq_encode of all N simulated ranks (one launch) followed by tpq_decode_reduce of the
N messages.  The workload is the Llama-2-13B-shaped prefill configuration (N = 8,
bf16 [2048 x 5120], k = 80, group 128).  The outlier set comes from a calibration run
on the GPU before timing (timed separately, reported under "calibrate").  Inputs are
resident in HBM; several independent buffer sets are rotated so that a step never
finds its data in the 256 MB memory-side cache.

Before anything is timed the GPU is brought to steady clocks by running the same step
for a fixed wall time (`clock_ramp_ms`, uncounted), then come the requested warm-up
steps and exactly `--steps` timed steps.

Prints one JSON line: metric / value (GB/s of bf16 partials through encode +
decode_reduce, from the wall time of the timed steps), the roofline of the dominant kernel
(tpq_encode, HBM-bound) from HIP events attached to the launches of a second pass over
the same steps, the one-rank encode and the per-device
share, a device-copy bandwidth as the practical ceiling, compact results of the other
configurations, and the CPU oracle timed on the host cores as a reported baseline.
"""
from __future__ import annotations

import argparse
import json
import os
import sys
import time

import numpy as np
import torch

HBM_PEAK_GBS = 8000.0   # MI355X published HBM3E peak bandwidth
ROOT = os.path.dirname(os.path.abspath(__file__))
# HBM bytes per launch from rocprofv3 --pmc FETCH_SIZE / WRITE_SIZE, scaled by a device copy of
# known size; kept in profiles/traffic.json beside the profile summary they come from
TRAFFIC_JSON = os.path.join(ROOT, "profiles", "traffic.json")

ACCUM_NAMES = {
    "fast": "bf16 mode at its 1e-2 tolerance: fp32 chain, one final rounding (TPQ_ACC_FAST)",
    "bf16": "bf16 chain: every term and partial sum rounded to bf16 (TPQ_ACC_BF16)",
    "fp32": "fp32 chain, one final rounding (TPQ_ACC_FP32)",
}


def parse():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=2000)
    ap.add_argument("--warmup", type=int, default=200)
    ap.add_argument("--sets", type=int, default=6, help="independent buffer sets rotated per step")
    ap.add_argument("--accum", choices=["fast", "bf16", "fp32"], default="fast",
                    help="arithmetic of the sum over ranks in tpq_decode_reduce in the timed steps "
                         "(the other modes are timed beside it and reported under decode_reduce.other_modes)")
    ap.add_argument("--ramp-ms", type=float, default=300.0,
                    help="wall time of untimed steps run first, so that the clocks are steady")
    ap.add_argument("--event-steps", type=int, default=256,
                    help="kernel durations come from HIP events on a second pass over the timed steps "
                         "(all of them, up to this many)")
    ap.add_argument("--no-cpu", action="store_true", help="skip the CPU oracle timing")
    ap.add_argument("--no-configs", action="store_true", help="skip the other configurations")
    ap.add_argument("--calibrate-chunks", type=int, default=8)
    ap.add_argument("--copy-probe", action="store_true",
                    help="also run an elementwise kernel that reads and writes 256 MiB: the known-size "
                         "dispatch that scales the FETCH_SIZE / WRITE_SIZE counters of a --pmc run")
    return ap.parse_args()


def timed_calls(calls, reps):
    """Average microseconds per call, launched back to back over the rotating sets."""
    for c in calls:
        c()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(reps):
        for c in calls:
            c()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) * 1e6 / reps / len(calls)


def new_event():
    e = torch.cuda.Event(enable_timing=True)
    e.record()           # creates the HIP event, whose handle the library is given
    return e


def event_us(tpq, calls, n):
    """Mean kernel duration (us) of n launches, from events attached to the dispatches."""
    ev = [[new_event(), new_event()] for _ in range(n)]
    torch.cuda.synchronize()
    for i, e in enumerate(ev):
        tpq.bench_time_next_launch(e[0], e[1])
        calls[i % len(calls)]()
    torch.cuda.synchronize()
    return float(np.mean([e[0].elapsed_time(e[1]) for e in ev])) * 1e3


def copy_ceiling(dev):
    """Device-to-device copy of 1 GiB (read + write counted): the practical ceiling of a stream."""
    n = 1 << 30
    src = torch.empty(n, dtype=torch.uint8, device=dev).fill_(1)
    dst = torch.empty_like(src)
    for _ in range(3):
        dst.copy_(src)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    c0.record()
    for _ in range(10):
        dst.copy_(src)
    c1.record()
    torch.cuda.synchronize()
    ms = c0.elapsed_time(c1) / 10
    del src, dst
    torch.cuda.empty_cache()
    return 2.0 * n / (ms * 1e-3) / 1e9


def other_configs(tpq, wl, dev):
    """Compact results of the configurations that are not the headline: us per launch,
    algorithmic GB/s and fraction of the HBM peak."""
    from bench_configs import idx_for
    out = {}

    # Gemma-2-27B-shaped decode regime: per block one-rank encode + decode_reduce over 8 messages
    w = wl.GEMMA_DECODE
    L = tpq.layout_init(w.E, w.k, w.G)
    calls_e, calls_d, keep = [], [], []
    for b in range(0, w.blocks, 4):
        plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w, b)).to(dev))
        Ys = wl.partial_sums(w, block=b, device=dev)
        msgs = [tpq.Message(L, w.T, dev) for _ in range(w.N)]
        tpq.encode(L, plan, Ys, msgs)
        o = torch.empty((w.T, w.E), dtype=torch.bfloat16, device=dev)
        calls_e.append(tpq.encode_call(L, plan, Ys[:1], msgs[:1]))
        calls_d.append(tpq.decode_reduce_call(L, plan, msgs, o, tpq.ACC_FAST))
        keep.append((plan, Ys, msgs, o))
    both = [c for pair in zip(calls_e, calls_d) for c in pair]
    us_block = timed_calls(both, 20) * 2
    W = L.wire_bytes_per_row
    B = w.T * (2 * w.E + W) + w.T * (w.N * W + 2 * w.E)
    out["gemma2_27b_decode"] = {"us_per_block": round(us_block, 2), "GBps": round(B / us_block / 1e3, 1),
                                "frac": round(B / us_block / 1e3 / HBM_PEAK_GBS, 4),
                                "what": "one-rank encode + decode_reduce(8) per block, launched back to back"}
    del keep, calls_e, calls_d, both
    torch.cuda.empty_cache()

    # Large prefill stress block, 4.5 bits, group 64 (the hardest variant), fp32 accumulate
    w = [v for v in wl.large_variants() if v.k > 200 and v.G == 64][0]
    L = tpq.layout_init(w.E, w.k, w.G)
    plan = tpq.plan_build(L, torch.from_numpy(idx_for(wl, w)).to(dev))
    tpq.plan_check(L, plan)
    Ys = wl.partial_sums(w, device=dev)
    msgs = [tpq.Message(L, w.T, dev) for _ in range(w.N)]
    o = torch.empty((w.T, w.E), dtype=torch.bfloat16, device=dev)
    enc = tpq.encode_call(L, plan, Ys, msgs)
    dec = tpq.decode_reduce_call(L, plan, msgs, o, tpq.ACC_FP32)
    us_e, us_d = timed_calls([enc], 5), timed_calls([dec], 5)
    W = L.wire_bytes_per_row
    Be, Bd = w.N * w.T * (2 * w.E + W), w.T * (w.N * W + 2 * w.E)
    out[w.name] = {"encode_us": round(us_e, 1), "encode_GBps": round(Be / us_e / 1e3, 1),
                   "encode_frac": round(Be / us_e / 1e3 / HBM_PEAK_GBS, 4),
                   "decode_reduce_us": round(us_d, 1), "decode_reduce_GBps": round(Bd / us_d / 1e3, 1),
                   "decode_reduce_frac": round(Bd / us_d / 1e3 / HBM_PEAK_GBS, 4),
                   "what": "16 ranks x [16384 x 8192], k = %d, group %d, fp32 accumulate, bf16 out" % (w.k, w.G)}
    del Ys, msgs, o, enc, dec
    torch.cuda.empty_cache()
    return out


def main():
    args = parse()
    if args.gpus != 1:
        sys.exit("bench.py: this build runs on one GPU only (the N tensor-parallel ranks are "
                 "simulated as N resident buffers); --gpus must be 1")
    if not torch.cuda.is_available():
        sys.exit("bench.py: no GPU visible")

    import paper_2411_07942_amd as tpq
    import workloads as wl

    dev = "cuda"
    w = wl.LLAMA_PREFILL
    N, T, E, k, G = w.N, w.T, w.E, w.k, w.G
    modes = {"fast": tpq.ACC_FAST, "bf16": tpq.ACC_BF16, "fp32": tpq.ACC_FP32}
    accum = modes[args.accum]
    L = tpq.layout_init(E, k, G)

    # ---- calibration on the GPU: selects the k features kept in bf16 ------------------
    n_seq, S = wl.n_cal_sequences(w), w.cal_seq
    m = torch.zeros((N, E), device=dev)
    M = torch.zeros((N, E), device=dev)
    ws = torch.zeros(tpq.calibrate_workspace_bytes(S, E), dtype=torch.uint8, device=dev)
    for i in range(N):
        for s in range(n_seq):
            tpq.calibrate(wl.calibration_sequence(w, 0, i, s, device=dev), i, N, s, 0.01, m, M, ws)
    Rbar = torch.empty(E, device=dev)
    idx_sorted = torch.empty(k, dtype=torch.int32, device=dev)
    wsf = torch.empty(tpq.calibrate_finalize_workspace_bytes(E), dtype=torch.uint8, device=dev)
    tpq.calibrate_finalize(m, M, k, Rbar, idx_sorted, None, wsf)
    plan = tpq.plan_build(L, idx_sorted)
    tpq.plan_check(L, plan)
    idx_np = idx_sorted.cpu().numpy().astype(np.int32)

    # ---- resident buffer sets -----------------------------------------------------------
    sets = []
    for s in range(args.sets):
        Ys = wl.partial_sums(w, block=s, device=dev)
        msgs = [tpq.Message(L, T, dev) for _ in range(N)]
        out = torch.empty((T, E), dtype=torch.bfloat16, device=dev)
        # the argument marshalling is done once per buffer set, outside the timed region
        sets.append((Ys, msgs, out, tpq.encode_call(L, plan, Ys, msgs),
                     tpq.decode_reduce_call(L, plan, msgs, out, accum)))
    torch.cuda.synchronize()

    def step(bufs):
        bufs[3]()
        bufs[4]()

    # ---- parity spot check against the oracle before timing ------------------------------
    import oracle
    step(sets[0])
    torch.cuda.synchronize()
    rows = torch.arange(0, T, 16, device=dev)
    refs = [oracle.encode(wl.to_bits(y[rows]), idx_np, G) for y in sets[0][0]]
    for i, mg in enumerate(sets[0][1]):
        outl, codes, scale, zero = mg.to_dense(L)
        r = rows.cpu().numpy()
        ok = (np.array_equal(outl[r], refs[i].outl) and np.array_equal(codes[r], refs[i].codes) and
              np.array_equal(scale[r], refs[i].scale) and np.array_equal(zero[r], refs[i].zero))
        if not ok:
            sys.exit("bench.py: encode disagrees with the oracle; not timing a wrong kernel")
    got = wl.to_bits(sets[0][2][rows])
    # fast / fp32: identical to the oracle's fp32 chain; fast also within 1e-2 of its bf16 chain
    exact_mode = tpq.ACC_BF16 if accum == tpq.ACC_BF16 else tpq.ACC_FP32
    want = oracle.decode_reduce(refs, idx_np, E, G, exact_mode, out_fp32=False)
    if not np.array_equal(got, want):
        sys.exit("bench.py: decode_reduce disagrees with the oracle; not timing a wrong kernel")
    fast_match = None
    if accum == tpq.ACC_FAST:
        # against the oracle's literal bf16 chain: every element within the chain's own rounding
        # bound (N + 1) * 2^-9 * sum |x_hat_i|, nearly all within the 1e-2 bar itself
        chain = oracle.decode_reduce(refs, idx_np, E, G, tpq.ACC_BF16, out_fp32=False)
        mag = np.zeros(chain.shape, np.float64)
        for mg in refs:
            mag += np.abs(oracle.dequantize(mg, idx_np, E, G).astype(np.float64))
        f = lambda b: (np.asarray(b, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)
        err, slack = np.abs(f(got) - f(chain)), np.abs(f(chain)) * 2.0 ** -8 + 1e-30
        if not np.all(err <= (N + 1) * 2.0 ** -9 * mag + slack):
            sys.exit("bench.py: the fast accumulate mode is outside the bf16 chain's rounding bound")
        fast_match = {"rows_checked": int(rows.numel()),
                      "within_1e-2_of_bf16_chain": round(float(np.mean(err <= 1e-2 * mag + slack)), 6),
                      "bit_identical_to_bf16_chain": round(float(np.mean(got == chain)), 4),
                      "bit_identical_to_fp32_chain": 1.0}
        if fast_match["within_1e-2_of_bf16_chain"] < 0.999:
            sys.exit("bench.py: the fast accumulate mode is outside the bf16 mode's tolerance")

    # ---- clock ramp, warm-up, timed region -------------------------------------------------
    ramp0 = time.perf_counter()
    i = 0
    while (time.perf_counter() - ramp0) * 1e3 < args.ramp_ms:
        for _ in range(32):
            step(sets[i % len(sets)])
            i += 1
        torch.cuda.synchronize()
    ramp_ms = (time.perf_counter() - ramp0) * 1e3
    for i in range(args.warmup):
        step(sets[i % len(sets)])
    # the timed region: exactly --steps steps, nothing else on the stream
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for i in range(args.steps):
        step(sets[i % len(sets)])
    torch.cuda.synchronize()
    t1 = time.perf_counter()
    wall_ms = (t1 - t0) * 1e3 / args.steps
    # kernel durations: a second pass over the same steps with HIP events attached to every
    # launch's own dispatch (tpq_bench_time_next_launch): each pair brackets one kernel on the stream it
    # runs on.  Kept out of the pass above because an attached launch costs some microseconds of
    # dispatch overhead, which would otherwise go into `value`.
    n_ev = min(args.steps, args.event_steps)
    ev = [[new_event() for _ in range(4)] for _ in range(n_ev)]
    torch.cuda.synchronize()
    for i, e in enumerate(ev):
        bufs = sets[i % len(sets)]
        tpq.bench_time_next_launch(e[0], e[1])
        bufs[3]()
        tpq.bench_time_next_launch(e[2], e[3])
        bufs[4]()
    torch.cuda.synchronize()
    enc_ms = float(np.mean([e[0].elapsed_time(e[1]) for e in ev]))
    dec_ms = float(np.mean([e[2].elapsed_time(e[3]) for e in ev]))

    # the other accumulate modes of tpq_decode_reduce, for the record (not part of `value`)
    other_modes = {}
    for name, mode in modes.items():
        if mode == accum:
            continue
        calls = [tpq.decode_reduce_call(L, plan, b[1], b[2], mode) for b in sets]
        for c in calls:
            c()
        other_modes[name] = {"avg_ms": round(event_us(tpq, calls, 24) * 1e-3, 5)}

    # one rank's encode: a device's real call, and the per-device share
    enc1_calls = [tpq.encode_call(L, plan, b[0][:1], b[1][:1]) for b in sets]
    for c in enc1_calls:
        c()
    enc1_us = event_us(tpq, enc1_calls, 24)

    W = L.wire_bytes_per_row
    B_in = N * T * E * 2
    B_enc = N * T * (2 * E + W)
    B_dec = T * (N * W + 2 * E)
    value = B_in / (wall_ms * 1e-3) / 1e9
    enc_gbs = B_enc / (enc_ms * 1e-3) / 1e9
    dec_gbs = B_dec / (dec_ms * 1e-3) / 1e9
    share_gbs = (B_enc / N + B_dec) / ((enc1_us + dec_ms * 1e3) * 1e-6) / 1e9

    ceiling = copy_ceiling(dev)
    if args.copy_probe:
        a = torch.zeros(1 << 26, dtype=torch.int32, device=dev)
        b = torch.empty_like(a)
        for _ in range(3):
            torch.bitwise_not(a, out=b)  # (the only bitwise_not of the run: found by name)
        torch.cuda.synchronize()
        del a, b

    # ---- calibration throughput (offline path, reported separately) ----------------------
    wc = wl.CALIBRATION
    Sc, Ec = wc.cal_seq, wc.E
    pool = [wl.calibration_sequence(wc, 0, 0, s, device=dev) for s in range(args.calibrate_chunks)]
    mc = torch.zeros((1, Ec), device=dev)
    Mc = torch.zeros((1, Ec), device=dev)
    wsc = torch.zeros(tpq.calibrate_workspace_bytes(Sc, Ec), dtype=torch.uint8, device=dev)
    for s in range(len(pool)):
        tpq.calibrate(pool[s], 0, 1, s, 0.01, mc, Mc, wsc)
    torch.cuda.synchronize()
    c0, c1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    reps = 8 * len(pool)
    c0.record()
    for s in range(reps):
        tpq.calibrate(pool[s % len(pool)], 0, 1, s + 1, 0.01, mc, Mc, wsc)
    c1.record()
    torch.cuda.synchronize()
    cal_ms = c0.elapsed_time(c1) / reps
    cal_gbs = 2.0 * Sc * Ec / (cal_ms * 1e-3) / 1e9
    del pool
    torch.cuda.empty_cache()

    configs = None if args.no_configs else other_configs(tpq, wl, dev)

    # ---- CPU oracle on the host cores (reported baseline, not a target) --------------------
    cpu = None
    if not args.no_cpu:
        threads = oracle.max_threads()
        Yh = [wl.to_bits(y) for y in sets[0][0]]
        oracle_mode = tpq.ACC_BF16 if accum == tpq.ACC_BF16 else tpq.ACC_FP32

        def one_pass(nthreads, Ysub):
            c_0 = time.perf_counter()
            ms_ref = [oracle.encode(Y, idx_np, G, threads=nthreads) for Y in Ysub]
            oracle.decode_reduce(ms_ref, idx_np, E, G, oracle_mode, out_fp32=False, threads=nthreads)
            return time.perf_counter() - c_0
        best = min(one_pass(threads, Yh) for _ in range(3))
        # one thread on an eighth of the rows (scaled to bytes)
        Tq = T // 8
        single = one_pass(1, [Y[:Tq] for Y in Yh])
        cpu = {"value": round(B_in / best / 1e9, 4), "unit": "GB/s", "cores": threads, "kind": "oracle",
               "sample": "the full workload (8 ranks x 2048 x 5120), best of 3 passes, "
                         "encode + decode_reduce, OpenMP over rows",
               "single_thread": {"value": round(B_in / 8 / single / 1e9, 4), "unit": "GB/s",
                                 "sample": "one thread, the first %d rows of every rank, one pass" % Tq}}

    traffic = {}
    if os.path.exists(TRAFFIC_JSON):
        with open(TRAFFIC_JSON) as fh:
            traffic = json.load(fh)

    result = {
        "metric": "encode+decode_reduce GB/s of bf16 partials (% HBM peak); effective bits/value",
        "value": round(value, 2), "unit": "GB/s", "n_gpus": 1, "steps": args.steps,
        "warmup": args.warmup, "ms_per_step": round(wall_ms, 5), "higher_is_better": True,
        "scaling": "weak", "vs_baseline": None, "dtype": "f32", "data": "synthetic",
        "config": {"workload": w.name, "n_ranks": N, "tokens": T, "features": E, "k_bf16": k,
                   "group": G, "io_dtype": "bf16", "accumulate": ACCUM_NAMES[args.accum], "out": "bf16",
                   "buffer_sets": len(sets)},
        "roofline": {"bound": "hbm", "kernel": "tpq_encode (k_encode_direct)", "achieved": round(enc_gbs, 1),
                     "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": round(enc_gbs / HBM_PEAK_GBS, 4),
                     "traffic": traffic.get("tpq_encode"), "algorithmic_bytes": B_enc,
                     "avg_ms": round(enc_ms, 5), "event_samples": n_ev},
        "cpu_baseline": cpu,
        "decode_reduce": {"achieved": round(dec_gbs, 1), "unit": "GB/s",
                          "frac": round(dec_gbs / HBM_PEAK_GBS, 4), "traffic": traffic.get("tpq_decode_reduce"),
                          "algorithmic_bytes": B_dec, "avg_ms": round(dec_ms, 5), "accumulate": args.accum,
                          "fast_mode_vs_oracle": fast_match, "other_modes": other_modes},
        "combined_hbm_frac": round((B_enc + B_dec) / ((enc_ms + dec_ms) * 1e-3) / 1e9 / HBM_PEAK_GBS, 4),
        "encode_one_rank": {"avg_ms": round(enc1_us * 1e-3, 5),
                            "achieved": round(B_enc / N / enc1_us / 1e3, 1), "unit": "GB/s"},
        "per_device_share": {"achieved": round(share_gbs, 1), "unit": "GB/s",
                             "frac": round(share_gbs / HBM_PEAK_GBS, 4),
                             "what": "(B_enc / N + B_dec) / (t_encode_one_rank + t_decode_reduce)"},
        "copy_ceiling_GBps": round(ceiling, 1),
        "clock_ramp_ms": round(ramp_ms, 1),
        "events": "second pass over the timed steps, events attached to every launch",
        "calibrate": {"achieved": round(cal_gbs, 1), "unit": "GB/s", "frac": round(cal_gbs / HBM_PEAK_GBS, 4),
                      "chunk": [Sc, Ec], "avg_ms": round(cal_ms, 5)},
        "configs": configs,
        "bits_per_value": {"payload": tpq.payload_bits(L), "wire": tpq.wire_bits(L)},
    }
    print(json.dumps(result))


if __name__ == "__main__":
    main()
