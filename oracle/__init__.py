"""CPU oracle for the low-bit tensor-parallel partial-sum codec.

TEST INFRASTRUCTURE ONLY.  This package wraps ``tpq_oracle.c`` (plain scalar C,
written from the paper: Sec. 2 for the compress / decompress-and-sum problem,
Sec. 3 Eq. (1)-(2) for calibration and the top-k selection, Fig. 2 for the
message structure) behind numpy arrays.  Only ``tests/``, the smoke check and the
benchmark's ``cpu_baseline`` leg may import it; the GPU library never does, and
nothing here imports the GPU package.

bf16 tensors travel as ``numpy.uint16`` arrays holding the raw 16-bit patterns.
All layouts are dense: ``outl [T,k]``, ``codes [T,ceil(r/2)]``, ``scale``/``zero``
``[T,ceil(r/G)]`` with ``r = E-k``.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tpq_oracle.c")
_LIB = os.path.join(_HERE, "libtpq_oracle.so")

ACC_FP32 = 0
ACC_BF16 = 1

# the flags matter: no contraction of a*b+c into an fma, no fast-math
CFLAGS = ["-O2", "-std=c11", "-ffp-contract=off", "-fno-fast-math", "-fopenmp",
          "-shared", "-fPIC", "-Wall", "-Wextra"]


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (always when ``force``; else only if absent)."""
    if force or not os.path.exists(_LIB):
        tmp = _LIB + ".tmp%d" % os.getpid()
        subprocess.run(["gcc", *CFLAGS, "-o", tmp, _SRC, "-lm"], check=True)
        os.replace(tmp, _LIB)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = ctypes.CDLL(_LIB)
        i64, i32, vp, f32 = ctypes.c_int64, ctypes.c_int, ctypes.c_void_p, ctypes.c_float
        lib.orc_max_threads.restype = i32
        lib.orc_calibrate_update.argtypes = [vp, i64, i64, i32, i32, f32, vp, vp]
        lib.orc_calibrate_finalize.argtypes = [vp, vp, i32, i32, i32, vp, vp, vp, vp]
        lib.orc_linear.argtypes = [vp, i64, i64, i32, vp, i32, i64, vp, i64, vp, i32]
        lib.orc_encode.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp, vp, i32]
        lib.orc_decode_reduce.argtypes = [i32, i64, i32, i32, i32, vp, vp, vp, vp, vp,
                                          i32, i32, vp, i32]
        lib.orc_decode_reduce_fused.argtypes = [i32, i64, i32, i32, i32, vp, vp, vp, vp, vp, vp, i64, vp,
                                                i32, i32, vp, i32]
        lib.orc_encode_bits.argtypes = [vp, i64, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp, i32]
        lib.orc_decode_reduce_bits.argtypes = [i32, i64, i32, i32, i32, i32, vp, vp, vp, vp, vp,
                                               i32, i32, vp, i32]
        lib.orc_static_params.argtypes = [vp, vp, i32, i32, vp, vp]
        lib.orc_static_params_bits.argtypes = [vp, vp, i32, i32, i32, vp, vp]
        lib.orc_encode_static_bits.argtypes = [vp, i64, i64, i32, i32, i32, vp, vp, vp, vp, i32]
        lib.orc_decode_reduce_static_bits.argtypes = [i32, i64, i32, i32, i32, vp, vp, vp, vp, i32, i32,
                                                      vp, i32]
        lib.orc_encode_static.argtypes = [vp, i64, i64, i32, i32, vp, vp, vp, vp, i32]
        lib.orc_decode_reduce_static.argtypes = [i32, i64, i32, i32, vp, vp, vp, vp, i32, i32,
                                                 vp, i32]
        _lib = lib
    return _lib


def max_threads() -> int:
    """Host threads the timed runs may use: OMP_NUM_THREADS if set, else the core count."""
    procs = int(_load().orc_max_threads())
    env = os.environ.get("OMP_NUM_THREADS", "")
    return max(1, min(procs, int(env))) if env.isdigit() else procs


def _ptr(a):
    return None if a is None else a.ctypes.data_as(ctypes.c_void_p)


def _u16(a) -> np.ndarray:
    a = np.ascontiguousarray(a)
    if a.dtype != np.uint16:
        raise TypeError("bf16 data must be passed as uint16 bit patterns")
    return a


def calibrate_update(Y, m, M, first: bool, gamma: float = 0.01) -> None:
    """One calibration sequence of one device: Eq. (1), (2); in-place on m, M [E]."""
    Y = _u16(Y)
    S, E = Y.shape
    assert m.dtype == np.float32 and M.dtype == np.float32 and m.shape == (E,) and M.shape == (E,)
    assert m.flags.c_contiguous and M.flags.c_contiguous
    rc = _load().orc_calibrate_update(_ptr(Y), S, E, E, int(bool(first)), gamma, _ptr(m), _ptr(M))
    if rc:
        raise ValueError("orc_calibrate_update: bad arguments")


def calibrate_finalize(m, M, k: int):
    """m, M fp32 [N,E] -> (R [N,E], Rbar [E], idx_sorted [k], idx_ranked [k])."""
    m = np.ascontiguousarray(m, dtype=np.float32)
    M = np.ascontiguousarray(M, dtype=np.float32)
    N, E = m.shape
    R = np.empty((N, E), np.float32)
    Rbar = np.empty(E, np.float32)
    idx_sorted = np.empty(k, np.int32)
    idx_ranked = np.empty(k, np.int32)
    rc = _load().orc_calibrate_finalize(_ptr(m), _ptr(M), N, E, k, _ptr(R), _ptr(Rbar),
                                        _ptr(idx_sorted), _ptr(idx_ranked))
    if rc:
        raise ValueError("orc_calibrate_finalize: bad arguments")
    return R, Rbar, idx_sorted, idx_ranked


@dataclass
class Message:
    """One device's message for one block (dense layouts)."""
    outl: np.ndarray   # uint16 [T,k]   selected features, verbatim bf16
    codes: np.ndarray  # uint8  [T,cb]  4-bit codes, two per byte, low nibble first
    scale: np.ndarray  # uint16 [T,ng]  bf16 step per group (0 => constant group)
    zero: np.ndarray   # uint16 [T,ng]  bf16 group minimum


def dims(E: int, k: int, G: int, bits: int = 4):
    r = E - k
    return r, (r * bits + 7) // 8, (r + G - 1) // G


def encode(Y, idx_sorted, G: int, threads: int = 1, bits: int = 4) -> Message:
    """bits = 4: the primary path; other widths (Sec. 4, Fig. 3) go through the generic routine."""
    Y = _u16(Y)
    T, E = Y.shape
    idx_sorted = np.ascontiguousarray(idx_sorted, dtype=np.int32)
    k = idx_sorted.shape[0]
    r, cb, ng = dims(E, k, G, bits)
    msg = Message(np.empty((T, k), np.uint16), np.empty((T, cb), np.uint8),
                  np.empty((T, ng), np.uint16), np.empty((T, ng), np.uint16))
    if bits == 4:
        rc = _load().orc_encode(_ptr(Y), T, E, E, k, G, _ptr(idx_sorted), _ptr(msg.outl),
                                _ptr(msg.codes), _ptr(msg.scale), _ptr(msg.zero), threads)
    else:
        rc = _load().orc_encode_bits(_ptr(Y), T, E, E, k, G, bits, _ptr(idx_sorted), _ptr(msg.outl),
                                     _ptr(msg.codes), _ptr(msg.scale), _ptr(msg.zero), threads)
    if rc:
        raise ValueError("orc_encode: bad arguments")
    return msg


def linear(X, Wt, threads: int = 1, with_magnitude: bool = False):
    """Sec. 2, f^(i)(x^(i)) = x^(i) W^(i): X bf16 [T,K], Wt bf16 [E,K] (W^(i) transposed) ->
    bf16 bits [T,E], every output summed in float64 and rounded once.  with_magnitude: also
    sum_k |x w| per output (float64), the scale of an accumulation-order error."""
    X, Wt = _u16(X), _u16(Wt)
    T, K = X.shape
    E, K2 = Wt.shape
    if K != K2:
        raise ValueError("orc_linear: inner dimensions differ")
    Y = np.empty((T, E), np.uint16)
    mag = np.empty((T, E), np.float64) if with_magnitude else None
    rc = _load().orc_linear(_ptr(X), T, K, K, _ptr(Wt), E, K, _ptr(Y), E,
                            _ptr(mag) if with_magnitude else None, threads)
    if rc:
        raise ValueError("orc_linear: bad arguments")
    return (Y, mag) if with_magnitude else Y


def encode_bits(Y, idx_sorted, G: int, bits: int, threads: int = 1) -> Message:
    """Always the generic routine (also for bits = 4: the cross-check of the two)."""
    Y = _u16(Y)
    T, E = Y.shape
    idx_sorted = np.ascontiguousarray(idx_sorted, dtype=np.int32)
    k = idx_sorted.shape[0]
    r, cb, ng = dims(E, k, G, bits)
    msg = Message(np.empty((T, k), np.uint16), np.empty((T, cb), np.uint8),
                  np.empty((T, ng), np.uint16), np.empty((T, ng), np.uint16))
    rc = _load().orc_encode_bits(_ptr(Y), T, E, E, k, G, bits, _ptr(idx_sorted), _ptr(msg.outl),
                                 _ptr(msg.codes), _ptr(msg.scale), _ptr(msg.zero), threads)
    if rc:
        raise ValueError("orc_encode_bits: bad arguments")
    return msg


def decode_reduce(msgs, idx_sorted, E: int, G: int, accum: int = ACC_FP32,
                  out_fp32: bool = False, threads: int = 1, bits: int = 4,
                  generic: bool = False) -> np.ndarray:
    """Dequantise the N messages and add them in ascending device order."""
    N = len(msgs)
    idx_sorted = np.ascontiguousarray(idx_sorted, dtype=np.int32)
    k = idx_sorted.shape[0]
    T = msgs[0].codes.shape[0] if k < E else msgs[0].outl.shape[0]
    r, cb, ng = dims(E, k, G, bits)
    keep = []

    def table(name, dtype, shape):
        arr = (ctypes.c_void_p * N)()
        for i, mg in enumerate(msgs):
            a = np.ascontiguousarray(getattr(mg, name), dtype=dtype)
            assert a.shape == shape, (name, a.shape, shape)
            keep.append(a)
            arr[i] = a.ctypes.data
        return arr

    codes = table("codes", np.uint8, (T, cb))
    scale = table("scale", np.uint16, (T, ng))
    zero = table("zero", np.uint16, (T, ng))
    outl = table("outl", np.uint16, (T, k))
    out = np.empty((T, E), np.float32 if out_fp32 else np.uint16)
    if bits == 4 and not generic:
        rc = _load().orc_decode_reduce(N, T, E, k, G, _ptr(idx_sorted), codes, scale, zero, outl,
                                       accum, int(bool(out_fp32)), _ptr(out), threads)
    else:
        rc = _load().orc_decode_reduce_bits(N, T, E, k, G, bits, _ptr(idx_sorted), codes, scale, zero,
                                            outl, accum, int(bool(out_fp32)), _ptr(out), threads)
    if rc:
        raise ValueError("orc_decode_reduce: bad arguments")
    return out


def decode_reduce_fused(msgs, idx_sorted, E: int, G: int, addend=None, bias=None,
                        accum: int = ACC_FP32, out_fp32: bool = False, threads: int = 1) -> np.ndarray:
    """decode_reduce, then + addend (bf16 bits [T,E]) and + bias (bf16 bits [E]) as further terms
    of the same accumulation (Sec. 2: the sum over the devices plus the bias)."""
    N = len(msgs)
    idx_sorted = np.ascontiguousarray(idx_sorted, dtype=np.int32)
    k = idx_sorted.shape[0]
    T = msgs[0].codes.shape[0] if k < E else msgs[0].outl.shape[0]
    r, cb, ng = dims(E, k, G)
    keep = []

    def table(name, dtype, shape):
        arr = (ctypes.c_void_p * N)()
        for i, mg in enumerate(msgs):
            a = np.ascontiguousarray(getattr(mg, name), dtype=dtype)
            assert a.shape == shape, (name, a.shape, shape)
            keep.append(a)
            arr[i] = a.ctypes.data
        return arr

    codes = table("codes", np.uint8, (T, cb))
    scale = table("scale", np.uint16, (T, ng))
    zero = table("zero", np.uint16, (T, ng))
    outl = table("outl", np.uint16, (T, k))
    add = None if addend is None else _u16(addend)
    bia = None if bias is None else np.ascontiguousarray(bias, dtype=np.uint16)
    assert add is None or add.shape == (T, E)
    assert bia is None or bia.shape == (E,)
    out = np.empty((T, E), np.float32 if out_fp32 else np.uint16)
    rc = _load().orc_decode_reduce_fused(N, T, E, k, G, _ptr(idx_sorted), codes, scale, zero, outl,
                                         None if add is None else _ptr(add), E,
                                         None if bia is None else _ptr(bia),
                                         accum, int(bool(out_fp32)), _ptr(out), threads)
    if rc:
        raise ValueError("orc_decode_reduce_fused: bad arguments")
    return out


def hop(msg_in: Message, Y, idx_sorted, G: int, accum: int = ACC_BF16, threads: int = 1) -> Message:
    """One step of a ring reduction (Sec. 5, the remark that the method could be adapted to ring
    all-reduce; the paper fixes none of it): a device receives a message, adds its own partial sum
    and sends the result on, quantised again.  Written out with the steps that exist already:
    the received message is dequantised and the device's bf16 partial sum Y added as one more
    term of the accumulation (decode_reduce_fused with the message as the only one and Y as the
    addend), the bf16 result is the tensor that encode compresses."""
    Y = _u16(Y)
    T, E = Y.shape
    V = decode_reduce_fused([msg_in], idx_sorted, E, G, addend=Y, bias=None, accum=accum,
                            out_fp32=False, threads=threads)
    return encode(V, idx_sorted, G, threads)


def dequantize(msg: Message, idx_sorted, E: int, G: int, bits: int = 4) -> np.ndarray:
    """x_hat fp32 [T,E] of one message (the N = 1, fp32 case of decode_reduce)."""
    return decode_reduce([msg], idx_sorted, E, G, ACC_FP32, out_fp32=True, bits=bits)


# ---- static symmetric mode (the paper's own quantiser, Sec. 3) ---------------------

@dataclass
class StaticMessage:
    """One device's message in the static mode: nothing but codes and BF16 features."""
    outl: np.ndarray   # uint16 [T,k]
    codes: np.ndarray  # uint8  [T,cb]  nibble = code + 8, two per byte, low nibble first


def static_params(m, M, bits: int = 4, generic: bool = False):
    """(step, inv) fp32 [N,E] from the calibrated (m, M) fp32 [N,E]."""
    m = np.ascontiguousarray(m, dtype=np.float32)
    M = np.ascontiguousarray(M, dtype=np.float32)
    N, E = m.shape
    step = np.empty((N, E), np.float32)
    inv = np.empty((N, E), np.float32)
    if bits == 4 and not generic:
        rc = _load().orc_static_params(_ptr(m), _ptr(M), N, E, _ptr(step), _ptr(inv))
    else:
        rc = _load().orc_static_params_bits(_ptr(m), _ptr(M), N, E, bits, _ptr(step), _ptr(inv))
    if rc:
        raise ValueError("orc_static_params: bad arguments")
    return step, inv


def encode_static(Y, idx_sorted, inv_row, threads: int = 1, bits: int = 4,
                  generic: bool = False) -> StaticMessage:
    """Y: one device's bf16 bits [T,E]; inv_row: that device's fp32 [E]."""
    Y = _u16(Y)
    T, E = Y.shape
    idx_sorted = np.ascontiguousarray(idx_sorted, dtype=np.int32)
    inv_row = np.ascontiguousarray(inv_row, dtype=np.float32)
    assert inv_row.shape == (E,)
    k = idx_sorted.shape[0]
    cb = ((E - k) * bits + 7) // 8
    msg = StaticMessage(np.empty((T, k), np.uint16), np.empty((T, cb), np.uint8))
    if bits == 4 and not generic:
        rc = _load().orc_encode_static(_ptr(Y), T, E, E, k, _ptr(idx_sorted), _ptr(inv_row),
                                       _ptr(msg.outl), _ptr(msg.codes), threads)
    else:
        rc = _load().orc_encode_static_bits(_ptr(Y), T, E, E, k, bits, _ptr(idx_sorted), _ptr(inv_row),
                                            _ptr(msg.outl), _ptr(msg.codes), threads)
    if rc:
        raise ValueError("orc_encode_static: bad arguments")
    return msg


def decode_reduce_static(msgs, idx_sorted, step, accum: int = ACC_FP32, out_fp32: bool = False,
                         threads: int = 1, bits: int = 4, generic: bool = False) -> np.ndarray:
    """step: fp32 [N,E].  Dequantise the N static-mode messages and add them."""
    N = len(msgs)
    step = np.ascontiguousarray(step, dtype=np.float32)
    E = step.shape[1]
    assert step.shape == (N, E)
    idx_sorted = np.ascontiguousarray(idx_sorted, dtype=np.int32)
    k = idx_sorted.shape[0]
    T = msgs[0].codes.shape[0] if k < E else msgs[0].outl.shape[0]
    cb = ((E - k) * bits + 7) // 8
    keep = []

    def table(name, dtype, shape):
        arr = (ctypes.c_void_p * N)()
        for i, mg in enumerate(msgs):
            a = np.ascontiguousarray(getattr(mg, name), dtype=dtype)
            assert a.shape == shape, (name, a.shape, shape)
            keep.append(a)
            arr[i] = a.ctypes.data
        return arr

    codes = table("codes", np.uint8, (T, cb))
    outl = table("outl", np.uint16, (T, k))
    out = np.empty((T, E), np.float32 if out_fp32 else np.uint16)
    if bits == 4 and not generic:
        rc = _load().orc_decode_reduce_static(N, T, E, k, _ptr(idx_sorted), codes, outl, _ptr(step),
                                              accum, int(bool(out_fp32)), _ptr(out), threads)
    else:
        rc = _load().orc_decode_reduce_static_bits(N, T, E, k, bits, _ptr(idx_sorted), codes, outl,
                                                   _ptr(step), accum, int(bool(out_fp32)), _ptr(out),
                                                   threads)
    if rc:
        raise ValueError("orc_decode_reduce_static: bad arguments")
    return out
