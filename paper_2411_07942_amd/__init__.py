"""Python binding of libtpq.so -- the MI355X codec for low-bit tensor-parallel
partial sums (calibration, encode, decode-and-reduce).

This module only marshals arguments: torch tensors provide device memory and the
current stream, every step of the path runs in the library's HIP kernels.  The
function names are those of ``include/tpq.h`` without the ``tpq_`` prefix.  There
is no CPU fallback: if ``libtpq.so`` has not been built
(``python -m paper_2411_07942_amd.build``), importing succeeds but the first call
raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

import torch

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libtpq.so")

OK = 0
ERR_NULL, ERR_SHAPE, ERR_INDEX, ERR_UNSUPPORTED, ERR_ALIGN, ERR_WORKSPACE, ERR_HIP = (
    -1, -2, -3, -4, -5, -6, -7)
ACC_FP32, ACC_BF16, ACC_FAST = 0, 1, 2
OUT_BF16, OUT_FP32 = 0, 1
MAX_RANKS = 64
MAX_E = 32768

EXPORTS = [
    "tpq_layout_init", "tpq_payload_bits", "tpq_wire_bits", "tpq_strerror", "tpq_last_hip_error",
    "tpq_bench_time_next_launch",
    "tpq_plan_bytes", "tpq_plan_build", "tpq_plan_check",
    "tpq_calibrate_workspace_bytes", "tpq_calibrate", "tpq_calibrate_fixed",
    "tpq_calibrate_finalize_workspace_bytes", "tpq_calibrate_finalize",
    "tpq_encode", "tpq_hop", "tpq_gemm_weights", "tpq_gemm_encode", "tpq_decode_reduce", "tpq_decode_reduce_fused",
    "tpq_static_table_floats", "tpq_static_params", "tpq_encode_static", "tpq_decode_reduce_static",
]


class Layout(ctypes.Structure):
    """Mirror of ``tpq_layout``."""
    _fields_ = [("E", ctypes.c_int32), ("k", ctypes.c_int32), ("G", ctypes.c_int32),
                ("bits", ctypes.c_int32), ("r", ctypes.c_int32), ("ng", ctypes.c_int32),
                ("code_bytes", ctypes.c_int32), ("reserved", ctypes.c_int32),
                ("pitch_codes", ctypes.c_int64), ("pitch_meta", ctypes.c_int64),
                ("pitch_outl", ctypes.c_int64), ("wire_bytes_per_row", ctypes.c_int64)]


class TpqError(RuntimeError):
    def __init__(self, code: int, where: str):
        self.code = code
        msg = _load().tpq_strerror(code).decode()
        if code == ERR_HIP:
            msg += " (hipError %d)" % _load().tpq_last_hip_error()
        super().__init__("%s: %s [%d]" % (where, msg, code))


_lib = None


def _load():
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError("libtpq.so is not built: run `python -m paper_2411_07942_amd.build` "
                           "(there is no fallback path)")
    lib = ctypes.CDLL(LIB_PATH)
    c_int, i64, vp, sz = ctypes.c_int, ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t
    LP = ctypes.POINTER(Layout)
    lib.tpq_layout_init.argtypes = [LP, c_int, c_int, c_int, c_int]
    lib.tpq_payload_bits.argtypes = [LP]
    lib.tpq_payload_bits.restype = ctypes.c_double
    lib.tpq_wire_bits.argtypes = [LP]
    lib.tpq_wire_bits.restype = ctypes.c_double
    lib.tpq_strerror.argtypes = [c_int]
    lib.tpq_strerror.restype = ctypes.c_char_p
    lib.tpq_last_hip_error.restype = c_int
    lib.tpq_plan_bytes.argtypes = [LP]
    lib.tpq_plan_bytes.restype = sz
    lib.tpq_plan_build.argtypes = [LP, vp, vp, sz, vp]
    lib.tpq_plan_check.argtypes = [LP, vp, vp]
    lib.tpq_calibrate_workspace_bytes.argtypes = [i64, c_int]
    lib.tpq_calibrate_workspace_bytes.restype = sz
    lib.tpq_calibrate.argtypes = [vp, i64, i64, c_int, c_int, c_int, i64, ctypes.c_float,
                                  vp, vp, vp, sz, vp]
    lib.tpq_calibrate_fixed.argtypes = [vp, i64, i64, c_int, c_int, c_int, i64, ctypes.c_float, vp, vp, vp]
    lib.tpq_calibrate_finalize_workspace_bytes.argtypes = [c_int]
    lib.tpq_calibrate_finalize_workspace_bytes.restype = sz
    lib.tpq_calibrate_finalize.argtypes = [vp, vp, c_int, c_int, c_int, vp, vp, vp, vp, vp, sz, vp]
    lib.tpq_encode.argtypes = [LP, vp, vp, i64, c_int, i64, vp, vp, vp, vp, vp]
    lib.tpq_bench_time_next_launch.argtypes = [vp, vp]
    lib.tpq_hop.argtypes = [LP, vp, vp, i64, c_int, i64, vp, vp, vp, vp, c_int, vp, vp, vp, vp, vp]
    lib.tpq_gemm_weights.argtypes = [LP, vp, vp, i64, c_int, vp, vp]
    lib.tpq_gemm_encode.argtypes = [LP, vp, i64, i64, c_int, vp, vp, vp, vp, vp, vp, i64, vp]
    lib.tpq_decode_reduce.argtypes = [LP, vp, c_int, i64, vp, vp, vp, vp, c_int, c_int, vp, i64, vp]
    lib.tpq_decode_reduce_fused.argtypes = [LP, vp, c_int, i64, vp, vp, vp, vp, vp, i64, vp, c_int, c_int,
                                            vp, i64, vp]
    lib.tpq_static_table_floats.argtypes = [LP]
    lib.tpq_static_table_floats.restype = sz
    lib.tpq_static_params.argtypes = [LP, vp, vp, vp, c_int, vp, vp, vp]
    lib.tpq_encode_static.argtypes = [LP, vp, vp, i64, c_int, i64, vp, vp, vp, vp]
    lib.tpq_decode_reduce_static.argtypes = [LP, vp, c_int, i64, vp, vp, vp, c_int, c_int, vp, i64, vp]
    _lib = lib
    return lib


def _check(rc: int, where: str) -> None:
    if rc != OK:
        raise TpqError(rc, where)


def _ptr(t: Optional[torch.Tensor]):
    return None if t is None else ctypes.c_void_p(t.data_ptr())


def _stream(stream=None):
    if stream is None:
        stream = torch.cuda.current_stream()
    return ctypes.c_void_p(stream.cuda_stream)


def _ptr_array(tensors: Optional[Sequence[torch.Tensor]], n: int):
    if tensors is None:
        return None
    arr = (ctypes.c_void_p * n)()
    for i in range(n):
        arr[i] = tensors[i].data_ptr()
    return arr


# ---- layout ----------------------------------------------------------------------

def layout_init(E: int, k: int, G: int, bits: int = 4) -> Layout:
    L = Layout()
    _check(_load().tpq_layout_init(ctypes.byref(L), E, k, G, bits), "tpq_layout_init")
    return L


def payload_bits(L: Layout) -> float:
    return float(_load().tpq_payload_bits(ctypes.byref(L)))


def wire_bits(L: Layout) -> float:
    return float(_load().tpq_wire_bits(ctypes.byref(L)))


# ---- plan ------------------------------------------------------------------------

def plan_bytes(L: Layout) -> int:
    return int(_load().tpq_plan_bytes(ctypes.byref(L)))


def plan_build(L: Layout, idx_sorted: torch.Tensor, plan: Optional[torch.Tensor] = None,
               stream=None) -> torch.Tensor:
    """idx_sorted: int32 device tensor [k].  Returns the (uint8, device) plan buffer."""
    if plan is None:
        plan = torch.empty(plan_bytes(L), dtype=torch.uint8, device=idx_sorted.device)
    _check(_load().tpq_plan_build(ctypes.byref(L), _ptr(idx_sorted), _ptr(plan), plan.numel(),
                                  _stream(stream)), "tpq_plan_build")
    return plan


def plan_check(L: Layout, plan: torch.Tensor, stream=None) -> None:
    _check(_load().tpq_plan_check(ctypes.byref(L), _ptr(plan), _stream(stream)), "tpq_plan_check")


# ---- calibration -----------------------------------------------------------------

def calibrate_workspace_bytes(S: int, E: int) -> int:
    return int(_load().tpq_calibrate_workspace_bytes(S, E))


def calibrate(Y: torch.Tensor, rank: int, n_ranks: int, seq_index: int, gamma: float,
              m: torch.Tensor, M: torch.Tensor, workspace: torch.Tensor, stream=None) -> None:
    """One sequence Y (bf16 [S,E], row stride Y.stride(0)) of device `rank`; m, M fp32 [n_ranks,E]."""
    S, E = Y.shape
    _check(_load().tpq_calibrate(_ptr(Y), S, Y.stride(0) if S > 1 else max(E, Y.stride(0)), E,
                                 rank, n_ranks, seq_index, gamma, _ptr(m), _ptr(M),
                                 _ptr(workspace), workspace.numel() * workspace.element_size(),
                                 _stream(stream)), "tpq_calibrate")


def calibrate_workspace(S: int, E: int, device) -> torch.Tensor:
    """A workspace for calibrate()."""
    return torch.empty(max(calibrate_workspace_bytes(S, E), 16), dtype=torch.uint8, device=device)


def calibrate_fixed(Y: torch.Tensor, rank: int, n_ranks: int, seq_index: int, gamma: float,
                    m: torch.Tensor, M: torch.Tensor, stream=None) -> None:
    """calibrate() with the library's own scratch buffer instead of a workspace (tpq_calibrate_fixed)."""
    S, E = Y.shape
    _check(_load().tpq_calibrate_fixed(_ptr(Y), S, Y.stride(0) if S > 1 else max(E, Y.stride(0)), E,
                                       rank, n_ranks, seq_index, gamma, _ptr(m), _ptr(M),
                                       _stream(stream)), "tpq_calibrate_fixed")


def calibrate_finalize_workspace_bytes(E: int) -> int:
    return int(_load().tpq_calibrate_finalize_workspace_bytes(E))


def calibrate_finalize(m: torch.Tensor, M: torch.Tensor, k: int, Rbar: torch.Tensor,
                       idx_sorted: torch.Tensor, idx_ranked: Optional[torch.Tensor],
                       workspace: torch.Tensor, R: Optional[torch.Tensor] = None,
                       stream=None) -> None:
    n_ranks, E = m.shape
    _check(_load().tpq_calibrate_finalize(_ptr(m), _ptr(M), n_ranks, E, k, _ptr(R), _ptr(Rbar),
                                          _ptr(idx_sorted), _ptr(idx_ranked), _ptr(workspace),
                                          workspace.numel() * workspace.element_size(),
                                          _stream(stream)), "tpq_calibrate_finalize")


# ---- messages --------------------------------------------------------------------

class Message:
    """Device buffers of one rank's message for one block (pitched rows)."""

    def __init__(self, L: Layout, T: int, device, fill: Optional[int] = None):
        def buf(pitch):
            n = max(int(pitch) * T, 16)
            t = torch.empty(n, dtype=torch.uint8, device=device)
            if fill is not None:
                t.fill_(fill)
            return t
        self.T = T
        self.codes = buf(L.pitch_codes)
        self.scale = buf(L.pitch_meta)
        self.zero = buf(L.pitch_meta)
        self.outl = buf(L.pitch_outl)

    def to_dense(self, L: Layout):
        """Logical content as CPU numpy arrays (pad bytes dropped)."""
        import numpy as np
        T = self.T

        def rows(t, pitch, nbytes):
            if T == 0 or nbytes == 0:
                return np.zeros((T, nbytes), np.uint8)
            a = t.cpu().numpy()[: pitch * T].reshape(T, pitch)
            return np.ascontiguousarray(a[:, :nbytes])
        codes = rows(self.codes, L.pitch_codes, L.code_bytes)
        scale = rows(self.scale, L.pitch_meta, 2 * L.ng).view(np.uint16)
        zero = rows(self.zero, L.pitch_meta, 2 * L.ng).view(np.uint16)
        outl = rows(self.outl, L.pitch_outl, 2 * L.k).view(np.uint16)
        return outl.reshape(T, L.k), codes, scale.reshape(T, L.ng), zero.reshape(T, L.ng)


def encode_call(L: Layout, plan: torch.Tensor, Y: Sequence[torch.Tensor],
                msgs: Sequence[Message]):
    """Marshal a tpq_encode call once; the returned function(stream=None) issues it.
    The tensors must stay alive (and in place) for as long as the function is used."""
    lib = _load()
    n = len(Y)
    T = Y[0].shape[0]
    ldY = Y[0].stride(0) if T > 1 else max(L.E, Y[0].stride(0))
    for y in Y:
        assert y.dtype == torch.bfloat16 and y.shape == Y[0].shape and y.stride(1) == 1
        assert T <= 1 or y.stride(0) == ldY
    args = (ctypes.byref(L), _ptr(plan), _ptr_array(Y, n), ldY, n, T,
            _ptr_array([m.codes for m in msgs], n), _ptr_array([m.scale for m in msgs], n),
            _ptr_array([m.zero for m in msgs], n), _ptr_array([m.outl for m in msgs], n))
    keep = (L, plan, list(Y), list(msgs))

    def call(stream=None, _keep=keep):
        _check(lib.tpq_encode(*args, _stream(stream)), "tpq_encode")
    return call


def encode(L: Layout, plan: torch.Tensor, Y: Sequence[torch.Tensor], msgs: Sequence[Message],
           stream=None) -> None:
    """Encode the ranks' partial sums Y[i] (bf16 [T,E]) into msgs[i] in one launch."""
    encode_call(L, plan, Y, msgs)(stream)


def bench_time_next_launch(start: Optional[torch.cuda.Event], stop: Optional[torch.cuda.Event]) -> None:
    """Attach two timing events to the next encode / ring step / decode kernel launched from this
    thread (tpq_bench_time_next_launch).  The events must exist already (recorded once before), so that
    their handles can be passed; afterwards start.elapsed_time(stop) is the kernel's duration."""
    if start is None:
        _check(_load().tpq_bench_time_next_launch(None, None), "tpq_bench_time_next_launch")
        return
    h0, h1 = start.cuda_event, stop.cuda_event
    if not h0 or not h1:
        raise ValueError("bench_time_next_launch: record each event once before handing it over")
    _check(_load().tpq_bench_time_next_launch(h0, h1), "tpq_bench_time_next_launch")


def hop_call(L: Layout, plan: torch.Tensor, Y: Sequence[torch.Tensor], in_msgs: Sequence[Message],
             out_msgs: Sequence[Message], accum: int = ACC_BF16):
    """Marshal a tpq_hop call once; the returned function(stream=None) issues it."""
    lib = _load()
    n = len(Y)
    T = Y[0].shape[0]
    ldY = Y[0].stride(0) if T > 1 else max(L.E, Y[0].stride(0))
    for y in Y:
        assert y.dtype == torch.bfloat16 and y.shape == Y[0].shape and y.stride(1) == 1
        assert T <= 1 or y.stride(0) == ldY
    assert len(in_msgs) == n and len(out_msgs) == n
    args = (ctypes.byref(L), _ptr(plan), _ptr_array(Y, n), ldY, n, T,
            _ptr_array([m.codes for m in in_msgs], n), _ptr_array([m.scale for m in in_msgs], n),
            _ptr_array([m.zero for m in in_msgs], n), _ptr_array([m.outl for m in in_msgs], n), accum,
            _ptr_array([m.codes for m in out_msgs], n), _ptr_array([m.scale for m in out_msgs], n),
            _ptr_array([m.zero for m in out_msgs], n), _ptr_array([m.outl for m in out_msgs], n))
    keep = (L, plan, list(Y), list(in_msgs), list(out_msgs))

    def call(stream=None, _keep=keep):
        _check(lib.tpq_hop(*args, _stream(stream)), "tpq_hop")
    return call


def hop(L: Layout, plan: torch.Tensor, Y: Sequence[torch.Tensor], in_msgs: Sequence[Message],
        out_msgs: Sequence[Message], accum: int = ACC_BF16, stream=None) -> None:
    """Ring step: out_msgs[i] = encode(bf16(dequantised in_msgs[i] (+) Y[i])), one launch."""
    hop_call(L, plan, Y, in_msgs, out_msgs, accum)(stream)


def gemm_weights(L: Layout, plan: torch.Tensor, Wt: torch.Tensor, stream=None) -> torch.Tensor:
    """Rows of Wt (bf16 [E, K], one row per output feature) in message order: the weights
    tpq_gemm_encode takes."""
    lib = _load()
    assert Wt.dtype == torch.bfloat16 and Wt.dim() == 2 and Wt.shape[0] == L.E and Wt.stride(1) == 1
    K = Wt.shape[1]
    Wp = torch.empty((L.E, K), dtype=torch.bfloat16, device=Wt.device)
    _check(lib.tpq_gemm_weights(ctypes.byref(L), _ptr(plan), _ptr(Wt), Wt.stride(0), K, _ptr(Wp),
                                _stream(stream)), "tpq_gemm_weights")
    return Wp


def gemm_encode_call(L: Layout, X: torch.Tensor, Wp: torch.Tensor, msg: Message,
                     Y_msg: Optional[torch.Tensor] = None):
    """Marshal a tpq_gemm_encode call once; the returned function(stream=None) issues it.
    X bf16 [T, K]; Wp from gemm_weights; Y_msg: optional bf16 [T, >= E] for the rounded product
    in message order."""
    lib = _load()
    assert X.dtype == torch.bfloat16 and X.dim() == 2 and X.stride(1) == 1
    assert Wp.dtype == torch.bfloat16 and Wp.is_contiguous() and Wp.shape == (L.E, X.shape[1])
    T, K = X.shape
    ldX = X.stride(0) if T > 1 else max(K, X.stride(0))
    ldYm = 0
    if Y_msg is not None:
        assert Y_msg.dtype == torch.bfloat16 and Y_msg.shape[0] == T and Y_msg.stride(1) == 1
        ldYm = Y_msg.stride(0) if T > 1 else max(L.E, Y_msg.stride(0))
    args = (ctypes.byref(L), _ptr(X), T, ldX, K, _ptr(Wp), _ptr(msg.codes), _ptr(msg.scale), _ptr(msg.zero),
            _ptr(msg.outl), _ptr(Y_msg) if Y_msg is not None else None, ldYm)
    keep = (L, X, Wp, msg, Y_msg)

    def call(stream=None, _keep=keep):
        _check(lib.tpq_gemm_encode(*args, _stream(stream)), "tpq_gemm_encode")
    return call


def gemm_encode(L: Layout, X: torch.Tensor, Wp: torch.Tensor, msg: Message,
                Y_msg: Optional[torch.Tensor] = None, stream=None) -> None:
    """msg = encode(bf16(X @ W)) for one device, the product never stored (unless Y_msg asks)."""
    gemm_encode_call(L, X, Wp, msg, Y_msg)(stream)


def decode_reduce_call(L: Layout, plan: torch.Tensor, msgs: Sequence[Message], out: torch.Tensor,
                       accum: int = ACC_FP32):
    """Marshal a tpq_decode_reduce call once; the returned function(stream=None) issues it."""
    lib = _load()
    n = len(msgs)
    T = out.shape[0]
    out_dtype = OUT_FP32 if out.dtype == torch.float32 else OUT_BF16
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    ldOut = out.stride(0) if T > 1 else max(L.E, out.stride(0))
    args = (ctypes.byref(L), _ptr(plan), n, T,
            _ptr_array([m.codes for m in msgs], n), _ptr_array([m.scale for m in msgs], n),
            _ptr_array([m.zero for m in msgs], n), _ptr_array([m.outl for m in msgs], n),
            accum, out_dtype, _ptr(out), ldOut)
    keep = (L, plan, list(msgs), out)

    def call(stream=None, _keep=keep):
        _check(lib.tpq_decode_reduce(*args, _stream(stream)), "tpq_decode_reduce")
    return call


def decode_reduce(L: Layout, plan: torch.Tensor, msgs: Sequence[Message], out: torch.Tensor,
                  accum: int = ACC_FP32, stream=None) -> None:
    """Dequantise and add msgs[0..n-1] into out ([T,E] bf16 or fp32)."""
    decode_reduce_call(L, plan, msgs, out, accum)(stream)


def decode_reduce_fused_call(L: Layout, plan: torch.Tensor, msgs: Sequence[Message], out: torch.Tensor,
                             addend: Optional[torch.Tensor] = None, bias: Optional[torch.Tensor] = None,
                             accum: int = ACC_FP32):
    """Marshal a tpq_decode_reduce_fused call once; the returned function(stream=None) issues it.
    addend: bf16 [T, E] (row stride free) or None; bias: bf16 [E] or None."""
    lib = _load()
    n = len(msgs)
    T = out.shape[0]
    out_dtype = OUT_FP32 if out.dtype == torch.float32 else OUT_BF16
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    ldOut = out.stride(0) if T > 1 else max(L.E, out.stride(0))
    ldAdd = 0
    if addend is not None:
        assert addend.dtype == torch.bfloat16 and addend.shape == (T, L.E) and addend.stride(1) == 1
        ldAdd = addend.stride(0) if T > 1 else max(L.E, addend.stride(0))
    if bias is not None:
        assert bias.dtype == torch.bfloat16 and bias.shape == (L.E,) and bias.is_contiguous()
    args = (ctypes.byref(L), _ptr(plan), n, T,
            _ptr_array([m.codes for m in msgs], n), _ptr_array([m.scale for m in msgs], n),
            _ptr_array([m.zero for m in msgs], n), _ptr_array([m.outl for m in msgs], n),
            _ptr(addend), ldAdd, _ptr(bias), accum, out_dtype, _ptr(out), ldOut)
    keep = (L, plan, list(msgs), out, addend, bias)

    def call(stream=None, _keep=keep):
        _check(lib.tpq_decode_reduce_fused(*args, _stream(stream)), "tpq_decode_reduce_fused")
    return call


def decode_reduce_fused(L, plan, msgs, out, addend=None, bias=None, accum: int = ACC_FP32, stream=None) -> None:
    """out = ((sum of the dequantised msgs) + addend) + bias, in one kernel."""
    decode_reduce_fused_call(L, plan, msgs, out, addend, bias, accum)(stream)


# ---- static symmetric mode -------------------------------------------------------

def static_table_floats(L: Layout) -> int:
    return int(_load().tpq_static_table_floats(ctypes.byref(L)))


def static_params(L: Layout, plan: torch.Tensor, m: torch.Tensor, M: torch.Tensor,
                  stream=None):
    """Calibration state m, M (fp32 [n_ranks, E]) -> (step, inv), fp32
    [n_ranks, static_table_floats(L)] in the plan's compacted feature order."""
    assert m.dtype == torch.float32 and M.dtype == torch.float32 and m.shape == M.shape
    assert m.is_contiguous() and M.is_contiguous() and m.shape[1] == L.E
    n = m.shape[0]
    w = max(static_table_floats(L), 4)
    step = torch.empty((n, w), dtype=torch.float32, device=m.device)
    inv = torch.empty((n, w), dtype=torch.float32, device=m.device)
    _check(_load().tpq_static_params(ctypes.byref(L), _ptr(plan), _ptr(m), _ptr(M), n,
                                     _ptr(step), _ptr(inv), _stream(stream)), "tpq_static_params")
    return step, inv


def encode_static_call(L: Layout, plan: torch.Tensor, Y: Sequence[torch.Tensor],
                       inv: torch.Tensor, msgs: Sequence[Message]):
    """Marshal a tpq_encode_static call once (inv: the rows of the ranks in Y, in order);
    the returned function(stream=None) issues it."""
    lib = _load()
    n = len(Y)
    T = Y[0].shape[0]
    ldY = Y[0].stride(0) if T > 1 else max(L.E, Y[0].stride(0))
    for y in Y:
        assert y.dtype == torch.bfloat16 and y.shape == Y[0].shape and y.stride(1) == 1
        assert T <= 1 or y.stride(0) == ldY
    assert inv.dtype == torch.float32 and inv.is_contiguous() and inv.shape[0] >= n
    args = (ctypes.byref(L), _ptr(plan), _ptr_array(Y, n), ldY, n, T, _ptr(inv),
            _ptr_array([m.codes for m in msgs], n), _ptr_array([m.outl for m in msgs], n))
    keep = (L, plan, list(Y), inv, list(msgs))

    def call(stream=None, _keep=keep):
        _check(lib.tpq_encode_static(*args, _stream(stream)), "tpq_encode_static")
    return call


def encode_static(L, plan, Y, inv, msgs, stream=None) -> None:
    encode_static_call(L, plan, Y, inv, msgs)(stream)


def decode_reduce_static_call(L: Layout, plan: torch.Tensor, msgs: Sequence[Message],
                              step: torch.Tensor, out: torch.Tensor, accum: int = ACC_FP32):
    """Marshal a tpq_decode_reduce_static call once; the returned function(stream=None)
    issues it."""
    lib = _load()
    n = len(msgs)
    T = out.shape[0]
    out_dtype = OUT_FP32 if out.dtype == torch.float32 else OUT_BF16
    assert out.dtype in (torch.float32, torch.bfloat16) and out.stride(1) == 1
    assert step.dtype == torch.float32 and step.is_contiguous() and step.shape[0] >= n
    ldOut = out.stride(0) if T > 1 else max(L.E, out.stride(0))
    args = (ctypes.byref(L), _ptr(plan), n, T,
            _ptr_array([m.codes for m in msgs], n), _ptr_array([m.outl for m in msgs], n),
            _ptr(step), accum, out_dtype, _ptr(out), ldOut)
    keep = (L, plan, list(msgs), step, out)

    def call(stream=None, _keep=keep):
        _check(lib.tpq_decode_reduce_static(*args, _stream(stream)), "tpq_decode_reduce_static")
    return call


def decode_reduce_static(L, plan, msgs, step, out, accum: int = ACC_FP32, stream=None) -> None:
    decode_reduce_static_call(L, plan, msgs, step, out, accum)(stream)
