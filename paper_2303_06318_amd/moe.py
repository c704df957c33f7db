"""Thin Python binding of the C-ABI library (include/moe.h): argument marshalling only.

Every function has the name and argument order of the C entry point; tensors are torch
tensors on the GPU (torch is used for device memory and the stream handle only) and are
passed as raw device pointers.  Nothing here computes anything: if ``libmoe_ted.so`` is not
built, importing the library raises -- there is no fallback path.
"""
from __future__ import annotations

import ctypes as C
import os

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libmoe_ted.so")

MOE_OK, MOE_ERR_INVALID_ARG, MOE_ERR_UNSUPPORTED, MOE_ERR_WORKSPACE_TOO_SMALL, MOE_ERR_HIP = range(5)
MOE_F32, MOE_BF16 = 0, 1
MOE_GELU_ERF, MOE_GELU_TANH = 0, 1

EXPORTS = ["moe_capacity", "moe_workspace_bytes", "moe_status_string", "moe_last_error", "moe_version", "moe_gate",
           "moe_dispatch", "moe_expert_ffn_fwd", "moe_combine", "moe_combine_bwd", "moe_expert_ffn_bwd",
           "moe_dispatch_bwd", "moe_gate_bwd", "moe_adamw_tiled", "moe_expert_ffn_fwd_fused",
           "moe_expert_ffn_fwd_static", "moe_launch_floor", "moe_dispatch_dtd", "moe_dtd_drop", "moe_dtd_gather",
           "moe_expert_ffn_fwd_dtd", "moe_dispatch_bwd_dtd"]
MOE_STATIC_SCRATCH_BYTES = 256 * 1024


class Shape(C.Structure):
    _fields_ = [("T", C.c_int64), ("h", C.c_int32), ("E", C.c_int32), ("f", C.c_int32), ("C", C.c_int64),
                ("dtype", C.c_int32), ("act", C.c_int32)]


class AdamwParams(C.Structure):
    _fields_ = [("lr", C.c_float), ("beta1", C.c_float), ("beta2", C.c_float), ("eps", C.c_float),
                ("weight_decay", C.c_float), ("grad_mult", C.c_float), ("step", C.c_int32)]


class MoeError(RuntimeError):
    def __init__(self, status: int, text: str):
        super().__init__(f"{status_string(status)}: {text}")
        self.status = status


_lib = None


def lib():
    """Load the HIP library; raises if it has not been built (python paper_2303_06318_amd/build.py)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is missing: build it with __graft_entry__.build() -- there is no fallback")
        L = C.CDLL(LIB_PATH)
        vp, i32, i64, sz = C.c_void_p, C.c_int32, C.c_int64, C.c_size_t
        sp = C.POINTER(Shape)
        L.moe_capacity.restype = i64
        L.moe_capacity.argtypes = [i64, i32, C.c_double]
        L.moe_workspace_bytes.restype = sz
        L.moe_workspace_bytes.argtypes = [sp, C.c_int]
        L.moe_status_string.restype = C.c_char_p
        L.moe_status_string.argtypes = [C.c_int]
        L.moe_last_error.restype = C.c_char_p
        L.moe_version.restype = C.c_int
        sig = {
            "moe_gate": [sp] + [vp] * 11 + [vp, sz, vp],
            "moe_dispatch": [sp, vp, vp, vp, vp],
            "moe_expert_ffn_fwd": [sp] + [vp] * 7 + [vp, sz, vp],
            "moe_expert_ffn_fwd_static": [sp] + [vp] * 7 + [vp],
            "moe_launch_floor": [i32, vp],
            "moe_dispatch_dtd": [sp, vp, vp, i32, i32, vp, vp],
            "moe_dtd_drop": [sp, vp, vp, i32, i32, vp, vp],
            "moe_dtd_gather": [sp, vp, vp, i32, vp, vp],
            "moe_expert_ffn_fwd_dtd": [sp, vp, i32] + [vp] * 6 + [vp, sz, vp],
            "moe_dispatch_bwd_dtd": [sp, vp, i32] + [vp] * 5 + [vp],
            "moe_combine": [sp] + [vp] * 5 + [vp],
            "moe_expert_ffn_fwd_fused": [sp] + [vp] * 12 + [vp, sz, vp],
            "moe_combine_bwd": [sp] + [vp] * 7 + [vp],
            "moe_expert_ffn_bwd": [sp] + [vp] * 10 + [vp, sz, vp],
            "moe_dispatch_bwd": [sp] + [vp] * 6 + [vp],
            "moe_gate_bwd": [sp] + [vp] * 8 + [vp, sz, vp],
            "moe_adamw_tiled": [i64, i64, C.POINTER(AdamwParams)] + [vp] * 6 + [i32, vp],
        }
        for name, args in sig.items():
            fn = getattr(L, name)
            fn.restype = C.c_int
            fn.argtypes = args
        _lib = L
    return _lib


def _ptr(t):
    if t is None:
        return None
    if isinstance(t, int):
        return C.c_void_p(t)
    return C.c_void_p(t.data_ptr())


def _stream(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream().cuda_stream
    return C.c_void_p(int(stream))


def _nbytes(t):
    return 0 if t is None else t.numel() * t.element_size()


def _check(st: int):
    if st != MOE_OK:
        raise MoeError(st, lib().moe_last_error().decode())


def status_string(st: int) -> str:
    return lib().moe_status_string(int(st)).decode()


def make_shape(T, h, E, f, Cap, dtype=MOE_BF16, act=MOE_GELU_ERF) -> Shape:
    return Shape(int(T), int(h), int(E), int(f), int(Cap), int(dtype), int(act))


def moe_capacity(T: int, E: int, capacity_factor: float) -> int:
    return int(lib().moe_capacity(int(T), int(E), float(capacity_factor)))


def moe_workspace_bytes(shape: Shape, for_backward) -> int:
    """for_backward: 0 / False forward only, 1 / True forward + backward, 2 with activation recomputation."""
    return int(lib().moe_workspace_bytes(C.byref(shape), int(for_backward)))


def moe_version() -> int:
    return int(lib().moe_version())


def moe_launch_floor(n, stream=None):
    _check(lib().moe_launch_floor(int(n), _stream(stream)))


def moe_gate(shape, x, w_gate, logit_bias, logits, probs, expert, gate_p, slot, counts, kept, token_of_slot, ws,
             stream=None):
    _check(lib().moe_gate(C.byref(shape), _ptr(x), _ptr(w_gate), _ptr(logit_bias), _ptr(logits), _ptr(probs),
                          _ptr(expert), _ptr(gate_p), _ptr(slot), _ptr(counts), _ptr(kept), _ptr(token_of_slot),
                          _ptr(ws), _nbytes(ws), _stream(stream)))


def moe_dispatch(shape, x, token_of_slot, buf, stream=None):
    _check(lib().moe_dispatch(C.byref(shape), _ptr(x), _ptr(token_of_slot), _ptr(buf), _stream(stream)))


def moe_expert_ffn_fwd(shape, buf, w1, w2, kept, z_save, hact, y, ws, stream=None):
    _check(lib().moe_expert_ffn_fwd(C.byref(shape), _ptr(buf), _ptr(w1), _ptr(w2), _ptr(kept), _ptr(z_save),
                                    _ptr(hact), _ptr(y), _ptr(ws), _nbytes(ws), _stream(stream)))


def moe_expert_ffn_fwd_static(shape, buf, w1, w2, kept, z_save, hact, y, stream=None):
    _check(lib().moe_expert_ffn_fwd_static(C.byref(shape), _ptr(buf), _ptr(w1), _ptr(w2), _ptr(kept), _ptr(z_save),
                                           _ptr(hact), _ptr(y), _stream(stream)))


def moe_expert_ffn_fwd_fused(shape, x, buf, token_of_slot, slot, gate_p, w1, w2, kept, z_save, hact, y, out, ws,
                             stream=None):
    _check(lib().moe_expert_ffn_fwd_fused(C.byref(shape), _ptr(x), _ptr(buf), _ptr(token_of_slot), _ptr(slot),
                                          _ptr(gate_p), _ptr(w1), _ptr(w2), _ptr(kept), _ptr(z_save), _ptr(hact),
                                          _ptr(y), _ptr(out), _ptr(ws), _nbytes(ws), _stream(stream)))


def moe_dispatch_dtd(shape, x, token_of_slot, tp_rank, tp_size, share, stream=None):
    _check(lib().moe_dispatch_dtd(C.byref(shape), _ptr(x), _ptr(token_of_slot), int(tp_rank), int(tp_size), _ptr(share),
                                  _stream(stream)))


def moe_dtd_drop(shape, buf, kept, tp_rank, tp_size, share, stream=None):
    _check(lib().moe_dtd_drop(C.byref(shape), _ptr(buf), _ptr(kept), int(tp_rank), int(tp_size), _ptr(share),
                              _stream(stream)))


def moe_dtd_gather(shape, shares, kept, tp_size, buf, stream=None):
    _check(lib().moe_dtd_gather(C.byref(shape), _ptr(shares), _ptr(kept), int(tp_size), _ptr(buf), _stream(stream)))


def moe_expert_ffn_fwd_dtd(shape, shares, tp_size, w1, w2, kept, z_save, hact, y, ws, stream=None):
    _check(lib().moe_expert_ffn_fwd_dtd(C.byref(shape), _ptr(shares), int(tp_size), _ptr(w1), _ptr(w2), _ptr(kept),
                                        _ptr(z_save), _ptr(hact), _ptr(y), _ptr(ws), _nbytes(ws), _stream(stream)))


def moe_dispatch_bwd_dtd(shape, d_shares, tp_size, expert, slot, d_x, d_logits=None, w_gate=None, stream=None):
    _check(lib().moe_dispatch_bwd_dtd(C.byref(shape), _ptr(d_shares), int(tp_size), _ptr(expert), _ptr(slot), _ptr(d_x),
                                      _ptr(d_logits), _ptr(w_gate), _stream(stream)))


def moe_combine(shape, y, expert, slot, gate_p, out, stream=None):
    _check(lib().moe_combine(C.byref(shape), _ptr(y), _ptr(expert), _ptr(slot), _ptr(gate_p), _ptr(out),
                             _stream(stream)))


def moe_combine_bwd(shape, d_out, y, token_of_slot, slot, gate_p, d_y, d_gate_p, stream=None):
    _check(lib().moe_combine_bwd(C.byref(shape), _ptr(d_out), _ptr(y), _ptr(token_of_slot), _ptr(slot), _ptr(gate_p),
                                 _ptr(d_y), _ptr(d_gate_p), _stream(stream)))


def moe_expert_ffn_bwd(shape, d_y, buf, z_save, hact, w1, w2, kept, d_buf, d_w1, d_w2, ws, stream=None):
    _check(lib().moe_expert_ffn_bwd(C.byref(shape), _ptr(d_y), _ptr(buf), _ptr(z_save), _ptr(hact), _ptr(w1), _ptr(w2),
                                    _ptr(kept), _ptr(d_buf), _ptr(d_w1), _ptr(d_w2), _ptr(ws), _nbytes(ws),
                                    _stream(stream)))


def moe_dispatch_bwd(shape, d_buf, expert, slot, d_x, d_logits=None, w_gate=None, stream=None):
    _check(lib().moe_dispatch_bwd(C.byref(shape), _ptr(d_buf), _ptr(expert), _ptr(slot), _ptr(d_x), _ptr(d_logits),
                                  _ptr(w_gate), _stream(stream)))


def moe_gate_bwd(shape, d_gate_p, probs, expert, x, w_gate, d_logits, d_w_gate, d_x_accum, ws, stream=None):
    _check(lib().moe_gate_bwd(C.byref(shape), _ptr(d_gate_p), _ptr(probs), _ptr(expert), _ptr(x), _ptr(w_gate),
                              _ptr(d_logits), _ptr(d_w_gate), _ptr(d_x_accum), _ptr(ws), _nbytes(ws),
                              _stream(stream)))


def make_adamw(lr, beta1, beta2, eps, weight_decay, step, grad_mult=1.0) -> AdamwParams:
    return AdamwParams(float(lr), float(beta1), float(beta2), float(eps), float(weight_decay), float(grad_mult),
                       int(step))


def moe_adamw_tiled(n, ts, hp, grad, master, exp_avg, exp_avg_sq, param, staging, dtype=MOE_BF16, stream=None):
    _check(lib().moe_adamw_tiled(int(n), int(ts), C.byref(hp), _ptr(grad), _ptr(master), _ptr(exp_avg),
                                 _ptr(exp_avg_sq), _ptr(param), _ptr(staging), int(dtype), _stream(stream)))
