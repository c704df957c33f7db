"""ctypes front end of the CPU oracle (oracle/moe_oracle.c).

TEST INFRASTRUCTURE ONLY: used by tests, the smoke check and the benchmark's
cpu_baseline leg.  The product path never imports this module, and this module
imports nothing from the GPU package.

Besides 1:1 wrappers of the C functions it offers ``layer_forward`` and
``layer_backward`` which chain them in the layer's order (paper Section 3,
Figure 3 steps 3-7 and their reverse).
"""
from __future__ import annotations

import ctypes as C
import math
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "moe_oracle.c")
_LIB = os.path.join(_HERE, "libmoe_oracle.so")

ACT_GELU_ERF, ACT_GELU_TANH = 0, 1


_LIB_SAN = os.path.join(_HERE, "libmoe_oracle_san.so")


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (plain -O2, OpenMP for the outer loops)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-o", _LIB, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


def build_sanitized(force: bool = False) -> str:
    """The same source with AddressSanitizer and UndefinedBehaviorSanitizer (host code only); any report
    aborts the process.  Loaded instead of the plain library when MOE_ORACLE_SANITIZE=1 is set, in a
    process that was started with the sanitizer runtime preloaded (tests/test_oracle_sanitizers.py)."""
    if force or not os.path.exists(_LIB_SAN) or os.path.getmtime(_LIB_SAN) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O1", "-g", "-fno-omit-frame-pointer", "-fsanitize=address,undefined",
               "-fno-sanitize-recover=all", "-fopenmp", "-fPIC", "-shared", "-std=gnu11", "-o", _LIB_SAN, _SRC, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB_SAN


def sanitizer_runtime() -> str:
    """Path of gcc's AddressSanitizer runtime (what such a process preloads)."""
    return subprocess.run(["gcc", "-print-file-name=libasan.so"], check=True, capture_output=True,
                          text=True).stdout.strip()


_lib = None


def lib():
    global _lib
    if _lib is None:
        if os.environ.get("MOE_ORACLE_SANITIZE") == "1":
            L = C.CDLL(build_sanitized())
        else:
            build()
            L = C.CDLL(_LIB)
        i64, i32, p, dbl = C.c_int64, C.c_int32, C.c_void_p, C.c_double
        L.orc_act.restype = dbl
        L.orc_act.argtypes = [dbl, i32]
        L.orc_act_grad.restype = dbl
        L.orc_act_grad.argtypes = [dbl, i32]
        L.orc_act_grad_array.restype = None
        L.orc_act_grad_array.argtypes = [i64, p, p, i32]
        L.orc_gate_logits.argtypes = [i64, i32, i32, p, p, p]
        L.orc_top1_softmax.argtypes = [i64, i32, p, p, p, p]
        L.orc_route.argtypes = [i64, i32, i64, p, p, p, p, p]
        L.orc_dispatch.argtypes = [i64, i32, i32, i64, p, p, p, p]
        L.orc_dtd_drop.restype = None
        L.orc_dtd_drop.argtypes = [i32, i64, i32, i32, i32, p, p]
        L.orc_dtd_gather.restype = None
        L.orc_dtd_gather.argtypes = [i32, i64, i32, i32, p, p]
        L.orc_ffn_fwd.argtypes = [i64, i32, i32, i32, p, p, p, p, p, p]
        L.orc_combine.argtypes = [i64, i32, i64, p, p, p, p, p]
        L.orc_combine_bwd.argtypes = [i64, i32, i32, i64, p, p, p, p, p, p, p]
        L.orc_ffn_bwd.argtypes = [i64, i32, i32, i32] + [p] * 10
        L.orc_dispatch_bwd.argtypes = [i64, i32, i64, p, p, p, p]
        L.orc_gate_bwd.argtypes = [i64, i32, i32] + [p] * 8
        L.orc_max_threads.restype = C.c_int
        L.orc_adamw_tiled.restype = None
        L.orc_adamw_tiled.argtypes = [i64, i64, dbl, dbl, dbl, dbl, dbl, i32, dbl] + [p] * 5 + [i32, p, p]
        for name in ("orc_gate_logits", "orc_top1_softmax", "orc_route", "orc_dispatch", "orc_ffn_fwd",
                     "orc_combine", "orc_combine_bwd", "orc_ffn_bwd", "orc_dispatch_bwd", "orc_gate_bwd"):
            getattr(L, name).restype = None
        _lib = L
    return _lib


def _a(x, dt):
    x = np.ascontiguousarray(x, dtype=dt)
    return x


def _p(x):
    return None if x is None else x.ctypes.data_as(C.c_void_p)


def capacity(T: int, E: int, capacity_factor: float) -> int:
    """C = ceil(capacity_factor * T / E), evaluated in double."""
    return int(math.ceil(float(capacity_factor) * float(T) / float(E)))


def act(x: float, mode: int = ACT_GELU_ERF) -> float:
    return lib().orc_act(float(x), mode)


def act_grad(x: float, mode: int = ACT_GELU_ERF) -> float:
    return lib().orc_act_grad(float(x), mode)


def act_grad_array(z, mode: int = ACT_GELU_ERF):
    """act'(z) element by element (float64)."""
    z = np.ascontiguousarray(z, dtype=np.float64)
    g = np.empty_like(z)
    lib().orc_act_grad_array(z.size, z.ctypes.data, g.ctypes.data, mode)
    return g


def gate_logits(x, wg):
    x, wg = _a(x, np.float32), _a(wg, np.float32)
    T, h = x.shape
    E = wg.shape[1]
    out = np.empty((T, E), np.float32)
    lib().orc_gate_logits(T, h, E, _p(x), _p(wg), _p(out))
    return out


def top1_softmax(logits):
    logits = _a(logits, np.float32)
    T, E = logits.shape
    expert = np.empty(T, np.int32)
    gate_p = np.empty(T, np.float32)
    probs = np.empty((T, E), np.float32)
    lib().orc_top1_softmax(T, E, _p(logits), _p(expert), _p(gate_p), _p(probs))
    return expert, gate_p, probs


def route(expert, E: int, Cap: int):
    expert = _a(expert, np.int32)
    T = expert.shape[0]
    slot = np.empty(T, np.int32)
    counts = np.empty(E, np.int32)
    kept = np.empty(E, np.int32)
    tok = np.empty(E * Cap, np.int32)
    lib().orc_route(T, E, Cap, _p(expert), _p(slot), _p(counts), _p(kept), _p(tok))
    return slot, counts, kept, tok.reshape(E, Cap)


def dispatch(x, expert, slot, E: int, Cap: int):
    x = _a(x, np.float32)
    T, h = x.shape
    D = np.empty((E, Cap, h), np.float32)
    lib().orc_dispatch(T, h, E, Cap, _p(x), _p(_a(expert, np.int32)), _p(_a(slot, np.int32)), _p(D))
    return D


def dtd_drop(buf, G: int, r: int):
    """Duplicate token dropping, the drop of rank r in a tensor-parallel group of G (paper Section 5.1):
    buf [E, C, w] -> share [E, ceil(C/G), w] holding rows r, r+G, r+2G, ... of every expert, zero beyond C."""
    buf = _a(buf, np.float32)
    E, Cap, w = buf.shape
    share = np.empty((E, (Cap + G - 1) // G, w), np.float32)
    lib().orc_dtd_drop(E, Cap, w, G, r, _p(buf), _p(share))
    return share


def dtd_gather(shares, Cap: int):
    """The all-gather's result put back in row order: shares [G, E, ceil(C/G), w] -> buf [E, C, w]."""
    shares = _a(shares, np.float32)
    G, E, Cg, w = shares.shape
    assert Cg == (Cap + G - 1) // G
    buf = np.empty((E, Cap, w), np.float32)
    lib().orc_dtd_gather(E, Cap, w, G, _p(shares), _p(buf))
    return buf


def ffn_fwd(D_e, W1_e, W2_e, mode: int = ACT_GELU_ERF):
    """One expert: returns (Z, H, Y) in double for the given rows of D_e."""
    D_e, W1_e, W2_e = _a(D_e, np.float32), _a(W1_e, np.float32), _a(W2_e, np.float32)
    rows, h = D_e.shape
    f = W1_e.shape[1]
    assert W1_e.shape == (h, f) and W2_e.shape[0] == f
    h2 = W2_e.shape[1]
    assert h2 == h
    Z = np.empty((rows, f), np.float64)
    H = np.empty((rows, f), np.float64)
    Y = np.empty((rows, h), np.float64)
    lib().orc_ffn_fwd(rows, h, f, mode, _p(D_e), _p(W1_e), _p(W2_e), _p(Z), _p(H), _p(Y))
    return Z, H, Y


def combine(Y, expert, slot, gate_p):
    Y = _a(Y, np.float64)
    E, Cap, h = Y.shape
    T = len(expert)
    out = np.empty((T, h), np.float64)
    lib().orc_combine(T, h, Cap, _p(Y), _p(_a(expert, np.int32)), _p(_a(slot, np.int32)),
                      _p(_a(gate_p, np.float32)), _p(out))
    return out


def combine_bwd(d_out, Y, expert, slot, gate_p):
    d_out, Y = _a(d_out, np.float32), _a(Y, np.float64)
    E, Cap, h = Y.shape
    T = d_out.shape[0]
    dY = np.empty((E, Cap, h), np.float64)
    dp = np.empty(T, np.float64)
    lib().orc_combine_bwd(T, h, E, Cap, _p(d_out), _p(Y), _p(_a(expert, np.int32)), _p(_a(slot, np.int32)),
                          _p(_a(gate_p, np.float32)), _p(dY), _p(dp))
    return dY, dp


def ffn_bwd(dY_e, D_e, Z_e, H_e, W1_e, W2_e, mode: int = ACT_GELU_ERF):
    """One expert: returns (dD, dW1, dW2, dZ) in double."""
    dY_e, Z_e, H_e = _a(dY_e, np.float64), _a(Z_e, np.float64), _a(H_e, np.float64)
    D_e, W1_e, W2_e = _a(D_e, np.float32), _a(W1_e, np.float32), _a(W2_e, np.float32)
    rows, h = D_e.shape
    f = W1_e.shape[1]
    dD = np.empty((rows, h), np.float64)
    dW1 = np.empty((h, f), np.float64)
    dW2 = np.empty((f, h), np.float64)
    dZ = np.empty((rows, f), np.float64)
    lib().orc_ffn_bwd(rows, h, f, mode, _p(dY_e), _p(D_e), _p(Z_e), _p(H_e), _p(W1_e), _p(W2_e), _p(dD),
                      _p(dW1), _p(dW2), _p(dZ))
    return dD, dW1, dW2, dZ


def dispatch_bwd(dD, expert, slot):
    dD = _a(dD, np.float64)
    E, Cap, h = dD.shape
    T = len(expert)
    dX = np.empty((T, h), np.float64)
    lib().orc_dispatch_bwd(T, h, Cap, _p(dD), _p(_a(expert, np.int32)), _p(_a(slot, np.int32)), _p(dX))
    return dX


def gate_bwd(dp, probs, expert, x, wg):
    dp, probs = _a(dp, np.float64), _a(probs, np.float32)
    x, wg = _a(x, np.float32), _a(wg, np.float32)
    T, h = x.shape
    E = wg.shape[1]
    dL = np.empty((T, E), np.float64)
    dWg = np.empty((h, E), np.float64)
    dXg = np.empty((T, h), np.float64)
    lib().orc_gate_bwd(T, h, E, _p(dp), _p(probs), _p(_a(expert, np.int32)), _p(x), _p(wg), _p(dL), _p(dWg),
                       _p(dXg))
    return dL, dWg, dXg


def adamw_tiled(grad, master, exp_avg, exp_avg_sq, ts: int, lr: float, beta1: float, beta2: float, eps: float,
                weight_decay: float, step: int, grad_mult: float = 1.0, round_bf16: bool = True):
    """One tiled mixed-precision AdamW step (paper Section 4; AdamW per the set-up in Section 6).

    ``grad`` holds the 16-bit gradients as float32 values; ``master``, ``exp_avg``, ``exp_avg_sq``
    are float32 and are NOT modified: the new (master, exp_avg, exp_avg_sq, param, staging_len) are
    returned, staging_len being the number of staging floats the step touched (<= ts).
    """
    grad = _a(grad, np.float32).ravel()
    w = np.array(master, dtype=np.float32).ravel().copy()
    m = np.array(exp_avg, dtype=np.float32).ravel().copy()
    v = np.array(exp_avg_sq, dtype=np.float32).ravel().copy()
    n = grad.size
    assert w.size == n and m.size == n and v.size == n and ts >= 1 and step >= 1
    param = np.empty(n, np.float32)
    staging = np.empty(ts, np.float32)
    hi = C.c_int64(0)
    lib().orc_adamw_tiled(n, ts, lr, beta1, beta2, eps, weight_decay, step, grad_mult, _p(grad), _p(w), _p(m),
                          _p(v), _p(param), 1 if round_bf16 else 0, _p(staging), C.addressof(hi))
    return w, m, v, param, int(hi.value)


def max_threads() -> int:
    return int(lib().orc_max_threads())


def layer_forward(x, wg, w1, w2, Cap: int, mode: int = ACT_GELU_ERF, logits=None, logit_bias=None,
                  experts=None):
    """Whole layer forward.  ``logits`` overrides the gate's linear map (routing given shared
    logits); ``logit_bias`` [E] fp32 is added in fp32 to the stored logits before the top-1 choice.
    ``experts`` restricts the FFN to a subset of expert ids (others' Z/H/Y rows stay zero)."""
    x = _a(x, np.float32)
    T, h = x.shape
    E = wg.shape[1]
    f = w1.shape[-1]
    if logits is None:
        logits = gate_logits(x, wg)
        if logit_bias is not None:
            logits = (logits + _a(logit_bias, np.float32)[None, :]).astype(np.float32)
    logits = _a(logits, np.float32)
    expert, gate_p, probs = top1_softmax(logits)
    slot, counts, kept, tok = route(expert, E, Cap)
    D = dispatch(x, expert, slot, E, Cap)
    Z = np.zeros((E, Cap, f), np.float64)
    H = np.zeros((E, Cap, f), np.float64)
    Y = np.zeros((E, Cap, h), np.float64)
    for e in (range(E) if experts is None else experts):
        k = int(kept[e])
        if k:
            Z[e, :k], H[e, :k], Y[e, :k] = ffn_fwd(D[e, :k], w1[e], w2[e], mode)
    out = combine(Y, expert, slot, gate_p)
    return dict(logits=logits, expert=expert, gate_p=gate_p, probs=probs, slot=slot, counts=counts, kept=kept,
                token_of_slot=tok, D=D, Z=Z, H=H, Y=Y, out=out)


def layer_backward(fw, d_out, x, wg, w1, w2, mode: int = ACT_GELU_ERF, experts=None):
    """Whole layer backward from the forward's saved dict ``fw`` and the upstream gradient."""
    E, Cap, h = fw["Y"].shape
    f = fw["Z"].shape[-1]
    dY, dp = combine_bwd(d_out, fw["Y"], fw["expert"], fw["slot"], fw["gate_p"])
    dD = np.zeros((E, Cap, h), np.float64)
    dZ = np.zeros((E, Cap, f), np.float64)
    dW1 = np.zeros((E, h, f), np.float64)
    dW2 = np.zeros((E, f, h), np.float64)
    for e in (range(E) if experts is None else experts):
        k = int(fw["kept"][e])
        if k:
            dD[e, :k], dW1[e], dW2[e], dZ[e, :k] = ffn_bwd(dY[e, :k], fw["D"][e, :k], fw["Z"][e, :k],
                                                            fw["H"][e, :k], w1[e], w2[e], mode)
    dX_disp = dispatch_bwd(dD, fw["expert"], fw["slot"])
    dL, dWg, dXg = gate_bwd(dp, fw["probs"], fw["expert"], x, wg)
    return dict(dY=dY, dp=dp, dD=dD, dZ=dZ, dW1=dW1, dW2=dW2, dX_dispatch=dX_disp, dL=dL, dWg=dWg, dX_gate=dXg,
                dX=dX_disp + dXg)
