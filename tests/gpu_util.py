"""Helpers shared by the GPU parity tests: upload seeded inputs, run the HIP layer, error metrics."""
from __future__ import annotations

import numpy as np
import torch

from paper_2303_06318_amd import moe, synth
from paper_2303_06318_amd.layer import MoeLayer


def relfro(a, b) -> float:
    a = np.asarray(a, np.float64)
    b = np.asarray(b, np.float64)
    d = np.linalg.norm(b)
    return float(np.linalg.norm(a - b) / (d if d > 0 else 1.0))


def to_dev(inp: synth.LayerInputs, name: str):
    """Upload one input tensor in its storage type."""
    a = getattr(inp, name)
    if a is None:
        return None
    if inp.wl.dtype == "bf16" and name in inp.bits:
        return torch.from_numpy(inp.bits[name].view(np.int16)).cuda().view(torch.bfloat16)
    return torch.from_numpy(np.ascontiguousarray(a)).cuda()


def host(t) -> np.ndarray:
    """Device tensor -> fp32/int numpy array (bf16 is widened exactly)."""
    if t.dtype == torch.bfloat16:
        return t.float().cpu().numpy()
    return t.cpu().numpy()


class DevInputs:
    def __init__(self, inp: synth.LayerInputs):
        self.x = to_dev(inp, "x")
        self.wg = torch.from_numpy(inp.wg).cuda()
        self.w1 = to_dev(inp, "w1")
        self.w2 = to_dev(inp, "w2")
        self.d_out = to_dev(inp, "d_out")
        self.bias = None if inp.logit_bias is None else torch.from_numpy(inp.logit_bias).cuda()


def make_layer(wl: synth.Workload, backward=None, act=moe.MOE_GELU_ERF, **modes) -> MoeLayer:
    dt = moe.MOE_BF16 if wl.dtype == "bf16" else moe.MOE_F32
    bw = wl.backward if backward is None else backward
    layer = MoeLayer(wl.T, wl.h, wl.E, wl.f, wl.C, dt, act, backward=bw, **modes)
    poison(layer)
    return layer


def poison(layer: MoeLayer) -> None:
    """Fill every intermediate buffer and the workspace with NaN bit patterns (all bytes 0xFF), so that a
    kernel that read a row nobody wrote (a slot beyond kept[e]) would show up as NaN in the results."""
    for name in ("buf", "hact", "z_save", "y", "d_y", "d_buf", "ws", "out", "d_x", "d_w1", "d_w2"):
        t = getattr(layer, name, None)
        if t is not None:
            t.view(torch.uint8).fill_(0xFF)


def kept_rows(a: np.ndarray, kept) -> np.ndarray:
    """Rows [0, kept[e]) of every expert of an [E, C, ...] array, concatenated."""
    return np.concatenate([a[e, :int(k)] for e, k in enumerate(kept)], axis=0)


def tol(wl: synth.Workload) -> float:
    """Relative Frobenius tolerance: 2e-2 for bf16 storage with fp32 accumulation, 1e-5 for fp32."""
    return 2e-2 if wl.dtype == "bf16" else 1e-5
