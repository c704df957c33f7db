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


# ---------------------------------------------------------------- fine-grained comparisons
# One norm over a whole tensor hides a wrong tile or row of a large result (a wrong 256 x 256 tile of a
# 16 x 4096 x 4096 gradient moves the whole-tensor relative error by 0.016).  These helpers apply the
# tolerance to every row and to every 256 x 256 tile, and bound single elements.

def _sq(a):
    a = np.asarray(a, np.float64)
    return a * a


def row_errors(g, o):
    """Relative Frobenius error of every row of a 2-d comparison (rows of norm 0 in the oracle: absolute)."""
    g = np.asarray(g, np.float64).reshape(-1, g.shape[-1])
    o = np.asarray(o, np.float64).reshape(-1, o.shape[-1])
    num = np.sqrt(_sq(g - o).sum(1))
    den = np.sqrt(_sq(o).sum(1))
    return num / np.where(den > 0, den, 1.0)


def tile_errors(g, o, tile=256):
    """Relative Frobenius error of every tile x tile block of the last two dimensions (ragged edges kept)."""
    g = np.asarray(g, np.float64)
    o = np.asarray(o, np.float64)
    lead = int(np.prod(g.shape[:-2])) if g.ndim > 2 else 1
    g = g.reshape(lead, *g.shape[-2:])
    o = o.reshape(lead, *o.shape[-2:])
    R, Cn = g.shape[-2:]
    rb = list(range(0, R, tile)) + [R]
    cb = list(range(0, Cn, tile))
    d2 = _sq(g - o)
    o2 = _sq(o)
    # column blocks by reduceat along the last axis, then row blocks
    d2 = np.add.reduceat(np.add.reduceat(d2, cb, axis=2), rb[:-1], axis=1)
    o2 = np.add.reduceat(np.add.reduceat(o2, cb, axis=2), rb[:-1], axis=1)
    return np.sqrt(d2) / np.where(o2 > 0, np.sqrt(o2), 1.0)


def assert_close_everywhere(name, g, o, t, tile=256, elem_rel=2.0 ** -7, elem_rms=0.03, rows_relative=True):
    """Every row and every tile x tile block within relative Frobenius t, and every element within
    elem_rel * |value| + elem_rms * rms(tensor).  The element bound: bf16 storage rounds the result by up
    to 2^-9 of its value and the bf16 intermediates add an error whose rms was measured at about 3e-3 of
    the tensor's rms; 2^-7 and 0.03 leave a factor of 4 and of 10 (a ten-sigma outlier) over those."""
    g = np.asarray(g, np.float64)
    o = np.asarray(o, np.float64)
    assert g.shape == o.shape, (name, g.shape, o.shape)
    assert np.isfinite(g).all(), name + ": non-finite values"
    if rows_relative:
        re = row_errors(g, o)
    else:
        # rows whose own norm can be far below their rounding error (a row scaled by a dot product whose terms
        # cancel): every row's error against the root-mean-square row norm instead of its own
        g2, o2 = g.reshape(-1, g.shape[-1]), o.reshape(-1, o.shape[-1])
        re = np.sqrt(_sq(g2 - o2).sum(1)) / np.sqrt(_sq(o2).sum(1).mean())
    assert re.max() <= t, "%s: row %d has relative error %.3e (tolerance %.1e)" % (name, int(re.argmax()), re.max(), t)
    if g.ndim >= 2 and g.shape[-1] > tile:
        te = tile_errors(g, o, tile)
        assert te.max() <= t, "%s: tile %s has relative error %.3e (tolerance %.1e)" % (
            name, np.unravel_index(int(te.argmax()), te.shape), te.max(), t)
    o2 = _sq(o).reshape(-1, o.shape[-1]).sum(1)
    live = o2 > 0                       # rows that are zero by definition (dropped tokens) do not dilute the scale
    rms = float(np.sqrt(o2[live].sum() / (live.sum() * o.shape[-1]))) if live.any() else 0.0
    excess = np.abs(g - o) - (elem_rel * np.abs(o) + elem_rms * rms)
    assert excess.max() <= 0, "%s: element %s off by %.3e beyond the bound (value %.3e, tensor rms %.3e)" % (
        name, np.unravel_index(int(excess.argmax()), excess.shape), float(np.abs(g - o).reshape(-1)[int(excess.argmax())]),
        float(o.reshape(-1)[int(excess.argmax())]), rms)
    return float(re.max())
