"""Seeded synthetic inputs for one MoE layer (tokens, gate weight, expert weights, upstream grad).

This module only draws random numbers and rounds them to the storage type; it
holds none of the layer's arithmetic.  Both the HIP path's tests and the CPU
oracle's tests take their inputs from here so that they see identical arrays.

Draw recipe
-----------
Every tensor is drawn from its own counter-based stream
``Philox(key = seed * 2**32 + tensor_id * 2**16 + chunk)``, where ``chunk`` is
the expert index for per-expert weights and a 0-based 4096-row block index for
token-shaped tensors.  Values are ``standard_normal(float32) * std``.  For the
bf16 workloads the fp32 draw is rounded to the nearest bf16 (ties to even) and
returned both as the uint16 bit pattern (what the GPU stores) and as the fp32
array holding exactly those values (what a CPU checker reads).

The five named workloads follow the shapes of the paper's models (Table 1:
hidden sizes 2048 and 4096, sequence length 2048; the FFN is four times the
hidden size because two thirds of a base model's parameters sit in FFN blocks,
Section 3.1; a tensor-parallel group of 4 for the 6.7B base, Section 7.4).
"""
from __future__ import annotations

import math
from concurrent.futures import ThreadPoolExecutor
from dataclasses import dataclass, field

import numpy as np

TENSOR_X, TENSOR_WG, TENSOR_W1, TENSOR_W2, TENSOR_DOUT = 0, 1, 2, 3, 4
TENSOR_OPT_GRAD, TENSOR_OPT_MASTER, TENSOR_OPT_M, TENSOR_OPT_V = 5, 6, 7, 8
_ROW_BLOCK = 4096


@dataclass(frozen=True)
class Workload:
    name: str
    T: int
    h: int
    E: int
    f: int
    capacity_factor: float
    dtype: str            # "f32" or "bf16" (storage type of x, w1, w2, d_out)
    seed: int
    x_std: float
    w_std: float
    wg_std: float
    zipf_bias: bool = False
    backward: bool = False
    # model sizes when the stored sizes h, f are those sizes rounded up to the library's multiple of 8:
    # columns h_model..h-1 of x / d_out / w2, rows h_model..h-1 of wg / w1, columns f_model..f-1 of w1 and
    # rows f_model..f-1 of w2 are drawn as zeros, which leaves every result of the model-size layer unchanged
    h_model: int = 0
    f_model: int = 0

    @property
    def C(self) -> int:
        return int(math.ceil(float(self.capacity_factor) * float(self.T) / float(self.E)))

    @property
    def hm(self) -> int:
        return self.h_model or self.h

    @property
    def fm(self) -> int:
        return self.f_model or self.f


WORKLOADS = {
    "cfg1_tiny_f32": Workload("cfg1_tiny_f32", 256, 64, 4, 256, 1.0, "f32", 0, 0.02, 0.02, 1.0),
    "cfg2_1p3b_fwd": Workload("cfg2_1p3b_fwd", 8192, 2048, 16, 8192, 1.25, "bf16", 1, 1.0, 0.02, 0.02),
    "cfg3_6p7b_tp4_fwd": Workload("cfg3_6p7b_tp4_fwd", 16384, 4096, 16, 4096, 1.25, "bf16", 2, 1.0, 0.02, 0.02),
    "cfg4_skewed_fwd": Workload("cfg4_skewed_fwd", 16384, 2048, 64, 4096, 1.0, "bf16", 3, 1.0, 0.02, 0.02,
                                zipf_bias=True),
    "cfg5_6p7b_tp4_fwdbwd": Workload("cfg5_6p7b_tp4_fwdbwd", 16384, 4096, 16, 4096, 1.25, "bf16", 4, 1.0, 0.02,
                                     0.02, backward=True),
    # the other two base models of the weak-scaling study (Section 7.4: 16 experts, tensor-parallel degrees 2 and 8;
    # Table 1: hidden sizes 2560 and 5140).  5140 and 4 * 5140 / 8 = 2570 are not multiples of 8: stored zero-padded.
    "cfg6_2p7b_tp2_fwdbwd": Workload("cfg6_2p7b_tp2_fwdbwd", 16384, 2560, 16, 5120, 1.25, "bf16", 5, 1.0, 0.02, 0.02,
                                     backward=True),
    "cfg7_13b_tp8_fwdbwd": Workload("cfg7_13b_tp8_fwdbwd", 16384, 5144, 16, 2576, 1.25, "bf16", 6, 1.0, 0.02, 0.02,
                                    backward=True, h_model=5140, f_model=2570),
}


def round_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """fp32 array -> uint16 bf16 bit patterns, round to nearest, ties to even (finite inputs)."""
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _draw(seed: int, tensor_id: int, chunk: int, shape, std: float) -> np.ndarray:
    key = (int(seed) << 32) + (int(tensor_id) << 16) + int(chunk)
    g = np.random.Generator(np.random.Philox(key=key))
    a = g.standard_normal(shape, dtype=np.float32)
    if std != 1.0:
        a *= np.float32(std)
    return a


def _draw_chunks(seed, tensor_id, n_chunks, chunk_shape_of, std, threads):
    with ThreadPoolExecutor(max_workers=threads) as ex:
        parts = list(ex.map(lambda c: _draw(seed, tensor_id, c, chunk_shape_of(c), std), range(n_chunks)))
    return parts


def _token_tensor(seed, tensor_id, T, h, std, threads):
    n_chunks = (T + _ROW_BLOCK - 1) // _ROW_BLOCK
    parts = _draw_chunks(seed, tensor_id, n_chunks,
                         lambda c: (min(_ROW_BLOCK, T - c * _ROW_BLOCK), h), std, threads)
    return np.concatenate(parts, axis=0) if parts else np.zeros((0, h), np.float32)


def token_blocks(seed: int, tensor_id: int, T: int, h: int, std: float):
    """The blocks of rows that _token_tensor concatenates, one at a time as (first row, fp32 block): for
    token tensors too large to hold twice on the host."""
    for c in range((T + _ROW_BLOCK - 1) // _ROW_BLOCK):
        yield c * _ROW_BLOCK, _draw(seed, tensor_id, c, (min(_ROW_BLOCK, T - c * _ROW_BLOCK), h), std)


@dataclass
class LayerInputs:
    wl: Workload
    # fp32 arrays holding exactly the stored values (bf16-representable for bf16 workloads)
    x: np.ndarray
    wg: np.ndarray
    w1: np.ndarray
    w2: np.ndarray
    d_out: np.ndarray | None
    logit_bias: np.ndarray | None      # [E] fp32 added to the gate logits (skewed workload), else None
    bits: dict = field(default_factory=dict)   # name -> uint16 bf16 patterns (bf16 workloads only)


def zipf_logit_bias(E: int) -> np.ndarray:
    """Per-expert additive logit offset 2*ln(1/(e+1)) for 0-based expert e, in fp32."""
    e = np.arange(E, dtype=np.float64)
    return (2.0 * np.log(1.0 / (e + 1.0))).astype(np.float32)


def make_inputs(wl: Workload, *, experts: int | None = None, threads: int = 8,
                need_bits: bool = True) -> LayerInputs:
    """Draw the layer's inputs.  ``experts`` limits how many experts' weights are drawn
    (the first ``experts`` ones; their values do not depend on the limit)."""
    nE = wl.E if experts is None else int(experts)
    x = _token_tensor(wl.seed, TENSOR_X, wl.T, wl.h, wl.x_std, threads)
    wg = _draw(wl.seed, TENSOR_WG, 0, (wl.h, wl.E), wl.wg_std)
    w1 = np.stack(_draw_chunks(wl.seed, TENSOR_W1, nE, lambda e: (wl.h, wl.f), wl.w_std, threads)) \
        if nE else np.zeros((0, wl.h, wl.f), np.float32)
    w2 = np.stack(_draw_chunks(wl.seed, TENSOR_W2, nE, lambda e: (wl.f, wl.h), wl.w_std, threads)) \
        if nE else np.zeros((0, wl.f, wl.h), np.float32)
    d_out = _token_tensor(wl.seed, TENSOR_DOUT, wl.T, wl.h, 1.0, threads) if wl.backward else None
    if wl.hm < wl.h or wl.fm < wl.f:
        x[:, wl.hm:] = 0
        wg[wl.hm:, :] = 0
        w1[:, wl.hm:, :] = 0
        w1[:, :, wl.fm:] = 0
        w2[:, wl.fm:, :] = 0
        w2[:, :, wl.hm:] = 0
        if d_out is not None:
            d_out[:, wl.hm:] = 0
    bits = {}
    if wl.dtype == "bf16":
        for name in ("x", "w1", "w2", "d_out"):
            a = {"x": x, "w1": w1, "w2": w2, "d_out": d_out}[name]
            if a is None:
                continue
            b = round_to_bf16_bits(a)
            a[...] = bf16_bits_to_f32(b)
            if need_bits:
                bits[name] = b
    bias = zipf_logit_bias(wl.E) if wl.zipf_bias else None
    return LayerInputs(wl, x, wg, w1, w2, d_out, bias, bits)


def scaled(wl: Workload, **kw) -> Workload:
    """A copy of a workload with some fields replaced (used for reduced-size parity cases)."""
    d = dict(wl.__dict__)
    d.update(kw)
    return Workload(**d)


@dataclass
class OptimizerInputs:
    """State of a flat parameter group before an optimizer step (all arrays have n elements)."""
    grad: np.ndarray           # fp32 values of the stored gradients (bf16-representable if dtype is bf16)
    master: np.ndarray         # fp32 master weights
    exp_avg: np.ndarray        # fp32 first moment
    exp_avg_sq: np.ndarray     # fp32 second moment, >= 0
    grad_bits: np.ndarray | None   # uint16 bf16 patterns of grad (bf16 only)


_OPT_BLOCK = 1 << 20


def make_optimizer_inputs(n: int, seed: int, dtype: str = "bf16", *, w_std: float = 0.02, g_std: float = 1e-3,
                          zero_fraction: float = 0.01, threads: int = 8) -> OptimizerInputs:
    """A flat expert-parameter group in mid-training: weights N(0, w_std) like the layer's expert
    weights, gradients N(0, g_std) with a fraction set to exactly zero (columns of an expert whose
    buffer rows were empty), a first moment of the gradients' scale and a second moment that is the
    square of a draw of that scale.  Streams are per 2**20-element block, so a prefix of a larger
    group equals the smaller group."""
    nb = (n + _OPT_BLOCK - 1) // _OPT_BLOCK

    def flat(tid, std):
        parts = _draw_chunks(seed, tid, nb, lambda c: (min(_OPT_BLOCK, n - c * _OPT_BLOCK),), std, threads)
        return np.concatenate(parts) if parts else np.zeros((0,), np.float32)

    grad = flat(TENSOR_OPT_GRAD, g_std)
    master = flat(TENSOR_OPT_MASTER, w_std)
    m = flat(TENSOR_OPT_M, 0.3 * g_std)
    v = flat(TENSOR_OPT_V, g_std)
    np.square(v, out=v)
    if zero_fraction > 0.0 and n:
        period = max(1, int(round(1.0 / zero_fraction)))
        grad[seed % period::period] = 0.0
    bits = None
    if dtype == "bf16":
        bits = round_to_bf16_bits(grad)
        grad = bf16_bits_to_f32(bits)
    return OptimizerInputs(grad, master, m, v, bits)
