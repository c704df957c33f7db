"""Tensors beyond 4 GiB: the token tensor, the expert buffers and their gradients each hold more than 2^32 bytes,
so every kernel that walks them has to address rows with 64-bit arithmetic (and the matrix-core dispatch backward,
which addresses through 32-bit windows, has to step aside for the general kernel).  The expert FFN is left out: one
expert's chunk stays below 2 GiB by the library's own limit, whatever the number of tokens.

Whole tensors of this size are beyond what the oracle holds in fp64, so the oracle is called on samples, re-indexed as
a small layer of its own (token i of the sample = expert i, slot 0): rows chosen at random, the first and last ones,
and the rows around byte offset 2^32 of every tensor.  Routing and the gate's gradients are compared in full."""
import numpy as np
import pytest
import torch

from paper_2303_06318_amd import moe, synth
from paper_2303_06318_amd.layer import MoeLayer
from gpu_util import relfro

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(900)]

T, H, E, F = 540_000, 4096, 8, 8
CAPACITY_FACTOR = 1.0
SEED = 11


def rows_f32(bits, idx):
    return synth.bf16_bits_to_f32(bits[idx])


def dev_rows(t2d, idx):
    """Rows idx of a [rows, h] device tensor as fp32 on the host (bf16 widened exactly)."""
    i = torch.from_numpy(np.asarray(idx, np.int64)).cuda()
    return t2d.index_select(0, i).float().cpu().numpy()


def test_tensors_beyond_4_GiB(orc):
    assert T * H * 2 > 2 ** 32
    C = int(np.ceil(CAPACITY_FACTOR * T / E))
    assert C * H * 2 < 2 ** 31
    # ---- inputs: drawn and uploaded block by block; the host keeps the bf16 bit patterns only
    x_bits = np.empty((T, H), np.uint16)
    x = torch.empty((T, H), dtype=torch.bfloat16, device="cuda")
    for r0, blk in synth.token_blocks(SEED, synth.TENSOR_X, T, H, 1.0):
        b = synth.round_to_bf16_bits(blk)
        x_bits[r0:r0 + len(b)] = b
        x[r0:r0 + len(b)] = torch.from_numpy(b.view(np.int16)).cuda().view(torch.bfloat16)
    wg_h = synth._draw(SEED, synth.TENSOR_WG, 0, (H, E), 0.02)
    wg = torch.from_numpy(wg_h).cuda()
    print("[beyond 4 GiB] inputs uploaded", flush=True)

    L = MoeLayer(T, H, E, F, C, moe.MOE_BF16, moe.MOE_GELU_ERF, backward=True)
    for name in ("buf", "y", "out", "d_y", "d_buf", "d_x"):
        getattr(L, name).view(torch.uint8).fill_(0xFF)            # NaN patterns: a row nobody wrote shows up
    rng = np.random.default_rng(SEED)
    edge = 2 ** 32 // (H * 2)                                      # first row beyond byte offset 2^32
    tok_s = np.unique(np.concatenate([rng.integers(0, T, 1500), np.arange(64), np.arange(T - 64, T),
                                      np.arange(edge - 16, edge + 16)])).astype(np.int64)

    # ---- gate: logits of the sampled tokens against the oracle, routing in full and bit for bit
    L.gate(x, wg)
    torch.cuda.synchronize()
    g_logits = L.logits.cpu().numpy()
    o_logits = orc.gate_logits(rows_f32(x_bits, tok_s), wg_h)
    assert relfro(g_logits[tok_s], o_logits) <= 1e-5
    e, p, P = orc.top1_softmax(g_logits)
    slot, counts, kept, tok = orc.route(e, E, C)
    assert np.array_equal(L.expert.cpu().numpy(), e)
    assert np.array_equal(L.slot.cpu().numpy(), slot)
    assert np.array_equal(L.counts.cpu().numpy(), counts)
    assert np.array_equal(L.kept.cpu().numpy(), kept)
    assert np.array_equal(L.token_of_slot.cpu().numpy(), tok)
    assert np.abs(L.gate_p.cpu().numpy() - p).max() <= 1e-5
    assert np.abs(L.probs.cpu().numpy() - P).max() <= 1e-5
    assert (slot < 0).sum() > 0 and (kept == C).any(), "some experts must overflow at capacity factor 1"
    assert (E - 1) * C + int(kept[E - 1]) > edge, "the last expert's rows must lie beyond byte offset 2^32"
    print("[beyond 4 GiB] gate and routing compared", flush=True)

    # ---- dispatch: a copy, bit for bit, on sampled slots (incl. the last filled one and those around 2^32 bytes)
    moe.moe_dispatch(L.shape, x, L.token_of_slot, L.buf)
    flat_tok = tok.reshape(-1)
    filled = np.flatnonzero(flat_tok >= 0)
    near = filled[(filled >= edge - 16) & (filled < edge + 16)]
    slot_s = np.unique(np.concatenate([rng.choice(filled, 1500), filled[:32], filled[-32:], near])).astype(np.int64)
    buf2d = L.buf.view(E * C, H)
    got = buf2d.index_select(0, torch.from_numpy(slot_s).cuda()).view(torch.int16).cpu().numpy().view(np.uint16)
    assert np.array_equal(got, x_bits[flat_tok[slot_s]])

    # the sample as a layer of its own for the oracle: token i -> expert i, slot 0 (or dropped)
    n = len(tok_s)
    e_s = np.arange(n, dtype=np.int32)
    slot_of = slot[tok_s]
    s_s = np.where(slot_of >= 0, 0, -1).astype(np.int32)
    row_of = np.where(slot_of >= 0, e[tok_s].astype(np.int64) * C + np.maximum(slot_of, 0), 0)   # buffer row of each sampled token
    x_s = rows_f32(x_bits, tok_s)
    Y_s = x_s[:, None, :].astype(np.float64)                        # y := buf, whose rows are the tokens' own x rows

    # ---- combine with y := buf: out[t] = p_t x[t], zero rows for dropped tokens
    moe.moe_combine(L.shape, L.buf, L.expert, L.slot, L.gate_p, L.out)
    o_out = orc.combine(Y_s, e_s, s_s, p[tok_s])
    g_out = dev_rows(L.out, tok_s)
    assert (g_out[slot_of < 0] == 0).all()
    assert (np.abs(g_out - o_out) <= 2.0 ** -8 * np.abs(o_out)).all()

    # ---- combine backward with d_out := x, y := buf
    moe.moe_combine_bwd(L.shape, x, L.buf, L.token_of_slot, L.slot, L.gate_p, L.d_y, L.d_gate_p)
    o_dY, o_dp = orc.combine_bwd(x_s, Y_s, e_s, s_s, p[tok_s])
    g_dp = L.d_gate_p.cpu().numpy()
    assert (g_dp[slot < 0] == 0).all()
    assert np.abs(g_dp[tok_s] - o_dp).max() <= 1e-4 * np.abs(o_dp).max()
    keep_s = slot_of >= 0
    g_dY = dev_rows(L.d_y.view(E * C, H), row_of[keep_s])
    assert (np.abs(g_dY - o_dY[keep_s, 0]) <= 2.0 ** -8 * np.abs(o_dY[keep_s, 0])).all()
    print("[beyond 4 GiB] dispatch, combine and combine backward compared", flush=True)

    # ---- dispatch backward alone (d_buf := d_y): a copy, zero rows for dropped tokens
    moe.moe_dispatch_bwd(L.shape, L.d_y, L.expert, L.slot, L.d_x)
    g_dx = dev_rows(L.d_x, tok_s)
    assert (g_dx[~keep_s] == 0).all()
    assert np.array_equal(g_dx[keep_s], g_dY)

    # ---- gate backward: d_logits and d_w_gate in full, the oracle taking the tokens in chunks (its d_w_gate is
    # a sum over tokens)
    moe.moe_gate_bwd(L.shape, L.d_gate_p, L.probs, L.expert, x, wg, L.d_logits, L.d_w_gate, None, L.ws)
    torch.cuda.synchronize()
    g_dL, g_dWg = L.d_logits.cpu().numpy(), L.d_w_gate.cpu().numpy()
    g_P = L.probs.cpu().numpy()
    o_dWg = np.zeros((H, E))
    o_dL = np.empty((T, E))
    step = 30_000
    for t0 in range(0, T, step):
        sl = slice(t0, min(T, t0 + step))
        dl, dwg, _ = orc.gate_bwd(g_dp[sl], g_P[sl], e[sl], rows_f32(x_bits, sl), wg_h)
        o_dL[sl] = dl
        o_dWg += dwg
    assert relfro(g_dL, o_dL) <= 1e-5
    assert relfro(g_dWg, o_dWg) <= 2e-2
    print("[beyond 4 GiB] gate backward compared", flush=True)

    # ---- dispatch backward with the gate term folded in (the general kernel: x spans more than 2 GiB)
    d_x2 = torch.full((T, H), float("nan"), dtype=torch.bfloat16, device="cuda")
    moe.moe_dispatch_bwd(L.shape, L.d_y, L.expert, L.slot, d_x2, L.d_logits, wg)
    _, _, o_dXg = orc.gate_bwd(g_dp[tok_s], g_P[tok_s], e[tok_s], x_s, wg_h)
    want = o_dXg + np.where(keep_s[:, None], g_dx, 0.0)
    g2 = dev_rows(d_x2, tok_s)
    assert np.isfinite(g2).all()
    err = np.linalg.norm(g2 - want, axis=1) / np.maximum(np.linalg.norm(want, axis=1), 1e-30)
    scale = np.sqrt((want ** 2).sum(1).mean())
    assert (np.linalg.norm(g2 - want, axis=1) <= 2e-2 * np.maximum(np.linalg.norm(want, axis=1), 0.05 * scale)).all(), err.max()
    print("[beyond 4 GiB] done", flush=True)
