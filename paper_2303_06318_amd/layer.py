"""Buffer owner and call sequencer for one MoE layer on one GPU.

Plumbing only: it allocates the device buffers the C ABI needs (torch tensors) and calls the
entry points in the layer's order (paper Section 3, Figure 3: routing, dispatch, expert FFN,
combine; the reverse for backward).  All arithmetic happens inside the HIP library.
"""
from __future__ import annotations

import torch

from . import moe


class MoeLayer:
    def __init__(self, T, h, E, f, Cap, dtype=moe.MOE_BF16, act=moe.MOE_GELU_ERF, backward=False, device="cuda:0",
                 recompute=False):
        """recompute=True: activation recomputation -- hact and z_save are not held between forward and
        backward (the backward recomputes them into the workspace)."""
        self.shape = moe.make_shape(T, h, E, f, Cap, dtype, act)
        self.T, self.h, self.E, self.f, self.C = T, h, E, f, Cap
        self.backward_enabled = backward
        self.tdtype = torch.bfloat16 if dtype == moe.MOE_BF16 else torch.float32
        dev = torch.device(device)
        self.device = dev
        f32, i32, td = torch.float32, torch.int32, self.tdtype

        def empty(shape, dt):
            return torch.empty(shape, dtype=dt, device=dev)

        self.logits = empty((T, E), f32)
        self.probs = empty((T, E), f32) if backward else None
        self.expert = empty((T,), i32)
        self.gate_p = empty((T,), f32)
        self.slot = empty((T,), i32)
        self.counts = empty((E,), i32)
        self.kept = empty((E,), i32)
        self.token_of_slot = empty((E, Cap), i32)
        self.buf = empty((E, Cap, h), td)
        self.recompute = bool(recompute)
        self.hact = None if recompute else empty((E, Cap, f), td)
        self.z_save = empty((E, Cap, f), td) if backward and not recompute else None
        self.y = empty((E, Cap, h), td)
        self.out = empty((T, h), td)
        nws = moe.moe_workspace_bytes(self.shape, 2 if recompute else (1 if backward else 0))
        if nws == 0:
            raise moe.MoeError(moe.MOE_ERR_UNSUPPORTED, moe.lib().moe_last_error().decode())
        self.ws = torch.empty((nws,), dtype=torch.uint8, device=dev)
        if backward:
            self.d_y = empty((E, Cap, h), td)
            self.d_gate_p = empty((T,), f32)
            self.d_buf = empty((E, Cap, h), td)
            self.d_w1 = empty((E, h, f), td)
            self.d_w2 = empty((E, f, h), td)
            self.d_x = empty((T, h), td)
            self.d_logits = empty((T, E), f32)
            self.d_w_gate = empty((h, E), f32)

    def gate(self, x, w_gate, logit_bias=None, logits_in=None):
        if logits_in is not None:
            self.logits.copy_(logits_in)
            x = None
        moe.moe_gate(self.shape, x, w_gate, logit_bias, self.logits, self.probs, self.expert, self.gate_p, self.slot,
                     self.counts, self.kept, self.token_of_slot, self.ws)

    def forward(self, x, w_gate, w1, w2, logit_bias=None, logits_in=None, fused=False):
        """fused=True: dispatch and combine folded into the expert GEMMs (bf16).  A layer that will run a
        backward still dispatches (the weight gradient reads buf); a forward-only layer gathers from x."""
        self.gate(x, w_gate, logit_bias, logits_in)
        if fused:
            if self.backward_enabled:
                moe.moe_dispatch(self.shape, x, self.token_of_slot, self.buf)
            moe.moe_expert_ffn_fwd_fused(self.shape, None if self.backward_enabled else x,
                                         self.buf if self.backward_enabled else None, self.token_of_slot, self.slot,
                                         self.gate_p, w1, w2, self.kept, self.z_save, self.hact,
                                         self.y if self.backward_enabled else None, self.out, self.ws)
            return self.out
        moe.moe_dispatch(self.shape, x, self.token_of_slot, self.buf)
        moe.moe_expert_ffn_fwd(self.shape, self.buf, w1, w2, self.kept, self.z_save, self.hact, self.y, self.ws)
        moe.moe_combine(self.shape, self.y, self.expert, self.slot, self.gate_p, self.out)
        return self.out

    def backward(self, d_out, x, w_gate, w1, w2, fused=True):
        assert self.backward_enabled
        moe.moe_combine_bwd(self.shape, d_out, self.y, self.token_of_slot, self.slot, self.gate_p, self.d_y,
                            self.d_gate_p)
        if fused:
            # gate backward first (it only needs d_gate_p), so that the token gradient is written once
            moe.moe_gate_bwd(self.shape, self.d_gate_p, self.probs, self.expert, x, w_gate, self.d_logits,
                             self.d_w_gate, None, self.ws)
        moe.moe_expert_ffn_bwd(self.shape, self.d_y, self.buf, self.z_save, self.hact, w1, w2, self.kept, self.d_buf,
                               self.d_w1, self.d_w2, self.ws)
        if fused:
            moe.moe_dispatch_bwd(self.shape, self.d_buf, self.expert, self.slot, self.d_x, self.d_logits, w_gate)
        else:
            moe.moe_dispatch_bwd(self.shape, self.d_buf, self.expert, self.slot, self.d_x)
            moe.moe_gate_bwd(self.shape, self.d_gate_p, self.probs, self.expert, x, w_gate, self.d_logits,
                             self.d_w_gate, self.d_x, self.ws)
        return self.d_x, self.d_w1, self.d_w2, self.d_w_gate
