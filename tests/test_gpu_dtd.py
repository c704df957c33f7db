"""Duplicate token dropping (paper Section 5.1), the local halves on one GPU: the drop fused with dispatch,
the expert FFN reading the all-gathered row shares in place, the reassembling copy, the backward's drop and
the dispatch backward from gradient shares.  The G ranks of a tensor-parallel group are played one after the
other on the one GPU (the all-to-all between experts that live on the same GPU, and the all-gather, move
nothing here).  Everything is compared with the oracle's drop / gather and bit for bit with the plain path."""
import numpy as np
import pytest
import torch

from paper_2303_06318_amd import moe, synth
from gpu_util import DevInputs, host, kept_rows, make_layer, relfro, tol

pytestmark = pytest.mark.gpu
W = synth.WORKLOADS

SHAPES = {
    # capacity 196: not a multiple of any G here; several m-tiles and a 9-block tile per expert
    "E16": synth.scaled(W["cfg5_6p7b_tp4_fwdbwd"], T=2500, h=520, f=648, E=16),
    # heavy dropping, empty experts, E above 32 (two expert k-steps in the dispatch backward)
    "E64_skewed": synth.scaled(W["cfg4_skewed_fwd"], T=3000, h=264, f=136, E=64, backward=True),
}


def nan_like(shape):
    return torch.full(shape, float("nan"), dtype=torch.bfloat16, device="cuda")


@pytest.mark.parametrize("G", [2, 3, 4, 8])
@pytest.mark.parametrize("name", list(SHAPES))
def test_duplicate_token_dropping_local_halves(orc, name, G):
    wl = SHAPES[name]
    inp = synth.make_inputs(wl)
    dev = DevInputs(inp)
    ref = make_layer(wl, backward=True)
    ref.forward(dev.x, dev.wg, dev.w1, dev.w2, logit_bias=dev.bias)
    ref.backward(dev.d_out, dev.x, dev.wg, dev.w1, dev.w2)
    torch.cuda.synchronize()
    sh, E, Cap, h, f = ref.shape, wl.E, wl.C, wl.h, wl.f
    Cg = -(-Cap // G)
    kept = host(ref.kept)
    fw = orc.layer_forward(inp.x, inp.wg, inp.w1, inp.w2, Cap, logits=host(ref.logits))
    bw = orc.layer_backward(fw, inp.d_out, inp.x, inp.wg, inp.w1, inp.w2)
    assert np.array_equal(kept, fw["kept"])

    def live(r):          # [E, Cg] mask of share rows that hold a kept row
        j = np.arange(Cg)[None, :]
        return (j * G + r) < kept[:, None]

    # 1. dispatch fused with the drop, one rank after the other
    shares = nan_like((G, E, Cg, h))
    for r in range(G):
        moe.moe_dispatch_dtd(sh, dev.x, ref.token_of_slot, r, G, shares[r])
    torch.cuda.synchronize()
    sh_host = host(shares)
    for r in range(G):
        want = orc.dtd_drop(fw["D"], G, r)
        m = live(r)
        assert np.array_equal(sh_host[r][m], want[m])              # a pure copy: bitwise
        assert np.isnan(sh_host[r][~m]).all()                      # rows of empty slots are not written
    # every kept row of every expert sits in exactly one share
    assert sum(int(live(r).sum()) for r in range(G)) == int(kept.sum())

    # 2. the FFN reading the shares in place: the same bits as the plain path, and the oracle's values
    z2, h2, y2 = nan_like((E, Cap, f)), nan_like((E, Cap, f)), nan_like((E, Cap, h))
    moe.moe_expert_ffn_fwd_dtd(sh, shares, G, dev.w1, dev.w2, ref.kept, z2, h2, y2, ref.ws)
    torch.cuda.synchronize()
    for a, b in ((z2, ref.z_save), (h2, ref.hact), (y2, ref.y)):
        assert np.array_equal(kept_rows(host(a), kept).view(np.uint32), kept_rows(host(b), kept).view(np.uint32))
    t = tol(wl)
    for e in range(E):
        k = int(kept[e])
        if k:
            assert relfro(host(y2)[e, :k], fw["Y"][e, :k]) <= t
            assert relfro(host(h2)[e, :k], fw["H"][e, :k]) <= t

    # 3. the reassembling copy
    buf2 = nan_like((E, Cap, h))
    moe.moe_dtd_gather(sh, shares, ref.kept, G, buf2)
    torch.cuda.synchronize()
    assert np.array_equal(kept_rows(host(buf2), kept), kept_rows(fw["D"], kept))
    assert np.array_equal(kept_rows(host(buf2), kept), kept_rows(orc.dtd_gather(np.nan_to_num(sh_host), Cap), kept))

    # 4. backward: the drop of d_buf, then the dispatch backward from the gathered gradient shares
    d_shares = nan_like((G, E, Cg, h))
    for r in range(G):
        moe.moe_dtd_drop(sh, ref.d_buf, ref.kept, r, G, d_shares[r])
    torch.cuda.synchronize()
    d_host = host(d_shares)
    d_buf = np.nan_to_num(host(ref.d_buf))
    for r in range(G):
        m = live(r)
        assert np.array_equal(d_host[r][m], orc.dtd_drop(d_buf, G, r)[m])           # the GPU's own rows, strided
        assert relfro(d_host[r][m], orc.dtd_drop(bw["dD"].astype(np.float32), G, r)[m]) <= t
        assert np.isnan(d_host[r][~m]).all()
    d_x2 = nan_like((wl.T, h))
    moe.moe_dispatch_bwd_dtd(sh, d_shares, G, ref.expert, ref.slot, d_x2, ref.d_logits, dev.wg)
    torch.cuda.synchronize()
    assert np.array_equal(host(d_x2).view(np.uint32), host(ref.d_x).view(np.uint32))
    assert relfro(host(d_x2), bw["dX"]) <= t
    # without the gate term: a plain gather, rows of dropped tokens zero
    d_x3, d_x4 = nan_like((wl.T, h)), nan_like((wl.T, h))
    moe.moe_dispatch_bwd_dtd(sh, d_shares, G, ref.expert, ref.slot, d_x3)
    moe.moe_dispatch_bwd(sh, ref.d_buf, ref.expert, ref.slot, d_x4)
    torch.cuda.synchronize()
    assert np.array_equal(host(d_x3).view(np.uint32), host(d_x4).view(np.uint32))
    assert relfro(host(d_x3), bw["dX_dispatch"]) <= t
    assert (host(d_x3)[host(ref.slot) < 0] == 0).all()
