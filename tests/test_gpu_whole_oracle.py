"""Every workload at its stated size against the WHOLE oracle.  First the benchmarked one (6.7B-base shard,
forward + backward, T=16384 h=4096 E=16 f=4096), element-wise: every output and every saved intermediate is compared per row and per
256 x 256 tile (not by one norm over the tensor), in the launch configuration bench.py times; then the
same comparison for the fused forward (dispatch / combine folded into the GEMMs) with the recomputing
backward.  The oracle pass takes about a minute of host time on the GPU machine's 16 cores."""
import time

import numpy as np
import pytest
import torch

from paper_2303_06318_amd import moe, synth
from gpu_util import DevInputs, assert_close_everywhere, host, kept_rows, make_layer, relfro

pytestmark = [pytest.mark.gpu, pytest.mark.timeout(1500)]


def _progress(msg, t0):
    print("[whole oracle] %s (%.0f s)" % (msg, time.time() - t0), flush=True)


def compare_with_oracle(orc, layer, inp, wl, fw, bw, what, t0):
    t = 2e-2
    kept = fw["kept"]
    worst = {}
    worst["out"] = assert_close_everywhere(what + " out", host(layer.out), fw["out"], t)
    dropped = fw["slot"] < 0
    assert (host(layer.out)[dropped] == 0).all()
    if layer.hact is not None:
        worst["hact"] = assert_close_everywhere(what + " hact", kept_rows(host(layer.hact), kept), kept_rows(fw["H"], kept), t)
        zg = kept_rows(host(layer.z_save), kept)
        worst["z_save"] = assert_close_everywhere(what + " z_save", zg, orc.act_grad_array(kept_rows(fw["Z"], kept)), t)
        del zg
    worst["y"] = assert_close_everywhere(what + " y", kept_rows(host(layer.y), kept), kept_rows(fw["Y"], kept), t)
    _progress(what + ": forward tensors compared", t0)
    worst["d_y"] = assert_close_everywhere(what + " d_y", kept_rows(host(layer.d_y), kept), kept_rows(bw["dY"], kept), t)
    worst["d_buf"] = assert_close_everywhere(what + " d_buf", kept_rows(host(layer.d_buf), kept), kept_rows(bw["dD"], kept), t)
    worst["d_x"] = assert_close_everywhere(what + " d_x", host(layer.d_x), bw["dX"], t)
    # d_gate_p: a dot product over h whose terms cancel, so single values can be smaller than their rounding
    # error: compared as a vector, and element-wise against the rms
    dp = host(layer.d_gate_p)
    assert relfro(dp, bw["dp"]) <= t
    assert np.abs(dp - bw["dp"]).max() <= 0.05 * np.sqrt((bw["dp"] ** 2).mean())
    assert (dp[dropped] == 0).all()
    _progress(what + ": activations' gradients compared", t0)
    for name, key in (("d_w1", "dW1"), ("d_w2", "dW2")):
        g = host(getattr(layer, name))
        for e in range(wl.E):        # per expert: every row and each of its 16 x 16 tiles
            worst[name] = max(worst.get(name, 0.0), assert_close_everywhere("%s %s[%d]" % (what, name, e), g[e], bw[key][e], t))
        del g
    # d_logits[t,:] is d_gate_p[t] times a vector: rows of tokens whose d_gate_p nearly cancels carry no relative accuracy
    assert relfro(host(layer.d_logits), bw["dL"]) <= t
    worst["d_logits"] = assert_close_everywhere(what + " d_logits", host(layer.d_logits), bw["dL"], 0.1, elem_rms=0.05,
                                                rows_relative=False)
    worst["d_w_gate"] = assert_close_everywhere(what + " d_w_gate", host(layer.d_w_gate).T, bw["dWg"].T, t)
    _progress(what + ": weight gradients compared; worst row errors " +
              ", ".join("%s %.2e" % kv for kv in worst.items()), t0)


def test_cfg5_every_row_and_tile_against_the_whole_oracle(orc):
    t0 = time.time()
    wl = synth.WORKLOADS["cfg5_6p7b_tp4_fwdbwd"]
    inp = synth.make_inputs(wl)
    dev = DevInputs(inp)
    _progress("inputs drawn and uploaded", t0)
    layer = make_layer(wl)
    layer.forward(dev.x, dev.wg, dev.w1, dev.w2)
    layer.backward(dev.d_out, dev.x, dev.wg, dev.w1, dev.w2)
    torch.cuda.synchronize()
    g_logits = host(layer.logits)
    # routing: bit-exact given the GPU's logits; everything downstream uses that routing on both sides
    fw = orc.layer_forward(inp.x, inp.wg, inp.w1, inp.w2, wl.C, logits=g_logits)
    _progress("oracle forward done", t0)
    for a, b in ((layer.expert, "expert"), (layer.slot, "slot"), (layer.counts, "counts"), (layer.kept, "kept"),
                 (layer.token_of_slot, "token_of_slot")):
        assert np.array_equal(host(a), fw[b]), b
    assert np.array_equal(kept_rows(host(layer.buf), fw["kept"]), kept_rows(fw["D"], fw["kept"]))
    assert relfro(g_logits, orc.gate_logits(inp.x, inp.wg)) <= 1e-5
    bw = orc.layer_backward(fw, inp.d_out, inp.x, inp.wg, inp.w1, inp.w2)
    _progress("oracle backward done", t0)
    compare_with_oracle(orc, layer, inp, wl, fw, bw, "three-call path", t0)

    # the fused forward (combine folded into GEMM2's epilogue; a training step still dispatches) and the
    # recomputing backward, compared with the oracle directly
    del layer
    torch.cuda.empty_cache()
    alt = make_layer(wl, recompute=True)
    alt.forward(dev.x, dev.wg, dev.w1, dev.w2, fused=True)
    alt.ws.fill_(0xFF)                      # nothing of the forward survives in the workspace
    alt.backward(dev.d_out, dev.x, dev.wg, dev.w1, dev.w2)
    torch.cuda.synchronize()
    assert np.array_equal(host(alt.logits).view(np.uint32), g_logits.view(np.uint32))
    compare_with_oracle(orc, alt, inp, wl, fw, bw, "fused forward + recomputing backward", t0)
    del alt
    torch.cuda.empty_cache()
    # forward-only fused form: rows gathered straight from x, no dispatch buffer, no y
    fwd = make_layer(wl, backward=False)
    fwd.forward(dev.x, dev.wg, dev.w1, dev.w2, fused=True)
    torch.cuda.synchronize()
    assert_close_everywhere("gathered forward out", host(fwd.out), fw["out"], 2e-2)
    assert_close_everywhere("gathered forward hact", kept_rows(host(fwd.hact), fw["kept"]), kept_rows(fw["H"], fw["kept"]), 2e-2)
    _progress("done", t0)


@pytest.mark.parametrize("name", ["cfg2_1p3b_fwd", "cfg3_6p7b_tp4_fwd", "cfg4_skewed_fwd"])
def test_forward_workloads_every_row_and_tile_against_the_whole_oracle(orc, name):
    """The three forward workloads at full size: routing bit-exact, the dispatch copy bitwise, hact / y / out per
    row, per 256 x 256 tile and per element against a full oracle pass (10-15 s of host time each), for the
    three-call path and for the gathered / scattered fused forward."""
    t0 = time.time()
    wl = synth.WORKLOADS[name]
    inp = synth.make_inputs(wl)
    dev = DevInputs(inp)
    layer = make_layer(wl)
    layer.forward(dev.x, dev.wg, dev.w1, dev.w2, logit_bias=dev.bias)
    torch.cuda.synchronize()
    g_logits = host(layer.logits)
    o_logits = orc.gate_logits(inp.x, inp.wg)
    if inp.logit_bias is not None:
        o_logits = (o_logits + inp.logit_bias[None, :]).astype(np.float32)
    assert relfro(g_logits, o_logits) <= 1e-5
    fw = orc.layer_forward(inp.x, inp.wg, inp.w1, inp.w2, wl.C, logits=g_logits)
    _progress(name + ": oracle forward done", t0)
    for a, b in ((layer.expert, "expert"), (layer.slot, "slot"), (layer.counts, "counts"), (layer.kept, "kept"),
                 (layer.token_of_slot, "token_of_slot")):
        assert np.array_equal(host(a), fw[b]), b
    kept = fw["kept"]
    assert np.abs(host(layer.gate_p) - fw["gate_p"]).max() <= 1e-5
    assert np.array_equal(kept_rows(host(layer.buf), kept), kept_rows(fw["D"], kept))
    if wl.zipf_bias:
        assert (fw["slot"] < 0).sum() > wl.T // 4 and (kept == 0).any()
    fused = make_layer(wl)
    fused.forward(dev.x, dev.wg, dev.w1, dev.w2, logit_bias=dev.bias, fused=True)
    torch.cuda.synchronize()
    for what, L in (("three-call path", layer), ("fused forward", fused)):
        assert_close_everywhere("%s %s hact" % (name, what), kept_rows(host(L.hact), kept), kept_rows(fw["H"], kept), 2e-2)
        if L is layer:
            assert_close_everywhere("%s %s y" % (name, what), kept_rows(host(L.y), kept), kept_rows(fw["Y"], kept), 2e-2)
        assert_close_everywhere("%s %s out" % (name, what), host(L.out), fw["out"], 2e-2)
        assert (host(L.out)[fw["slot"] < 0] == 0).all()
    _progress(name + ": done", t0)
