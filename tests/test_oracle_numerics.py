"""Pins for the oracle's floating point parts: GeLU, softmax, the matmuls, dispatch/combine,
the whole layer against a dense one-hot formulation in torch fp64, and the backward against
autograd and finite differences.  No GPU, no GPU library."""
import math
import os

import numpy as np
import pytest
import torch

from paper_2303_06318_amd import synth

GOLD = os.path.join(os.path.dirname(__file__), "golden")


def relerr(a, b):
    a, b = np.asarray(a, np.float64), np.asarray(b, np.float64)
    d = np.linalg.norm(b)
    return np.linalg.norm(a - b) / (d if d > 0 else 1.0)


# ---------------------------------------------------------------- GeLU
@pytest.mark.parametrize("x", [-8.0, -3.0, -1.0, -0.3, 0.0, 0.2, 1.0, 2.5, 9.0])
def test_gelu_closed_forms(orc, x):
    erf_form = 0.5 * x * (1.0 + math.erf(x / math.sqrt(2.0)))
    assert abs(orc.act(x, orc.ACT_GELU_ERF) - erf_form) < 1e-15
    xt = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    for mode, approx in ((orc.ACT_GELU_ERF, "none"), (orc.ACT_GELU_TANH, "tanh")):
        y = torch.nn.functional.gelu(xt, approximate=approx)
        (g,) = torch.autograd.grad(y, xt)
        assert abs(orc.act(x, mode) - y.item()) < 1e-14
        assert abs(orc.act_grad(x, mode) - g.item()) < 1e-13


def test_gelu_limits(orc):
    assert orc.act(0.0) == 0.0
    assert abs(orc.act(30.0) - 30.0) < 1e-12 and abs(orc.act(-30.0)) < 1e-12
    assert abs(orc.act_grad(0.0) - 0.5) < 1e-15
    # derivative agrees with a central difference
    for x in (-2.0, -0.5, 0.7, 3.0):
        for mode in (0, 1):
            fd = (orc.act(x + 1e-6, mode) - orc.act(x - 1e-6, mode)) / 2e-6
            assert abs(fd - orc.act_grad(x, mode)) < 1e-8


def test_gelu_derivative_array_against_autograd_and_differences(orc):
    """The array form of act' (the checker of the z_save the GPU keeps for the backward): against the
    library's GeLU differentiated by autograd in fp64, against central differences of the oracle's own
    forward, and against the closed form with math.erf -- over a ragged 3-d array, so that a wrong
    length, stride or mode argument shows."""
    rng = np.random.default_rng(11)
    z = np.concatenate([rng.standard_normal(997) * 2.5, [-9.0, -1e-3, 0.0, 1e-3, 9.0, 30.0, -30.0]]).reshape(4, 251)
    for mode, approx in ((orc.ACT_GELU_ERF, "none"), (orc.ACT_GELU_TANH, "tanh")):
        g = orc.act_grad_array(z, mode)
        assert g.shape == z.shape and g.dtype == np.float64
        zt = torch.from_numpy(z.copy()).requires_grad_(True)
        (ref,) = torch.autograd.grad(torch.nn.functional.gelu(zt, approximate=approx).sum(), zt)
        assert np.abs(g - ref.numpy()).max() < 1e-13
        fd = np.array([(orc.act(v + 1e-6, mode) - orc.act(v - 1e-6, mode)) / 2e-6 for v in z.ravel()]).reshape(z.shape)
        assert np.abs(g - fd).max() < 1e-8
    closed = np.array([0.5 * (1.0 + math.erf(v / math.sqrt(2.0))) + v * math.exp(-0.5 * v * v) / math.sqrt(2.0 * math.pi)
                       for v in z.ravel()]).reshape(z.shape)
    assert np.abs(orc.act_grad_array(z, orc.ACT_GELU_ERF) - closed).max() < 1e-15
    # the two forms differ (by up to a few 1e-4 near |z| = 2): a swapped mode argument cannot pass both
    assert np.abs(orc.act_grad_array(z, 0) - orc.act_grad_array(z, 1)).max() > 1e-4
    assert orc.act_grad_array(np.zeros((0,)), 0).shape == (0,)


# ---------------------------------------------------------------- softmax / logits
def test_softmax_against_library_and_invariants(orc):
    rng = np.random.default_rng(0)
    L = (rng.standard_normal((300, 16)) * 3).astype(np.float32)
    e, p, P = orc.top1_softmax(L)
    ref = torch.softmax(torch.from_numpy(L).double(), dim=1).numpy()
    assert np.abs(P - ref).max() < 1e-7
    assert np.abs(P.astype(np.float64).sum(1) - 1).max() < 1e-6
    assert np.array_equal(e, ref.argmax(1))
    assert np.abs(p - ref.max(1)).max() < 1e-7
    assert (p >= 1.0 / 16 - 1e-7).all()
    # shift invariance (exact power-of-two shift keeps fp32 differences exact)
    e2, p2, P2 = orc.top1_softmax((L + np.float32(4.0)).astype(np.float32))
    assert np.array_equal(e, e2)
    assert np.abs(P2 - P).max() < 1e-5


def test_gate_logits_against_library_matmul(orc):
    rng = np.random.default_rng(1)
    x = rng.standard_normal((70, 96)).astype(np.float32)
    wg = rng.standard_normal((96, 5)).astype(np.float32)
    L = orc.gate_logits(x, wg)
    ref = (torch.from_numpy(x).double() @ torch.from_numpy(wg).double()).numpy()
    assert np.abs(L - ref).max() <= 1e-6 * np.abs(ref).max()
    # not transposed: a one-hot x row picks a row of wg
    x1 = np.zeros((1, 96), np.float32)
    x1[0, 7] = 1
    assert np.array_equal(orc.gate_logits(x1, wg)[0], wg[7])


# ---------------------------------------------------------------- FFN
def test_ffn_special_case_dense_mlp(orc):
    """E = 1, capacity >= T and a zero gate weight make the layer a plain two-layer MLP on all
    tokens in order with p = 1: compare with torch fp64 matmul + gelu."""
    rng = np.random.default_rng(2)
    T, h, f = 37, 24, 40
    x = rng.standard_normal((T, h)).astype(np.float32)
    w1 = (rng.standard_normal((1, h, f)) * 0.3).astype(np.float32)
    w2 = (rng.standard_normal((1, f, h)) * 0.3).astype(np.float32)
    wg = np.zeros((h, 1), np.float32)
    for mode, approx in ((orc.ACT_GELU_ERF, "none"), (orc.ACT_GELU_TANH, "tanh")):
        fw = orc.layer_forward(x, wg, w1, w2, orc.capacity(T, 1, 1.0), mode)
        assert (fw["gate_p"] == 1.0).all() and fw["slot"].tolist() == list(range(T))
        xd = torch.from_numpy(x).double()
        ref = torch.nn.functional.gelu(xd @ torch.from_numpy(w1[0]).double(), approximate=approx) \
            @ torch.from_numpy(w2[0]).double()
        assert relerr(fw["out"], ref.numpy()) < 1e-14


def test_ffn_not_transposed(orc):
    """Rectangular shapes with one-hot inputs: a transposed or mis-strided weight read would
    pick the wrong entries."""
    h, f = 3, 5
    w1 = np.arange(h * f, dtype=np.float32).reshape(h, f) / 10
    w2 = (np.arange(f * h, dtype=np.float32).reshape(f, h) - 7) / 10
    D = np.zeros((1, h), np.float32)
    D[0, 2] = 1.0
    Z, H, Y = orc.ffn_fwd(D, w1, w2)
    assert np.allclose(Z[0], w1[2])
    Hd = np.array([orc.act(float(v)) for v in w1[2]])
    assert np.allclose(H[0], Hd)
    assert np.allclose(Y[0], Hd @ w2.astype(np.float64))


# ---------------------------------------------------------------- dispatch / combine
def test_dispatch_combine_round_trip(orc):
    rng = np.random.default_rng(3)
    T, h, E = 200, 16, 4
    Cap = orc.capacity(T, E, 0.8)
    x = rng.standard_normal((T, h)).astype(np.float32)
    expert = rng.integers(0, E, T).astype(np.int32)
    slot, counts, kept, tok = orc.route(expert, E, Cap)
    assert (slot < 0).any()
    D = orc.dispatch(x, expert, slot, E, Cap)
    # pure copy, bitwise; unfilled rows are zero
    for e in range(E):
        assert np.array_equal(D[e, :kept[e]], x[tok[e, :kept[e]]])
        assert (D[e, kept[e]:] == 0).all()
    # identity FFN (Y := D) and p = 1: combine returns the token itself, dropped tokens give exactly zero
    out = orc.combine(D.astype(np.float64), expert, slot, np.ones(T, np.float32))
    keep = slot >= 0
    assert np.array_equal(out[keep], x[keep].astype(np.float64))
    assert (out[~keep] == 0).all()
    p = rng.random(T).astype(np.float32)
    out = orc.combine(D.astype(np.float64), expert, slot, p)
    assert np.array_equal(out[keep], p[keep, None].astype(np.float64) * x[keep].astype(np.float64))


# ---------------------------------------------------------------- whole layer vs dense one-hot formulation
def dense_onehot_layer(x, wg, w1, w2, Cap, approx="none", logit_bias=None):
    """Independent formulation in torch fp64: one-hot masks, cumsum positions, einsum dispatch."""
    xd = torch.tensor(x, dtype=torch.float64, requires_grad=True)
    wgd = torch.tensor(wg, dtype=torch.float64, requires_grad=True)
    w1d = torch.tensor(w1, dtype=torch.float64, requires_grad=True)
    w2d = torch.tensor(w2, dtype=torch.float64, requires_grad=True)
    logits = xd @ wgd
    if logit_bias is not None:
        logits = logits + torch.tensor(logit_bias, dtype=torch.float64)
    T, E = logits.shape
    l32 = logits.detach().float()
    e = torch.argmax(l32, dim=1)
    mask = torch.nn.functional.one_hot(e, E).to(torch.int64)
    pos = torch.cumsum(mask, 0) - 1
    keep = (pos < Cap) & (mask > 0)
    disp = (keep[:, :, None] & (pos[:, :, None] == torch.arange(Cap)[None, None, :])).double()   # [T,E,C]
    probs = torch.softmax(logits, dim=1)
    gate = (probs * mask.double()).sum(1)
    D = torch.einsum("tec,th->ech", disp, xd)
    Z = torch.einsum("ech,ehf->ecf", D, w1d)
    H = torch.nn.functional.gelu(Z, approximate=approx)
    Y = torch.einsum("ecf,efh->ech", H, w2d)
    out = torch.einsum("tec,ech->th", disp * gate[:, None, None], Y)
    return out, (xd, wgd, w1d, w2d), dict(expert=e.numpy(), keep=keep.any(1).numpy(), probs=probs, Y=Y)


def small_case(seed, T=96, h=20, E=4, f=28, cf=0.75, x_std=1.0, w_std=0.3):
    rng = np.random.default_rng(seed)
    x = (rng.standard_normal((T, h)) * x_std).astype(np.float32)
    wg = (rng.standard_normal((h, E)) * 0.5).astype(np.float32)
    w1 = (rng.standard_normal((E, h, f)) * w_std).astype(np.float32)
    w2 = (rng.standard_normal((E, f, h)) * w_std).astype(np.float32)
    d_out = rng.standard_normal((T, h)).astype(np.float32)
    return x, wg, w1, w2, d_out


@pytest.mark.parametrize("mode,approx", [(0, "none"), (1, "tanh")])
def test_layer_forward_against_dense_onehot(orc, mode, approx):
    x, wg, w1, w2, d_out = small_case(10)
    T, E = x.shape[0], wg.shape[1]
    Cap = orc.capacity(T, E, 0.75)
    fw = orc.layer_forward(x, wg, w1, w2, Cap, mode)
    out, _, aux = dense_onehot_layer(x, wg, w1, w2, Cap, approx)
    assert np.array_equal(fw["expert"], aux["expert"])
    assert np.array_equal(fw["slot"] >= 0, aux["keep"])
    assert (fw["slot"] < 0).any(), "case must exercise drops"
    assert relerr(fw["out"], out.detach().numpy()) < 1e-7    # p is rounded to fp32 in the oracle
    assert (fw["out"][fw["slot"] < 0] == 0).all()


def test_layer_forward_with_logit_bias(orc):
    x, wg, w1, w2, d_out = small_case(11, E=8, cf=1.0)
    bias = synth.zipf_logit_bias(8)
    assert np.allclose(bias, [-2 * math.log(e + 1) for e in range(8)], atol=1e-6)
    Cap = orc.capacity(x.shape[0], 8, 1.0)
    fw = orc.layer_forward(x, wg, w1, w2, Cap, 0, logit_bias=bias)
    out, _, aux = dense_onehot_layer(x, wg, w1, w2, Cap, "none", logit_bias=bias)
    assert np.array_equal(fw["expert"], aux["expert"])
    assert relerr(fw["out"], out.detach().numpy()) < 1e-7
    assert fw["counts"][0] > Cap      # the favoured expert overflows


@pytest.mark.parametrize("mode,approx", [(0, "none"), (1, "tanh")])
def test_layer_backward_against_autograd(orc, mode, approx):
    x, wg, w1, w2, d_out = small_case(12)
    T, E = x.shape[0], wg.shape[1]
    Cap = orc.capacity(T, E, 0.75)
    fw = orc.layer_forward(x, wg, w1, w2, Cap, mode)
    bw = orc.layer_backward(fw, d_out, x, wg, w1, w2, mode)
    out, (xd, wgd, w1d, w2d), aux = dense_onehot_layer(x, wg, w1, w2, Cap, approx)
    out.backward(torch.tensor(d_out, dtype=torch.float64))
    # the oracle rounds p and P to fp32 once; everything else is double
    assert relerr(bw["dW1"], w1d.grad.numpy()) < 1e-6
    assert relerr(bw["dW2"], w2d.grad.numpy()) < 1e-6
    assert relerr(bw["dWg"], wgd.grad.numpy()) < 1e-6
    assert relerr(bw["dX"], xd.grad.numpy()) < 1e-6
    drop = fw["slot"] < 0
    assert (bw["dX_dispatch"][drop] == 0).all() and (bw["dp"][drop] == 0).all()
    assert (bw["dL"][drop] == 0).all()


def test_layer_backward_finite_differences(orc):
    """Central differences in double on the oracle's own forward, away from argmax ties.
    Catches a wrong sign / missing term independent of torch."""
    x, wg, w1, w2, d_out = small_case(13, T=24, h=6, E=3, f=7, cf=1.0)
    T, E = x.shape[0], wg.shape[1]
    Cap = orc.capacity(T, E, 1.0)
    fw = orc.layer_forward(x, wg, w1, w2, Cap, 0)
    srt = np.sort(fw["logits"], axis=1)
    assert (srt[:, -1] - srt[:, -2]).min() > 1e-3
    bw = orc.layer_backward(fw, d_out, x, wg, w1, w2, 0)

    def loss(xx, wgg, w11, w22):
        # fp64 forward written directly (no fp32 rounding), routing frozen from fw
        L = xx @ wgg
        P = np.exp(L - L.max(1, keepdims=True))
        P /= P.sum(1, keepdims=True)
        tot = 0.0
        for t in range(T):
            if fw["slot"][t] < 0:
                continue
            e = fw["expert"][t]
            z = xx[t] @ w11[e]
            hh = np.array([orc.act(float(v)) for v in z])
            tot += P[t, e] * float((hh @ w22[e]) @ d_out[t].astype(np.float64))
        return tot

    args = [a.astype(np.float64) for a in (x, wg, w1, w2)]
    grads = [bw["dX"], bw["dWg"], bw["dW1"], bw["dW2"]]
    rng = np.random.default_rng(5)
    eps = 1e-5
    for ai, (a, g) in enumerate(zip(args, grads)):
        for _ in range(6):
            idx = tuple(int(rng.integers(0, s)) for s in a.shape)
            ap, am = [v.copy() for v in args], [v.copy() for v in args]
            ap[ai][idx] += eps
            am[ai][idx] -= eps
            fd = (loss(*ap) - loss(*am)) / (2 * eps)
            assert abs(fd - g[idx]) <= 2e-5 * max(1.0, abs(fd)), (ai, idx, fd, g[idx])


def test_backward_linear_in_upstream_grad(orc):
    x, wg, w1, w2, d_out = small_case(14)
    Cap = orc.capacity(x.shape[0], wg.shape[1], 0.75)
    fw = orc.layer_forward(x, wg, w1, w2, Cap, 0)
    b1 = orc.layer_backward(fw, d_out, x, wg, w1, w2, 0)
    b2 = orc.layer_backward(fw, (2 * d_out).astype(np.float32), x, wg, w1, w2, 0)
    for k in ("dX", "dW1", "dW2", "dWg"):
        assert relerr(b2[k], 2 * b1[k]) < 1e-14


# ---------------------------------------------------------------- workload shapes and generator
def test_model_shape_closed_forms():
    """Section 3.1, Eq. 2 + Eq. 3: total = (E+2)/3 * NP_base must give the totals the paper prints,
    and an FFN of width 4h holds two thirds of a layer's 12 h^2 parameters."""
    with open(os.path.join(GOLD, "model_shapes.txt")) as fh:
        rows = [l.split() for l in fh if l.strip() and not l.startswith("#")]
    for base, E, total, layers, hidden in rows:
        base, E, total, layers, hidden = float(base), int(E), float(total), int(layers), int(hidden)
        assert abs((E + 2) / 3 * base - total) / total < 0.02
        ffn = 2 * hidden * (4 * hidden)
        assert abs(ffn / (12 * hidden * hidden) - 2 / 3) < 1e-12
        assert abs(12 * hidden * hidden * layers / 1e9 - base) / base < 0.1
    w3 = synth.WORKLOADS["cfg3_6p7b_tp4_fwd"]
    assert w3.h == 4096 and w3.f == 4 * 4096 // 4 and w3.C == 1280
    w2 = synth.WORKLOADS["cfg2_1p3b_fwd"]
    assert w2.h == 2048 and w2.f == 4 * 2048 and w2.C == 640
    assert synth.WORKLOADS["cfg4_skewed_fwd"].C == 256 and synth.WORKLOADS["cfg1_tiny_f32"].C == 64


def test_synth_generator_is_seeded_and_bf16_exact():
    wl = synth.scaled(synth.WORKLOADS["cfg5_6p7b_tp4_fwdbwd"], T=300, h=64, f=96, E=3)
    a, b = synth.make_inputs(wl), synth.make_inputs(wl)
    for n in ("x", "wg", "w1", "w2", "d_out"):
        assert np.array_equal(getattr(a, n), getattr(b, n))
    # stored values are exactly bf16-representable and equal the bit patterns
    for n in ("x", "w1", "w2", "d_out"):
        v = getattr(a, n)
        assert np.array_equal(synth.bf16_bits_to_f32(a.bits[n]), v)
        assert (v.view(np.uint32) & 0xFFFF == 0).all()
    assert abs(a.x.std() - 1.0) < 0.05 and abs(a.w1.std() - 0.02) < 0.002
    # round-to-nearest-even on known patterns
    vals = np.array([1.0, 1.00390625, 1.005859375, 1.01171875], np.float32)   # 1, 1+2^-8 (tie), 1+1.5*2^-8, 1+3*2^-8
    bits = synth.round_to_bf16_bits(vals)
    assert synth.bf16_bits_to_f32(bits).tolist() == [1.0, 1.0, 1.0078125, 1.015625]
    # per-expert streams do not depend on how many experts are drawn
    c = synth.make_inputs(wl, experts=1)
    assert np.array_equal(c.w1[0], a.w1[0])


def test_zero_padding_of_h_and_f_changes_nothing(orc):
    """A model whose sizes are not multiples of 8 (13B base: h = 5140, f = 2570) is stored zero-padded; the padded
    layer must give the model-size layer's results in the model's columns and zeros in the padding."""
    hm, fm, E, T = 20, 10, 3, 64
    wl = synth.Workload("pad", T, 24, E, 16, 1.0, "f32", 9, 1.0, 0.3, 0.5, backward=True, h_model=hm, f_model=fm)
    a = synth.make_inputs(wl)
    assert not a.x[:, hm:].any() and not a.w1[:, hm:, :].any() and not a.w1[:, :, fm:].any()
    assert not a.w2[:, fm:, :].any() and not a.w2[:, :, hm:].any() and not a.wg[hm:].any() and not a.d_out[:, hm:].any()
    fw_p = orc.layer_forward(a.x, a.wg, a.w1, a.w2, wl.C)
    bw_p = orc.layer_backward(fw_p, a.d_out, a.x, a.wg, a.w1, a.w2)
    c = np.ascontiguousarray
    x, wg, w1, w2, do = c(a.x[:, :hm]), c(a.wg[:hm]), c(a.w1[:, :hm, :fm]), c(a.w2[:, :fm, :hm]), c(a.d_out[:, :hm])
    fw = orc.layer_forward(x, wg, w1, w2, wl.C)
    bw = orc.layer_backward(fw, do, x, wg, w1, w2)
    assert np.array_equal(fw["expert"], fw_p["expert"]) and np.array_equal(fw["slot"], fw_p["slot"])
    assert np.allclose(fw_p["out"][:, :hm], fw["out"], rtol=1e-12, atol=1e-300) and not fw_p["out"][:, hm:].any()
    assert np.allclose(bw_p["dX"][:, :hm], bw["dX"], rtol=1e-12, atol=1e-300) and not bw_p["dX"][:, hm:].any()
    assert np.allclose(bw_p["dW1"][:, :hm, :fm], bw["dW1"], rtol=1e-12, atol=1e-300)
    assert np.allclose(bw_p["dW2"][:, :fm, :hm], bw["dW2"], rtol=1e-12, atol=1e-300)
    assert np.allclose(bw_p["dWg"][:hm], bw["dWg"], rtol=1e-12, atol=1e-300)
    # every padded weight entry has a zero gradient (GeLU(0) = 0 and W2's padded rows are zero), so the padding
    # stays zero under training
    assert not bw_p["dW1"][:, hm:, :].any() and not bw_p["dW1"][:, :, fm:].any()
    assert not bw_p["dW2"][:, :, hm:].any() and not bw_p["dW2"][:, fm:, :].any() and not bw_p["dWg"][hm:].any()
