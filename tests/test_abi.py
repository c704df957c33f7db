"""Host-side checks of the C-ABI library that need no GPU: it loads, exports every symbol the
header declares, and rejects bad arguments before launching anything."""
import ctypes as C
import os
import re

import pytest

from paper_2303_06318_amd import moe

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "moe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(moe_[a-z0-9_]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = moe.lib()
    names = declared_functions()
    assert len(names) >= 13
    for n in names:
        assert hasattr(L, n), n
    assert sorted(moe.EXPORTS) == names
    # the binding offers the same names
    for n in names:
        if n not in ("moe_status_string", "moe_last_error"):
            assert hasattr(moe, n), n


def test_capacity_and_workspace_are_pure_host_functions():
    assert moe.moe_capacity(16384, 16, 1.25) == 1280
    assert moe.moe_capacity(256, 4, 1.0) == 64
    assert moe.moe_capacity(10, 3, 1.0) == 4
    assert moe.moe_capacity(0, 3, 1.0) == 0 and moe.moe_capacity(10, 0, 1.0) == 0
    sh = moe.make_shape(16384, 4096, 16, 4096, 1280)
    fw, bw = moe.moe_workspace_bytes(sh, False), moe.moe_workspace_bytes(sh, True)
    assert 0 < fw < bw
    assert bw >= 16 * 1280 * 4096 * 2


@pytest.mark.parametrize("kw,status", [
    (dict(T=0), moe.MOE_ERR_INVALID_ARG),
    (dict(E=0), moe.MOE_ERR_INVALID_ARG),
    (dict(Cap=-1), moe.MOE_ERR_INVALID_ARG),
    (dict(h=4100), moe.MOE_ERR_UNSUPPORTED),      # not a multiple of 8 for bf16
    (dict(E=257), moe.MOE_ERR_UNSUPPORTED),
    (dict(dtype=7), moe.MOE_ERR_UNSUPPORTED),
    (dict(act=9), moe.MOE_ERR_UNSUPPORTED),
    # beyond the 32-bit windows the kernels address through: a token tensor of 2^37 bytes, a row of 2^21 elements,
    # an expert chunk of 2 GiB, an expert weight matrix of 2 GiB
    (dict(T=1 << 24, h=4096), moe.MOE_ERR_UNSUPPORTED),
    (dict(h=1 << 21, f=8), moe.MOE_ERR_UNSUPPORTED),
    (dict(Cap=1 << 22, h=256), moe.MOE_ERR_UNSUPPORTED),
    (dict(h=32768, f=32768), moe.MOE_ERR_UNSUPPORTED),
])
def test_bad_shapes_are_rejected_without_launch(kw, status):
    base = dict(T=1024, h=512, E=8, f=512, Cap=128, dtype=moe.MOE_BF16, act=moe.MOE_GELU_ERF)
    base.update(kw)
    sh = moe.make_shape(**base)
    assert moe.moe_workspace_bytes(sh, False) == 0
    fake = 4096   # never dereferenced: validation fails first
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_dispatch(sh, fake, fake, fake, stream=0)
    assert ei.value.status == status


def test_null_misaligned_and_workspace_errors():
    sh = moe.make_shape(1024, 512, 8, 512, 128)
    a = 4096
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_combine(sh, a, a, None, a, a, stream=0)
    assert ei.value.status == moe.MOE_ERR_INVALID_ARG and "slot" in str(ei.value)
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_combine(sh, a, a, a + 4, a, a, stream=0)
    assert ei.value.status == moe.MOE_ERR_INVALID_ARG and "aligned" in str(ei.value)
    # workspace too small: pass a raw pointer with a byte count through the C function directly
    L = moe.lib()
    p = C.c_void_p(a)
    st = L.moe_gate(C.byref(sh), p, p, None, p, None, p, p, p, p, p, p, p, 16, None)
    assert st == moe.MOE_ERR_WORKSPACE_TOO_SMALL
    assert b"workspace" in L.moe_last_error()
    assert moe.status_string(st) == "MOE_ERR_WORKSPACE_TOO_SMALL"


@pytest.mark.parametrize("kw,status,word", [
    (dict(step=0), moe.MOE_ERR_INVALID_ARG, "step"),
    (dict(ts=0), moe.MOE_ERR_INVALID_ARG, "ts"),
    (dict(n=-1), moe.MOE_ERR_INVALID_ARG, "n="),
    (dict(beta1=1.0), moe.MOE_ERR_INVALID_ARG, "beta1"),
    (dict(lr=float("nan")), moe.MOE_ERR_INVALID_ARG, "lr"),
    (dict(eps=-1e-8), moe.MOE_ERR_INVALID_ARG, "eps"),
    (dict(dtype=5), moe.MOE_ERR_UNSUPPORTED, "dtype"),
    (dict(n=1 << 40), moe.MOE_ERR_UNSUPPORTED, "2^40"),
    (dict(ts=1001), moe.MOE_ERR_UNSUPPORTED, "multiple of 8"),
    (dict(master=None), moe.MOE_ERR_INVALID_ARG, "master"),
    (dict(staging=4100), moe.MOE_ERR_INVALID_ARG, "aligned"),
])
def test_adamw_bad_arguments_are_rejected_without_launch(kw, status, word):
    a = 4096      # never dereferenced: validation fails first
    args = dict(n=100000, ts=1000, lr=1e-3, beta1=0.9, beta2=0.95, eps=1e-8, weight_decay=0.1, step=1, dtype=moe.MOE_BF16,
                master=a, staging=a)
    args.update(kw)
    hp = moe.make_adamw(args["lr"], args["beta1"], args["beta2"], args["eps"], args["weight_decay"], args["step"])
    with pytest.raises(moe.MoeError) as ei:
        moe.moe_adamw_tiled(args["n"], args["ts"], hp, a, args["master"], a, a, a, args["staging"], args["dtype"], stream=0)
    assert ei.value.status == status and word in str(ei.value)


def test_adamw_empty_group_is_a_no_op():
    hp = moe.make_adamw(1e-3, 0.9, 0.95, 1e-8, 0.1, 1)
    moe.moe_adamw_tiled(0, 8, hp, None, None, None, None, None, None, moe.MOE_BF16, stream=0)


def test_recompute_mode_arguments():
    sh = moe.make_shape(1024, 512, 8, 512, 128)
    w0, w1, w2 = (moe.moe_workspace_bytes(sh, m) for m in (0, 1, 2))
    assert 0 < w0 < w1 < w2 and moe.moe_workspace_bytes(sh, 3) == 0
    assert w2 >= 3 * 8 * 128 * 512 * 2
    a = 4096
    L = moe.lib()
    p = C.c_void_p(a)
    # z_save without hact (or the reverse) is rejected
    st = L.moe_expert_ffn_bwd(C.byref(sh), p, p, p, None, p, p, p, p, p, p, p, w2, None)
    assert st == moe.MOE_ERR_INVALID_ARG and b"together" in L.moe_last_error()
    # recomputation needs the larger workspace
    st = L.moe_expert_ffn_bwd(C.byref(sh), p, p, None, None, p, p, p, p, p, p, p, w1, None)
    assert st == moe.MOE_ERR_WORKSPACE_TOO_SMALL
    st = L.moe_expert_ffn_fwd(C.byref(sh), p, p, p, p, None, None, p, p, w0, None)
    assert st == moe.MOE_ERR_WORKSPACE_TOO_SMALL


def test_fused_forward_arguments():
    a = 4096
    L = moe.lib()
    p = C.c_void_p(a)
    sh = moe.make_shape(1024, 512, 8, 512, 128)
    big = 1 << 40
    # both x and buf, or neither
    assert L.moe_expert_ffn_fwd_fused(C.byref(sh), p, p, p, p, p, p, p, p, None, None, None, p, p, big, None) == moe.MOE_ERR_INVALID_ARG
    assert L.moe_expert_ffn_fwd_fused(C.byref(sh), None, None, p, p, p, p, p, p, None, None, None, p, p, big, None) == moe.MOE_ERR_INVALID_ARG
    assert b"either x" in L.moe_last_error()
    # fp32 storage is not served by the fused call
    sh32 = moe.make_shape(1024, 512, 8, 512, 128, moe.MOE_F32)
    assert L.moe_expert_ffn_fwd_fused(C.byref(sh32), p, None, p, p, p, p, p, p, None, None, None, p, p, big, None) == moe.MOE_ERR_UNSUPPORTED
    # x too large for a gathered operand
    shb = moe.make_shape(1 << 19, 4096, 8, 512, 1 << 16)
    assert L.moe_expert_ffn_fwd_fused(C.byref(shb), p, None, p, p, p, p, p, p, None, None, None, p, p, big, None) == moe.MOE_ERR_UNSUPPORTED
    assert b"2 GiB" in L.moe_last_error()
    # workspace
    assert L.moe_expert_ffn_fwd_fused(C.byref(sh), p, None, p, p, p, p, p, p, None, None, None, p, p, 64, None) == moe.MOE_ERR_WORKSPACE_TOO_SMALL


def test_static_scratch_forward_arguments():
    """The entry point without a workspace refuses, before anything touches the GPU, a missing hact and a
    shape whose tile plans exceed the library's static array."""
    L = moe.lib()
    p = C.c_void_p(4096)
    ok = moe.make_shape(16384, 4096, 16, 4096, 1280)
    assert L.moe_expert_ffn_fwd_static(C.byref(ok), p, p, p, p, None, None, p, None) == moe.MOE_ERR_INVALID_ARG
    assert b"hact" in L.moe_last_error()
    big = moe.make_shape(1 << 18, 2048, 256, 2048, 1024)     # 2 x (128 + 16 * 256 * 4 * 8) bytes of plans > 256 KiB
    assert L.moe_expert_ffn_fwd_static(C.byref(big), p, p, p, p, None, p, p, None) == moe.MOE_ERR_UNSUPPORTED
    assert b"static scratch" in L.moe_last_error() and str(moe.MOE_STATIC_SCRATCH_BYTES).encode() in L.moe_last_error()


def test_duplicate_token_dropping_arguments():
    sh = moe.make_shape(1024, 512, 8, 512, 128)
    a = 4096
    for rank, size in ((0, 0), (2, 2), (-1, 4), (0, 129)):
        with pytest.raises(moe.MoeError) as ei:
            moe.moe_dispatch_dtd(sh, a, a, rank, size, a, stream=0)
        assert ei.value.status == moe.MOE_ERR_INVALID_ARG and "tp_size" in str(ei.value)
    sh32 = moe.make_shape(1024, 512, 8, 512, 128, moe.MOE_F32)
    with pytest.raises(moe.MoeError) as ei:
        moe.lib()  # ws is passed as a raw pointer below
        st = moe.lib().moe_expert_ffn_fwd_dtd(C.byref(sh32), C.c_void_p(a), 2, C.c_void_p(a), C.c_void_p(a), C.c_void_p(a), None,
                                              C.c_void_p(a), C.c_void_p(a), C.c_void_p(a), 1 << 40, None)
        raise moe.MoeError(st, moe.lib().moe_last_error().decode())
    assert ei.value.status == moe.MOE_ERR_UNSUPPORTED


def test_missing_library_fails_loudly(monkeypatch):
    monkeypatch.setattr(moe, "_lib", None)
    monkeypatch.setattr(moe, "LIB_PATH", "/nonexistent/libmoe_ted.so")
    with pytest.raises(RuntimeError, match="no fallback"):
        moe.lib()
