"""Host-side checks that need no GPU: the C-ABI library loads, exports every symbol the header
declares, and rejects bad arguments before touching the device."""
import ctypes
import os
import re

import pytest

from conftest import ROOT
from paper_2405_01067_amd import binding as abt

HEADER = os.path.join(ROOT, "include", "abtrain.h")


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(abt._LIB_PATH):
        import __graft_entry__ as ge
        ge.build()
    return abt.load()


def declared_functions():
    text = open(HEADER).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = re.findall(r"^\s*(?:const\s+char\s*\*|int|size_t|double)\s+(\w+)\s*\(", text, flags=re.M)
    return sorted(set(names))


def test_header_functions_are_exported(lib):
    names = declared_functions()
    assert {"lr_linear_fwd", "lr_linear_bwd", "ab_merge", "ab_merge_batched"} <= set(names)
    for n in names:
        assert hasattr(lib, n), n
    assert set(names) == set(abt.EXPORTS)


def test_status_strings(lib):
    assert abt.status_string(0) == "ABT_OK"
    for code in range(-9, 0):
        s = abt.status_string(code)
        assert s.startswith("ABT_E"), s
    assert "unknown" in abt.status_string(-99)


def test_workspace_queries(lib):
    # bf16 forward keeps T on chip: no workspace
    assert lib.lr_linear_fwd_workspace_bytes(12608, 3072, 768, 192, abt.ABT_BF16) == 0
    assert lib.lr_linear_fwd_workspace_bytes(64, 256, 256, 32, abt.ABT_F32) >= 64 * 32 * 4
    b = lib.lr_linear_bwd_workspace_bytes(12608, 3072, 768, 192, abt.ABT_BF16)
    # A^T, B^T, dT, T and at least one fp32 partial of dA and dB
    assert b >= 2 * (3072 * 192 + 768 * 192 + 2 * 12608 * 192) + 4 * (3072 + 768) * 192
    assert b % 256 == 0
    # unsupported shapes report 0
    assert lib.lr_linear_bwd_workspace_bytes(128, 100, 768, 192, abt.ABT_BF16) == 0
    assert lib.lr_linear_bwd_workspace_bytes(128, 128, 128, 416, abt.ABT_BF16) == 0
    w0 = lib.ab_merge_workspace_bytes(4, 3072, 768, 384, 384, 0)
    w1 = lib.ab_merge_workspace_bytes(4, 3072, 768, 96, 384, 1)  # same K = 384 by concatenation
    assert w0 > 0 and w1 > 0
    assert w0 >= 4 * (3072 + 768) * 384 + 5 * 8 * 384 * 384
    assert lib.ab_merge_workspace_bytes(0, 10, 10, 32, 32, 0) == 0


def test_argument_validation_without_device(lib):
    buf = ctypes.create_string_buffer(4096 + 256)
    base = (ctypes.addressof(buf) + 255) // 256 * 256          # fake, aligned, never dereferenced
    p = ctypes.c_void_p(base)
    null = ctypes.c_void_p(0)
    odd = ctypes.c_void_p(base + 2)
    f = lib.lr_linear_fwd
    assert f(null, p, p, p, null, 64, 256, 256, 32, abt.ABT_BF16, null, 0, null) == -1      # EINVAL
    assert f(p, p, p, p, null, 64, 256, 256, 32, 7, null, 0, null) == -5                    # EDTYPE
    assert f(p, p, p, p, null, 0, 256, 256, 32, abt.ABT_BF16, null, 0, null) == -2          # ESHAPE
    assert f(p, p, p, p, null, 64, 250, 256, 32, abt.ABT_BF16, null, 0, null) == -2
    assert f(p, p, p, p, null, 64, 256, 256, 48, abt.ABT_BF16, null, 0, null) == -2
    assert f(p, p, p, p, null, 64, 256, 256, 512, abt.ABT_BF16, null, 0, null) == -2
    assert f(odd, p, p, p, null, 64, 256, 256, 32, abt.ABT_BF16, null, 0, null) == -3       # EALIGN
    assert f(p, p, p, p, null, 64, 256, 256, 32, abt.ABT_F32, null, 0, null) == -4          # EWORKSPACE (T needs a home)
    g = lib.lr_linear_bwd
    assert g(p, p, p, p, p, p, p, p, 64, 256, 256, 32, abt.ABT_BF16, 0, null, 0, null) == -4
    assert g(null, p, p, p, p, p, p, p, 64, 256, 256, 32, abt.ABT_BF16, 0, p, 1 << 30, null) == -1
    assert g(p, p, p, p, p, p, p, p, 64, 256, 256, 33, abt.ABT_BF16, 0, p, 1 << 30, null) == -2

    ptrs = (ctypes.c_void_p * 2)(base, base)
    pp = ctypes.cast(ptrs, ctypes.POINTER(ctypes.c_void_p))
    h = lib.ab_merge
    ok_args = dict(G=2, m=64, n=64, k=32, tau=0.1, k_fixed=0, mode=0)

    def call(**kw):
        a = dict(ok_args); a.update(kw)
        return h(pp, pp, a["G"], a["m"], a["n"], a["k"], a["tau"], a["k_fixed"], a["mode"],
                 a.get("A_out", p), p, p, p, a.get("k_cap", 32), null, a.get("ws", null), a.get("wsb", 0), null)

    assert call() == -4                       # no workspace
    assert call(G=0) == -1
    assert call(tau=1.5) == -1
    assert call(tau=-0.1) == -1
    assert call(mode=2) == -1
    assert call(k=40) == -2
    assert call(k=1024, G=4, mode=1) == -2    # K = G k > 2048
    assert call(k_cap=0) == -2
    assert call(A_out=null) == -1
    assert call(A_out=odd) == -3
    assert call(ws=odd, wsb=1 << 40) == -3


def test_factorize_validation_without_device(lib):
    buf = ctypes.create_string_buffer(4096 + 256)
    base = (ctypes.addressof(buf) + 255) // 256 * 256          # fake, aligned, never dereferenced
    p, null, odd = ctypes.c_void_p(base), ctypes.c_void_p(0), ctypes.c_void_p(base + 2)
    f = lib.ab_factorize
    big = 1 << 40
    assert lib.ab_factorize_workspace_bytes(3072, 768, 384) > 4 * 768 * 768
    descs = (abt.FactorizeDesc * 2)()
    for d, (m, n) in zip(descs, ((3072, 768), (768, 768))):
        d.m, d.n, d.k_cap = m, n, 384
    both = lib.ab_factorize_batched_workspace_bytes(descs, 2)
    # the two layers share one 768 x 768 identity
    assert both < lib.ab_factorize_workspace_bytes(3072, 768, 384) + lib.ab_factorize_workspace_bytes(768, 768, 384)
    assert both > lib.ab_factorize_workspace_bytes(3072, 768, 384)
    assert lib.ab_factorize_workspace_bytes(768, 3072, 384) > 4 * 768 * 768
    assert lib.ab_factorize_workspace_bytes(100, 70, 32) == 0
    assert lib.ab_factorize_workspace_bytes(4096, 2080, 32) == 0
    assert f(null, 256, 256, 0.1, 0, p, p, p, p, 256, p, big, null) == -1        # EINVAL
    assert f(p, 100, 70, 0.1, 0, p, p, p, p, 64, p, big, null) == -2             # ESHAPE
    assert f(p, 4096, 2080, 0.1, 0, p, p, p, p, 64, p, big, null) == -2
    assert f(p, 256, 256, 0.1, 0, p, p, p, p, 0, p, big, null) == -2
    assert f(odd, 256, 256, 0.1, 0, p, p, p, p, 256, p, big, null) == -3         # EALIGN
    assert f(p, 256, 256, 0.1, 0, p, p, p, p, 256, null, 0, null) == -4          # EWORKSPACE
    assert f(p, 256, 256, 0.1, 0, p, p, p, p, 256, p, 1024, null) == -4
    assert f(p, 256, 256, 1.5, 0, p, p, p, p, 256, p, big, null) == -1           # tau out of range
    assert f(p, 256, 256, 0.1, 0, null, p, p, p, 256, p, big, null) == -1


def test_group_step_validation_and_rebound_factor_without_device(lib):
    from oracle import ab_oracle as orc
    buf = ctypes.create_string_buffer(4096 + 256)
    base = (ctypes.addressof(buf) + 255) // 256 * 256          # fake, aligned, never dereferenced
    p, null = ctypes.c_void_p(base), ctypes.c_void_p(0)
    step = lib.ab_adamw_step
    t = (abt.AdamwTensor * 2)()
    for e in t:
        e.param = e.grad = e.exp_avg = e.exp_avg_sq = base
        e.count = 100
    ok = (1e-3, 1.0, 0.9, 0.999, 1e-8, 0.01)
    assert step(t, 0, 1, *ok, null) == 0                        # nothing to do
    t[0].count = t[1].count = 0
    assert step(t, 2, 1, *ok, null) == 0                        # empty tensors are skipped
    t[0].count = 100
    assert step(t, 2, 0, *ok, null) == -1                       # step counts from 1
    assert step(None, 2, 1, *ok, null) == -1
    assert step(t, -1, 1, *ok, null) == -1
    assert step(t, 2, 1, 1e-3, 1.0, 1.0, 0.999, 1e-8, 0.01, null) == -1      # beta1 = 1
    assert step(t, 2, 1, 1e-3, 1.0, 0.9, -0.1, 1e-8, 0.01, null) == -1
    assert step(t, 2, 1, 1e-3, 1.0, 0.9, 0.999, -1.0, 0.01, null) == -1
    assert step(t, 2, 1, float("nan"), 1.0, 0.9, 0.999, 1e-8, 0.01, null) == -1
    t[0].count = -5
    assert step(t, 2, 1, *ok, null) == -2
    t[0].count = 100
    t[0].grad = 0
    assert step(t, 2, 1, *ok, null) == -1
    t[0].grad = base + 4
    assert step(t, 2, 1, *ok, null) == -3
    t[0].grad = base
    t[0].param_bf16 = base + 2
    assert step(t, 2, 1, *ok, null) == -3
    # the learning-rate factor is host arithmetic: the library's and the oracle's must agree
    for n in (0, 1, 3, 8, 1000):
        for i in range(0, 12):
            assert lib.ab_lr_rebound_scale(i, n) == pytest.approx(orc.lr_rebound_scale(i, n), rel=1e-15)
    assert lib.ab_lr_rebound_scale(-3, 8) == pytest.approx(1 / 8)
    r = lib.ab_reconstruct
    assert r(null, p, p, 8, 8, 4, null) == -1
    assert r(p, p, p, 0, 8, 4, null) == -2
    assert r(p, p, ctypes.c_void_p(base + 4), 8, 8, 4, null) == -3


def test_conv_validation_without_device(lib):
    buf = ctypes.create_string_buffer(4096 + 256)
    base = (ctypes.addressof(buf) + 255) // 256 * 256          # fake, aligned, never dereferenced
    p, null, odd = ctypes.c_void_p(base), ctypes.c_void_p(0), ctypes.c_void_p(base + 2)
    BF = abt.ABT_BF16
    good = abt.ConvGeom(2, 14, 14, 256, 3, 3)
    need = lib.lr_conv_bwd_workspace_bytes(ctypes.byref(good), 256, 64, BF)
    M = 2 * 14 * 14
    assert need >= 2 * M * 64 * 2 + 256 * 9 * 64 * 2            # dT, T, the re-laid-out factor
    assert lib.lr_conv_bwd_workspace_bytes(ctypes.byref(good), 256, 64, abt.ABT_F32) == 0
    fwd = lambda g, m=256, r=64, dt=BF, act=p, Y=p: lib.lr_conv_fwd(act, p, p, Y, null, ctypes.byref(g), m, r, dt, null)
    assert fwd(good, dt=abt.ABT_F32) == -5                      # bf16 only
    assert lib.lr_conv_fwd(p, p, p, p, null, None, 256, 64, BF, null) == -1
    assert fwd(good, act=null) == -1
    assert fwd(good, Y=odd) == -3
    for bad in (abt.ConvGeom(2, 14, 14, 48, 3, 3),              # C not a multiple of 64
                abt.ConvGeom(2, 14, 14, 256, 2, 3),             # even window
                abt.ConvGeom(0, 14, 14, 256, 3, 3),
                abt.ConvGeom(2, 14, 14, 256, 17, 3),
                abt.ConvGeom(2, 14, 14, 1 << 20, 3, 3),         # kh kw C too wide
                abt.ConvGeom(1 << 31, 14, 14, 64, 3, 3),        # too many pixels
                abt.ConvGeom(2, 14, 14, 256, 3, 3, 3),          # stride other than 1 or 2
                abt.ConvGeom(2, 14, 14, 256, 3, 3, 0)):
        assert fwd(bad) == -2
        assert lib.lr_conv_bwd_workspace_bytes(ctypes.byref(bad), 256, 64, BF) == 0
    assert fwd(good, m=100) == -2 and fwd(good, r=48) == -2 and fwd(good, r=224) == -2 and fwd(good, r=416) == -2
    bwd = lambda ws, wsb, dY=p: lib.lr_conv_bwd(dY, p, p, p, p, p, p, p, ctypes.byref(good), 256, 64, BF, 0, ws, wsb, null)
    assert bwd(null, 0) == -4 and bwd(p, need - 1) == -4
    assert bwd(odd, 1 << 40) == -3
    assert bwd(p, 1 << 40, dY=null) == -1


def test_binding_refuses_cpu_tensors(lib):
    import torch
    x = torch.zeros(4, 64, dtype=torch.bfloat16)
    a = torch.zeros(64, 32, dtype=torch.bfloat16)
    b = torch.zeros(32, 64, dtype=torch.bfloat16)
    with pytest.raises(abt.AbtError):
        abt.lr_linear_fwd(x, a, b)
    with pytest.raises(abt.AbtError):
        abt.ab_merge([a.float()], [b.float()], tau=0.1)


def test_chain_shape_setters(lib):
    assert abt.set_chain_rows(128) == 0
    assert abt.set_chain_rows(77) == 128          # ignored value, setting kept
    assert abt.set_chain_rows(64) == 128
    assert abt.set_chain_rows(0) == 64
    assert abt.set_chain_parts(3) == 0
    assert abt.set_chain_parts(99) == 3           # ignored
    assert abt.set_chain_parts(0) == 3
    assert abt.set_chain_parts(0) == 0 and abt.set_chain_rows(0) == 0


def test_sweep_cap_setter(lib):
    prev = abt.set_jacobi_max_sweeps(5)
    assert abt.set_jacobi_max_sweeps(1000) == 5
    assert abt.set_jacobi_max_sweeps(prev) == 64


def test_merge_group_setter(lib):
    prev = abt.set_merge_groups(2)
    assert abt.set_merge_groups(-5) == 2          # negative: back to "as many as allowed"
    assert abt.set_merge_groups(prev) == 0
