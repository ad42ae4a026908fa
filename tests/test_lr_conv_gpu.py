"""Parity of the factored convolution on the GPU (lr_conv_fwd / lr_conv_bwd, through the C ABI)
against the CPU oracle, element by element on the same seeded inputs.  The kernels gather the
patch matrix from the channels-last activation; the oracle builds it explicitly.

Tolerance: relative Frobenius error 1e-2 (bf16 storage, fp32 accumulation), as for the linear
layer.  Where the gathered kernels must do exactly what the plain ones do on an explicit patch
matrix (same products in the same order), the comparison is bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ab_oracle as orc
from paper_2405_01067_amd import binding as abt
from paper_2405_01067_amd import inputs as gen

pytestmark = pytest.mark.gpu

TOL = 1e-2
BF = torch.bfloat16


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def dev(x, dtype=BF):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0").to(dtype)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def run(c, **bwd_kw):
    act, dY, A, B = (dev(c[k]) for k in ("act", "dY", "A", "B"))
    Y, T = abt.lr_conv_fwd(act, A, B, c["kh"], c["kw"], save_T=True, stride=c.get("stride", 1))
    dAct, dA, dB = abt.lr_conv_bwd(dY, act, T, A, B, c["kh"], c["kw"], stride=c.get("stride", 1), **bwd_kw)
    torch.cuda.synchronize()
    return act, dY, A, B, Y, T, dAct, dA, dB


def check(c):
    act, dY, A, B, Y, T, dAct, dA, dB = run(c)
    st = c.get("stride", 1)
    Yo, To = orc.lr_conv_fwd(c["act"], c["A"], c["B"], c["kh"], c["kw"], st)
    dActo, dAo, dBo, _ = orc.lr_conv_bwd(c["dY"], c["act"], c["A"], c["B"], c["kh"], c["kw"], st)
    errs = {"T": rel(host(T), To), "Y": rel(host(Y), Yo), "dAct": rel(host(dAct), dActo),
            "dA": rel(host(dA), dAo), "dB": rel(host(dB), dBo)}
    assert all(e < TOL for e in errs.values()), errs
    return errs


CASES = [
    # N, H, W, C, m, r, kh, kw
    (3, 7, 5, 64, 128, 32, 3, 3),      # 105 pixels: one full row block and a ragged one
    (2, 9, 9, 128, 64, 96, 3, 3),      # r = 96: taps padded to 128 columns in the activation gradient
    (5, 4, 6, 192, 192, 64, 1, 1),     # 1 x 1: the plain factored layer on the pixels
    (2, 6, 4, 64, 64, 160, 5, 3),      # window wider than the image is tall enough for; unequal sides
    (1, 8, 8, 512, 64, 32, 3, 3),      # activation gradient in two blocks of 256 channels
    (4, 3, 2, 64, 64, 384, 3, 3),      # widest rank; image narrower than the window
    (37, 14, 14, 64, 256, 64, 3, 3),   # 7252 pixels: several row splits of the factor gradients
    (8, 56, 56, 64, 64, 32, 3, 3),     # ResNet-50's widest feature map: a patch reaches 57 pixels, nearly a row block
    (2, 5, 40, 128, 128, 128, 7, 7),   # 7 x 7 window: taller than the image, reach 123 pixels
]


@pytest.mark.parametrize("N,H,W,C,m,r,kh,kw", CASES)
def test_conv_step_against_oracle(N, H, W, C, m, r, kh, kw):
    c = gen.conv_case(N, H, W, C, m, r, kh, kw, seed=N * 1000 + H * 100 + C + r)
    check(c)


@pytest.mark.parametrize("N,H,W,C,m,r,kh,kw", [CASES[0], CASES[1], CASES[6], (3, 10, 10, 64, 128, 192, 3, 3)])
def test_conv_step_with_tall_work_groups(N, H, W, C, m, r, kh, kw):
    # the 128-row chain kernel (chosen by itself only for large batches) forced on small ones
    prev = abt.set_chain_rows(128)
    try:
        c = gen.conv_case(N, H, W, C, m, r, kh, kw, seed=N * 1000 + H * 100 + C + r + 1)
        check(c)
    finally:
        abt.set_chain_rows(prev)


STRIDED = [
    # N, H, W, C, m, r, kh, kw: stride 2, output grid ceil(H / 2) x ceil(W / 2)
    (3, 8, 8, 64, 128, 32, 3, 3),      # even sides: 4 x 4 outputs per image, 48 rows
    (5, 7, 5, 64, 64, 64, 3, 3),       # odd sides: 4 x 3 outputs, the last window hangs over the edge
    (4, 9, 6, 128, 64, 96, 1, 1),      # 1 x 1, stride 2: the shortcut projection of a down-sampling block
    (2, 14, 14, 128, 128, 32, 3, 3),   # 98 rows: two row blocks, ragged
    (9, 6, 10, 64, 64, 128, 5, 3),     # wide window, unequal sides, 135 rows
    (40, 8, 8, 64, 64, 32, 3, 3),      # 640 rows from 2560 pixels: several splits and row blocks
]


@pytest.mark.parametrize("N,H,W,C,m,r,kh,kw", STRIDED)
def test_strided_conv_step_against_oracle(N, H, W, C, m, r, kh, kw):
    c = gen.conv_case(N, H, W, C, m, r, kh, kw, seed=900 + N + H + r, stride=2)
    check(c)


@pytest.mark.parametrize("N,H,W,C,m,r,kh,kw", STRIDED[:4])
def test_strided_conv_step_with_tall_work_groups(N, H, W, C, m, r, kh, kw):
    prev = abt.set_chain_rows(128)
    try:
        check(gen.conv_case(N, H, W, C, m, r, kh, kw, seed=950 + N + H + r, stride=2))
    finally:
        abt.set_chain_rows(prev)


def test_resnet50_downsampling_convolutions():
    """The two strided convolutions of a ResNet-50 down-sampling block (stage 3: 28 x 28 -> 14 x 14), at a
    batch the oracle's explicit patch matrix still fits: 3 x 3 stride 2 on 128 channels, and the
    1 x 1 stride 2 shortcut 256 -> 512."""
    check(gen.conv_case(16, 28, 28, 128, 128, 32, 3, 3, seed=31, stride=2))
    check(gen.conv_case(16, 28, 28, 256, 512, 128, 1, 1, seed=32, stride=2))


def test_conv_equals_linear_layer_on_explicit_patches():
    # the gathered kernels and the plain kernels on an explicit patch matrix run the same products
    # in the same order: forward bit for bit; the factor gradients too
    c = gen.conv_case(6, 10, 7, 128, 128, 64, 3, 3, seed=5)
    act, dY, A, B, Y, T, dAct, dA, dB = run(c)
    Xcol = dev(orc.conv_patches(c["act"], 3, 3).astype(np.float32))      # entries are bf16 values: exact
    Y2, T2 = abt.lr_linear_fwd(Xcol, A, B, save_T=True)
    dX2, dA2, dB2 = abt.lr_linear_bwd(dY, Xcol, T2, A, B)
    torch.cuda.synchronize()
    assert torch.equal(T, T2) and torch.equal(Y, Y2)
    assert torch.equal(dA, dA2)
    assert rel(host(dB), host(dB2)) < 1e-6          # same products; the row splits may differ
    # the activation gradient is the adjoint of the patch extraction applied to dXcol
    fold = orc.conv_patches_adjoint(host(dX2), c["act"].shape, 3, 3)
    assert rel(host(dAct), fold) < TOL


def test_conv_bwd_options():
    c = gen.conv_case(4, 6, 6, 64, 128, 96, 3, 3, seed=17)
    act, dY, A, B, Y, T, dAct, dA, dB = run(c)
    kh, kw = c["kh"], c["kw"]
    # frozen-factor variants
    g1 = abt.lr_conv_bwd(dY, act, T, A, B, kh, kw, need_dB=False)
    assert g1[2] is None and torch.equal(g1[0], dAct) and torch.equal(g1[1], dA)
    g2 = abt.lr_conv_bwd(dY, act, T, A, B, kh, kw, need_dA=False, need_dAct=False)
    assert g2[0] is None and g2[1] is None and torch.equal(g2[2], dB)
    # T recomputed
    g3 = abt.lr_conv_bwd(dY, act, None, A, B, kh, kw)
    assert all(torch.equal(x, y) for x, y in zip(g3, (dAct, dA, dB)))
    # accumulate
    accA, accB = dA.clone(), dB.clone()
    abt.lr_conv_bwd(dY, act, T, A, B, kh, kw, need_dAct=False, dA=accA, dB=accB, accumulate=True)
    torch.cuda.synchronize()
    assert rel(host(accA), 2 * host(dA)) < 1e-6 and rel(host(accB), 2 * host(dB)) < 1e-6
    # forward without saving T; reruns are bit-identical
    Y2, T2 = abt.lr_conv_fwd(act, A, B, kh, kw, save_T=False)
    assert T2 is None and torch.equal(Y2, Y)
    again = run(c)
    assert all(torch.equal(x, y) for x, y in zip(again[4:], (Y, T, dAct, dA, dB)))


def test_conv_refuses_unsupported_shapes():
    act = torch.zeros((1, 4, 4, 48), dtype=BF, device="cuda:0")      # C not a multiple of 64
    A = torch.zeros((64, 32), dtype=BF, device="cuda:0")
    B = torch.zeros((32, 9 * 48), dtype=BF, device="cuda:0")
    with pytest.raises(abt.AbtError):
        abt.lr_conv_fwd(act, A, B, 3, 3)
    act = torch.zeros((1, 4, 4, 64), dtype=BF, device="cuda:0")
    B = torch.zeros((32, 4 * 64), dtype=BF, device="cuda:0")
    with pytest.raises(abt.AbtError):
        abt.lr_conv_fwd(act, A, B, 2, 2)                              # even window
    A = torch.zeros((64, 224), dtype=BF, device="cuda:0")
    B = torch.zeros((224, 9 * 64), dtype=BF, device="cuda:0")
    with pytest.raises(abt.AbtError):
        abt.lr_conv_fwd(act, A, B, 3, 3)                              # rank the gathered kernel does not cover


@pytest.mark.parametrize("case", gen.RESNET50_CONVS_NATIVE, ids=lambda cs: cs[0])
def test_config4_native_full_size(case):
    name, N, H, W, C, m, r = case
    c = gen.conv_case(N, H, W, C, m, r, 3, 3, seed=3 + 200 + N + C)
    errs = check(c)
    print(name, errs)
