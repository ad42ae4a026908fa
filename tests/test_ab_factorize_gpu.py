"""Parity of ab_factorize (Eq. 3 for a dense weight, the abDecomposition step of Algorithm 1)
against the CPU oracle's ab_decomposition: singular values (1e-4 relative on the kept ones), the
selected rank (exact on spectra with a gap at the threshold), the product A B = U_k Sigma_k V_k^T,
the projectors on the singular subspaces and the balanced split A^T A = Sigma_k = B B^T."""
import math

import numpy as np
import pytest
import torch

from oracle import ab_oracle as orc
from paper_2405_01067_amd import binding as abt
from paper_2405_01067_amd import inputs as gen

pytestmark = pytest.mark.gpu

TOL = 1e-4


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda:0")


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


def check(W32, out, tau=None, k_fixed=None, expect_k=None):
    """W32: the fp32 values the GPU got; the oracle factorises exactly those."""
    A_o, B_o, s_o, k_o = orc.ab_decomposition(W32.astype(np.float64), tau=tau, k=k_fixed)
    k = int(out["k"].item())
    assert k == k_o, (k, k_o)
    if expect_k is not None:
        assert k == expect_k
    S = host(out["S"])
    errs = {"sigma": float(np.max(np.abs(S[:k] - s_o[:k]) / s_o[:k]))}
    A, B = host(out["A"]), host(out["B"])
    assert not A[:, k:].any() and not B[k:, :].any(), "columns/rows beyond k' must be zero"
    A, B = A[:, :k], B[:k, :]
    errs["AB"] = rel(A @ B, A_o @ B_o)
    errs["AtA"] = rel(A.T @ A, np.diag(s_o[:k]))
    errs["BBt"] = rel(B @ B.T, np.diag(s_o[:k]))
    U_o = A_o / np.sqrt(s_o[:k])[None, :]
    V_o = (B_o / np.sqrt(s_o[:k])[:, None]).T
    U = A / np.sqrt(s_o[:k])[None, :]
    V = (B / np.sqrt(s_o[:k])[:, None]).T
    errs["projU"] = float(np.linalg.norm(U @ U.T - U_o @ U_o.T) / math.sqrt(k))
    errs["projV"] = float(np.linalg.norm(V @ V.T - V_o @ V_o.T) / math.sqrt(k))
    assert all(e < TOL for e in errs.values()), errs
    return errs


def planted(m, n, gap, seed, tail=0.1):
    """Dense m x n matrix with spectrum i^-0.8 and a drop by `tail` after position `gap`."""
    rng = np.random.default_rng(seed)
    K = min(m, n)
    sigma = gen.power_law_spectrum(K, gap_at=gap, gap_factor=tail)
    L, R, _, _ = gen.planted_factor_pair(rng, m, n, sigma)
    return (L @ R).astype(np.float32), sigma


def test_config1_dense_weight_fixed_rank():
    # config 1's W (256 x 256, N(0, 1/256)): the rank-32 factors the step of config 1 starts from
    c = gen.config1_dense(0)
    W32 = c["W"].astype(np.float32)
    out = abt.ab_factorize(dev(W32), tau=0.0, k_fixed=32, k_cap=32)
    check(W32, out, k_fixed=32, expect_k=32)


@pytest.mark.parametrize("m,n,gap", [(320, 192, 40), (192, 320, 40), (256, 256, 100), (512, 96, 17), (64, 1024, 9)])
def test_planted_gap_selects_the_rank(m, n, gap):
    W32, sigma = planted(m, n, gap, seed=m + n + gap)
    tau = float(math.sqrt(sigma[gap - 1] * sigma[gap]) / sigma[0])
    out = abt.ab_factorize(dev(W32), tau=tau)
    check(W32, out, tau=tau, expect_k=gap)


def test_vit_attention_projection_shape():
    # 768 x 768 (ViT-B/16 proj): K = 768 runs the wide-core Jacobi kernels
    W32, sigma = planted(768, 768, 192, seed=5)
    tau = float(math.sqrt(sigma[191] * sigma[192]) / sigma[0])
    out = abt.ab_factorize(dev(W32), tau=tau, k_cap=384)
    check(W32, out, tau=tau, expect_k=192)


def test_widest_core_the_boundary_admits():
    # min(m, n) = 2048, the documented limit, with n > m (the I W route): blocks of 4 columns,
    # 511 cross rounds per sweep in the general Jacobi kernels
    W32, sigma = planted(2048, 2304, 300, seed=21)
    tau = float(math.sqrt(sigma[299] * sigma[300]) / sigma[0])
    out = abt.ab_factorize(dev(W32), tau=tau, k_cap=512)
    check(W32, out, tau=tau, expect_k=300)


def test_rank_deficient_weight_and_k_cap():
    # rank 48 exactly (in fp64; fp32 rounding leaves a tail ~1e-8): tau picks the 48, k_cap clips
    rng = np.random.default_rng(11)
    sigma = gen.power_law_spectrum(48)
    L, R, _, _ = gen.planted_factor_pair(rng, 256, 160, sigma)
    W32 = (L @ R).astype(np.float32)
    out = abt.ab_factorize(dev(W32), tau=1e-3)
    check(W32, out, tau=1e-3, expect_k=48)
    out = abt.ab_factorize(dev(W32), tau=1e-3, k_cap=32)
    assert int(out["k"].item()) == 32 and out["A"].shape == (256, 32)
    A, B = host(out["A"]), host(out["B"])
    A_o, B_o, _, _ = orc.ab_decomposition(W32.astype(np.float64), k=32)
    assert rel(A @ B, A_o @ B_o) < TOL


def test_batched_matches_single_calls():
    specs = [(320, 192, 40), (192, 320, 40), (256, 256, 100), (768, 96, 17)]
    mats, taus = [], []
    for m, n, gap in specs:
        W32, sigma = planted(m, n, gap, seed=3 * m + n)
        mats.append(W32)
        taus.append(float(math.sqrt(sigma[gap - 1] * sigma[gap]) / sigma[0]))
    outs = abt.ab_factorize_batched([dict(W=dev(W), tau=t) for W, t in zip(mats, taus)])
    for (m, n, gap), W32, tau, o in zip(specs, mats, taus, outs):
        check(W32, o, tau=tau, expect_k=gap)
        single = abt.ab_factorize(dev(W32), tau=tau)
        assert torch.equal(single["S"], o["S"]) and torch.equal(single["A"], o["A"]) and torch.equal(single["B"], o["B"])


def test_unsupported_shapes_are_refused():
    with pytest.raises(abt.AbtError):
        abt.ab_factorize(torch.zeros((100, 70), device="cuda:0"), tau=0.1)      # min(m, n) % 32
    with pytest.raises(abt.AbtError):
        abt.ab_factorize(torch.zeros((4096, 2080), device="cuda:0"), tau=0.1)   # min(m, n) > 2048
