"""One low-rank phase of Algorithm 1 composed from the library's entry points, on one layer with
two emulated groups, against the same composition of the CPU oracle's functions:

    A, B <- abDecomposition(W) with the cut-off rule          ab_factorize
    group 0 trains A, group 1 trains B, the other factor      lr_linear_fwd, lr_linear_bwd (masked),
      frozen, a few AdamW steps under a learning-rate rebound   ab_adamw_step, ab_lr_rebound_scale
    average the factors over the groups and re-factorise       ab_merge
    W <- A B                                                    ab_reconstruct

fp32 path throughout.  The upstream gradient is that of a least-squares loss, formed by the test
(dY = Y - target): it belongs to the model, not to the path.  Both sides start from the factors the
GPU factorisation produced (factorisation parity has its own tests; singular vectors are only
defined up to sign, and per-element Adam is equivariant under such sign changes, so only products
would be comparable otherwise)."""
import math

import numpy as np
import pytest
import torch

from oracle import ab_oracle as orc
from paper_2405_01067_amd import binding as abt
from paper_2405_01067_amd import inputs as gen

pytestmark = pytest.mark.gpu

HYPER = dict(beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def dev(x):
    return torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to("cuda:0")


def host(t):
    return t.detach().cpu().numpy().astype(np.float64)


def test_low_rank_phase_two_groups():
    rng = np.random.default_rng(2024)
    m, n, gap, M, steps, rebound, lr = 256, 192, 32, 300, 5, 3, 1e-3
    sigma = gen.power_law_spectrum(min(m, n), gap_at=gap)
    Lf, Rf, _, _ = gen.planted_factor_pair(rng, m, n, sigma)
    W32 = (Lf @ Rf).astype(np.float32)
    tau = float(math.sqrt(sigma[gap - 1] * sigma[gap]) / sigma[0])

    # ---- decomposition with the cut-off rule
    fz = abt.ab_factorize(dev(W32), tau=tau, k_cap=64)
    k = int(fz["k"].item())
    assert k == gap == orc.ab_decomposition(W32.astype(np.float64), tau=tau)[3]
    A0 = fz["A"][:, :k].contiguous()
    B0 = fz["B"][:k, :].contiguous()
    A0h, B0h = host(A0), host(B0)                      # both sides start here

    # ---- group training: group 0 trains A, group 1 trains B
    data = []
    for g in range(2):
        X = gen.gaussian(rng, (M, n))
        Yt = (X.astype(np.float64) @ W32.astype(np.float64).T + 0.1 * rng.standard_normal((M, m))).astype(np.float32)
        data.append((X, Yt))
    gpu_factors, cpu_factors = [], []
    for g, target in enumerate(("A", "B")):
        X, Yt = data[g]
        Xd, Ytd = dev(X), dev(Yt)
        A, B = A0.clone(), B0.clone()
        trained = A if target == "A" else B
        mom, var = torch.zeros_like(trained), torch.zeros_like(trained)
        Ao, Bo = A0h.copy(), B0h.copy()
        state = (np.zeros_like(Ao if target == "A" else Bo), np.zeros_like(Ao if target == "A" else Bo))
        for t in range(1, steps + 1):
            scale = abt.lr_rebound_scale(t - 1, rebound)
            Y, T = abt.lr_linear_fwd(Xd, A, B, save_T=True)
            dY = Y - Ytd
            dX, dA, dB = abt.lr_linear_bwd(dY, Xd, T, A, B, need_dA=(target == "A"), need_dB=(target == "B"))
            assert (dB if target == "A" else dA) is None
            abt.ab_adamw_step([dict(param=trained, grad=dA if target == "A" else dB, exp_avg=mom, exp_avg_sq=var)],
                              step=t, lr=lr, lr_scale=scale, **HYPER)
            # oracle: the same step in fp64
            Yo, _ = orc.lr_linear_fwd(X, Ao, Bo)
            out = orc.group_train_step(X, Yo - Yt, Ao, Bo, target, state, t, lr,
                                       lr_scale=orc.lr_rebound_scale(t - 1, rebound), **HYPER)
            Ao, Bo, state = out["A"], out["B"], out["state"]
        torch.cuda.synchronize()
        frozen_ok = torch.equal(B, B0) if target == "A" else torch.equal(A, A0)
        assert frozen_ok
        assert rel(host(A), Ao) < 1e-4 and rel(host(B), Bo) < 1e-4, (target, rel(host(A), Ao), rel(host(B), Bo))
        # the trained factor really moved, by about lr per step and element
        moved = rel(host(trained), A0h if target == "A" else B0h)
        assert moved > 1e-3
        gpu_factors.append((A, B))
        cpu_factors.append((Ao, Bo))

    # ---- synchronisation: average the factors over the groups, re-factorise with the cut-off rule
    mg = abt.ab_merge([a for a, _ in gpu_factors], [b for _, b in gpu_factors], tau=tau, k_cap=64, want_W=True)
    ref = orc.ab_merge([a for a, _ in cpu_factors], [b for _, b in cpu_factors], tau=tau)
    k2 = int(mg["k"].item())
    assert k2 == ref["k"]
    S = host(mg["S"])[:k2]
    assert np.max(np.abs(S - ref["s"][:k2]) / ref["s"][:k2]) < 1e-4
    assert rel(host(mg["W"]), ref["W"]) < 1e-4

    # ---- hand-off to the full-rank weight
    A2, B2 = mg["A"][:, :k2].contiguous(), mg["B"][:k2, :].contiguous()
    Wn = abt.ab_reconstruct(A2, B2)
    torch.cuda.synchronize()
    Wo = orc.reconstruct(ref["A"], ref["B"])
    assert rel(host(Wn), Wo) < 1e-4
    # what the phase changed, not just the unchanged bulk of W, must agree
    W_start = A0h @ B0h
    assert rel(host(Wn) - W_start, Wo - W_start) < 1e-2
    assert rel(Wo, W_start) > 1e-4
