"""Pins for the CPU oracle: each oracle function is checked against something other than
itself -- hand-worked values, closed forms, finite differences, planted spectra, a brute-force
Jacobi eigen-solver written here, and invariants the paper's Eq. 3 / Algorithm 1 imply.
CPU only."""
import math
import os

import numpy as np
import pytest

from conftest import GOLDEN, read_golden_matrices
from oracle import ab_oracle as orc
from paper_2405_01067_amd import inputs as gen


def rel(a, b):
    return np.linalg.norm(np.asarray(a) - np.asarray(b)) / max(np.linalg.norm(np.asarray(b)), 1e-300)


# ------------------------------------------------------------------ forward / backward

def test_hand_worked_factored_layer():
    g = read_golden_matrices(os.path.join(GOLDEN, "hand_factored_layer.txt"))
    Y, T = orc.lr_linear_fwd(g["X"], g["A"], g["B"])
    assert np.array_equal(T, g["T"]) and np.array_equal(Y, g["Y"])
    dX, dA, dB, dT = orc.lr_linear_bwd(g["dY"], g["X"], g["A"], g["B"])
    assert np.array_equal(dT, g["dT"]) and np.array_equal(dA, g["dA"])
    assert np.array_equal(dB, g["dB"]) and np.array_equal(dX, g["dX"])


def test_fwd_equals_dense_layer_with_W_eq_AB():
    rng = np.random.default_rng(11)
    M, m, n, r = 37, 29, 23, 7
    X, A, B = rng.standard_normal((M, n)), rng.standard_normal((m, r)), rng.standard_normal((r, n))
    Y, T = orc.lr_linear_fwd(X, A, B)
    # explicit triple sums, element by element, through the dense weight W = A B
    W = np.zeros((m, n))
    for i in range(m):
        for j in range(n):
            W[i, j] = sum(A[i, t] * B[t, j] for t in range(r))
    Yd = np.zeros((M, m))
    for p in range(M):
        for i in range(m):
            Yd[p, i] = sum(X[p, j] * W[i, j] for j in range(n))
    assert rel(Y, Yd) < 1e-13
    assert T.shape == (M, r)


def test_fwd_identity_blocks_pad_and_crop():
    # A = [I; 0], B = [I 0]: T is the first r inputs, Y is T zero-padded to m outputs
    M, m, n, r = 5, 6, 8, 3
    X = np.arange(M * n, dtype=np.float64).reshape(M, n)
    A = np.zeros((m, r)); A[:r, :r] = np.eye(r)
    B = np.zeros((r, n)); B[:r, :r] = np.eye(r)
    Y, T = orc.lr_linear_fwd(X, A, B)
    assert np.array_equal(T, X[:, :r])
    assert np.array_equal(Y[:, :r], X[:, :r]) and not Y[:, r:].any()


def test_bwd_matches_central_finite_differences():
    rng = np.random.default_rng(5)
    M, m, n, r = 6, 5, 7, 3
    X, A, B = rng.standard_normal((M, n)), rng.standard_normal((m, r)), rng.standard_normal((r, n))
    dY = rng.standard_normal((M, m))

    def loss(X_, A_, B_):
        # L = <Y, dY> computed with explicit loops, not through the oracle
        tot = 0.0
        for p in range(M):
            t = [sum(X_[p, j] * B_[q, j] for j in range(n)) for q in range(r)]
            for i in range(m):
                tot += dY[p, i] * sum(t[q] * A_[i, q] for q in range(r))
        return tot

    dX, dA, dB, _ = orc.lr_linear_bwd(dY, X, A, B)
    h = 1e-5
    for name, arr, grad in (("X", X, dX), ("A", A, dA), ("B", B, dB)):
        num = np.zeros_like(arr)
        for idx in np.ndindex(arr.shape):
            orig = arr[idx]
            arr[idx] = orig + h
            up = loss(X, A, B)
            arr[idx] = orig - h
            dn = loss(X, A, B)
            arr[idx] = orig
            num[idx] = (up - dn) / (2 * h)
        assert rel(grad, num) < 1e-8, name


def test_bwd_dense_layer_identities():
    rng = np.random.default_rng(6)
    M, m, n, r = 40, 17, 19, 5
    X, A, B = rng.standard_normal((M, n)), rng.standard_normal((m, r)), rng.standard_normal((r, n))
    dY = rng.standard_normal((M, m))
    dX, dA, dB, dT = orc.lr_linear_bwd(dY, X, A, B)
    dW = np.einsum("pi,pj->ij", dY, X)           # dense-layer weight gradient
    assert rel(dA, np.einsum("ij,tj->it", dW, B)) < 1e-13      # dA = dW B^T
    assert rel(dB, np.einsum("it,ij->tj", A, dW)) < 1e-13      # dB = A^T dW
    assert rel(dX, np.einsum("pi,ij->pj", dY, A @ B)) < 1e-13  # dX = dY W
    assert dT.shape == (M, r)


# ------------------------------------------------------------------ SVD

def _golden_svd_cases():
    cases = []
    with open(os.path.join(GOLDEN, "closed_form_svd.txt")) as fh:
        for line in fh:
            line = line.strip()
            if not line or line.startswith("#"):
                continue
            name, mat, sv = [p.strip() for p in line.split("|")]
            parts = mat.split()
            rows, cols = int(parts[0]), int(parts[1])
            W = np.array([float(v) for v in parts[2:]]).reshape(rows, cols)
            cases.append((name, W, np.array([float(v) for v in sv.split()])))
    return cases


@pytest.mark.parametrize("name,W,sv", _golden_svd_cases())
def test_svd_closed_forms(name, W, sv):
    U, s, Vt = orc.svd(W)
    assert np.allclose(s, sv, rtol=1e-14, atol=0)
    assert rel((U * s) @ Vt, W) < 1e-14
    assert U.shape == (W.shape[0], len(sv)) and Vt.shape == (len(sv), W.shape[1])


def test_rank1_truncation_of_sym2_is_closed_form():
    A, B, s, k = orc.ab_decomposition(np.array([[3.0, 2.0], [2.0, 3.0]]), k=1)
    assert np.allclose(A @ B, 2.5 * np.ones((2, 2)), atol=1e-14)
    assert np.allclose(np.abs(A[:, 0]), math.sqrt(5.0 / 2.0)) and np.allclose(np.abs(B[0]), math.sqrt(2.5))


def _jacobi_eigenvalues(S, sweeps=60):
    """Brute force: classical two-sided Jacobi on a small symmetric matrix, pure loops."""
    S = np.array(S, dtype=np.float64)
    n = S.shape[0]
    for _ in range(sweeps):
        off = 0.0
        for p in range(n - 1):
            for q in range(p + 1, n):
                if abs(S[p, q]) < 1e-300:
                    continue
                off += S[p, q] ** 2
                theta = (S[q, q] - S[p, p]) / (2.0 * S[p, q])
                t = (1.0 if theta >= 0 else -1.0) / (abs(theta) + math.sqrt(theta * theta + 1.0))
                c = 1.0 / math.sqrt(t * t + 1.0)
                sn = t * c
                J = np.eye(n)
                J[p, p] = c; J[q, q] = c; J[p, q] = sn; J[q, p] = -sn
                S = J.T @ S @ J
        if off < 1e-30:
            break
    return np.sort(np.diag(S))[::-1]


@pytest.mark.parametrize("shape", [(3, 3), (6, 4), (4, 7), (8, 8)])
def test_svd_against_brute_force_jacobi(shape):
    rng = np.random.default_rng(shape[0] * 10 + shape[1])
    W = rng.standard_normal(shape)
    small = W.T @ W if shape[0] >= shape[1] else W @ W.T
    ev = _jacobi_eigenvalues(small)
    U, s, Vt = orc.svd(W)
    assert np.allclose(s, np.sqrt(np.maximum(ev, 0)), rtol=1e-10)
    k = min(shape)
    assert np.allclose(U.T @ U, np.eye(k), atol=1e-13) and np.allclose(Vt @ Vt.T, np.eye(k), atol=1e-13)
    assert rel((U * s) @ Vt, W) < 1e-13
    assert abs(np.sum(s ** 2) - np.sum(W ** 2)) < 1e-11 * np.sum(W ** 2)


@pytest.mark.parametrize("m,n", [(40, 24), (24, 40)])
def test_svd_recovers_planted_spectrum_and_subspaces(m, n):
    rng = np.random.default_rng(3)
    sigma = np.array([7.0, 5.0, 3.0, 2.0, 1.0, 0.5, 0.25, 0.01])
    L, R, P, Q = gen.planted_factor_pair(rng, m, n, sigma)
    U, s, Vt = orc.svd(L @ R)
    assert np.allclose(s[:8], sigma, rtol=1e-12)
    assert np.all(s[8:] < 1e-13)
    # distinct values: each singular vector equals the planted one up to sign
    assert np.allclose(np.abs(np.sum(U[:, :8] * P, axis=0)), 1.0, atol=1e-10)
    assert np.allclose(np.abs(np.sum(Vt[:8].T * Q, axis=0)), 1.0, atol=1e-10)
    # and the signs of u_i and v_i are consistent: u_i^T W v_i = +sigma_i
    assert np.allclose(np.einsum("ij,ij->j", U[:, :8], (L @ R) @ Vt[:8].T), sigma, rtol=1e-12)


# ------------------------------------------------------------------ Eq. 3 split, Eckart-Young, rank rule

def _spectral_norm_power(E, iters=2000):
    rng = np.random.default_rng(0)
    v = rng.standard_normal(E.shape[1])
    for _ in range(iters):
        v = E.T @ (E @ v)
        v /= np.linalg.norm(v)
    return np.linalg.norm(E @ v)


def test_ab_decomposition_balanced_split_and_eckart_young():
    rng = np.random.default_rng(9)
    m, n, k = 30, 20, 6
    sigma = np.array([9, 8, 6.5, 5, 4, 3, 2.2, 1.7, 1.1, 0.6, 0.3, 0.2, 0.1, 0.05, 0.02, 0.01, 5e-3, 2e-3, 1e-3, 5e-4])
    L, R, P, Q = gen.planted_factor_pair(rng, m, n, sigma)
    W = L @ R
    A, B, s, kk = orc.ab_decomposition(W, k=k)
    assert kk == k and A.shape == (m, k) and B.shape == (k, n)
    # A^T A = Sigma_k = B B^T (the Sigma^(1/2) goes to both sides)
    assert np.allclose(A.T @ A, np.diag(sigma[:k]), atol=1e-12)
    assert np.allclose(B @ B.T, np.diag(sigma[:k]), atol=1e-12)
    # A B = U_k Sigma_k V_k^T built from the planted frames
    assert rel(A @ B, (P[:, :k] * sigma[:k]) @ Q[:, :k].T) < 1e-12
    # Eckart-Young: Frobenius error^2 = sum of discarded sigma^2; spectral error = sigma_{k+1}
    E = W - A @ B
    assert abs(np.sum(E ** 2) - np.sum(sigma[k:] ** 2)) < 1e-11 * np.sum(sigma[k:] ** 2)
    assert abs(_spectral_norm_power(E) - sigma[k]) < 1e-9 * sigma[k]
    # no rank-k matrix from random perturbations of (A, B) does better
    for _ in range(20):
        A2 = A + 1e-3 * rng.standard_normal(A.shape)
        B2 = B + 1e-3 * rng.standard_normal(B.shape)
        assert np.sum((W - A2 @ B2) ** 2) >= np.sum(E ** 2) - 1e-12


def test_select_rank_rule():
    s = np.array([10.0, 5.0, 1.0, 0.999, 0.5, 0.0])
    assert orc.select_rank(s, 0.1) == 3            # 1.0 >= 0.1*10 kept (non-strict), 0.999 dropped
    assert orc.select_rank(s, 0.0999) == 4
    assert orc.select_rank(s, 0.5) == 2
    assert orc.select_rank(s, 0.0) == 6            # tau = 0 keeps everything >= 0
    assert orc.select_rank(s, 1.0) == 1
    assert orc.select_rank(np.array([3.0, 3.0, 3.0]), 1.0) == 3
    assert orc.select_rank(np.array([0.0, 0.0]), 0.5) == 2   # 0 >= 0
    A, B, sv, k = orc.ab_decomposition(np.diag([4.0, 2.0, 0.3, 0.1]), tau=0.25)
    assert k == 2 and np.allclose(A @ B, np.diag([4.0, 2.0, 0.0, 0.0]), atol=1e-14)


# ------------------------------------------------------------------ merge

def _factors(rng, m, n, k):
    sigma = np.linspace(3.0, 1.0, k)
    L, R, _, _ = gen.planted_factor_pair(rng, m, n, sigma)
    return L, R, sigma


def test_merge_identical_copies_is_idempotent():
    rng = np.random.default_rng(21)
    L, R, sigma = _factors(rng, 26, 18, 5)
    for mode in (0, 1):
        out = orc.ab_merge([L, L, L], [R, R, R], tau=0.1, mode=mode)
        assert out["k"] == 5
        assert np.allclose(out["s"][:5], sigma, rtol=1e-12)
        assert rel(out["A"] @ out["B"], L @ R) < 1e-12
        assert rel(out["W"], L @ R) < 1e-13


def test_merge_permutation_invariance_and_uniform_weights():
    rng = np.random.default_rng(22)
    L, R, _ = _factors(rng, 20, 24, 4)
    As = [L + 0.05 * rng.standard_normal(L.shape) for _ in range(3)]
    Bs = [R + 0.05 * rng.standard_normal(R.shape) for _ in range(3)]
    for mode in (0, 1):
        o1 = orc.ab_merge(As, Bs, tau=0.0, mode=mode)
        o2 = orc.ab_merge(As[::-1], Bs[::-1], tau=0.0, mode=mode)
        assert rel(o1["W"], o2["W"]) < 1e-14 and np.allclose(o1["s"], o2["s"], rtol=1e-12, atol=1e-14)
    # explicit element-wise uniform average (allReduce of A / worldSize)
    Abar = (As[0] + As[1] + As[2]) / 3.0
    Bbar = (Bs[0] + Bs[1] + Bs[2]) / 3.0
    Wm = np.zeros((20, 24))
    for i in range(20):
        for j in range(24):
            Wm[i, j] = sum(Abar[i, t] * Bbar[t, j] for t in range(4))
    assert rel(orc.merged_matrix(As, Bs, 0), Wm) < 1e-14


def test_merge_scaling_separates_the_two_readings():
    # copies a_g * A, b_g * B: mean of factors scales sigma by mean(a)*mean(b); mean of
    # products by mean(a*b).  With a = (1,3), b = (2,6): 2*4 = 8 against (2+18)/2 = 10.
    rng = np.random.default_rng(23)
    L, R, sigma = _factors(rng, 16, 12, 3)
    a, b = (1.0, 3.0), (2.0, 6.0)
    As = [a[0] * L, a[1] * L]
    Bs = [b[0] * R, b[1] * R]
    s0 = orc.ab_merge(As, Bs, tau=0.0, mode=0)["s"][:3]
    s1 = orc.ab_merge(As, Bs, tau=0.0, mode=1)["s"][:3]
    assert np.allclose(s0, 8.0 * sigma, rtol=1e-12)
    assert np.allclose(s1, 10.0 * sigma, rtol=1e-12)
    assert np.allclose(orc.merged_spectrum(As, Bs, 0)[:3], 8.0 * sigma, rtol=1e-12)


def test_merge_rank_rule_on_planted_gap_and_weyl_bound():
    rng = np.random.default_rng(24)
    m, n, k_in, gap = 96, 64, 24, 10
    sigma = gen.power_law_spectrum(k_in, 0.8, gap, 0.1)
    L, R, _, _ = gen.planted_factor_pair(rng, m, n, sigma)
    tau = math.sqrt(sigma[gap - 1] * sigma[gap]) / sigma[0]
    clean = orc.ab_merge([L, L], [R, R], tau=tau)
    assert clean["k"] == gap and np.allclose(clean["s"][:k_in], sigma, rtol=1e-11)
    As, Bs = gen.perturbed_copies(rng, L, R, 4, 1e-4)
    noisy = orc.ab_merge(As, Bs, tau=tau)
    assert noisy["k"] == gap
    # Weyl: every singular value moves by at most the spectral norm of the perturbation
    shift = np.linalg.norm(noisy["W"] - L @ R, 2)
    assert np.all(np.abs(noisy["s"][:k_in] - sigma) <= shift * (1 + 1e-9) + 1e-15)
    # A' B' is the best rank-k' approximation of the merged matrix (Eckart-Young again)
    E = noisy["W"] - noisy["A"] @ noisy["B"]
    assert abs(np.sum(E ** 2) - np.sum(noisy["s"][gap:] ** 2)) < 1e-10 * np.sum(noisy["s"] ** 2)
    assert np.allclose(noisy["A"].T @ noisy["A"], np.diag(noisy["s"][:gap]), atol=1e-12)
    # k_fixed overrides the threshold
    assert orc.ab_merge(As, Bs, tau=tau, k_fixed=7)["k"] == 7


def test_merge_mode1_rank_can_exceed_k():
    rng = np.random.default_rng(25)
    L1, R1, _ = _factors(rng, 20, 20, 3)
    L2, R2, _ = _factors(rng, 20, 20, 3)
    s0 = orc.ab_merge([L1, L2], [R1, R2], tau=0.0, mode=0)["s"]
    s1 = orc.ab_merge([L1, L2], [R1, R2], tau=0.0, mode=1)["s"]
    assert np.sum(s0 > 1e-10) == 3 and np.sum(s1 > 1e-10) == 6
    assert rel(orc.merged_matrix([L1, L2], [R1, R2], 1), 0.5 * (L1 @ R1 + L2 @ R2)) < 1e-14


# ------------------------------------------------------------------ benchmark configs behave as designed

def test_config1_reading_rank_is_32_in_both_modes():
    c = gen.config1_dense(0)
    A, B, s, k = orc.ab_decomposition(c["W"], k=32)
    assert 1.8 < s[0] < 2.2                      # N(0, var 1/256) on 256x256: sigma_max about 2
    As = [A.astype(np.float32), (A + c["noise_A"]).astype(np.float32)]
    Bs = [B.astype(np.float32), (B + c["noise_B"]).astype(np.float32)]
    for mode in (0, 1):
        assert orc.ab_merge(As, Bs, tau=c["tau"], mode=mode)["k"] == 32


def test_config5_layer_thresholds():
    lay = gen.merge_layer(768, 768, seed=101, k_in=384)
    s = orc.merged_spectrum(lay["A_copies"], lay["B_copies"], 0)
    k_gap = orc.select_rank(s, gen.CFG5_TAU_GAP)
    assert k_gap == gen.CFG5_GAP_AT
    assert s[191] / (gen.CFG5_TAU_GAP * s[0]) > 2.0 and s[192] / (gen.CFG5_TAU_GAP * s[0]) < 0.6
    k_lit = orc.select_rank(s, gen.CFG5_TAU_LITERAL)
    assert 15 <= k_lit <= 19


def test_bf16_rounding_helper_is_rne():
    x = np.array([1.0, 1.00390625, 1.005859375, -2.5, 3.1415927, 1e-40, np.inf], dtype=np.float32)
    r = gen.round_to_bf16(x)
    assert r[0] == 1.0
    assert r[1] == 1.0                # exactly halfway between 1.0 and 1.0078125 -> even (1.0)
    assert r[2] == np.float32(1.0078125)
    assert r[3] == -2.5 and r[6] == np.inf
    assert abs(r[4] - 3.140625) < 1e-7
    assert np.all(np.abs(r[:5] - x[:5]) <= np.abs(x[:5]) * 2.0 ** -8)


# ---------------------------------------------------------------------------------------------
# group-training step: AdamW, learning-rate rebound, frozen factor, reconstruction
# ---------------------------------------------------------------------------------------------

def test_adamw_first_step_closed_form():
    # from a zero state the bias-corrected moments are g and g^2: theta moves by lr g/(|g|+eps),
    # whatever the betas are; the decay term is lr * lambda * theta.
    rng = np.random.default_rng(5)
    th = rng.standard_normal(50)
    g = rng.standard_normal(50) * 10.0 ** rng.integers(-6, 3, 50)
    for b1, b2 in ((0.9, 0.999), (0.5, 0.7)):
        th1, m1, v1 = orc.adamw_step(th, g, 0 * th, 0 * th, 1, 1e-2, b1, b2, 1e-8, 0.0)
        np.testing.assert_allclose(th1, th - 1e-2 * g / (np.abs(g) + 1e-8), rtol=1e-13, atol=0)
        np.testing.assert_allclose(m1, (1 - b1) * g, rtol=1e-14)
        np.testing.assert_allclose(v1, (1 - b2) * g * g, rtol=1e-14)
    th2, _, _ = orc.adamw_step(th, g, 0 * th, 0 * th, 1, 1e-2, 0.9, 0.999, 1e-8, 0.3)
    np.testing.assert_allclose(th2 - th1, -1e-2 * 0.3 * th, rtol=1e-10, atol=1e-16)


def test_adamw_constant_gradient_and_pure_decay():
    # a constant gradient keeps mh = g, vh = g^2 at every step: t equal moves of lr*sign(g)
    g = np.array([3.0, -0.25, 1e-3])
    th, m, v = np.zeros(3), np.zeros(3), np.zeros(3)
    for t in range(1, 8):
        th, m, v = orc.adamw_step(th, g, m, v, t, 1e-3, 0.9, 0.999, 0.0, 0.0)
        np.testing.assert_allclose(th, -t * 1e-3 * np.sign(g), rtol=1e-12)
    # zero gradient: only the decoupled decay acts, theta_t = theta_0 (1 - lr lambda)^t
    th0 = np.array([2.0, -5.0])
    th, m, v = th0.copy(), np.zeros(2), np.zeros(2)
    for t in range(1, 6):
        th, m, v = orc.adamw_step(th, np.zeros(2), m, v, t, 0.1, weight_decay=0.5)
        np.testing.assert_allclose(th, th0 * (1 - 0.05) ** t, rtol=1e-13)
        assert np.all(m == 0) and np.all(v == 0)


def test_adamw_against_library_optimizer():
    torch = pytest.importorskip("torch")
    rng = np.random.default_rng(11)
    th0 = rng.standard_normal((7, 5))
    p = torch.nn.Parameter(torch.tensor(th0, dtype=torch.float64))
    opt = torch.optim.AdamW([p], lr=3e-3, betas=(0.8, 0.95), eps=1e-6, weight_decay=0.1)
    th, m, v = th0.copy(), np.zeros_like(th0), np.zeros_like(th0)
    for t in range(1, 13):
        g = rng.standard_normal((7, 5)) * (0.1 if t % 3 else 10.0)
        scale = orc.lr_rebound_scale(t - 1, 6)
        for group in opt.param_groups:
            group["lr"] = 3e-3 * scale
        p.grad = torch.tensor(g, dtype=torch.float64)
        opt.step()
        th, m, v = orc.adamw_step(th, g, m, v, t, 3e-3, 0.8, 0.95, 1e-6, 0.1, lr_scale=scale)
        np.testing.assert_allclose(th, p.detach().numpy(), rtol=1e-12, atol=1e-14)
    st = opt.state[p]
    np.testing.assert_allclose(m, st["exp_avg"].numpy(), rtol=1e-13)
    np.testing.assert_allclose(v, st["exp_avg_sq"].numpy(), rtol=1e-13)


def test_lr_rebound_scale_ramp():
    n = 8
    s = [orc.lr_rebound_scale(i, n) for i in range(12)]
    assert s[0] == pytest.approx(1.0 / n) and s[0] < 0.2          # starts near zero
    assert all(b > a for a, b in zip(s[:n - 1], s[1:n]))           # climbs
    assert np.allclose(np.diff(s[:n]), 1.0 / n)                    # linearly
    assert s[n - 1] == 1.0 and all(x == 1.0 for x in s[n:])        # back at the scheduled rate
    assert orc.lr_rebound_scale(0, 0) == 1.0


def test_group_step_freezes_the_other_factor_and_descends():
    rng = np.random.default_rng(2)
    M, m, n, k = 40, 12, 9, 4
    X = rng.standard_normal((M, n)); A = rng.standard_normal((m, k)); B = rng.standard_normal((k, n))
    Yt = rng.standard_normal((M, m))
    loss = lambda A_, B_: 0.5 * np.sum((orc.lr_linear_fwd(X, A_, B_)[0] - Yt) ** 2)
    for target in ("A", "B"):
        Y, _ = orc.lr_linear_fwd(X, A, B)
        dY = Y - Yt
        tr = A if target == "A" else B
        out = orc.group_train_step(X, dY, A, B, target, (0 * tr, 0 * tr), 1, 1e-3, weight_decay=0.0)
        frozen_new, frozen_old = (out["B"], B) if target == "A" else (out["A"], A)
        assert np.array_equal(frozen_new, frozen_old)
        moved = out["A"] - A if target == "A" else out["B"] - B
        # first Adam step: every entry moves by lr against the sign of its gradient
        np.testing.assert_allclose(moved, -1e-3 * np.sign(out["grad"]), rtol=1e-6)
        assert loss(out["A"], out["B"]) < loss(A, B)
        # the gradient is the one of the full backward
        ref = orc.lr_linear_bwd(dY, X, A, B)
        assert np.array_equal(out["grad"], ref[1] if target == "A" else ref[2])
        assert np.array_equal(out["dX"], ref[0])


def test_reconstruct_is_the_dense_weight_of_the_layer():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((6, 3)); B = rng.standard_normal((3, 5)); X = rng.standard_normal((4, 5))
    W = orc.reconstruct(A, B)
    np.testing.assert_allclose(X @ W.T, orc.lr_linear_fwd(X, A, B)[0], rtol=1e-13, atol=1e-13)
    assert np.linalg.matrix_rank(W) == 3


# ---------------------------------------------------------------------------------------------
# convolutional layer carried as factors
# ---------------------------------------------------------------------------------------------

def test_conv_patches_hand_example_and_shift():
    # one 3 x 3 single-channel image, 3 x 3 window: the patch of the centre pixel is the image
    # itself, row-major; the patch of the top-left pixel has the image's top-left 2 x 2 block in
    # its bottom-right corner and zeros elsewhere
    img = np.arange(1.0, 10.0).reshape(1, 3, 3, 1)
    P = orc.conv_patches(img, 3, 3)
    assert P.shape == (9, 9)
    np.testing.assert_array_equal(P[4], np.arange(1.0, 10.0))
    np.testing.assert_array_equal(P[0], [0, 0, 0, 0, 1, 2, 0, 4, 5])
    np.testing.assert_array_equal(P[8], [5, 6, 0, 8, 9, 0, 0, 0, 0])
    # a weight with a single one at tap (ky, kx) = (0, 2) shifts the image down-left by (1, -1)
    w = np.zeros((1, 9)); w[0, 0 * 3 + 2] = 1.0
    out = (P @ w.T).reshape(3, 3)
    np.testing.assert_array_equal(out, [[0, 0, 0], [2, 3, 0], [5, 6, 0]])


def test_conv_fwd_against_library_correlation():
    sig = pytest.importorskip("scipy.signal")
    rng = np.random.default_rng(8)
    N, H, W, C, m, k = 2, 5, 6, 3, 4, 2
    for kh, kw in ((3, 3), (1, 1), (3, 1), (5, 3)):
        act = rng.standard_normal((N, H, W, C))
        A = rng.standard_normal((m, k)); B = rng.standard_normal((k, kh * kw * C))
        Y, T = orc.lr_conv_fwd(act, A, B, kh, kw)
        Wd = (A @ B).reshape(m, kh, kw, C)                      # dense weight, tap-major flattening
        for b in range(N):
            for o in range(m):
                ref = sum(sig.correlate2d(act[b, :, :, c], Wd[o, :, :, c], mode="same") for c in range(C))
                np.testing.assert_allclose(Y.reshape(N, H, W, m)[b, :, :, o], ref, rtol=1e-11, atol=1e-11)
    # stride 2: the library's stride-1 correlation at every second pixel (5 x 6 -> 3 x 3 outputs)
    kh, kw = 3, 3
    act = rng.standard_normal((N, H, W, C))
    A = rng.standard_normal((m, k)); B = rng.standard_normal((k, kh * kw * C))
    Y, T = orc.lr_conv_fwd(act, A, B, kh, kw, stride=2)
    assert Y.shape == (N * 3 * 3, m) and T.shape == (N * 3 * 3, k)
    Wd = (A @ B).reshape(m, kh, kw, C)
    for b in range(N):
        for o in range(m):
            ref = sum(sig.correlate2d(act[b, :, :, c], Wd[o, :, :, c], mode="same") for c in range(C))
            np.testing.assert_allclose(Y.reshape(N, 3, 3, m)[b, :, :, o], ref[::2, ::2], rtol=1e-11, atol=1e-11)
    # a 1 x 1 window with stride 2 is the plain factored layer on every second pixel
    Bp = rng.standard_normal((k, C))
    np.testing.assert_array_equal(orc.lr_conv_fwd(act, A, Bp, 1, 1, stride=2)[0],
                                  orc.lr_linear_fwd(act[:, ::2, ::2].reshape(-1, C), A, Bp)[0])
    # a 1 x 1 window is the plain factored linear layer on the pixels
    act = rng.standard_normal((N, H, W, C)); A = rng.standard_normal((m, k)); B = rng.standard_normal((k, C))
    np.testing.assert_array_equal(orc.lr_conv_fwd(act, A, B, 1, 1)[0],
                                  orc.lr_linear_fwd(act.reshape(-1, C), A, B)[0])


def test_conv_patches_adjoint_identity():
    rng = np.random.default_rng(9)
    shape = (2, 4, 5, 3)
    for kh, kw in ((3, 3), (1, 3), (5, 5)):
        act = rng.standard_normal(shape)
        G = rng.standard_normal((2 * 4 * 5, kh * kw * 3))
        lhs = np.sum(orc.conv_patches(act, kh, kw) * G)
        rhs = np.sum(act * orc.conv_patches_adjoint(G, shape, kh, kw))
        assert lhs == pytest.approx(rhs, rel=1e-12)
        # stride 2: 4 x 5 -> 2 x 3 patches
        G2 = rng.standard_normal((2 * 2 * 3, kh * kw * 3))
        lhs = np.sum(orc.conv_patches(act, kh, kw, 2) * G2)
        rhs = np.sum(act * orc.conv_patches_adjoint(G2, shape, kh, kw, 2))
        assert lhs == pytest.approx(rhs, rel=1e-12)


@pytest.mark.parametrize("stride", [1, 2])
def test_conv_bwd_matches_central_finite_differences(stride):
    rng = np.random.default_rng(10)
    N, H, W, C, m, k, kh, kw = 2, 4, 3, 2, 3, 2, 3, 3
    rows = N * (-(-H // stride)) * (-(-W // stride))
    act = rng.standard_normal((N, H, W, C)); A = rng.standard_normal((m, k))
    B = rng.standard_normal((k, kh * kw * C)); R = rng.standard_normal((rows, m))
    loss = lambda a_, A_, B_: float(np.sum(orc.lr_conv_fwd(a_, A_, B_, kh, kw, stride)[0] * R))
    dAct, dA, dB, _ = orc.lr_conv_bwd(R, act, A, B, kh, kw, stride)
    eps = 1e-6
    for arr, grad, which in ((act, dAct, 0), (A, dA, 1), (B, dB, 2)):
        for _ in range(12):
            idx = tuple(rng.integers(0, s) for s in arr.shape)
            hi = [act.copy(), A.copy(), B.copy()]; lo = [act.copy(), A.copy(), B.copy()]
            hi[which][idx] += eps; lo[which][idx] -= eps
            fd = (loss(*hi) - loss(*lo)) / (2 * eps)
            assert fd == pytest.approx(grad[idx], rel=1e-6, abs=1e-8)


# ------------------------------------------------------------------ Algorithm 1 as a whole

def test_schedule_fractions_and_the_driver_agree():
    """The oracle's phase lengths (floating-point fractions of Sec. "Hyperparameter considerations")
    and the driver's integer arithmetic give the same whole steps for every run length."""
    from paper_2405_01067_amd import driver as drv
    assert orc.ab_schedule(3000) == (600, 100, 25, 50)        # 20 %, 3.33 %, a quarter, a half
    for n in range(1, 3001):
        s = drv.schedule(n)
        assert (s.warmup_steps, s.ab_steps, s.rebound_steps, s.lr_rebound_steps) == orc.ab_schedule(n), n
    assert [drv.group_target(g, 4) for g in range(4)] == ["A", "A", "B", "B"]
    assert [drv.group_target(g, 3) for g in range(3)] == ["A", "A", "B"]


def test_training_run_with_zero_learning_rate_is_eckart_young_truncation():
    """With a learning rate of zero the group phase leaves the factors alone, so one cycle of
    Algorithm 1 must map W to its best rank-k approximation (k from the cut-off rule), whatever the
    number of groups, and a cut-off of zero must give W back."""
    rng = np.random.default_rng(5)
    W = [rng.standard_normal((12, 9)), rng.standard_normal((7, 12))]
    X = rng.standard_normal((20, 9))
    calls = []
    def full_rank(Wl, phase, i, scale):
        calls.append((phase, i, scale))
    for groups in (1, 3):
        calls.clear()
        out, hist = orc.ab_training_run(W, groups, 0.3, 0.0, lambda g, s: X, lambda Y, g, s: Y, full_rank, 7)
        # 7 steps: warm-up 1, then decomposition, 1 group step, synchronisation, 1 rebound step, ...
        assert orc.ab_schedule(7) == (1, 1, 1, 1)
        assert [c[0] for c in calls] == ["warmup", "rebound", "rebound", "rebound"]
        assert len(hist) == 3 and hist[0][0] == 2
        for l, w in enumerate(W):
            u, s, vt = np.linalg.svd(w)
            k = int(np.sum(s >= 0.3 * s[0]))
            assert hist[0][1][l] == k
            best = (u[:, :k] * s[:k]) @ vt[:k]
            assert np.allclose(out[l], best, atol=1e-12)
    out, _ = orc.ab_training_run(W, 2, 0.0, 0.0, lambda g, s: X, lambda Y, g, s: Y, full_rank, 4)
    for l in range(2):
        assert np.allclose(out[l], W[l], atol=1e-12)


def test_training_run_one_group_one_step_is_one_adamw_step_on_A():
    """One group (it trains A), one layer, a single group step: the synchronised weight is
    (A - step) B with the AdamW step of the oracle's own optimiser on the gradient dY^T T."""
    rng = np.random.default_rng(6)
    W = rng.standard_normal((8, 6))
    X = rng.standard_normal((15, 6))
    Yt = rng.standard_normal((15, 8))
    hyper = dict(beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)
    # 4 steps: warm-up 1, then one cycle of 1 group step + 1 rebound step, then another group step
    out, hist = orc.ab_training_run([W], 1, 0.0, 1e-2, lambda g, s: X, lambda Y, g, s: Y - Yt,
                                    lambda Wl, ph, i, sc: None, 3, **hyper)
    A, B, _, k = orc.ab_decomposition(W, tau=0.0)
    T = X @ B.T
    dA = (T @ A.T - Yt).T @ T
    # first AdamW step: bias-corrected moments give g / (|g| + eps) elementwise
    A1 = A - 1e-2 * (dA / (np.abs(dA) + 1e-8) + 0.01 * A)
    assert np.allclose(hist[0][2][0], A1 @ B, atol=1e-10)
