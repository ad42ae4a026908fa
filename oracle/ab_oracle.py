"""CPU oracle for the AB-training hot path (arxiv 2405.01067).  TEST INFRASTRUCTURE ONLY.

A plain, slow, fp64 NumPy statement of what the factored-layer training step and the merge
compute, written from the paper.  It shares no code with the HIP library and must never be
imported by the product path: only tests, the smoke check and the bench's `cpu_baseline`
leg may use it.

Notation follows the paper's Eq. 3: a layer weight W (m x n, out x in) is carried as
W = A B with A = U_k Sigma_k^(1/2) (m x k) and B = Sigma_k^(1/2) V_k^T (k x n).
The layer acts as y = x W^T, so for a batch X (M x n):  T = X B^T (M x k),  Y = T A^T (M x m).

Pins (tests/test_oracle_pins.py): every function below is checked against closed forms,
finite differences, planted spectra, brute-force Jacobi on tiny matrices, invariants and, for
the optimiser step, a library optimiser run in fp64.  Nothing here is "parity unpinned".
"""
from __future__ import annotations

import numpy as np

_F64 = np.float64


def _f64(x):
    return np.asarray(x, dtype=_F64)


# --------------------------------------------------------------------------------------
# factored layer: forward and backward (Eq. 3 and the chain rule through it)
# --------------------------------------------------------------------------------------

def lr_linear_fwd(X, A, B):
    """Forward of a layer whose weight is W = A B (Eq. 3): T = X B^T, Y = T A^T.

    No intermediate rounding.  Returns (Y, T) in fp64."""
    X, A, B = _f64(X), _f64(A), _f64(B)
    T = X @ B.T
    Y = T @ A.T
    return Y, T


def lr_linear_bwd(dY, X, A, B):
    """Backward of the same layer for a loss L with dL/dY = dY (chain rule on Eq. 3; the
    group phase of Algorithm 1 trains A or B, so both factor gradients are defined):

        dT = dY A,   dA = dY^T T,   dB = dT^T X,   dX = dT B.

    Returns (dX, dA, dB, dT) in fp64."""
    dY, X, A, B = _f64(dY), _f64(X), _f64(A), _f64(B)
    T = X @ B.T
    dT = dY @ A
    dA = dY.T @ T
    dB = dT.T @ X
    dX = dT @ B
    return dX, dA, dB, dT


# --------------------------------------------------------------------------------------
# SVD, rank rule, AB decomposition (Sec. "Methodology", Eq. 3)
# --------------------------------------------------------------------------------------

def svd(W):
    """Full thin SVD W = U diag(s) V^T in fp64, s descending.  LAPACK (numpy.linalg.svd) is
    the library step; a wide matrix (n > m) is transposed first, as the paper prescribes
    for unfavourable shapes, and the bases are swapped back."""
    W = _f64(W)
    m, n = W.shape
    if n > m:
        U, s, Vt = np.linalg.svd(W.T, full_matrices=False)
        return Vt.T, s, U.T
    U, s, Vt = np.linalg.svd(W, full_matrices=False)
    return U, s, Vt


def select_rank(s, tau):
    """Rank rule of the AB decomposition: singular values smaller than sigmaCutoff times the
    largest one are removed, i.e. keep sigma_i iff sigma_i >= tau * sigma_1.  The comparison
    is taken in fp32 (the precision the library stores sigma in).  At least one is kept."""
    s32 = np.asarray(s, dtype=np.float32)
    if s32.size == 0:
        return 0
    cut = np.float32(tau) * s32[0]
    return max(1, int(np.count_nonzero(s32 >= cut)))


def ab_decomposition(W, tau=None, k=None):
    """Eq. 3: A = U_k Sigma_k^(1/2), B = Sigma_k^(1/2) V_k^T from the SVD of W; k given, or
    chosen by the rank rule with threshold tau.  Returns (A, B, s, k) with s the full
    descending spectrum."""
    U, s, Vt = svd(W)
    if k is None:
        k = select_rank(s, tau)
    k = int(k)
    root = np.sqrt(s[:k])
    A = U[:, :k] * root[None, :]
    B = root[:, None] * Vt[:k, :]
    return A, B, s, k


# --------------------------------------------------------------------------------------
# merge (Algorithm 1: all-reduce of A and of B over all workers, then W <- A B; followed by
# the re-decomposition with the rank rule)
# --------------------------------------------------------------------------------------

def merged_matrix(A_copies, B_copies, mode=0):
    """The merged dense weight.
    mode 0 (the paper): average A and B separately over the copies, then W = A_mean B_mean.
    mode 1 (mean of reconstructions): W = (1/G) sum_g A_g B_g."""
    G = len(A_copies)
    assert G == len(B_copies) and G >= 1
    if mode == 0:
        A_mean = sum(_f64(a) for a in A_copies) / G
        B_mean = sum(_f64(b) for b in B_copies) / G
        return A_mean @ B_mean
    if mode == 1:
        return sum(_f64(a) @ _f64(b) for a, b in zip(A_copies, B_copies)) / G
    raise ValueError("mode must be 0 or 1")


def ab_merge(A_copies, B_copies, tau, k_fixed=0, mode=0):
    """Merge G group copies of the factors and re-factorise the result.

    Returns a dict: W (merged dense matrix, m x n), s (its full descending spectrum),
    k (selected rank: k_fixed if > 0 else the rank rule with tau), A (m x k), B (k x n)
    with A B the best rank-k approximation of W split as in Eq. 3, and U, V (the leading k
    singular vectors, columns)."""
    W = merged_matrix(A_copies, B_copies, mode)
    U, s, Vt = svd(W)
    k = int(k_fixed) if k_fixed and k_fixed > 0 else select_rank(s, tau)
    k = min(k, len(s))
    root = np.sqrt(s[:k])
    return {
        "W": W, "s": s, "k": k,
        "A": U[:, :k] * root[None, :],
        "B": root[:, None] * Vt[:k, :],
        "U": U[:, :k], "V": Vt[:k, :].T,
    }


def merged_spectrum(A_copies, B_copies, mode=0):
    """Singular values only of the merged matrix (descending, fp64)."""
    W = merged_matrix(A_copies, B_copies, mode)
    if W.shape[1] > W.shape[0]:
        W = W.T
    return np.linalg.svd(W, compute_uv=False)


# --------------------------------------------------------------------------------------
# group training step (Sec. "Methodology", group-training phase of Algorithm 1; Sec. "Learning
# rate rebound"; the experiments train with AdamW, Sec. "Experiments")
# --------------------------------------------------------------------------------------

def lr_rebound_scale(i, rebound_steps):
    """Factor applied to the scheduled learning rate i steps (0-based) after a change of the
    parameters' shape.  The paper says the rate drops to near zero and climbs back to its
    scheduled value over `rebound_steps` steps; the shape of the climb is not given.  Reading:
    linear, (i + 1) / rebound_steps, capped at 1; rebound_steps <= 0 means no rebound."""
    if rebound_steps <= 0:
        return 1.0
    return min(1.0, (int(i) + 1) / float(rebound_steps))


def adamw_step(theta, g, m, v, t, lr, beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01,
               lr_scale=1.0):
    """One step of Adam with decoupled weight decay (the optimiser the paper's experiments
    name), step counter t >= 1, on fp64 copies of the arguments:

        m' = b1 m + (1 - b1) g                 v' = b2 v + (1 - b2) g^2
        mh = m' / (1 - b1^t)                   vh = v' / (1 - b2^t)
        theta' = theta - eta (mh / (sqrt(vh) + eps) + lambda theta),   eta = lr * lr_scale.

    The rebound factor multiplies the whole step (gradient part and decay part alike), as a
    change of the learning rate does.  Returns (theta', m', v')."""
    theta, g, m, v = _f64(theta), _f64(g), _f64(m), _f64(v)
    assert t >= 1
    m1 = beta1 * m + (1.0 - beta1) * g
    v1 = beta2 * v + (1.0 - beta2) * g * g
    mh = m1 / (1.0 - beta1 ** t)
    vh = v1 / (1.0 - beta2 ** t)
    eta = lr * lr_scale
    return theta - eta * (mh / (np.sqrt(vh) + eps) + weight_decay * theta), m1, v1


def group_train_step(X, dY, A, B, target, state, t, lr, lr_scale=1.0, **hyper):
    """One step of the group-training phase for one layer and a given upstream gradient dY:
    forward and backward of the factored layer, then an AdamW step on the factor this group
    trains (target 'A' or 'B'); the other factor is frozen and keeps its value.  `state` is the
    pair (m, v) of the trained factor.  Returns a dict with Y, dX, the gradient used, the new
    factors and the new state."""
    Y, _ = lr_linear_fwd(X, A, B)
    dX, dA, dB, _ = lr_linear_bwd(dY, X, A, B)
    m, v = state
    if target == "A":
        A1, m1, v1 = adamw_step(A, dA, m, v, t, lr, lr_scale=lr_scale, **hyper)
        return {"Y": Y, "dX": dX, "grad": dA, "A": A1, "B": _f64(B), "state": (m1, v1)}
    if target == "B":
        B1, m1, v1 = adamw_step(B, dB, m, v, t, lr, lr_scale=lr_scale, **hyper)
        return {"Y": Y, "dX": dX, "grad": dB, "A": _f64(A), "B": B1, "state": (m1, v1)}
    raise ValueError("target must be 'A' or 'B'")


def reconstruct(A, B):
    """W <- A B, the hand-off from the factors back to the full-rank weight (Algorithm 1)."""
    return _f64(A) @ _f64(B)


def ab_schedule(total_steps):
    """Phase lengths of Algorithm 1 for a run of `total_steps` steps with the fractions of Sec.
    "Hyperparameter considerations": warmupSteps 20 %, numABSteps 3.33 % (1/30),
    fullRankReboundSteps 0.25 numABSteps, learning-rate rebound 0.5 numABSteps.  Reading: each is
    rounded to the nearest whole step (halves up) and is at least one step.
    Returns (warmup, num_ab, full_rank_rebound, lr_rebound)."""
    def whole(x):
        return max(1, int(np.floor(x + 0.5)))
    warm = whole(0.2 * total_steps)
    num_ab = whole(total_steps / 30.0)
    return warm, num_ab, whole(0.25 * num_ab), whole(0.5 * num_ab)


def ab_training_run(weights, groups, tau, lr, batch, loss_grad, full_rank_step, total_steps, **hyper):
    """Algorithm 1 for a chain of linear layers (the output of layer l feeds layer l + 1, no
    activations) and `groups` emulated workers, composed of the functions above, in fp64.

    The first half of the groups trains A, the second half B (odd counts: the extra group trains
    A); the other factor is frozen.  The optimiser state of the trained factors starts at zero in
    every group-training phase and its step counter at 1 (the parameters have changed shape; the
    learning-rate rebound is the paper's answer to exactly that).  batch(g, step) gives the input
    of group g, loss_grad(Y, g, step) the gradient at the last layer's output, and
    full_rank_step(weights, phase, i, lr_scale) trains the dense weights in place: those three
    belong to the model, not to the method.  Returns (weights, history): history has one entry
    per synchronisation, (step, ranks selected at the decomposition, copies of the weights)."""
    W = [_f64(w).copy() for w in weights]
    warm, num_ab, reb, lr_reb = ab_schedule(total_steps)
    step, history = 0, []
    for i in range(min(warm, total_steps)):
        full_rank_step(W, "warmup", i, 1.0)
        step += 1
    while step < total_steps:
        factors = [ab_decomposition(w, tau=tau) for w in W]
        ranks = [f[3] for f in factors]
        A = [[f[0].copy() for f in factors] for _ in range(groups)]
        B = [[f[1].copy() for f in factors] for _ in range(groups)]
        targets = ["A" if g < (groups + 1) // 2 else "B" for g in range(groups)]
        state = [[(np.zeros_like(A[g][l] if targets[g] == "A" else B[g][l]),) * 2 for l in range(len(W))]
                 for g in range(groups)]
        n_ab = min(num_ab, total_steps - step)
        for i in range(n_ab):
            scale = lr_rebound_scale(i, lr_reb)
            for g in range(groups):
                acts = [_f64(batch(g, step))]
                for l in range(len(W)):
                    acts.append(lr_linear_fwd(acts[-1], A[g][l], B[g][l])[0])
                dY = _f64(loss_grad(acts[-1], g, step))
                for l in reversed(range(len(W))):
                    out = group_train_step(acts[l], dY, A[g][l], B[g][l], targets[g], state[g][l], i + 1, lr,
                                           lr_scale=scale, **hyper)
                    dY = out["dX"]
                    A[g][l], B[g][l], state[g][l] = out["A"], out["B"], out["state"]
            step += 1
        for l in range(len(W)):
            # A <- allReduce(A / worldSize), B <- allReduce(B / worldSize), W <- A B
            W[l] = merged_matrix([A[g][l] for g in range(groups)], [B[g][l] for g in range(groups)], mode=0)
        history.append((step, ranks, [w.copy() for w in W]))
        for i in range(min(reb, total_steps - step)):
            full_rank_step(W, "rebound", i, lr_rebound_scale(i, lr_reb))
            step += 1
    return W, history


# --------------------------------------------------------------------------------------
# convolutional layer carried as factors (Sec. "Methodology": a weight with more than two
# dimensions is flattened over its trailing dimensions to give the matrix W of Eq. 3)
# --------------------------------------------------------------------------------------
# A convolution weight [m, C, kh, kw] flattened to W [m, kh kw C] factors as W = A B with
# A [m, k] and B [k, kh kw C]: B is a kh x kw convolution to k channels, A a 1 x 1 convolution.
# Layout here: activations N x H x W x C (channels last); the flattened axis is ordered tap-major,
# column (ky kw + kx) C + c.  (The order of the flattened axis only permutes the columns of W
# and of B; it does not change the factorisation.)  Zero padding (kh-1)/2, (kw-1)/2, kh and kw odd,
# stride s >= 1 in both directions: output pixel (y', x') is centred on input pixel (s y', s x') and
# the output has ceil(H / s) x ceil(W / s) pixels: the 3x3 and 1x1 convolutions of ResNet-50's
# bottleneck blocks, the down-sampling ones (s = 2) included.

def conv_patches(act, kh, kw, stride=1):
    """Patch matrix of a channels-last activation: Xcol [N H' W', kh kw C] with
    Xcol[(b, y', x'), (ky, kx, c)] = act[b, s y' + ky - ph, s x' + kx - pw, c], zero outside the
    image (H' = ceil(H / s), W' = ceil(W / s)): the patches of every s-th pixel in both directions."""
    act = _f64(act)
    N, H, W, C = act.shape
    assert kh % 2 == 1 and kw % 2 == 1
    ph, pw = kh // 2, kw // 2
    padded = np.zeros((N, H + 2 * ph, W + 2 * pw, C), dtype=_F64)
    padded[:, ph:ph + H, pw:pw + W, :] = act
    cols = np.empty((N, H, W, kh * kw, C), dtype=_F64)
    for ky in range(kh):
        for kx in range(kw):
            cols[:, :, :, ky * kw + kx, :] = padded[:, ky:ky + H, kx:kx + W, :]
    cols = cols[:, ::stride, ::stride]
    return np.ascontiguousarray(cols).reshape(-1, kh * kw * C)


def conv_patches_adjoint(G, shape, kh, kw, stride=1):
    """Adjoint of conv_patches: sums every entry of G [N H' W', kh kw C] back onto the activation
    element it was read from.  Returns [N, H, W, C]."""
    N, H, W, C = shape
    Gs = _f64(G).reshape(N, -(-H // stride), -(-W // stride), kh * kw, C)
    G = np.zeros((N, H, W, kh * kw, C), dtype=_F64)     # the pixels between the strided ones had no patch
    G[:, ::stride, ::stride] = Gs
    ph, pw = kh // 2, kw // 2
    padded = np.zeros((N, H + 2 * ph, W + 2 * pw, C), dtype=_F64)
    for ky in range(kh):
        for kx in range(kw):
            padded[:, ky:ky + H, kx:kx + W, :] += G[:, :, :, ky * kw + kx, :]
    return padded[:, ph:ph + H, pw:pw + W, :]


def lr_conv_fwd(act, A, B, kh, kw, stride=1):
    """Forward of a convolution whose flattened weight is W = A B: the factored linear layer
    applied to the patch matrix.  Returns (Y [N H' W', m], T [N H' W', k])."""
    return lr_linear_fwd(conv_patches(act, kh, kw, stride), A, B)


def lr_conv_bwd(dY, act, A, B, kh, kw, stride=1):
    """Backward of the same layer: the factored layer's gradients on the patch matrix, and the
    activation gradient as the adjoint of the patch extraction applied to dXcol = dT B.
    Returns (dAct [N, H, W, C], dA, dB, dT)."""
    act = _f64(act)
    dXcol, dA, dB, dT = lr_linear_bwd(dY, conv_patches(act, kh, kw, stride), A, B)
    return conv_patches_adjoint(dXcol, act.shape, kh, kw, stride), dA, dB, dT
