"""Seeded synthetic inputs shared by the CPU oracle's tests and the HIP path's tests/bench.

This module only draws random numbers and lays them out: no factored products, no SVD, no rank
rule, nothing the oracle or the kernels compute.  The one linear-algebra routine it calls, a QR
of a Gaussian matrix, draws random orthonormal frames; `planted_factor_pair` scales such frames
by the square roots of a chosen spectrum, because the workloads prescribe inputs of that form
(factor copies that look like the output of a decomposition with a known spectrum).  Neither the
oracle nor the library calls it to do their own arithmetic.  Everything is NumPy on the host;
callers upload the arrays they need.

The workloads mirror the layer shapes of the paper's experiments (ViT-B/16 and ResNet-50 at
local batch 64/256, Sec. "Experiments"); the paper's datasets and trained weights are replaced
by Gaussians of the same shape.
"""
from __future__ import annotations

import numpy as np

# ----------------------------------------------------------------------------------------
# bf16 storage helpers (format conversion only: IEEE round-to-nearest-even on the top 16 bits)
# ----------------------------------------------------------------------------------------

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """float32 array -> uint16 array of bf16 bit patterns, round-to-nearest-even."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    nan = (u & 0x7FFFFFFF) > 0x7F800000
    rounded = (u + (0x7FFF + ((u >> 16) & 1))) >> 16
    rounded = np.where(nan, (u >> 16) | 0x0040, rounded)
    return rounded.astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """uint16 bf16 bit patterns -> the float32 values they denote (exact)."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << 16).view(np.float32)


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """float32 array rounded to the nearest bf16-representable float32 values."""
    return bf16_bits_to_f32(f32_to_bf16_bits(x))


# ----------------------------------------------------------------------------------------
# basic draws
# ----------------------------------------------------------------------------------------

def gaussian(rng: np.random.Generator, shape, std: float = 1.0) -> np.ndarray:
    """iid N(0, std^2) float32 array."""
    out = rng.standard_normal(size=shape, dtype=np.float32)
    if std != 1.0:
        out *= np.float32(std)
    return out


def orthonormal_frame(rng: np.random.Generator, rows: int, cols: int) -> np.ndarray:
    """rows x cols float64 matrix with orthonormal columns, Haar-distributed (cols <= rows)."""
    g = rng.standard_normal(size=(rows, cols))
    q, r = np.linalg.qr(g)
    q *= np.sign(np.diag(r))[None, :]  # fix the sign so the draw is Haar and reproducible
    return q


def power_law_spectrum(count: int, decay: float = 0.8, gap_at: int = 0,
                       gap_factor: float = 0.1) -> np.ndarray:
    """sigma_i = i^-decay (i = 1..count); entries after position gap_at are multiplied by
    gap_factor, which plants a spectral gap there (gap_at = 0: no gap)."""
    i = np.arange(1, count + 1, dtype=np.float64)
    s = i ** (-decay)
    if gap_at:
        s[gap_at:] *= gap_factor
    return s


def planted_factor_pair(rng: np.random.Generator, m: int, n: int, sigma: np.ndarray):
    """A test matrix with a known spectrum, handed over as two thin matrices.

    Draws orthonormal frames P (m x k), Q (n x k) and returns float64
    L = P * sqrt(sigma) (columns scaled) and R = sqrt(sigma) * Q^T (rows scaled), so that
    L @ R has exactly the singular values `sigma` (k = len(sigma)).  Also returns P, Q.
    """
    k = len(sigma)
    p = orthonormal_frame(rng, m, k)
    q = orthonormal_frame(rng, n, k)
    root = np.sqrt(np.asarray(sigma, dtype=np.float64))
    return p * root[None, :], root[:, None] * q.T, p, q


def perturbed_copies(rng: np.random.Generator, a: np.ndarray, b: np.ndarray, g: int,
                     std: float, first_exact: bool = False):
    """g float32 copies of (a, b), each with independent N(0, std^2) noise on every entry.
    first_exact keeps copy 0 unperturbed (config 1: copy 2 = copy 1 + noise)."""
    a32 = np.asarray(a, dtype=np.float32)
    b32 = np.asarray(b, dtype=np.float32)
    a_copies, b_copies = [], []
    for i in range(g):
        if first_exact and i == 0:
            a_copies.append(a32.copy())
            b_copies.append(b32.copy())
        else:
            a_copies.append(a32 + gaussian(rng, a32.shape, std))
            b_copies.append(b32 + gaussian(rng, b32.shape, std))
    return a_copies, b_copies


# ----------------------------------------------------------------------------------------
# the five benchmark configurations
# ----------------------------------------------------------------------------------------

# ViT-B/16 linear layers as (name, m = out features, n = in features)
VIT_B16_LINEARS = (("qkv", 2304, 768), ("proj", 768, 768), ("fc1", 3072, 768), ("fc2", 768, 3072))
VIT_B16_BLOCKS = 12
VIT_TOKENS = 197

# ResNet-50 convolutions as im2col GEMMs: (name, M rows, n = K of the GEMM, m = out channels, r)
RESNET50_CONVS = (
    ("conv3x3_256_14", 50176, 2304, 256, 64),
    ("conv1x1_1024_256_14", 50176, 1024, 256, 96),
    ("conv3x3_512_7", 12544, 4608, 512, 128),
)

CFG5_TAU_LITERAL = 0.1         # threshold as stated: keeps sigma >= 0.1 sigma_max
CFG5_TAU_GAP = 0.004704        # geometric middle of the planted gap at position 192
CFG5_K_IN = 384
CFG5_GAP_AT = 192
CFG5_G = 4
CFG5_NOISE_STD = 1e-3


def config1_dense(seed: int = 0):
    """Config 1 raw draws (float32): W 256x256 ~ N(0, var 1/256), X 64x256 ~ N(0,1),
    dY 64x256 ~ N(0,1), and the noise added to copy 2's factors (256x32 and 32x256,
    std 1e-3).  The factorisation of W is the caller's business."""
    rng = np.random.default_rng(seed)
    w = gaussian(rng, (256, 256), std=1.0 / 16.0)
    x = gaussian(rng, (64, 256))
    dy = gaussian(rng, (64, 256))
    noise_a = gaussian(rng, (256, 32), std=1e-3)
    noise_b = gaussian(rng, (32, 256), std=1e-3)
    return {"W": w, "X": x, "dY": dy, "noise_A": noise_a, "noise_B": noise_b,
            "r": 32, "tau": 0.1, "G": 2}


def lr_case(M: int, m: int, n: int, r: int, seed: int, relu_x: bool = False,
            dy_std: float = 1e-2, bf16: bool = True):
    """One factored-layer training step's inputs (configs 2-4).

    X  M x n ~ N(0,1) (relu_x: max(0, .), about half exact zeros, the im2col'd ResNet case)
    dY M x m ~ N(0, dy_std^2)
    A  m x r ~ N(0, 1/r), B r x n ~ N(0, 1/n): well-scaled factors, T and Y come out O(1).
    With bf16=True every array is rounded to bf16-representable float32 values, so the oracle
    and the GPU consume identical numbers.
    """
    rng = np.random.default_rng(seed)
    a = gaussian(rng, (m, r), std=r ** -0.5)
    b = gaussian(rng, (r, n), std=n ** -0.5)
    x = gaussian(rng, (M, n))
    if relu_x:
        np.maximum(x, 0.0, out=x)
    dy = gaussian(rng, (M, m), std=dy_std)
    if bf16:
        a, b, x, dy = (round_to_bf16(t) for t in (a, b, x, dy))
    return {"X": x, "dY": dy, "A": a, "B": b, "M": M, "m": m, "n": n, "r": r}


def config2(seed: int = 1):
    """ViT-B/16 MLP fc1 at batch 64 x 197 tokens, r = 192."""
    return lr_case(64 * VIT_TOKENS, 3072, 768, 192, seed)


def config3_cases():
    """(name, M, m, n, r, seed) for the 12 ViT-B/16 cases at batch 256 x 197 tokens."""
    out, idx = [], 0
    for r in (96, 192, 384):
        for name, m, n in VIT_B16_LINEARS:
            out.append((f"{name}_r{r}", 256 * VIT_TOKENS, m, n, r, 2 + idx))
            idx += 1
    return out


def config4_cases():
    """(name, M, m, n, r, seed) for the three ResNet-50 im2col cases at batch 256."""
    return [(name, M, m, n, r, 3 + 100 + i) for i, (name, M, n, m, r) in enumerate(RESNET50_CONVS)]


def conv_case(N: int, H: int, W: int, C: int, m: int, r: int, kh: int, kw: int, seed: int,
              relu_act: bool = True, dy_std: float = 1e-2, stride: int = 1):
    """One factored convolution's training-step inputs, channels last, all bf16-representable:
    act N x H x W x C ~ max(0, N(0,1)) (post-ReLU feature map; relu_act=False keeps the Gaussian),
    dY (N H' W') x m ~ N(0, dy_std^2) (H' = ceil(H / stride)), A m x r ~ N(0, 1/r), B r x (kh kw C) ~ N(0, 1/(kh kw C)),
    B's columns ordered tap-major: (ky kw + kx) C + c."""
    rng = np.random.default_rng(seed)
    n = kh * kw * C
    a = gaussian(rng, (m, r), std=r ** -0.5)
    b = gaussian(rng, (r, n), std=n ** -0.5)
    act = gaussian(rng, (N, H, W, C))
    if relu_act:
        np.maximum(act, 0.0, out=act)
    rows = N * (-(-H // stride)) * (-(-W // stride))      # output pixels: ceil(H / stride) x ceil(W / stride) per image
    dy = gaussian(rng, (rows, m), std=dy_std)
    a, b, act, dy = (round_to_bf16(t) for t in (a, b, act, dy))
    return {"act": act, "dY": dy, "A": a, "B": b, "N": N, "H": H, "W": W, "C": C, "m": m, "r": r,
            "kh": kh, "kw": kw, "stride": stride}


# ResNet-50 3x3 convolutions of config 4 in their native form: (name, N, H, W, C, m, r)
RESNET50_CONVS_NATIVE = (
    ("conv3x3_256_14", 256, 14, 14, 256, 256, 64),
    ("conv3x3_512_7", 256, 7, 7, 512, 512, 128),
)
# down-sampling convolutions of ResNet-50's stage 3 (28 x 28 -> 14 x 14): (name, N, H, W, C, m, r, kh, kw), stride 2
RESNET50_CONVS_STRIDED = (
    ("conv3x3_s2_128_28", 256, 28, 28, 128, 128, 64, 3, 3),
    ("conv1x1_s2_256_512_28", 256, 28, 28, 256, 512, 128, 1, 1),
)


def merge_layer(m: int, n: int, seed: int, k_in: int = CFG5_K_IN, g: int = CFG5_G,
                gap_at: int = CFG5_GAP_AT, noise_std: float = CFG5_NOISE_STD):
    """One layer of config 5: planted spectrum sigma_i = i^-0.8 with a 10x drop after
    position gap_at, carried as rank-k_in thin matrices, then g noisy float32 copies."""
    rng = np.random.default_rng(seed)
    sigma = power_law_spectrum(k_in, 0.8, gap_at, 0.1)
    left, right, _, _ = planted_factor_pair(rng, m, n, sigma)
    a_copies, b_copies = perturbed_copies(rng, left, right, g, noise_std)
    return {"A_copies": a_copies, "B_copies": b_copies, "sigma_planted": sigma,
            "m": m, "n": n, "k": k_in, "G": g}


def config5_layers(blocks: int = VIT_B16_BLOCKS):
    """(layer index, name, m, n, seed) for the full ViT-B/16 linear set: blocks x 4 layers."""
    out = []
    for blk in range(blocks):
        for name, m, n in VIT_B16_LINEARS:
            idx = len(out)
            out.append((idx, f"blk{blk}.{name}", m, n, 100 + idx))
    return out
