"""Parity of the HIP factored-layer step (lr_linear_fwd / lr_linear_bwd, through the C ABI)
against the CPU oracle, element by element on the same seeded inputs.

Tolerances (relative Frobenius error): 1e-2 for the bf16 path, 1e-4 for the fp32 path.
The benchmark configurations (2, all twelve cases of 3, the three of 4) are compared in full,
every element of T, Y, dX, dA, dB.  sampled_check evaluates the oracle on sampled rows (Y, dX are
row-independent) and on sampled columns of dA / rows of dB (each needs only one column of T / dT);
it serves the cases that only probe a launch shape."""
import gc

import numpy as np
import pytest
import torch

from oracle import ab_oracle as orc
from paper_2405_01067_amd import binding as abt
from paper_2405_01067_amd import inputs as gen

pytestmark = pytest.mark.gpu

TOL_BF16 = 1e-2
TOL_F32 = 1e-4


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def dev(x, dtype):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0").to(dtype)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def run_step(c, dtype, **bwd_kw):
    X, dY, A, B = (dev(c[k], dtype) for k in ("X", "dY", "A", "B"))
    Y, T = abt.lr_linear_fwd(X, A, B, save_T=True)
    dX, dA, dB = abt.lr_linear_bwd(dY, X, T, A, B, **bwd_kw)
    torch.cuda.synchronize()
    return X, dY, A, B, Y, T, dX, dA, dB


def check_full(c, dtype, tol):
    X, dY, A, B, Y, T, dX, dA, dB = run_step(c, dtype)
    Yo, To = orc.lr_linear_fwd(c["X"], c["A"], c["B"])
    dXo, dAo, dBo, _ = orc.lr_linear_bwd(c["dY"], c["X"], c["A"], c["B"])
    errs = {"T": rel(host(T), To), "Y": rel(host(Y), Yo), "dX": rel(host(dX), dXo),
            "dA": rel(host(dA), dAo), "dB": rel(host(dB), dBo)}
    assert all(e < tol for e in errs.values()), errs
    return errs


# ------------------------------------------------------------------ config 1 (fp32)

def test_config1_fp32_step():
    c1 = gen.config1_dense(0)
    A, B, _, _ = orc.ab_decomposition(c1["W"], k=c1["r"])
    c = {"X": c1["X"], "dY": c1["dY"], "A": A.astype(np.float32), "B": B.astype(np.float32)}
    check_full(c, torch.float32, TOL_F32)


@pytest.mark.parametrize("M,m,n,r", [(1, 8, 8, 1), (130, 200, 72, 24), (257, 129, 131, 33), (300, 64, 640, 160)])
def test_fp32_ragged_shapes(M, m, n, r):
    c = gen.lr_case(M, m, n, r, seed=M + r, bf16=False, dy_std=1.0)
    check_full(c, torch.float32, TOL_F32)


# ------------------------------------------------------------------ bf16: every rank, several tiles, ragged tail

@pytest.mark.parametrize("r", [32, 64, 96, 128, 160, 192, 224, 256, 288, 320, 352, 384])
def test_bf16_every_rank(r):
    c = gen.lr_case(M=128 * 2 + 45, m=192, n=320, r=r, seed=40 + r)
    check_full(c, torch.bfloat16, TOL_BF16)


@pytest.mark.parametrize("M", [1, 31, 32, 33, 127, 128, 129, 1000])
def test_bf16_row_counts(M):
    c = gen.lr_case(M=M, m=128, n=64, r=64, seed=900 + M)
    check_full(c, torch.bfloat16, TOL_BF16)


def test_bf16_many_splits_and_wide():
    # enough rows for several row splits of the dA / dB reduction, wide n and m
    c = gen.lr_case(M=5000, m=640, n=1216, r=96, seed=77)
    check_full(c, torch.bfloat16, TOL_BF16)


def test_bf16_relu_inputs_half_zero():
    c = gen.lr_case(M=777, m=256, n=1152, r=64, seed=78, relu_x=True)
    assert 0.45 < np.mean(c["X"] == 0) < 0.55
    check_full(c, torch.bfloat16, TOL_BF16)


# ------------------------------------------------------------------ largest sizes

@pytest.mark.parametrize("m,n", [(1 << 20, 64), (64, 1 << 20)], ids=["m=2^20", "n=2^20"])
def test_bf16_widest_factor_dimension(m, n):
    # the documented limit of m and n: row pitches of 2 MiB, 16384 contraction slabs or output tiles
    c = gen.lr_case(M=70, m=m, n=n, r=32, seed=4242)
    check_full(c, torch.bfloat16, TOL_BF16)


def test_bf16_row_offsets_beyond_4_GiB():
    # dY and Y of 5.2 GB each: byte offsets of rows pass 2^32.  The inputs are a seeded block of
    # 40000 rows repeated 32 times plus 37 more rows (the period is not a power of two, so a row
    # offset that wrapped at 2^32 bytes = 2^20 rows would land on different data); every output
    # row must then repeat with the same period, the first period is compared with the oracle
    # in full, and dA, dB are 32 times the block's plus those of the 37 extra rows.
    blk, reps, extra, m, n, r = 40000, 32, 37, 2048, 64, 64
    c = gen.lr_case(M=blk, m=m, n=n, r=r, seed=808)
    M = blk * reps + extra
    Xb, dYb = dev(c["X"], torch.bfloat16), dev(c["dY"], torch.bfloat16)
    X = torch.cat([Xb.repeat(reps, 1), Xb[:extra]])
    dY = torch.cat([dYb.repeat(reps, 1), dYb[:extra]])
    assert dY.numel() * 2 > (1 << 32) and tuple(dY.shape) == (M, m)
    A, B = dev(c["A"], torch.bfloat16), dev(c["B"], torch.bfloat16)
    Y, T = abt.lr_linear_fwd(X, A, B, save_T=True)
    dX, dA, dB = abt.lr_linear_bwd(dY, X, T, A, B)
    torch.cuda.synchronize()
    for out in (Y, T):
        first = out[:blk]
        for k in range(1, reps):
            assert torch.equal(out[k * blk:(k + 1) * blk], first), k
        assert torch.equal(out[reps * blk:], first[:extra])
    # dX: work-groups start the 32 contraction slabs of dT = dY A at different slabs, so the fp32
    # sums of two periods are taken in different orders and a few bf16 roundings fall the other way
    first = dX[:blk].float()
    for k in range(1, reps):
        d = (dX[k * blk:(k + 1) * blk].float() - first).norm() / first.norm()
        assert float(d) < 1e-3, (k, float(d))
    assert float((dX[reps * blk:].float() - first[:extra]).norm() / first[:extra].norm()) < 1e-3
    Yo, To = orc.lr_linear_fwd(c["X"], c["A"], c["B"])
    dXo, dAo, dBo, _ = orc.lr_linear_bwd(c["dY"], c["X"], c["A"], c["B"])
    _, dAe, dBe, _ = orc.lr_linear_bwd(c["dY"][:extra], c["X"][:extra], c["A"], c["B"])
    errs = {"Y": rel(host(Y[:blk]), Yo), "T": rel(host(T[:blk]), To), "dX": rel(host(dX[:blk]), dXo),
            "dA": rel(host(dA), reps * dAo + dAe), "dB": rel(host(dB), reps * dBo + dBe)}
    assert all(e < TOL_BF16 for e in errs.values()), errs


# ------------------------------------------------------------------ options

def test_bwd_skips_accumulate_recompute_and_determinism():
    c = gen.lr_case(M=700, m=256, n=192, r=96, seed=5)
    X, dY, A, B, Y, T, dX, dA, dB = run_step(c, torch.bfloat16)
    # frozen-factor variants: a group that trains A skips dB and vice versa
    dX2, dA2, dB2 = abt.lr_linear_bwd(dY, X, T, A, B, need_dB=False)
    assert dB2 is None and torch.equal(dA2, dA) and torch.equal(dX2, dX)
    dX3, dA3, dB3 = abt.lr_linear_bwd(dY, X, T, A, B, need_dA=False, need_dX=False)
    assert dA3 is None and dX3 is None and torch.equal(dB3, dB)
    # T = None: recomputed from X and B, same values the forward saved
    dX4, dA4, dB4 = abt.lr_linear_bwd(dY, X, None, A, B)
    assert torch.equal(dA4, dA) and torch.equal(dB4, dB) and torch.equal(dX4, dX)
    # accumulate adds into existing gradients
    accA, accB = dA.clone(), dB.clone()
    abt.lr_linear_bwd(dY, X, T, A, B, need_dX=False, dA=accA, dB=accB, accumulate=True)
    torch.cuda.synchronize()
    assert rel(host(accA), 2 * host(dA)) < 1e-6 and rel(host(accB), 2 * host(dB)) < 1e-6
    # forward without saving T gives the same Y
    Y2, T2 = abt.lr_linear_fwd(X, A, B, save_T=False)
    assert T2 is None and torch.equal(Y2, Y)
    # bit-identical reruns (fixed split and summation order)
    for _ in range(3):
        _, _, _, _, Yr, Tr, dXr, dAr, dBr = run_step(c, torch.bfloat16)
        assert torch.equal(Yr, Y) and torch.equal(dXr, dX) and torch.equal(dAr, dA) and torch.equal(dBr, dB)


def test_saved_T_is_what_stage_two_consumed():
    # T_save holds T rounded to bf16; Y must equal the oracle's second product applied to exactly it
    c = gen.lr_case(M=200, m=128, n=256, r=64, seed=9)
    X, dY, A, B, Y, T, *_ = run_step(c, torch.bfloat16)
    Y_from_T = host(T) @ c["A"].astype(np.float64).T
    assert rel(host(Y), Y_from_T) < 3e-3      # only the final bf16 rounding of Y remains


def test_fp32_options():
    c = gen.lr_case(M=150, m=96, n=80, r=16, seed=3, bf16=False, dy_std=1.0)
    X, dY, A, B, Y, T, dX, dA, dB = run_step(c, torch.float32)
    dX4, dA4, dB4 = abt.lr_linear_bwd(dY, X, None, A, B)
    torch.cuda.synchronize()
    assert torch.equal(dA4, dA) and torch.equal(dB4, dB)
    accA = dA.clone()
    abt.lr_linear_bwd(dY, X, T, A, B, need_dX=False, need_dB=False, dA=accA, accumulate=True)
    torch.cuda.synchronize()
    assert rel(host(accA), 2 * host(dA)) < 1e-6


# ------------------------------------------------------------------ full benchmark sizes

def sampled_check(c, tol, n_rows=384, n_cols=8, seed=0):
    M, m, n, r = c["M"], c["m"], c["n"], c["r"]
    X, dY, A, B, Y, T, dX, dA, dB = run_step(c, torch.bfloat16)
    rng = np.random.default_rng(seed)
    rows = np.unique(np.concatenate([np.arange(0, 40), np.arange(M - 70, M),
                                     rng.integers(0, M, size=n_rows)]))
    A64, B64 = c["A"].astype(np.float64), c["B"].astype(np.float64)
    Yo, To = orc.lr_linear_fwd(c["X"][rows], A64, B64)
    dXo, _, _, dTo = orc.lr_linear_bwd(c["dY"][rows], c["X"][rows], A64, B64)
    errs = {"T": rel(host(T[rows]), To), "Y": rel(host(Y[rows]), Yo), "dX": rel(host(dX[rows]), dXo)}
    # dA[:, j] = dY^T T[:, j] and dB[i, :] = dT[:, i]^T X need one column of T / dT over ALL rows:
    # the oracle's own products restricted to that column (B[j,:] resp. A[:, i])
    js = np.unique(np.concatenate([[0, r - 1], rng.integers(0, r, size=n_cols)]))
    # with A, B restricted to the columns/rows js, T and dT restrict the same way
    # (T[:, js] = X B[js]^T, dT[:, js] = dY A[:, js]), so the oracle returns dA[:, js] and dB[js, :]
    _, dA_cols, dB_rows, _ = orc.lr_linear_bwd(c["dY"], c["X"], A64[:, js], B64[js, :])
    errs["dA"] = rel(host(dA[:, js]), dA_cols)
    errs["dB"] = rel(host(dB[js, :]), dB_rows)
    assert all(e < tol for e in errs.values()), errs
    return errs


def test_config2_full_size():
    c = gen.config2()
    assert (c["M"], c["m"], c["n"], c["r"]) == (12608, 3072, 768, 192)
    errs = check_full(c, torch.bfloat16, TOL_BF16)
    print("config 2 errors:", errs)


@pytest.fixture
def release_memory():
    # the full-size cases hold a few GB each on the host (fp64 oracle results) and on the device
    yield
    gc.collect()
    torch.cuda.empty_cache()


@pytest.mark.parametrize("case", gen.config3_cases(), ids=lambda cs: cs[0])
def test_config3_full_size(case, release_memory):
    # all twelve ViT-B/16 cases, every element of T, Y, dX, dA, dB against the oracle
    name, M, m, n, r, seed = case
    assert M == 50432
    c = gen.lr_case(M, m, n, r, seed)
    errs = check_full(c, torch.bfloat16, TOL_BF16)
    print(name, errs)


@pytest.mark.parametrize("case", gen.config4_cases(), ids=lambda cs: cs[0])
def test_config4_full_size(case, release_memory):
    # the three ResNet-50 im2col cases (post-ReLU inputs), every element
    name, M, m, n, r, seed = case
    c = gen.lr_case(M, m, n, r, seed, relu_x=True)
    errs = check_full(c, torch.bfloat16, TOL_BF16)
    print(name, errs)


# ------------------------------------------------------------------ HIP graph capture

def test_step_replays_from_a_captured_graph():
    # The step only enqueues kernels on the caller's stream (no allocation, no synchronisation, no
    # memset), so a caller may capture it once and replay it.  Every replay, with the program's own
    # eager work and synchronisations in between and fresh inputs copied into the captured buffers,
    # must reproduce the eager result bit for bit.
    M, m, n, r = 1000, 256, 192, 96
    cases = [gen.lr_case(M=M, m=m, n=n, r=r, seed=600 + i) for i in range(3)]
    bf = torch.bfloat16
    X, dY, A, B = (torch.empty(s, dtype=bf, device="cuda:0") for s in ((M, n), (M, m), (m, r), (r, n)))
    Y = torch.empty((M, m), dtype=bf, device="cuda:0")
    T = torch.empty((M, r), dtype=bf, device="cuda:0")
    dX = torch.empty((M, n), dtype=bf, device="cuda:0")
    dA = torch.empty((m, r), dtype=torch.float32, device="cuda:0")
    dB = torch.empty((r, n), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(abt.load().lr_linear_bwd_workspace_bytes(M, m, n, r, abt.ABT_BF16), dtype=torch.uint8, device="cuda:0")

    def load_case(c):
        for dst, key in ((X, "X"), (dY, "dY"), (A, "A"), (B, "B")):
            dst.copy_(dev(c[key], bf))

    def step():
        abt.lr_linear_fwd(X, A, B, save_T=True, Y=Y, T=T, workspace=ws)
        abt.lr_linear_bwd(dY, X, T, A, B, dX=dX, dA=dA, dB=dB, workspace=ws)

    eager = []
    for c in cases:                      # eager results (also the warm-up that sets kernel attributes)
        load_case(c)
        step()
        torch.cuda.synchronize()
        eager.append([t.clone() for t in (Y, T, dX, dA, dB)])
    graph = torch.cuda.CUDAGraph()
    load_case(cases[0])
    torch.cuda.synchronize()
    with torch.cuda.graph(graph):
        step()
    for rep in range(2):
        for c, want in zip(cases, eager):
            load_case(c)
            for t in (Y, T, dX, dA, dB):
                t.fill_(7.0)             # eager work between the replays; stale results must not survive
            torch.cuda.synchronize()
            graph.replay()
            torch.cuda.synchronize()
            for got, ref in zip((Y, T, dX, dA, dB), want):
                assert torch.equal(got, ref)


# ------------------------------------------------------------------ 128-row work-groups (large batches)

@pytest.fixture
def tall_chain():
    prev = abt.set_chain_rows(128)
    yield
    abt.set_chain_rows(prev)


@pytest.mark.parametrize("r", [32, 64, 96, 128, 192, 256, 384])
@pytest.mark.parametrize("M", [1, 64, 129, 1000])
def test_bf16_tall_work_groups(tall_chain, M, r):
    # forced on small batches so that the oracle can check every element: one row, one row group,
    # a ragged second work-group, several work-groups; n, m give several slabs and a ragged last tile
    c = gen.lr_case(M=M, m=320, n=192, r=r, seed=7000 + M + r)
    check_full(c, torch.bfloat16, TOL_BF16)


@pytest.mark.parametrize("parts", [2, 3, 8])
@pytest.mark.parametrize("M,r", [(129, 192), (1000, 96), (300, 32), (200, 384), (257, 256)])
def test_bf16_tall_work_groups_with_column_parts(tall_chain, M, r, parts):
    # several work-groups per row block, each doing a share of the output tiles (m = 448: four
    # tiles, the last ragged; 8 parts are capped to 4)
    prev = abt.set_chain_parts(parts)
    try:
        c = gen.lr_case(M=M, m=448, n=192, r=r, seed=7100 + M + r + parts)
        check_full(c, torch.bfloat16, TOL_BF16)
    finally:
        abt.set_chain_parts(prev)


@pytest.mark.parametrize("M", [64 * 259, 64 * 258 + 17])
def test_bf16_last_round_shared_by_output_tiles(M):
    # more than one round of 64-row work-groups and a last round of three row blocks: those are
    # split four ways by output tiles (m = 512: four tiles) and repeat the single stage-1 slab
    prev = abt.set_chain_rows(64)
    try:
        c = gen.lr_case(M=M, m=512, n=64, r=32, seed=7300 + M % 97)
        check_full(c, torch.bfloat16, TOL_BF16)
    finally:
        abt.set_chain_rows(prev)


@pytest.mark.parametrize("r", [256, 384])
def test_bf16_wide_rank_last_round_shared_by_output_tiles(tall_chain, r):
    # 259 row blocks of 128 rows: the three of the last round are split four ways by output tiles
    # (m = 512: four tiles) in the kernel of eight equal waves; the last block is ragged
    c = gen.lr_case(M=128 * 258 + 17, m=512, n=64, r=r, seed=7400 + r)
    check_full(c, torch.bfloat16, TOL_BF16)


@pytest.mark.parametrize("r", [192, 256, 384])
def test_bf16_wide_rank_many_blocks_outputs_below_the_streaming_size(tall_chain, r):
    # 300 row blocks (more than one round of the chip, the last 44 shared by output tiles), four output
    # tiles (the last ragged), outputs just under the size from which they are stored with the
    # non-temporal hint: the finished tiles leave by plain stores while the next slabs are loading
    c = gen.lr_case(M=128 * 300, m=448, n=64, r=r, seed=7500 + r)
    assert c["X"].shape[0] * (448 + r) * 2 < 64 << 20
    check_full(c, torch.bfloat16, TOL_BF16)


def test_bf16_tall_work_groups_chosen_for_large_batches():
    # above one round of 64-row work-groups the library picks the 128-row kernel by itself; the
    # result must agree with the 64-row kernel's up to summation order, and with the oracle on samples
    c = gen.lr_case(M=20000, m=768, n=768, r=192, seed=31)
    sampled_check(c, TOL_BF16, seed=1)
    X, dY, A, B, Y, T, dX, dA, dB = run_step(c, torch.bfloat16)
    prev = abt.set_chain_rows(64)
    try:
        _, _, _, _, Y64, T64, dX64, dA64, dB64 = run_step(c, torch.bfloat16)
    finally:
        abt.set_chain_rows(prev)
    for a, b in ((Y, Y64), (T, T64), (dX, dX64), (dA, dA64), (dB, dB64)):
        assert rel(host(a), host(b)) < 2e-3
