"""Parity of the group-training step on the GPU (ab_adamw_step, the frozen-factor backward,
ab_reconstruct, through the C ABI) against the CPU oracle, element by element.

Optimiser tolerances.  The kernel evaluates the update in fp32 with IEEE division and square
root; the oracle in fp64 from the same fp32 state.  With E = beta1 |m| + (1 - beta1) |g| (the
magnitude the new first moment is rounded at) and U = E / (1 - beta1^t) / (sqrt(vh) + eps):
    |dm| <= 3e-7 E,   |dv| <= 4e-7 v' (all terms of v' are positive),
    |dtheta| <= 1.2e-7 |theta'| + eta * 2e-6 * (U + lambda |theta|)
(a handful of fp32 roundings each: half an ulp is 6e-8).  The bf16 copy must be the
round-to-nearest-even image of the fp32 parameter the kernel wrote, bit for bit.

A gradient that the bf16 layer kernels computed differs from the fp64 one by bf16 rounding, and
Adam's first steps depend on a gradient's sign: an entry whose gradient is near zero may move
the other way.  The composed step is therefore checked link by link: the gradients against the
oracle in the Frobenius norm (the layer tests' bar), then the update against the oracle's update
of the same gradient values."""
import numpy as np
import pytest
import torch

from oracle import ab_oracle as orc
from paper_2405_01067_amd import binding as abt
from paper_2405_01067_amd import inputs as gen

pytestmark = pytest.mark.gpu

HYPER = dict(beta1=0.9, beta2=0.999, eps=1e-8, weight_decay=0.01)


def dev(x, dtype=torch.float32):
    return torch.from_numpy(np.ascontiguousarray(x)).to("cuda:0").to(dtype)


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def bf16_bits(t):
    return t.view(torch.int16).cpu().numpy().view(np.uint16)


def check_update(before, after, t, lr, lr_scale, hyper, bf16=None):
    """before/after: (theta, g, m, v) float32 host arrays around one kernel step."""
    th0, g, m0, v0 = (np.asarray(x, dtype=np.float64) for x in before)
    th1, m1, v1 = (np.asarray(x, dtype=np.float64) for x in after)
    tho, mo, vo = orc.adamw_step(th0, g, m0, v0, t, lr, hyper["beta1"], hyper["beta2"], hyper["eps"],
                                 hyper["weight_decay"], lr_scale=lr_scale)
    b1, b2 = hyper["beta1"], hyper["beta2"]
    E = b1 * np.abs(m0) + (1 - b1) * np.abs(g)
    assert np.all(np.abs(m1 - mo) <= 3e-7 * E + 1e-45), float(np.max(np.abs(m1 - mo) - 3e-7 * E))
    assert np.all(np.abs(v1 - vo) <= 4e-7 * vo + 1e-45)
    U = E / (1 - b1 ** t) / (np.sqrt(vo / (1 - b2 ** t)) + hyper["eps"])
    eta = lr * lr_scale
    bound = 1.2e-7 * np.abs(tho) + eta * 2e-6 * (U + hyper["weight_decay"] * np.abs(th0)) + 1e-45
    err = np.abs(th1 - tho)
    assert np.all(err <= bound), (float(err.max()), int(np.argmax(err - bound)))
    if bf16 is not None:
        assert np.array_equal(bf16, gen.f32_to_bf16_bits(np.asarray(after[0], dtype=np.float32)))


def make_state(rng, count, started=True):
    th = gen.gaussian(rng, (count,), std=0.05)
    g = gen.gaussian(rng, (count,)) * np.float32(10.0) ** rng.integers(-5, 2, count).astype(np.float32)
    if started:
        m = gen.gaussian(rng, (count,), std=0.1)
        v = np.square(gen.gaussian(rng, (count,), std=0.1))
    else:
        m = np.zeros(count, np.float32)
        v = np.zeros(count, np.float32)
    return th, g, m, v


@pytest.mark.parametrize("count", [1, 3, 4, 5, 4095, 4096, 4097, 3 * 4096 + 7, 768 * 192])
@pytest.mark.parametrize("with_bf16", [False, True])
def test_adamw_one_tensor(count, with_bf16):
    rng = np.random.default_rng(1000 + count)
    state = make_state(rng, count)
    th, g, m, v = (dev(x) for x in state)
    pb = torch.full((count,), 7.0, dtype=torch.bfloat16, device="cuda:0") if with_bf16 else None
    g_before = g.clone()
    abt.ab_adamw_step([dict(param=th, grad=g, exp_avg=m, exp_avg_sq=v, param_bf16=pb)], step=5, lr=1e-3,
                      lr_scale=0.5, **HYPER)
    torch.cuda.synchronize()
    assert torch.equal(g, g_before)
    check_update(state, (th.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()), 5, 1e-3, 0.5, HYPER,
                 bf16_bits(pb) if with_bf16 else None)


def test_adamw_many_tensors_two_launches_and_empty_ones():
    # 60 tensors of unequal sizes (more than one launch holds), two of them empty, every third
    # with a bf16 copy; guard elements around every buffer must stay untouched
    rng = np.random.default_rng(77)
    counts = [int(c) for c in rng.integers(1, 20000, 60)]
    counts[7] = 0
    counts[48] = 0
    items, states = [], []
    for i, c in enumerate(counts):
        st = make_state(rng, c, started=(i % 2 == 0))
        bufs = []
        for x in st:
            b = torch.full((c + 8,), -3.0, dtype=torch.float32, device="cuda:0")
            b[4:4 + c] = dev(x)
            bufs.append(b)
        pbuf = torch.full((c + 16,), -3.0, dtype=torch.bfloat16, device="cuda:0") if i % 3 == 0 else None
        d = dict(param=bufs[0][4:4 + c], grad=bufs[1][4:4 + c], exp_avg=bufs[2][4:4 + c], exp_avg_sq=bufs[3][4:4 + c],
                 param_bf16=pbuf[8:8 + c] if pbuf is not None else None)
        items.append((d, bufs, pbuf))
        states.append(st)
    abt.ab_adamw_step([d for d, _, _ in items], step=1, lr=3e-3, lr_scale=1.0, **HYPER)
    torch.cuda.synchronize()
    for (d, bufs, pbuf), st, c in zip(items, states, counts):
        for b in bufs:
            assert torch.all(b[:4] == -3.0) and torch.all(b[4 + c:] == -3.0)
        if pbuf is not None:
            assert torch.all(pbuf[:8] == -3.0) and torch.all(pbuf[8 + c:] == -3.0)
        if c == 0:
            continue
        check_update(st, tuple(d[k].cpu().numpy() for k in ("param", "exp_avg", "exp_avg_sq")), 1, 3e-3, 1.0, HYPER,
                     bf16_bits(d["param_bf16"]) if pbuf is not None else None)


def test_adamw_trajectory_with_rebound_and_determinism():
    # twenty steps from a zero state with a fresh gradient each step and the rebound factor of an
    # eight-step climb; each step is checked against the oracle's step from the same state, the end
    # point against the oracle's own fp64 trajectory
    rng = np.random.default_rng(9)
    count = 50000
    th0 = gen.gaussian(rng, (count,), std=0.05)
    hyper = dict(beta1=0.8, beta2=0.95, eps=1e-6, weight_decay=0.1)
    th, m, v = dev(th0), dev(np.zeros(count, np.float32)), dev(np.zeros(count, np.float32))
    th_b, m_b, v_b = th.clone(), m.clone(), v.clone()
    g_buf = torch.empty(count, dtype=torch.float32, device="cuda:0")
    plan_b = abt.AdamwPlan([dict(param=th_b, grad=g_buf, exp_avg=m_b, exp_avg_sq=v_b)])   # table built once
    o_th, o_m, o_v = th0.astype(np.float64), np.zeros(count), np.zeros(count)
    for t in range(1, 21):
        g_np = gen.gaussian(rng, (count,), std=(0.1 if t % 3 else 5.0))
        g = dev(g_np)
        scale = abt.lr_rebound_scale(t - 1, 8)
        assert scale == pytest.approx(orc.lr_rebound_scale(t - 1, 8))
        before = (th.cpu().numpy(), g_np, m.cpu().numpy(), v.cpu().numpy())
        abt.ab_adamw_step([dict(param=th, grad=g, exp_avg=m, exp_avg_sq=v)], step=t, lr=2e-3, lr_scale=scale, **hyper)
        g_buf.copy_(g)
        abt.ab_adamw_step(plan_b, step=t, lr=2e-3, lr_scale=scale, **hyper)
        torch.cuda.synchronize()
        check_update(before, (th.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()), t, 2e-3, scale, hyper)
        o_th, o_m, o_v = orc.adamw_step(o_th, g_np, o_m, o_v, t, 2e-3, lr_scale=scale, **hyper)
    assert torch.equal(th, th_b) and torch.equal(m, m_b) and torch.equal(v, v_b)
    # twenty steps of at most eta each: the trajectories stay within a small fraction of one step
    assert np.max(np.abs(host(th) - o_th)) < 2e-3 * 1e-3
    assert rel(host(m), o_m) < 1e-6 and rel(host(v), o_v) < 1e-6


def test_adamw_large_step_count_bias_corrections():
    # after many steps the corrections are close to one; at step 1 they are 1/(1-beta)
    rng = np.random.default_rng(4)
    for t in (1, 2, 1000, 10 ** 6):
        state = make_state(rng, 5000)
        th, g, m, v = (dev(x) for x in state)
        abt.ab_adamw_step([dict(param=th, grad=g, exp_avg=m, exp_avg_sq=v)], step=t, lr=1e-2, **HYPER)
        torch.cuda.synchronize()
        check_update(state, (th.cpu().numpy(), m.cpu().numpy(), v.cpu().numpy()), t, 1e-2, 1.0, HYPER)


@pytest.mark.parametrize("target", ["A", "B"])
@pytest.mark.parametrize("dtype", [torch.bfloat16, torch.float32])
def test_group_step_frozen_factor(target, dtype):
    bf = dtype == torch.bfloat16
    c = gen.lr_case(M=700, m=256, n=192, r=64, seed=31, bf16=bf) if bf else \
        gen.lr_case(M=150, m=70, n=50, r=12, seed=32, bf16=False)
    tol = 1e-2 if bf else 1e-4
    X, dY, A, B = (dev(c[k], dtype) for k in ("X", "dY", "A", "B"))
    master = dev(c[target])                                      # fp32 master copy of the trained factor
    frozen_before = (B if target == "A" else A).clone()
    Y, T = abt.lr_linear_fwd(X, A, B, save_T=True)
    dX, dA, dB = abt.lr_linear_bwd(dY, X, T, A, B, need_dA=(target == "A"), need_dB=(target == "B"))
    assert (dB if target == "A" else dA) is None
    grad = dA if target == "A" else dB
    ref = orc.group_train_step(c["X"], c["dY"], c["A"], c["B"], target,
                               (np.zeros_like(c[target]), np.zeros_like(c[target])), 1, 1e-3, **HYPER)
    assert rel(host(Y), ref["Y"]) < tol and rel(host(dX), ref["dX"]) < tol and rel(host(grad), ref["grad"]) < tol
    m = torch.zeros_like(master)
    v = torch.zeros_like(master)
    trained = A if target == "A" else B
    g_np = grad.cpu().numpy().copy()
    before = (master.cpu().numpy().ravel(), g_np.ravel(), m.cpu().numpy().ravel(), v.cpu().numpy().ravel())
    abt.ab_adamw_step([dict(param=master, grad=grad, exp_avg=m, exp_avg_sq=v, param_bf16=trained if bf else None)],
                      step=1, lr=1e-3, **HYPER)
    torch.cuda.synchronize()
    check_update(before, tuple(x.cpu().numpy().ravel() for x in (master, m, v)), 1, 1e-3, 1.0, HYPER,
                 bf16_bits(trained).ravel() if bf else None)
    assert torch.equal(B if target == "A" else A, frozen_before)
    # the next forward reads the updated factor: it must match the oracle's forward of that factor
    if bf:
        Y2, _ = abt.lr_linear_fwd(X, A, B, save_T=False)
    else:
        Y2, _ = abt.lr_linear_fwd(X, master if target == "A" else A, master if target == "B" else B, save_T=False)
    newA = host(A) if bf else (host(master) if target == "A" else c["A"])
    newB = host(B) if bf else (host(master) if target == "B" else c["B"])
    assert rel(host(Y2), orc.lr_linear_fwd(c["X"], newA, newB)[0]) < tol


def test_group_step_all_vit_factors_full_size():
    # the trained factors of all 48 ViT-B/16 layers at rank 192 in one call (A for half of the
    # layers, B for the others, as the two kinds of groups hold them); sampled elements
    rng = np.random.default_rng(12)
    items, keep = [], []
    for blk in range(gen.VIT_B16_BLOCKS):
        for li, (name, mm, nn) in enumerate(gen.VIT_B16_LINEARS):
            shape = (mm, 192) if (blk + li) % 2 == 0 else (192, nn)
            cnt = shape[0] * shape[1]
            th = torch.randn(cnt, device="cuda:0") * 0.05
            g = torch.randn(cnt, device="cuda:0") * 1e-3
            m = torch.randn(cnt, device="cuda:0") * 1e-3
            v = torch.rand(cnt, device="cuda:0") * 1e-6
            pb = torch.empty(cnt, dtype=torch.bfloat16, device="cuda:0")
            idx = torch.from_numpy(rng.integers(0, cnt, 4000)).to("cuda:0")
            idx[:3] = torch.tensor([0, cnt - 1, cnt // 2])
            keep.append((idx, tuple(x[idx].cpu().numpy() for x in (th, g, m, v))))
            items.append(dict(param=th, grad=g, exp_avg=m, exp_avg_sq=v, param_bf16=pb))
    abt.ab_adamw_step(items, step=40, lr=1e-3, lr_scale=0.7, **HYPER)
    torch.cuda.synchronize()
    for d, (idx, before) in zip(items, keep):
        after = tuple(d[k][idx].cpu().numpy() for k in ("param", "exp_avg", "exp_avg_sq"))
        check_update(before, after, 40, 1e-3, 0.7, HYPER, bf16_bits(d["param_bf16"][idx].contiguous()))


@pytest.mark.parametrize("m,n,k", [(70, 50, 7), (256, 256, 32), (3072, 768, 192), (768, 3072, 384)])
def test_reconstruct(m, n, k):
    rng = np.random.default_rng(m + n + k)
    A = gen.gaussian(rng, (m, k), std=k ** -0.5)
    B = gen.gaussian(rng, (k, n))
    W = abt.ab_reconstruct(dev(A), dev(B))
    torch.cuda.synchronize()
    assert rel(host(W), orc.reconstruct(A, B)) < 1e-4


# ------------------------------------------------------------------ G groups per launch

@pytest.mark.parametrize("dtype,shape", [(torch.bfloat16, (700, 256, 192, 64)), (torch.bfloat16, (1500, 320, 128, 192)),
                                          (torch.float32, (150, 70, 50, 12))],
                         ids=["bf16-r64", "bf16-r192", "fp32"])
def test_grouped_step_matches_the_oracle_and_the_single_group_calls(dtype, shape):
    grouped_step_check(dtype, shape)


@pytest.mark.parametrize("r", [256, 384])
def test_grouped_step_wide_rank_128_row_work_groups(r):
    # the kernel of eight equal waves (plain 128-row launches at r = 256, 384), four groups per launch,
    # a ragged last row block and a ragged last output tile
    prev = abt.set_chain_rows(128)
    try:
        grouped_step_check(torch.bfloat16, (700, 320, 192, r))
    finally:
        abt.set_chain_rows(prev)


def grouped_step_check(dtype, shape):
    """Four groups of one shape, each with its own batch and its own factors, two training A and two
    training B (one of the B groups without dX, one A group without a saved T): one grouped forward
    and one grouped backward against the oracle, element by element, and against the single-group
    calls (same kernels; the factor gradients may differ in summation order only)."""
    M, m, n, r = shape
    bf = dtype == torch.bfloat16
    tol = 1e-2 if bf else 1e-4
    G = 4
    cases = [gen.lr_case(M=M, m=m, n=n, r=r, seed=500 + g, bf16=bf, dy_std=1e-2 if bf else 1.0) for g in range(G)]
    groups = [dict(X=dev(c["X"], dtype), A=dev(c["A"], dtype), B=dev(c["B"], dtype), dY=dev(c["dY"], dtype)) for c in cases]
    fwd = abt.lr_linear_fwd_grouped(groups)
    for g, (Y, T) in enumerate(fwd):
        groups[g]["T"] = T
    plan = [dict(dX=True, dA=True), dict(dX=True, dA=True, T=None), dict(dX=True, dB=True), dict(dB=True)]
    for g in range(G):
        groups[g].update(plan[g])
    bwd = abt.lr_linear_bwd_grouped(groups)
    again = abt.lr_linear_bwd_grouped(groups)
    torch.cuda.synchronize()
    for g, c in enumerate(cases):
        Yo, To = orc.lr_linear_fwd(c["X"], c["A"], c["B"])
        dXo, dAo, dBo, _ = orc.lr_linear_bwd(c["dY"], c["X"], c["A"], c["B"])
        Y, T = fwd[g]
        dX, dA, dB = bwd[g]
        assert rel(host(Y), Yo) < tol and rel(host(T), To) < tol
        assert (dX is None) == ("dX" not in plan[g]) and (dA is None) == ("dA" not in plan[g]) and (dB is None) == ("dB" not in plan[g])
        Y1, T1 = abt.lr_linear_fwd(groups[g]["X"], groups[g]["A"], groups[g]["B"], save_T=True)
        assert rel(host(Y), host(Y1)) < (2e-3 if bf else 1e-6)
        s_dX, s_dA, s_dB = abt.lr_linear_bwd(groups[g]["dY"], groups[g]["X"], T1, groups[g]["A"], groups[g]["B"],
                                             need_dX=dX is not None, need_dA=dA is not None, need_dB=dB is not None)
        for got, ref, single, name in ((dX, dXo, s_dX, "dX"), (dA, dAo, s_dA, "dA"), (dB, dBo, s_dB, "dB")):
            if got is None:
                continue
            assert rel(host(got), ref) < tol, (g, name, rel(host(got), ref))
            assert rel(host(got), host(single)) < (2e-3 if bf else 1e-5), (g, name)
        for a, b in zip(bwd[g], again[g]):
            assert (a is None and b is None) or torch.equal(a, b)      # fixed split and summation order


def test_grouped_backward_accumulates_and_fills_the_chip_shape():
    """config-2 shape, four groups: accumulate adds into the gradients; the 128-row kernel is the
    one chosen for 4 x 197 row blocks."""
    c = gen.lr_case(M=12608, m=3072, n=768, r=192, seed=77)
    bf = torch.bfloat16
    base = dict(X=dev(c["X"], bf), A=dev(c["A"], bf), B=dev(c["B"], bf), dY=dev(c["dY"], bf))
    groups = [dict(base) for _ in range(4)]
    for g, (Y, T) in enumerate(abt.lr_linear_fwd_grouped(groups)):
        groups[g]["T"] = T
    for g in range(4):
        groups[g].update(dict(dX=True, dA=True) if g < 2 else dict(dX=True, dB=True))
    outs = abt.lr_linear_bwd_grouped(groups)
    torch.cuda.synchronize()
    dXo, dAo, dBo, _ = orc.lr_linear_bwd(c["dY"], c["X"], c["A"], c["B"])
    for g, (dX, dA, dB) in enumerate(outs):
        assert rel(host(dX), dXo) < 1e-2
        assert rel(host(dA if g < 2 else dB), dAo if g < 2 else dBo) < 1e-2
    # the groups hold the same inputs here, so they must agree bit for bit among themselves
    assert torch.equal(outs[0][0], outs[3][0]) and torch.equal(outs[0][1], outs[1][1]) and torch.equal(outs[2][2], outs[3][2])
    acc = [dict(g) for g in groups]
    for g in range(4):
        key = "dA" if g < 2 else "dB"
        acc[g][key] = outs[g][1 if g < 2 else 2].clone()
        acc[g]["dX"] = None
    abt.lr_linear_bwd_grouped(acc, accumulate=True)
    torch.cuda.synchronize()
    for g in range(4):
        key = "dA" if g < 2 else "dB"
        assert rel(host(acc[g][key]), 2 * host(outs[g][1 if g < 2 else 2])) < 1e-6
