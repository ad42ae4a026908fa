"""lr_linear_bwd_static (the backward that allocates nothing and keeps its workspace in a static
device array of the library) against lr_linear_bwd on the same inputs, through the C ABI.

Both run the same kernels on the same workspace layout, so the gradients must agree bit for bit
(well inside the bf16 tolerance of the parity tests); the first call is also compared with the
oracle.  The second call is smaller than the first: whatever the first left in the array must
not reach the second's results."""
import numpy as np
import pytest
import torch

from oracle import ab_oracle as orc
from paper_2405_01067_amd import binding as abt
from paper_2405_01067_amd import inputs as gen

pytestmark = pytest.mark.gpu

TOL_BF16 = 1e-2


def rel(a, b):
    a = np.asarray(a, dtype=np.float64)
    b = np.asarray(b, dtype=np.float64)
    return float(np.linalg.norm(a - b) / max(np.linalg.norm(b), 1e-300))


def host(t):
    return t.detach().float().cpu().numpy().astype(np.float64)


def both_paths(c, dtype, with_T):
    dev = lambda k: torch.from_numpy(np.ascontiguousarray(c[k])).to("cuda:0").to(dtype)
    X, dY, A, B = dev("X"), dev("dY"), dev("A"), dev("B")
    M, n = X.shape
    m, r = A.shape
    T = abt.lr_linear_fwd(X, A, B, save_T=True)[1] if with_T else None
    ref = abt.lr_linear_bwd(dY, X, T, A, B)
    # outputs of the allocation-free call exist before it; poisoned so that a skipped write shows
    dX = torch.full((M, n), 7.0, dtype=dtype, device="cuda:0")
    dA = torch.full((m, r), 7.0, dtype=torch.float32, device="cuda:0")
    dB = torch.full((r, n), 7.0, dtype=torch.float32, device="cuda:0")
    torch.cuda.synchronize()
    abt.lr_linear_bwd_static(dY, X, T, A, B, dX=dX, dA=dA, dB=dB)
    torch.cuda.synchronize()
    return ref, (dX, dA, dB)


def test_static_scratch_backward_matches_the_workspace_backward():
    lib = abt.load()
    big = gen.lr_case(M=3000, m=640, n=448, r=96, seed=5151)
    small = gen.lr_case(M=301, m=192, n=128, r=64, seed=5152)
    assert lib.lr_linear_bwd_workspace_bytes(3000, 640, 448, 96, abt.ABT_BF16) > \
        lib.lr_linear_bwd_workspace_bytes(301, 192, 128, 64, abt.ABT_BF16) > 0
    for c, with_T in ((big, True), (small, False)):
        ref, got = both_paths(c, torch.bfloat16, with_T)
        for a, b, nm in zip(got, ref, ("dX", "dA", "dB")):
            assert torch.equal(a, b), nm
        dXo, dAo, dBo, _ = orc.lr_linear_bwd(c["dY"], c["X"], c["A"], c["B"])
        errs = {"dX": rel(host(got[0]), dXo), "dA": rel(host(got[1]), dAo), "dB": rel(host(got[2]), dBo)}
        assert all(e < TOL_BF16 for e in errs.values()), errs


def test_static_scratch_backward_fp32_and_accumulate():
    c = gen.lr_case(M=260, m=96, n=80, r=16, seed=5153, bf16=False, dy_std=1.0)
    ref, got = both_paths(c, torch.float32, True)
    for a, b in zip(got, ref):
        assert torch.equal(a, b)
    # accumulate adds into the caller's gradients, skipped outputs stay untouched
    dev = lambda k: torch.from_numpy(np.ascontiguousarray(c[k])).to("cuda:0")
    accA = ref[1].clone()
    abt.lr_linear_bwd_static(dev("dY"), dev("X"), None, dev("A"), dev("B"), dA=accA, accumulate=True)
    torch.cuda.synchronize()
    assert rel(host(accA), 2 * host(ref[1])) < 1e-6


def test_static_scratch_backward_rejects_shapes_beyond_its_array():
    lib = abt.load()
    M, m, n, r = 50432, 3072, 768, 384
    assert lib.lr_linear_bwd_workspace_bytes(M, m, n, r, abt.ABT_BF16) > abt.STATIC_SCRATCH_BYTES
    bf = torch.bfloat16
    # the shape is refused before any pointer is used: small stand-in tensors are never touched
    t = torch.zeros(64, dtype=bf, device="cuda:0")
    f = torch.zeros(64, dtype=torch.float32, device="cuda:0")
    st = lib.lr_linear_bwd_static(t.data_ptr(), t.data_ptr(), None, t.data_ptr(), t.data_ptr(),
                                  t.data_ptr(), f.data_ptr(), f.data_ptr(), M, m, n, r, abt.ABT_BF16, 0, None)
    assert st == abt.ABT_ETOOLARGE
    assert "static scratch" in abt.status_string(st)
    torch.cuda.synchronize()
    assert not t.any() and not f.any()
