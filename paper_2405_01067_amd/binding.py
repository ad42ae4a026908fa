"""Thin ctypes binding of libabtrain.so: same names as the C ABI in include/abtrain.h,
argument marshalling only.  torch supplies device memory and the current stream; every step
of the computation runs in the library's HIP kernels.  There is no fallback: if the library
is missing or a call returns an error, this raises.
"""
from __future__ import annotations

import ctypes
import os
from typing import List, Optional, Sequence

ABT_F32, ABT_BF16 = 0, 1
ABT_ENOCONV = -6
ABT_ETOOLARGE = -9

_LIB_PATH = os.path.join(os.path.dirname(os.path.abspath(__file__)), "lib", "libabtrain.so")
_lib = None

EXPORTS = (
    "abt_status_string", "abt_set_jacobi_max_sweeps", "abt_set_merge_groups", "abt_set_merge_stage_timing",
    "ab_merge_stage_ms", "abt_set_chain_rows", "abt_set_chain_parts",
    "lr_linear_fwd", "lr_linear_fwd_workspace_bytes",
    "lr_linear_bwd", "lr_linear_bwd_workspace_bytes", "lr_linear_bwd_static",
    "lr_linear_fwd_grouped", "lr_linear_bwd_grouped", "lr_linear_bwd_grouped_workspace_bytes",
    "ab_merge", "ab_merge_workspace_bytes",
    "ab_merge_batched", "ab_merge_batched_workspace_bytes", "ab_merge_info",
    "ab_factorize", "ab_factorize_workspace_bytes",
    "ab_factorize_batched", "ab_factorize_batched_workspace_bytes",
    "ab_adamw_step", "ab_lr_rebound_scale", "ab_reconstruct",
    "lr_conv_fwd", "lr_conv_bwd", "lr_conv_bwd_workspace_bytes",
)


class AbtError(RuntimeError):
    pass


class FactorizeDesc(ctypes.Structure):
    _fields_ = [("W", ctypes.c_void_p), ("m", ctypes.c_int64), ("n", ctypes.c_int64),
                ("tau", ctypes.c_float), ("k_fixed", ctypes.c_int64),
                ("A_out", ctypes.c_void_p), ("B_out", ctypes.c_void_p), ("S_out", ctypes.c_void_p),
                ("k_out", ctypes.c_void_p), ("k_cap", ctypes.c_int64)]


class ConvGeom(ctypes.Structure):
    _fields_ = [("N", ctypes.c_int64), ("H", ctypes.c_int64), ("W", ctypes.c_int64), ("C", ctypes.c_int64),
                ("kh", ctypes.c_int32), ("kw", ctypes.c_int32), ("stride", ctypes.c_int32), ("reserved", ctypes.c_int32)]

    def __init__(self, N=0, H=0, W=0, C=0, kh=1, kw=1, stride=1):
        super().__init__(N, H, W, C, kh, kw, stride, 0)


class AdamwTensor(ctypes.Structure):
    _fields_ = [("param", ctypes.c_void_p), ("grad", ctypes.c_void_p), ("exp_avg", ctypes.c_void_p),
                ("exp_avg_sq", ctypes.c_void_p), ("param_bf16", ctypes.c_void_p), ("count", ctypes.c_int64)]


class LrGroup(ctypes.Structure):
    """abt_lr_group"""
    _fields_ = [(name, ctypes.c_void_p) for name in ("X", "A", "B", "Y", "T_save", "dY", "T", "dX", "dA", "dB")]


MAX_GROUPS = 8   # ABT_MAX_GROUPS


class MergeDesc(ctypes.Structure):
    """abt_merge_desc"""
    _fields_ = [
        ("A_copies", ctypes.POINTER(ctypes.c_void_p)),
        ("B_copies", ctypes.POINTER(ctypes.c_void_p)),
        ("G", ctypes.c_int32),
        ("mode", ctypes.c_int32),
        ("m", ctypes.c_int64), ("n", ctypes.c_int64), ("k", ctypes.c_int64),
        ("tau", ctypes.c_float),
        ("k_fixed", ctypes.c_int64),
        ("A_out", ctypes.c_void_p), ("B_out", ctypes.c_void_p), ("S_out", ctypes.c_void_p),
        ("k_out", ctypes.c_void_p),
        ("k_cap", ctypes.c_int64),
        ("W_out", ctypes.c_void_p),
    ]


def load():
    """dlopen the library and declare the prototypes.  Needs no GPU."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise AbtError(f"{_LIB_PATH} is missing: run `python __graft_entry__.py` (build) first")
    lib = ctypes.CDLL(_LIB_PATH)
    for name in EXPORTS:
        if not hasattr(lib, name):
            raise AbtError(f"libabtrain.so does not export {name}")
    i64, vp, sz, ci = ctypes.c_int64, ctypes.c_void_p, ctypes.c_size_t, ctypes.c_int
    lib.abt_status_string.restype = ctypes.c_char_p
    lib.abt_status_string.argtypes = [ci]
    lib.abt_set_chain_rows.restype = ci
    lib.abt_set_chain_rows.argtypes = [ci]
    lib.abt_set_chain_parts.restype = ci
    lib.abt_set_chain_parts.argtypes = [ci]
    lib.abt_set_jacobi_max_sweeps.restype = ci
    lib.abt_set_jacobi_max_sweeps.argtypes = [ci]
    lib.abt_set_merge_groups.restype = ci
    lib.abt_set_merge_groups.argtypes = [ci]
    lib.abt_set_merge_stage_timing.restype = ci
    lib.abt_set_merge_stage_timing.argtypes = [ci]
    lib.ab_merge_stage_ms.restype = ci
    lib.ab_merge_stage_ms.argtypes = [ctypes.POINTER(ctypes.c_float)]
    lib.lr_linear_fwd.restype = ci
    lib.lr_linear_fwd.argtypes = [vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, vp, sz, vp]
    lib.lr_linear_fwd_workspace_bytes.restype = sz
    lib.lr_linear_fwd_workspace_bytes.argtypes = [i64, i64, i64, i64, ci]
    lib.lr_linear_bwd.restype = ci
    lib.lr_linear_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, vp, sz, vp]
    lib.lr_linear_bwd_workspace_bytes.restype = sz
    lib.lr_linear_fwd_grouped.restype = ci
    lib.lr_linear_fwd_grouped.argtypes = [ctypes.POINTER(LrGroup), ci, i64, i64, i64, i64, ci, vp, sz, vp]
    lib.lr_linear_bwd_grouped.restype = ci
    lib.lr_linear_bwd_grouped.argtypes = [ctypes.POINTER(LrGroup), ci, i64, i64, i64, i64, ci, ci, vp, sz, vp]
    lib.lr_linear_bwd_grouped_workspace_bytes.restype = sz
    lib.lr_linear_bwd_grouped_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, ci]
    lib.lr_linear_bwd_static.restype = ci
    lib.lr_linear_bwd_static.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, i64, i64, i64, i64, ci, ci, vp]
    lib.lr_linear_bwd_workspace_bytes.argtypes = [i64, i64, i64, i64, ci]
    pvp = ctypes.POINTER(ctypes.c_void_p)
    lib.ab_merge.restype = ci
    lib.ab_merge.argtypes = [pvp, pvp, ci, i64, i64, i64, ctypes.c_float, i64, ci,
                             vp, vp, vp, vp, i64, vp, vp, sz, vp]
    lib.ab_merge_workspace_bytes.restype = sz
    lib.ab_merge_workspace_bytes.argtypes = [ci, i64, i64, i64, i64, ci]
    lib.ab_merge_batched.restype = ci
    lib.ab_merge_batched.argtypes = [ctypes.POINTER(MergeDesc), ci, vp, sz, vp]
    lib.ab_merge_batched_workspace_bytes.restype = sz
    lib.ab_merge_batched_workspace_bytes.argtypes = [ctypes.POINTER(MergeDesc), ci]
    lib.ab_merge_info.restype = ci
    lib.ab_merge_info.argtypes = [vp, ci, ctypes.POINTER(ctypes.c_int32), ctypes.POINTER(ctypes.c_int32), vp]
    lib.ab_factorize.restype = ci
    lib.ab_factorize.argtypes = [vp, i64, i64, ctypes.c_float, i64, vp, vp, vp, vp, i64, vp, sz, vp]
    lib.ab_factorize_workspace_bytes.restype = sz
    lib.ab_factorize_workspace_bytes.argtypes = [i64, i64, i64]
    lib.ab_factorize_batched.restype = ci
    lib.ab_factorize_batched.argtypes = [ctypes.POINTER(FactorizeDesc), ci, vp, sz, vp]
    lib.ab_factorize_batched_workspace_bytes.restype = sz
    lib.ab_factorize_batched_workspace_bytes.argtypes = [ctypes.POINTER(FactorizeDesc), ci]
    lib.ab_adamw_step.restype = ci
    cd = ctypes.c_double
    lib.ab_adamw_step.argtypes = [ctypes.POINTER(AdamwTensor), ci, i64, cd, cd, cd, cd, cd, cd, vp]
    lib.ab_lr_rebound_scale.restype = ctypes.c_double
    lib.ab_lr_rebound_scale.argtypes = [i64, i64]
    lib.ab_reconstruct.restype = ci
    lib.ab_reconstruct.argtypes = [vp, vp, vp, i64, i64, i64, vp]
    pg = ctypes.POINTER(ConvGeom)
    lib.lr_conv_fwd.restype = ci
    lib.lr_conv_fwd.argtypes = [vp, vp, vp, vp, vp, pg, i64, i64, ci, vp]
    lib.lr_conv_bwd.restype = ci
    lib.lr_conv_bwd.argtypes = [vp, vp, vp, vp, vp, vp, vp, vp, pg, i64, i64, ci, ci, vp, sz, vp]
    lib.lr_conv_bwd_workspace_bytes.restype = sz
    lib.lr_conv_bwd_workspace_bytes.argtypes = [pg, i64, i64, ci]
    _lib = lib
    return lib


def status_string(code: int) -> str:
    return load().abt_status_string(int(code)).decode()


def _check(code: int, what: str):
    if code != 0:
        raise AbtError(f"{what} failed: {status_string(code)} ({code})")


def set_chain_rows(rows: int) -> int:
    """Force the chain kernel's work-group height (64 or 128; 0 = automatic); returns the previous setting."""
    return load().abt_set_chain_rows(int(rows))


def set_chain_parts(parts: int) -> int:
    """Force the column parts of the 128-row chain kernel (1..8; 0 = automatic); returns the previous setting."""
    return load().abt_set_chain_parts(int(parts))


def set_jacobi_max_sweeps(n: int) -> int:
    return load().abt_set_jacobi_max_sweeps(int(n))


def set_merge_groups(n: int) -> int:
    return load().abt_set_merge_groups(int(n))


MERGE_STAGES = ("mean_gram", "cholesky", "core_product", "jacobi", "rank_and_projectors", "back_projection")


def set_merge_stage_timing(on: bool) -> int:
    return load().abt_set_merge_stage_timing(int(bool(on)))


def merge_stage_ms() -> dict:
    """Elapsed milliseconds of the stages of the last batched merge / factorisation that ran with
    the stage timers on (waits for it)."""
    buf = (ctypes.c_float * len(MERGE_STAGES))()
    _check(load().ab_merge_stage_ms(buf), "ab_merge_stage_ms")
    return dict(zip(MERGE_STAGES, (float(x) for x in buf)))


# --------------------------------------------------------------------------------------
# torch-facing wrappers (allocation of outputs/workspace + pointer marshalling only)
# --------------------------------------------------------------------------------------

def _torch():
    import torch
    return torch


def _dt(t):
    torch = _torch()
    if t.dtype == torch.bfloat16:
        return ABT_BF16
    if t.dtype == torch.float32:
        return ABT_F32
    raise AbtError(f"unsupported dtype {t.dtype}")


def _ptr(t):
    return ctypes.c_void_p(t.data_ptr()) if t is not None else ctypes.c_void_p(0)


def _stream():
    return ctypes.c_void_p(_torch().cuda.current_stream().cuda_stream)


def _dev_tensor(t, name):
    if not t.is_cuda:
        raise AbtError(f"{name} must live on the GPU: the library has no CPU path")
    if not t.is_contiguous():
        raise AbtError(f"{name} must be contiguous")
    return t


def _workspace(nbytes: int, device, workspace=None):
    torch = _torch()
    if workspace is not None:
        if workspace.numel() * workspace.element_size() < nbytes:
            raise AbtError("workspace tensor too small")
        return workspace
    return torch.empty(max(int(nbytes), 256), dtype=torch.uint8, device=device)


def lr_linear_fwd(X, A, B, save_T: bool = True, Y=None, T=None, workspace=None):
    """Y = (X B^T) A^T.  Returns (Y, T) (T is None when save_T is False)."""
    torch = _torch()
    lib = load()
    X, A, B = _dev_tensor(X, "X"), _dev_tensor(A, "A"), _dev_tensor(B, "B")
    M, n = X.shape
    m, r = A.shape
    if tuple(B.shape) != (r, n) or A.dtype != X.dtype or B.dtype != X.dtype:
        raise AbtError("shape/dtype mismatch: X [M,n], A [m,r], B [r,n], one dtype")
    dt = _dt(X)
    if Y is None:
        Y = torch.empty((M, m), dtype=X.dtype, device=X.device)
    if save_T and T is None:
        T = torch.empty((M, r), dtype=X.dtype, device=X.device)
    nbytes = lib.lr_linear_fwd_workspace_bytes(M, m, n, r, dt)
    ws = _workspace(nbytes, X.device, workspace)
    _check(lib.lr_linear_fwd(_ptr(X), _ptr(A), _ptr(B), _ptr(Y), _ptr(T if save_T else None),
                             M, m, n, r, dt, _ptr(ws), ws.numel(), _stream()), "lr_linear_fwd")
    return Y, (T if save_T else None)


def lr_linear_bwd(dY, X, T, A, B, need_dX: bool = True, need_dA: bool = True, need_dB: bool = True,
                  dX=None, dA=None, dB=None, accumulate: bool = False, workspace=None):
    """dX = (dY A) B, dA = dY^T T, dB = (dY A)^T X.  T may be None (recomputed).
    Returns (dX, dA, dB); skipped gradients are None."""
    torch = _torch()
    lib = load()
    dY, X, A, B = (_dev_tensor(t, nm) for t, nm in ((dY, "dY"), (X, "X"), (A, "A"), (B, "B")))
    M, n = X.shape
    m, r = A.shape
    if tuple(dY.shape) != (M, m) or tuple(B.shape) != (r, n):
        raise AbtError("shape mismatch: dY [M,m], X [M,n], A [m,r], B [r,n]")
    if T is not None and tuple(_dev_tensor(T, "T").shape) != (M, r):
        raise AbtError("T must be [M,r]")
    dt = _dt(X)
    for t, nm in ((dY, "dY"), (A, "A"), (B, "B"), (T, "T")):
        if t is not None and t.dtype != X.dtype:
            raise AbtError(f"{nm} must have the dtype of X ({X.dtype}), got {t.dtype}")
    for t, nm, want in ((dX, "dX", X.dtype), (dA, "dA", torch.float32), (dB, "dB", torch.float32)):
        if t is not None and t.dtype != want:
            raise AbtError(f"{nm} must be {want}, got {t.dtype}")
    if need_dX and dX is None:
        dX = torch.empty((M, n), dtype=X.dtype, device=X.device)
    if need_dA and dA is None:
        if accumulate:
            raise AbtError("accumulate needs existing dA")
        dA = torch.empty((m, r), dtype=torch.float32, device=X.device)
    if need_dB and dB is None:
        if accumulate:
            raise AbtError("accumulate needs existing dB")
        dB = torch.empty((r, n), dtype=torch.float32, device=X.device)
    nbytes = lib.lr_linear_bwd_workspace_bytes(M, m, n, r, dt)
    ws = _workspace(nbytes, X.device, workspace)
    _check(lib.lr_linear_bwd(_ptr(dY), _ptr(X), _ptr(T), _ptr(A), _ptr(B),
                             _ptr(dX if need_dX else None), _ptr(dA if need_dA else None),
                             _ptr(dB if need_dB else None), M, m, n, r, dt, int(bool(accumulate)),
                             _ptr(ws), ws.numel(), _stream()), "lr_linear_bwd")
    return (dX if need_dX else None), (dA if need_dA else None), (dB if need_dB else None)


def _group_shapes(groups, keys):
    torch = _torch()
    if not 1 <= len(groups) <= MAX_GROUPS:
        raise AbtError(f"between 1 and {MAX_GROUPS} groups per call")
    X0, A0 = groups[0]["X"], groups[0]["A"]
    M, n = X0.shape
    m, r = A0.shape
    shapes = {"X": (M, n), "A": (m, r), "B": (r, n), "Y": (M, m), "T": (M, r), "dY": (M, m), "dX": (M, n)}
    for g in groups:
        for k in keys:
            t = g.get(k)
            if t is None:
                continue
            _dev_tensor(t, k)
            if tuple(t.shape) != shapes[k] or t.dtype != X0.dtype:
                raise AbtError(f"{k} of every group must be {shapes[k]} of {X0.dtype}")
    return M, m, n, r, _dt(X0)


def lr_linear_fwd_grouped(groups: List[dict], save_T: bool = True):
    """lr_linear_fwd for up to 8 groups of one shape in one call.  Each dict: X, A, B (GPU tensors of one
    dtype) and optionally preallocated Y, T.  Returns a list of (Y, T)."""
    torch = _torch()
    lib = load()
    M, m, n, r, dt = _group_shapes(groups, ("X", "A", "B", "Y", "T"))
    G = len(groups)
    table = (LrGroup * G)()
    outs = []
    for i, g in enumerate(groups):
        X = g["X"]
        Y = g.get("Y")
        if Y is None:
            Y = torch.empty((M, m), dtype=X.dtype, device=X.device)
        T = g.get("T") if save_T else None
        if save_T and T is None:
            T = torch.empty((M, r), dtype=X.dtype, device=X.device)
        e = table[i]
        e.X, e.A, e.B, e.Y, e.T_save = _ptr(X), _ptr(g["A"]), _ptr(g["B"]), _ptr(Y), _ptr(T)
        outs.append((Y, T))
    each = lib.lr_linear_fwd_workspace_bytes(M, m, n, r, dt) if not save_T else 0
    ws = _workspace(each * G, groups[0]["X"].device, None)
    _check(lib.lr_linear_fwd_grouped(table, G, M, m, n, r, dt, _ptr(ws), ws.numel(), _stream()), "lr_linear_fwd_grouped")
    return outs


def lr_linear_bwd_grouped(groups: List[dict], accumulate: bool = False, workspace=None):
    """lr_linear_bwd for up to 8 groups of one shape in one call.  Each dict: dY, X, A, B, optionally T,
    and the outputs wanted, preallocated or True to have them allocated: dX, dA, dB (absent, None or
    False = skipped).  Returns a list of (dX, dA, dB)."""
    torch = _torch()
    lib = load()
    M, m, n, r, dt = _group_shapes(groups, ("X", "A", "B", "dY", "T"))
    G = len(groups)
    table = (LrGroup * G)()
    outs = []
    dev = groups[0]["X"].device
    for i, g in enumerate(groups):
        def want(key, shape, dtype):
            v = g.get(key)
            if v is None or v is False:
                return None
            if v is True:
                if accumulate and key != "dX":
                    raise AbtError(f"accumulate needs an existing {key}")
                return torch.empty(shape, dtype=dtype, device=dev)
            _dev_tensor(v, key)
            if tuple(v.shape) != shape or v.dtype != dtype:
                raise AbtError(f"{key} must be {shape} of {dtype}")
            return v
        dX = want("dX", (M, n), g["X"].dtype)
        dA = want("dA", (m, r), torch.float32)
        dB = want("dB", (r, n), torch.float32)
        e = table[i]
        e.X, e.A, e.B, e.dY, e.T = _ptr(g["X"]), _ptr(g["A"]), _ptr(g["B"]), _ptr(g["dY"]), _ptr(g.get("T"))
        e.dX, e.dA, e.dB = _ptr(dX), _ptr(dA), _ptr(dB)
        outs.append((dX, dA, dB))
    nbytes = lib.lr_linear_bwd_grouped_workspace_bytes(G, M, m, n, r, dt)
    if nbytes == 0:
        raise AbtError("lr_linear_bwd_grouped: unsupported shape")
    ws = _workspace(nbytes, dev, workspace)
    _check(lib.lr_linear_bwd_grouped(table, G, M, m, n, r, dt, int(bool(accumulate)), _ptr(ws), ws.numel(), _stream()),
           "lr_linear_bwd_grouped")
    return outs


STATIC_SCRATCH_BYTES = 64 << 20   # ABT_STATIC_SCRATCH_BYTES of the header


def lr_linear_bwd_static(dY, X, T, A, B, dX=None, dA=None, dB=None, accumulate: bool = False):
    """lr_linear_bwd through the entry point that allocates nothing: the caller passes every output
    it wants (None skips that gradient) and the library uses its own static scratch array.
    Returns (dX, dA, dB) as passed."""
    torch = _torch()
    lib = load()
    dY, X, A, B = (_dev_tensor(t, nm) for t, nm in ((dY, "dY"), (X, "X"), (A, "A"), (B, "B")))
    M, n = X.shape
    m, r = A.shape
    if tuple(dY.shape) != (M, m) or tuple(B.shape) != (r, n):
        raise AbtError("shape mismatch: dY [M,m], X [M,n], A [m,r], B [r,n]")
    for t, nm, shape, want in ((T, "T", (M, r), X.dtype), (dY, "dY", (M, m), X.dtype), (A, "A", (m, r), X.dtype),
                               (B, "B", (r, n), X.dtype), (dX, "dX", (M, n), X.dtype),
                               (dA, "dA", (m, r), torch.float32), (dB, "dB", (r, n), torch.float32)):
        if t is None:
            continue
        _dev_tensor(t, nm)
        if tuple(t.shape) != shape or t.dtype != want:
            raise AbtError(f"{nm} must be {shape} of {want}, got {tuple(t.shape)} of {t.dtype}")
    _check(lib.lr_linear_bwd_static(_ptr(dY), _ptr(X), _ptr(T), _ptr(A), _ptr(B), _ptr(dX), _ptr(dA), _ptr(dB),
                                    M, m, n, r, _dt(X), int(bool(accumulate)), _stream()), "lr_linear_bwd_static")
    return dX, dA, dB


def _conv_geom(act, B, kh, kw, stride=1):
    torch = _torch()
    _dev_tensor(act, "act")
    if act.dim() != 4 or act.dtype != torch.bfloat16:
        raise AbtError("act must be a bf16 tensor [N, H, W, C] (channels last)")
    N, H, W, C = act.shape
    if B.dim() != 2 or B.shape[1] != kh * kw * C:
        raise AbtError("B must be [r, kh*kw*C] with tap-major columns")
    if stride not in (1, 2):
        raise AbtError("stride must be 1 or 2")
    return ConvGeom(N, H, W, C, kh, kw, stride), N * (-(-H // stride)) * (-(-W // stride))


def lr_conv_fwd(act, A, B, kh: int, kw: int, save_T: bool = True, Y=None, T=None, stride: int = 1):
    """Factored kh x kw convolution (zero padding kh/2, kw/2; stride 1 or 2): Y [N*H'*W', m],
    T [N*H'*W', r] with H' = ceil(H / stride), from the channels-last activation act [N, H, W, C],
    A [m, r], B [r, kh*kw*C] (all bf16, on the GPU)."""
    torch = _torch()
    lib = load()
    A, B = _dev_tensor(A, "A"), _dev_tensor(B, "B")
    geom, M = _conv_geom(act, B, kh, kw, stride)
    m, r = A.shape
    if B.shape[0] != r:
        raise AbtError("shape mismatch: A [m,r], B [r, kh*kw*C]")
    if Y is None:
        Y = torch.empty((M, m), dtype=act.dtype, device=act.device)
    if save_T and T is None:
        T = torch.empty((M, r), dtype=act.dtype, device=act.device)
    if not save_T:
        T = None
    _check(lib.lr_conv_fwd(_ptr(act), _ptr(A), _ptr(B), _ptr(Y), _ptr(T), ctypes.byref(geom), m, r, _dt(act), _stream()),
           "lr_conv_fwd")
    return Y, T


def lr_conv_bwd(dY, act, T, A, B, kh: int, kw: int, need_dAct: bool = True, need_dA: bool = True,
                need_dB: bool = True, dAct=None, dA=None, dB=None, accumulate: bool = False, workspace=None,
                stride: int = 1):
    """Gradients of the factored convolution: dAct [N,H,W,C] bf16, dA [m,r] fp32, dB [r, kh*kw*C] fp32;
    skipped gradients are None.  T may be None (recomputed).  dY and T have N*H'*W' rows."""
    torch = _torch()
    lib = load()
    dY, A, B = _dev_tensor(dY, "dY"), _dev_tensor(A, "A"), _dev_tensor(B, "B")
    geom, M = _conv_geom(act, B, kh, kw, stride)
    m, r = A.shape
    if tuple(dY.shape) != (M, m) or B.shape[0] != r or (T is not None and tuple(_dev_tensor(T, "T").shape) != (M, r)):
        raise AbtError("shape mismatch: dY [N*H*W, m], A [m,r], B [r, kh*kw*C], T [N*H*W, r]")
    dev = act.device
    if need_dAct and dAct is None:
        dAct = torch.empty_like(act)
    if need_dA and dA is None:
        dA = torch.zeros((m, r), dtype=torch.float32, device=dev) if accumulate else \
            torch.empty((m, r), dtype=torch.float32, device=dev)
    if need_dB and dB is None:
        dB = torch.zeros(tuple(B.shape), dtype=torch.float32, device=dev) if accumulate else \
            torch.empty(tuple(B.shape), dtype=torch.float32, device=dev)
    if not need_dAct:
        dAct = None
    if not need_dA:
        dA = None
    if not need_dB:
        dB = None
    need = lib.lr_conv_bwd_workspace_bytes(ctypes.byref(geom), m, r, _dt(act))
    if need == 0:
        raise AbtError("lr_conv_bwd: unsupported shape")
    ws = _workspace(need, dev, workspace)
    _check(lib.lr_conv_bwd(_ptr(dY), _ptr(act), _ptr(T), _ptr(A), _ptr(B), _ptr(dAct), _ptr(dA), _ptr(dB),
                           ctypes.byref(geom), m, r, _dt(act), 1 if accumulate else 0,
                           _ptr(ws), ws.numel() * ws.element_size(), _stream()), "lr_conv_bwd")
    return dAct, dA, dB


def _ptr_array(tensors: Sequence):
    arr = (ctypes.c_void_p * len(tensors))(*[t.data_ptr() for t in tensors])
    return arr


def ab_merge(A_copies: Sequence, B_copies: Sequence, tau: float, k_fixed: int = 0, mode: int = 0,
             k_cap: Optional[int] = None, want_W: bool = False, workspace=None, check_converged: bool = True):
    """Merge G copies of one layer.  Returns dict(A [m,k_cap], B [k_cap,n], S [k_cap], k (0-d int32
    tensor on the GPU), W or None, workspace)."""
    outs = ab_merge_batched([dict(A_copies=A_copies, B_copies=B_copies, tau=tau, k_fixed=k_fixed,
                                  mode=mode, k_cap=k_cap, want_W=want_W)], workspace=workspace,
                            check_converged=check_converged, _single=True)
    return outs[0]


def ab_merge_batched(layers: List[dict], workspace=None, check_converged: bool = True, _single: bool = False):
    """Merge L layers in one call.  Each layer dict: A_copies, B_copies (lists of fp32 GPU tensors),
    tau, and optionally k_fixed, mode, k_cap, want_W, or preallocated A_out/B_out/S_out/k_out/W_out."""
    torch = _torch()
    lib = load()
    L = len(layers)
    descs = (MergeDesc * L)()
    keep = []
    outs = []
    dev = None
    for i, lay in enumerate(layers):
        As = [_dev_tensor(a, "A copy") for a in lay["A_copies"]]
        Bs = [_dev_tensor(b, "B copy") for b in lay["B_copies"]]
        G = len(As)
        if G < 1 or len(Bs) != G:
            raise AbtError("need G >= 1 copies of A and of B")
        m, k = As[0].shape
        k2, n = Bs[0].shape
        for a, b in zip(As, Bs):
            if tuple(a.shape) != (m, k) or tuple(b.shape) != (k, n) or a.dtype != torch.float32 or b.dtype != torch.float32:
                raise AbtError("all copies must be fp32 with identical shapes A [m,k], B [k,n]")
        dev = As[0].device
        mode = int(lay.get("mode", 0))
        K = k if mode == 0 else k * G
        k_cap = lay.get("k_cap") or K
        A_out = lay.get("A_out")
        if A_out is None:
            A_out = torch.empty((m, k_cap), dtype=torch.float32, device=dev)
        B_out = lay.get("B_out")
        if B_out is None:
            B_out = torch.empty((k_cap, n), dtype=torch.float32, device=dev)
        S_out = lay.get("S_out")
        if S_out is None:
            S_out = torch.empty((k_cap,), dtype=torch.float32, device=dev)
        k_out = lay.get("k_out")
        if k_out is None:
            k_out = torch.zeros((), dtype=torch.int32, device=dev)
        W_out = lay.get("W_out")
        if W_out is None and lay.get("want_W"):
            W_out = torch.empty((m, n), dtype=torch.float32, device=dev)
        pa, pb = _ptr_array(As), _ptr_array(Bs)
        keep.append((As, Bs, pa, pb))
        d = descs[i]
        d.A_copies = ctypes.cast(pa, ctypes.POINTER(ctypes.c_void_p))
        d.B_copies = ctypes.cast(pb, ctypes.POINTER(ctypes.c_void_p))
        d.G, d.mode, d.m, d.n, d.k = G, mode, m, n, k
        d.tau, d.k_fixed = float(lay["tau"]), int(lay.get("k_fixed", 0))
        d.A_out, d.B_out, d.S_out, d.k_out = A_out.data_ptr(), B_out.data_ptr(), S_out.data_ptr(), k_out.data_ptr()
        d.k_cap = int(k_cap)
        d.W_out = W_out.data_ptr() if W_out is not None else None
        outs.append({"A": A_out, "B": B_out, "S": S_out, "k": k_out, "W": W_out})
    nbytes = lib.ab_merge_batched_workspace_bytes(descs, L)
    if nbytes == 0:
        raise AbtError("ab_merge_batched_workspace_bytes rejected the layer list")
    ws = _workspace(nbytes, dev, workspace)
    _check(lib.ab_merge_batched(descs, L, _ptr(ws), ws.numel(), _stream()), "ab_merge_batched")
    for o in outs:
        o["workspace"] = ws
    if check_converged:
        for i in range(L):
            sweeps, nsig = merge_info(ws, i)
            outs[i]["sweeps"] = sweeps
    return outs


def ab_factorize(W, tau: float, k_fixed: int = 0, k_cap: Optional[int] = None, workspace=None,
                 check_converged: bool = True):
    """Truncated SVD factors of a dense fp32 GPU matrix W [m, n] (Eq. 3).  Returns dict(A [m,k_cap],
    B [k_cap,n], S [k_cap], k (0-d int32 tensor on the GPU), workspace)."""
    return ab_factorize_batched([dict(W=W, tau=tau, k_fixed=k_fixed, k_cap=k_cap)], workspace=workspace,
                                check_converged=check_converged)[0]


def ab_factorize_batched(layers: List[dict], workspace=None, check_converged: bool = True):
    """Factorise L dense weights in one call.  Each layer dict: W (fp32 GPU tensor [m, n]), tau, and
    optionally k_fixed, k_cap.  Returns a list of dicts as ab_factorize."""
    torch = _torch()
    lib = load()
    L = len(layers)
    descs = (FactorizeDesc * L)()
    outs = []
    dev = None
    for i, lay in enumerate(layers):
        W = _dev_tensor(lay["W"], "W")
        if W.dtype != torch.float32 or W.dim() != 2:
            raise AbtError("W must be a 2-d fp32 tensor")
        m, n = W.shape
        k_cap = int(lay.get("k_cap") or min(m, n))
        dev = W.device
        o = dict(A=torch.empty((m, k_cap), dtype=torch.float32, device=dev),
                 B=torch.empty((k_cap, n), dtype=torch.float32, device=dev),
                 S=torch.empty((k_cap,), dtype=torch.float32, device=dev),
                 k=torch.zeros((), dtype=torch.int32, device=dev), _W=W)
        d = descs[i]
        d.W = _ptr(W); d.m = m; d.n = n; d.tau = float(lay["tau"]); d.k_fixed = int(lay.get("k_fixed", 0))
        d.A_out = _ptr(o["A"]); d.B_out = _ptr(o["B"]); d.S_out = _ptr(o["S"]); d.k_out = _ptr(o["k"])
        d.k_cap = k_cap
        outs.append(o)
    need = lib.ab_factorize_batched_workspace_bytes(descs, L)
    if need == 0:
        raise AbtError("ab_factorize: unsupported shape (min(m, n) must be a multiple of 32, <= 2048)")
    if workspace is None or workspace.numel() < need:
        workspace = torch.empty(need, dtype=torch.uint8, device=dev)
    _check(lib.ab_factorize_batched(descs, L, _ptr(workspace), workspace.numel(), _stream()), "ab_factorize_batched")
    for i, o in enumerate(outs):
        o["workspace"] = workspace
        o.pop("_W")
        if check_converged:
            merge_info(workspace, i)
    return outs


def lr_rebound_scale(i: int, rebound_steps: int) -> float:
    """Learning-rate factor i steps (0-based) after a change of the parameters' shape."""
    return float(load().ab_lr_rebound_scale(int(i), int(rebound_steps)))


class AdamwPlan:
    """The tensor table of ab_adamw_step, marshalled once: a training loop updates the same
    tensors every step, and building the table costs more host time than the kernel runs.
    Holds references to the tensors so that their memory stays alive."""

    def __init__(self, tensors: Sequence[dict]):
        torch = _torch()
        self.n = len(tensors)
        self.table = (AdamwTensor * max(self.n, 1))()
        self.tensors = list(tensors)
        for i, t in enumerate(tensors):
            p = _dev_tensor(t["param"], "param")
            cnt = p.numel()
            for key in ("param", "grad", "exp_avg", "exp_avg_sq"):
                x = _dev_tensor(t[key], key)
                if x.dtype != torch.float32 or x.numel() != cnt:
                    raise AbtError(f"{key} must be fp32 with as many elements as param")
            pb = t.get("param_bf16")
            if pb is not None:
                _dev_tensor(pb, "param_bf16")
                if pb.dtype != torch.bfloat16 or pb.numel() != cnt:
                    raise AbtError("param_bf16 must be bf16 with as many elements as param")
            e = self.table[i]
            e.param = _ptr(t["param"]); e.grad = _ptr(t["grad"]); e.exp_avg = _ptr(t["exp_avg"])
            e.exp_avg_sq = _ptr(t["exp_avg_sq"]); e.param_bf16 = _ptr(pb); e.count = cnt


def ab_adamw_step(tensors, step: int, lr: float, lr_scale: float = 1.0, beta1: float = 0.9,
                  beta2: float = 0.999, eps: float = 1e-8, weight_decay: float = 0.01):
    """One AdamW step, in place.  `tensors` is an AdamwPlan, or a list of dicts with fp32 GPU
    tensors param, grad, exp_avg, exp_avg_sq of equal element count and optionally param_bf16
    (bf16, same count) that receives the rounded new parameter."""
    plan = tensors if isinstance(tensors, AdamwPlan) else AdamwPlan(tensors)
    _check(load().ab_adamw_step(plan.table, plan.n, int(step), float(lr), float(lr_scale), float(beta1),
                                float(beta2), float(eps), float(weight_decay), _stream()), "ab_adamw_step")


def ab_reconstruct(A, B, W=None):
    """W [m, n] = A [m, k] . B [k, n] for fp32 GPU tensors."""
    torch = _torch()
    _dev_tensor(A, "A"); _dev_tensor(B, "B")
    if A.dtype != torch.float32 or B.dtype != torch.float32 or A.dim() != 2 or B.dim() != 2 or A.shape[1] != B.shape[0]:
        raise AbtError("ab_reconstruct: A [m, k] and B [k, n] must be fp32 matrices")
    m, k = A.shape
    n = B.shape[1]
    if W is None:
        W = torch.empty((m, n), dtype=torch.float32, device=A.device)
    else:
        _dev_tensor(W, "W")
        if W.dtype != torch.float32 or tuple(W.shape) != (m, n):
            raise AbtError("ab_reconstruct: W must be fp32 [m, n]")
    _check(load().ab_reconstruct(_ptr(A), _ptr(B), _ptr(W), m, n, k, _stream()), "ab_reconstruct")
    return W


def merge_info(workspace, layer: int = 0):
    """(sweeps, n_sigma) of a finished merge; raises if the Jacobi sweep cap was hit."""
    lib = load()
    sweeps, nsig = ctypes.c_int32(0), ctypes.c_int32(0)
    code = lib.ab_merge_info(_ptr(workspace), int(layer), ctypes.byref(sweeps), ctypes.byref(nsig), _stream())
    _check(code, "ab_merge_info")
    return sweeps.value, nsig.value
