"""ctypes binding of libdad's C ABI (include/dad.h).

Argument marshalling only: torch supplies device memory and the current HIP
stream; every step of the path runs inside the library's kernels.  There is no
fallback: if libdad.so is missing or a call fails, an exception is raised.
"""
from __future__ import annotations

import ctypes as C
import os

import torch

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_HERE, "libdad.so")

DAD_F32, DAD_BF16 = 0, 1
DAD_OK, DAD_ERR_NULL, DAD_ERR_SHAPE, DAD_ERR_ALIGN, DAD_ERR_WORKSPACE, DAD_ERR_DTYPE, DAD_ERR_NUMERIC, \
    DAD_ERR_HIP = range(8)
DAD_MAX_RANK = 64
DAD_GRAM_MAX_ROWS = 1024
DAD_ACT = {"identity": 0, "relu": 1, "tanh": 2, "sigmoid": 3}

_lib = None


class RebuildDesc(C.Structure):
    """dad_rebuild_desc"""
    _fields_ = [("L", C.c_void_p), ("R", C.c_void_p), ("G", C.c_void_p), ("K", C.c_int64), ("h_in", C.c_int64),
                ("h_out", C.c_int64)]


class CompressDesc(C.Structure):
    """dad_compress_desc"""
    _fields_ = [("A", C.c_void_p), ("D", C.c_void_p), ("G0", C.c_void_p), ("Pt", C.c_void_p), ("Gt", C.c_void_p),
                ("N", C.c_int64), ("h_in", C.c_int64), ("h_out", C.c_int64),
                ("S", C.c_int), ("A_sites", C.POINTER(C.c_void_p)), ("D_sites", C.POINTER(C.c_void_p)),
                ("rows", C.POINTER(C.c_int64))]


class DadError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = status
        super().__init__(f"{where}: {lib().dad_status_string(status).decode()}")


def lib() -> C.CDLL:
    """Load libdad.so (built by paper_2102_09631_amd.build) and declare its prototypes."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(LIB_PATH):
        raise RuntimeError(f"{LIB_PATH} is missing: run `python -m paper_2102_09631_amd.build` first "
                           "(there is no fallback path)")
    L = C.CDLL(LIB_PATH)
    vp, i64, sz = C.c_void_p, C.c_int64, C.c_size_t
    L.dad_status_string.restype = C.c_char_p
    L.dad_status_string.argtypes = [C.c_int]
    L.dad_init.restype = C.c_int
    L.dad_init.argtypes = []
    L.dad_stack_factors.restype = C.c_int
    L.dad_stack_factors.argtypes = [C.c_int, C.POINTER(vp), C.POINTER(vp), C.POINTER(i64), i64, i64, C.c_int,
                                    vp, vp, vp]
    L.dad_compress_workspace_bytes.restype = sz
    L.dad_compress_workspace_bytes.argtypes = [i64, i64, i64, C.c_int, C.c_int]
    L.dad_compress_rank.restype = C.c_int
    L.dad_compress_rank.argtypes = [vp, vp, i64, i64, i64, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, sz, vp]
    L.dad_compress_rank_noalloc.restype = C.c_int
    L.dad_compress_rank_noalloc.argtypes = [vp, vp, i64, i64, i64, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp]
    L.dad_reconstruct_workspace_bytes.restype = sz
    L.dad_reconstruct_workspace_bytes.argtypes = [i64, i64, i64, C.c_int]
    L.dad_reconstruct_grad.restype = C.c_int
    L.dad_reconstruct_grad.argtypes = [vp, vp, i64, i64, i64, C.c_int, vp, vp, sz, vp]
    L.dad_compress_gram_workspace_bytes.restype = sz
    L.dad_compress_gram_workspace_bytes.argtypes = [i64, i64, i64, C.c_int, C.c_int]
    L.dad_compress_rank_gram.restype = C.c_int
    L.dad_compress_rank_gram.argtypes = [vp, vp, i64, i64, i64, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, sz, vp]
    L.dad_compress_sequential_workspace_bytes.restype = sz
    L.dad_compress_sequential_workspace_bytes.argtypes = [i64, i64, i64, C.c_int]
    L.dad_compress_rank_sequential.restype = C.c_int
    L.dad_compress_rank_sequential.argtypes = [vp, vp, i64, i64, i64, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp, vp, sz, vp]
    L.dad_compress_rank_adaptive.restype = C.c_int
    L.dad_compress_rank_adaptive.argtypes = [vp, vp, i64, i64, i64, C.c_int, C.c_int, C.c_int, C.c_float, vp, vp, vp, vp,
                                             vp, vp, vp, sz, vp]
    L.dad_backprop_delta.restype = C.c_int
    L.dad_backprop_delta.argtypes = [vp, vp, vp, i64, i64, i64, C.c_int, C.c_int, vp, vp]
    L.dad_poll_numeric_status.restype = C.c_int
    L.dad_poll_numeric_status.argtypes = [vp, vp]
    L.dad_profile_enable.restype = C.c_int
    L.dad_profile_enable.argtypes = [C.c_int]
    L.dad_profile_reset.restype = C.c_int
    L.dad_profile_reset.argtypes = []
    L.dad_profile_kernel_count.restype = C.c_int
    L.dad_profile_kernel_count.argtypes = []
    L.dad_profile_kernel_name.restype = C.c_char_p
    L.dad_profile_kernel_name.argtypes = [C.c_int]
    L.dad_profile_get.restype = C.c_int
    L.dad_profile_get.argtypes = [C.c_int, C.POINTER(C.c_double), C.POINTER(C.c_int64)]
    L.dad_reconstruct_grouped_workspace_bytes.restype = sz
    L.dad_reconstruct_grouped_workspace_bytes.argtypes = [C.c_int, C.POINTER(RebuildDesc), C.c_int]
    L.dad_reconstruct_grad_grouped.restype = C.c_int
    L.dad_reconstruct_grad_grouped.argtypes = [C.c_int, C.POINTER(RebuildDesc), C.c_int, vp, sz, vp]
    L.dad_compress_grouped_workspace_bytes.restype = sz
    L.dad_compress_grouped_workspace_bytes.argtypes = [C.c_int, C.POINTER(CompressDesc), C.c_int, C.c_int, C.c_int]
    L.dad_compress_rank_grouped.restype = C.c_int
    L.dad_compress_rank_grouped.argtypes = [C.c_int, C.POINTER(CompressDesc), C.c_int, C.c_int, C.c_int, C.c_int, vp, sz, vp]
    pvp, pi64 = C.POINTER(vp), C.POINTER(i64)
    L.dad_compress_sites_workspace_bytes.restype = sz
    L.dad_compress_sites_workspace_bytes.argtypes = [C.c_int, pi64, i64, i64, C.c_int, C.c_int]
    L.dad_compress_rank_sites.restype = C.c_int
    L.dad_compress_rank_sites.argtypes = [C.c_int, pvp, pvp, pi64, i64, i64, C.c_int, C.c_int, C.c_int, vp, vp, vp, vp,
                                          sz, vp]
    L.dad_reconstruct_sites_workspace_bytes.restype = sz
    L.dad_reconstruct_sites_workspace_bytes.argtypes = [C.c_int, pi64, i64, i64, C.c_int]
    L.dad_reconstruct_grad_sites.restype = C.c_int
    L.dad_reconstruct_grad_sites.argtypes = [C.c_int, pvp, pvp, pi64, i64, i64, C.c_int, vp, vp, sz, vp]
    L.dad_probe_mfma_loop.restype = C.c_int
    L.dad_probe_mfma_loop.argtypes = [vp, sz, C.c_int, vp, vp, C.POINTER(C.c_double)]
    L.dad_probe_read_stream.restype = C.c_int
    L.dad_probe_read_stream.argtypes = [vp, sz, vp, vp, C.POINTER(C.c_double)]
    _lib = L
    return L


def _dt(t: torch.Tensor) -> int:
    if t.dtype == torch.float32:
        return DAD_F32
    if t.dtype == torch.bfloat16:
        return DAD_BF16
    raise TypeError(f"factor dtype must be float32 or bfloat16, got {t.dtype}")


def _stream() -> int:
    return torch.cuda.current_stream().cuda_stream


def _check(rc: int, where: str):
    if rc != DAD_OK:
        raise DadError(rc, where)


def _dense2d(t: torch.Tensor, name: str):
    if t.dim() != 2 or not t.is_contiguous() or not t.is_cuda:
        raise ValueError(f"{name} must be a contiguous 2-D CUDA tensor")


def _factor_args(A, D, G0, r):
    """Checks shared by the reductions: A (N x h_in) and Delta (N x h_out) dense CUDA tensors of one dtype,
    G0 float32 r x h_out.  Returns (N, h_in, h_out, dad_dtype)."""
    _dense2d(A, "A")
    _dense2d(D, "Delta")
    _dense2d(G0, "G0")
    N, h_in = A.shape
    h_out = D.shape[1]
    if D.shape[0] != N or D.dtype != A.dtype:
        raise ValueError("A and Delta disagree in rows or dtype")
    if G0.dtype != torch.float32 or tuple(G0.shape) != (r, h_out):
        raise ValueError("G0 must be float32 of shape (r, h_out)")
    return N, h_in, h_out, _dt(A)


def init():
    """dad_init: one-time set-up of the current device (needed only before a first call under graph capture)."""
    _check(lib().dad_init(), "dad_init")


def stack_factors(A_sites, D_sites, A_out=None, D_out=None):
    """dad_stack_factors: vertical concatenation of the sites' (A_s, Delta_s)."""
    S = len(A_sites)
    if S == 0 or len(D_sites) != S:
        raise ValueError("need the same non-zero number of A and Delta blocks")
    for a, d in zip(A_sites, D_sites):
        _dense2d(a, "A_s")
        _dense2d(d, "Delta_s")
        if a.shape[0] != d.shape[0] or a.dtype != A_sites[0].dtype or d.dtype != a.dtype:
            raise ValueError("site blocks disagree in rows or dtype")
    h_in, h_out = A_sites[0].shape[1], D_sites[0].shape[1]
    if any(a.shape[1] != h_in for a in A_sites) or any(d.shape[1] != h_out for d in D_sites):
        raise ValueError("site blocks disagree in width")
    rows = [int(a.shape[0]) for a in A_sites]
    N = sum(rows)
    dev, dt = A_sites[0].device, A_sites[0].dtype
    if A_out is None:
        A_out = torch.empty((N, h_in), dtype=dt, device=dev)
    if D_out is None:
        D_out = torch.empty((N, h_out), dtype=dt, device=dev)
    pa = (C.c_void_p * S)(*[a.data_ptr() for a in A_sites])
    pd = (C.c_void_p * S)(*[d.data_ptr() for d in D_sites])
    pr = (C.c_int64 * S)(*rows)
    _check(lib().dad_stack_factors(S, pa, pd, pr, h_in, h_out, _dt(A_sites[0]), A_out.data_ptr(), D_out.data_ptr(),
                                   _stream()), "dad_stack_factors")
    return A_out, D_out


def _site_tables(A_sites, D_sites):
    """Checks a list of site blocks and marshals it: (S, pointer arrays, row array, rows, h_in, h_out, dt)."""
    S = len(A_sites)
    if S == 0 or len(D_sites) != S:
        raise ValueError("need the same non-zero number of A and Delta blocks")
    h_in, h_out = A_sites[0].shape[1], D_sites[0].shape[1]
    dt = _dt(A_sites[0])
    for a, d in zip(A_sites, D_sites):
        _dense2d(a, "A_s")
        _dense2d(d, "Delta_s")
        if a.shape[0] != d.shape[0] or a.dtype != A_sites[0].dtype or d.dtype != a.dtype:
            raise ValueError("site blocks disagree in rows or dtype")
        if a.shape[1] != h_in or d.shape[1] != h_out:
            raise ValueError("site blocks disagree in width")
    rows = [int(a.shape[0]) for a in A_sites]
    pa = (C.c_void_p * S)(*[a.data_ptr() for a in A_sites])
    pd = (C.c_void_p * S)(*[d.data_ptr() for d in D_sites])
    pr = (C.c_int64 * S)(*rows)
    return S, pa, pd, pr, rows, h_in, h_out, dt


def compress_rank_sites(A_sites, D_sites, r, n_iter, G0, Pt=None, Gt=None, workspace=None, check=False):
    """dad_compress_rank_sites: compress_rank on the sites' blocks, without the stacked copy where the
    blocks can be read in place."""
    S, pa, pd, pr, rows, h_in, h_out, dt = _site_tables(A_sites, D_sites)
    _dense2d(G0, "G0")
    if G0.dtype != torch.float32 or tuple(G0.shape) != (r, h_out):
        raise ValueError("G0 must be float32 of shape (r, h_out)")
    dev = A_sites[0].device
    if workspace is None:
        nbytes = lib().dad_compress_sites_workspace_bytes(S, pr, h_in, h_out, r, dt)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=dev)
    if Pt is None:
        Pt = torch.empty((r, h_in), dtype=torch.float32, device=dev)
    if Gt is None:
        Gt = torch.empty((r, h_out), dtype=torch.float32, device=dev)
    _check(lib().dad_compress_rank_sites(S, pa, pd, pr, h_in, h_out, dt, r, n_iter, G0.data_ptr(), Pt.data_ptr(),
                                         Gt.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()),
           "dad_compress_rank_sites")
    if check:
        _check(lib().dad_poll_numeric_status(workspace.data_ptr(), _stream()), "dad_poll_numeric_status")
    return Pt, Gt


def reconstruct_grad_sites(A_sites, D_sites, G=None, workspace=None):
    """dad_reconstruct_grad_sites: G = A^T Delta (h_in x h_out fp32) from the sites' blocks."""
    S, pa, pd, pr, rows, h_in, h_out, dt = _site_tables(A_sites, D_sites)
    dev = A_sites[0].device
    if workspace is None:
        nbytes = lib().dad_reconstruct_sites_workspace_bytes(S, pr, h_in, h_out, dt)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=dev) if nbytes else None
    if G is None:
        G = torch.empty((h_in, h_out), dtype=torch.float32, device=dev)
    _check(lib().dad_reconstruct_grad_sites(S, pa, pd, pr, h_in, h_out, dt, G.data_ptr(),
                                            workspace.data_ptr() if workspace is not None else None,
                                            workspace.numel() if workspace is not None else 0, _stream()),
           "dad_reconstruct_grad_sites")
    return G


def reconstruct_sites_workspace_bytes(rows, h_in, h_out, dtype) -> int:
    pr = (C.c_int64 * len(rows))(*rows)
    return lib().dad_reconstruct_sites_workspace_bytes(len(rows), pr, h_in, h_out,
                                                       DAD_BF16 if dtype == torch.bfloat16 else DAD_F32)


def compress_workspace_bytes(N, h_in, h_out, r, dtype) -> int:
    return lib().dad_compress_workspace_bytes(N, h_in, h_out, r, DAD_BF16 if dtype == torch.bfloat16 else DAD_F32)


def compress_rank(A, D, r, n_iter, G0, Pt=None, Gt=None, workspace=None, check=False):
    """dad_compress_rank: (A, Delta, G0) -> (Pt r x h_in, Gt r x h_out), fp32.

    `workspace` is a uint8 CUDA tensor of at least compress_workspace_bytes(...);
    one is allocated when omitted.  With check=True the stream is synchronised
    and a latched numerical breakdown raises DadError(DAD_ERR_NUMERIC).
    """
    N, h_in, h_out, dt = _factor_args(A, D, G0, r)
    if workspace is None:
        nbytes = lib().dad_compress_workspace_bytes(N, h_in, h_out, r, dt)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=A.device)
    if Pt is None:
        Pt = torch.empty((r, h_in), dtype=torch.float32, device=A.device)
    if Gt is None:
        Gt = torch.empty((r, h_out), dtype=torch.float32, device=A.device)
    _check(lib().dad_compress_rank(A.data_ptr(), D.data_ptr(), N, h_in, h_out, dt, r, n_iter, G0.data_ptr(),
                                   Pt.data_ptr(), Gt.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()),
           "dad_compress_rank")
    if check:
        _check(lib().dad_poll_numeric_status(workspace.data_ptr(), _stream()), "dad_poll_numeric_status")
    return Pt, Gt


DAD_STATIC_SCRATCH_BYTES = 32 << 20


def compress_rank_noalloc(A, D, r, n_iter, G0, Pt, Gt, numeric_flag=None):
    """dad_compress_rank_noalloc: compress_rank on the library's static scratch.  Every buffer is the
    caller's (Pt r x h_in, Gt r x h_out fp32; numeric_flag an int32 tensor of one element or None);
    nothing is allocated here or in the library."""
    N, h_in, h_out, dt = _factor_args(A, D, G0, r)
    if tuple(Pt.shape) != (r, h_in) or tuple(Gt.shape) != (r, h_out) or Pt.dtype != torch.float32 \
            or Gt.dtype != torch.float32:
        raise ValueError("Pt, Gt must be float32 of shape (r, h_in), (r, h_out)")
    if numeric_flag is not None and (numeric_flag.dtype != torch.int32 or numeric_flag.numel() != 1):
        raise ValueError("numeric_flag must be one int32")
    _check(lib().dad_compress_rank_noalloc(A.data_ptr(), D.data_ptr(), N, h_in, h_out, _dt(A), r, n_iter, G0.data_ptr(),
                                           Pt.data_ptr(), Gt.data_ptr(),
                                           numeric_flag.data_ptr() if numeric_flag is not None else None, _stream()),
           "dad_compress_rank_noalloc")
    return Pt, Gt


def compress_gram_workspace_bytes(N, h_in, h_out, r, dtype) -> int:
    return lib().dad_compress_gram_workspace_bytes(N, h_in, h_out, r, DAD_BF16 if dtype == torch.bfloat16 else DAD_F32)


def compress_rank_gram(A, D, r, n_iter, G0, Pt=None, Gt=None, workspace=None, check=False):
    """dad_compress_rank_gram: dad_compress_rank for N <= DAD_GRAM_MAX_ROWS rows, iterating on A A^T and
    Delta Delta^T; same arguments and outputs as compress_rank."""
    N, h_in, h_out, dt = _factor_args(A, D, G0, r)
    if workspace is None:
        nbytes = lib().dad_compress_gram_workspace_bytes(N, h_in, h_out, r, dt)
        workspace = torch.empty(max(nbytes, 256), dtype=torch.uint8, device=A.device)
    if Pt is None:
        Pt = torch.empty((r, h_in), dtype=torch.float32, device=A.device)
    if Gt is None:
        Gt = torch.empty((r, h_out), dtype=torch.float32, device=A.device)
    _check(lib().dad_compress_rank_gram(A.data_ptr(), D.data_ptr(), N, h_in, h_out, dt, r, n_iter, G0.data_ptr(),
                                        Pt.data_ptr(), Gt.data_ptr(), workspace.data_ptr(), workspace.numel(), _stream()),
           "dad_compress_rank_gram")
    if check:
        _check(lib().dad_poll_numeric_status(workspace.data_ptr(), _stream()), "dad_poll_numeric_status")
    return Pt, Gt


def compress_rank_sequential(A, D, r, n_iter, G0, Qt=None, sGt=None, sigma=None, workspace=None, check=False):
    """dad_compress_rank_sequential: the one-vector-at-a-time recurrence with peeling.

    Returns (Qt r x h_in unit rows, sGt r x h_out rows sigma_j g_j, sigma r).
    """
    N, h_in, h_out, dt = _factor_args(A, D, G0, r)
    dev = A.device
    Qt = torch.empty((r, h_in), dtype=torch.float32, device=dev) if Qt is None else Qt
    sGt = torch.empty((r, h_out), dtype=torch.float32, device=dev) if sGt is None else sGt
    sigma = torch.empty((r,), dtype=torch.float32, device=dev) if sigma is None else sigma
    if workspace is None:
        workspace = torch.empty(lib().dad_compress_sequential_workspace_bytes(N, h_in, h_out, dt), dtype=torch.uint8,
                                device=dev)
    _check(lib().dad_compress_rank_sequential(A.data_ptr(), D.data_ptr(), N, h_in, h_out, dt, r, n_iter, G0.data_ptr(),
                                              Qt.data_ptr(), sGt.data_ptr(), sigma.data_ptr(), workspace.data_ptr(),
                                              workspace.numel(), _stream()), "dad_compress_rank_sequential")
    if check:
        _check(lib().dad_poll_numeric_status(workspace.data_ptr(), _stream()), "dad_poll_numeric_status")
    return Qt, sGt, sigma


def compress_rank_adaptive(A, D, r, max_iter, theta, G0, workspace=None, check=False):
    """dad_compress_rank_adaptive: the one-vector recurrence with the theta stop tests.

    Returns (Qt, sGt, sigma, effective_rank, iterations): device tensors, the last two int32.
    """
    N, h_in, h_out, dt = _factor_args(A, D, G0, r)
    dev = A.device
    Qt = torch.empty((r, h_in), dtype=torch.float32, device=dev)
    sGt = torch.empty((r, h_out), dtype=torch.float32, device=dev)
    sigma = torch.empty((r,), dtype=torch.float32, device=dev)
    rank = torch.full((1,), -1, dtype=torch.int32, device=dev)
    iters = torch.full((r,), -1, dtype=torch.int32, device=dev)
    if workspace is None:
        workspace = torch.empty(lib().dad_compress_sequential_workspace_bytes(N, h_in, h_out, dt), dtype=torch.uint8,
                                device=dev)
    _check(lib().dad_compress_rank_adaptive(A.data_ptr(), D.data_ptr(), N, h_in, h_out, dt, r, max_iter, theta,
                                            G0.data_ptr(), Qt.data_ptr(), sGt.data_ptr(), sigma.data_ptr(),
                                            rank.data_ptr(), iters.data_ptr(), workspace.data_ptr(), workspace.numel(),
                                            _stream()), "dad_compress_rank_adaptive")
    if check:
        _check(lib().dad_poll_numeric_status(workspace.data_ptr(), _stream()), "dad_poll_numeric_status")
    return Qt, sGt, sigma, rank, iters


def reconstruct_workspace_bytes(K, h_in, h_out, dtype) -> int:
    return lib().dad_reconstruct_workspace_bytes(K, h_in, h_out, DAD_BF16 if dtype == torch.bfloat16 else DAD_F32)


def reconstruct_grad(L, R, G=None, workspace=None):
    """dad_reconstruct_grad: G = L^T R (h_in x h_out fp32) from K-row factors."""
    _dense2d(L, "L")
    _dense2d(R, "R")
    K, h_in = L.shape
    h_out = R.shape[1]
    if R.shape[0] != K or R.dtype != L.dtype:
        raise ValueError("L and R disagree in rows or dtype")
    dt = _dt(L)
    if workspace is None:
        nbytes = lib().dad_reconstruct_workspace_bytes(K, h_in, h_out, dt)
        workspace = torch.empty(nbytes, dtype=torch.uint8, device=L.device) if nbytes else None
    if G is None:
        G = torch.empty((h_in, h_out), dtype=torch.float32, device=L.device)
    _check(lib().dad_reconstruct_grad(L.data_ptr(), R.data_ptr(), K, h_in, h_out, dt, G.data_ptr(),
                                      workspace.data_ptr() if workspace is not None else None,
                                      workspace.numel() if workspace is not None else 0, _stream()),
           "dad_reconstruct_grad")
    return G


DAD_MAX_LANES = 8


class CompressGroup:
    """Arguments of dad_compress_rank_grouped marshalled once.  layers: list of (A, D, G0) tensors, or
    (A_sites, D_sites, G0) with two lists of site blocks for a layer that is not stacked;
    outputs Pt, Gt are allocated unless given.  run() is one call of the entry point."""

    def __init__(self, layers, r, n_iter, lanes=2, Pts=None, Gts=None, workspace=None):
        if not layers:
            raise ValueError("need at least one layer")
        self.n, self.r, self.n_iter, self.lanes = len(layers), r, n_iter, lanes
        self.descs = (CompressDesc * self.n)()
        self.Pt, self.Gt = [], []
        self._tables = []
        first = layers[0][0]
        dev = (first[0] if isinstance(first, (list, tuple)) else first).device
        self.dt = _dt(first[0] if isinstance(first, (list, tuple)) else first)
        for i, (A, D, G0) in enumerate(layers):
            _dense2d(G0, "G0")
            if isinstance(A, (list, tuple)):
                S, pa, pd, pr, rows, h_in, h_out, dt = _site_tables(A, D)
                self._tables.append((pa, pd, pr))
                N, a_ptr, d_ptr = 0, None, None
            else:
                _dense2d(A, "A")
                _dense2d(D, "Delta")
                N, h_in = A.shape
                h_out = D.shape[1]
                if D.shape[0] != N or D.dtype != A.dtype:
                    raise ValueError("A and Delta disagree in rows or dtype")
                S, pa, pd, pr, dt = 0, None, None, None, _dt(A)
                a_ptr, d_ptr = A.data_ptr(), D.data_ptr()
            if dt != self.dt:
                raise ValueError("the layers of a group share one dtype")
            if G0.dtype != torch.float32 or tuple(G0.shape) != (r, h_out):
                raise ValueError("G0 must be float32 of shape (r, h_out)")
            Pt = Pts[i] if Pts is not None else torch.empty((r, h_in), dtype=torch.float32, device=dev)
            Gt = Gts[i] if Gts is not None else torch.empty((r, h_out), dtype=torch.float32, device=dev)
            self.Pt.append(Pt)
            self.Gt.append(Gt)
            self.descs[i] = CompressDesc(a_ptr, d_ptr, G0.data_ptr(), Pt.data_ptr(), Gt.data_ptr(), N, h_in, h_out,
                                         S, pa, pd, pr)
        self._keep = layers
        need = lib().dad_compress_grouped_workspace_bytes(self.n, self.descs, self.dt, r, lanes)
        if need == 0:
            raise ValueError("invalid sizes for dad_compress_rank_grouped")
        self.need = need        # bytes of workspace one run() takes
        if workspace is None:
            workspace = torch.zeros(need, dtype=torch.uint8, device=dev)
        self.workspace = workspace

    def run(self, check=False):
        ws = self.workspace
        _check(lib().dad_compress_rank_grouped(self.n, self.descs, self.dt, self.r, self.n_iter, self.lanes,
                                               ws.data_ptr(), ws.numel(), _stream()), "dad_compress_rank_grouped")
        if check:
            _check(lib().dad_poll_numeric_status(ws.data_ptr(), _stream()), "dad_poll_numeric_status")
        return self.Pt, self.Gt


class RebuildGroup:
    """Arguments of dad_reconstruct_grad_grouped marshalled once: the descriptor table, its workspace
    and the outputs.  run() is one call of the entry point."""

    def __init__(self, pairs, Gs=None, workspace=None):
        if not pairs:
            raise ValueError("need at least one (L, R) pair")
        dt = _dt(pairs[0][0])
        self.n = len(pairs)
        self.dt = dt
        self.G = []
        self.descs = (RebuildDesc * self.n)()
        for i, (L, R) in enumerate(pairs):
            _dense2d(L, "L")
            _dense2d(R, "R")
            if R.shape[0] != L.shape[0] or R.dtype != L.dtype or _dt(L) != dt:
                raise ValueError("L and R disagree in rows or dtype")
            G = Gs[i] if Gs is not None else torch.empty((L.shape[1], R.shape[1]), dtype=torch.float32, device=L.device)
            if tuple(G.shape) != (L.shape[1], R.shape[1]) or G.dtype != torch.float32 or not G.is_contiguous():
                raise ValueError("G must be contiguous float32 h_in x h_out")
            self.G.append(G)
            self.descs[i] = RebuildDesc(L.data_ptr(), R.data_ptr(), G.data_ptr(), L.shape[0], L.shape[1], R.shape[1])
        self._keep = pairs
        need = lib().dad_reconstruct_grouped_workspace_bytes(self.n, self.descs, dt)
        if workspace is None and need:
            workspace = torch.empty(need, dtype=torch.uint8, device=pairs[0][0].device)
        self.workspace = workspace

    def run(self):
        ws = self.workspace
        _check(lib().dad_reconstruct_grad_grouped(self.n, self.descs, self.dt, ws.data_ptr() if ws is not None else None,
                                                  ws.numel() if ws is not None else 0, _stream()),
               "dad_reconstruct_grad_grouped")
        return self.G


def reconstruct_grad_grouped(pairs, Gs=None, workspace=None):
    """dad_reconstruct_grad_grouped: [G_i = L_i^T R_i] for a list of (L_i, R_i) pairs in one call."""
    return RebuildGroup(pairs, Gs, workspace).run()


def backprop_delta(D_next, W_next, Z, act, D_out=None):
    """dad_backprop_delta: D_out = (D_next W_next^T) * phi'(Z), rows of D_out dense with pitch h.

    D_out may be a row slice of a larger (stacked) buffer of the same width.
    """
    _dense2d(D_next, "D_next")
    _dense2d(W_next, "W_next")
    _dense2d(Z, "Z")
    N, h_next = D_next.shape
    h = W_next.shape[0]
    if W_next.shape[1] != h_next or tuple(Z.shape) != (N, h) or not (D_next.dtype == W_next.dtype == Z.dtype):
        raise ValueError("D_next (N x h_next), W_next (h x h_next) and Z (N x h) disagree in shape or dtype")
    if act not in DAD_ACT:
        raise ValueError(f"unknown activation {act!r}")
    if D_out is None:
        D_out = torch.empty((N, h), dtype=Z.dtype, device=Z.device)
    _dense2d(D_out, "D_out")
    if tuple(D_out.shape) != (N, h) or D_out.dtype != Z.dtype:
        raise ValueError("D_out must be N x h of the factors' dtype")
    _check(lib().dad_backprop_delta(D_next.data_ptr(), W_next.data_ptr(), Z.data_ptr(), N, h, h_next, _dt(Z),
                                    DAD_ACT[act], D_out.data_ptr(), _stream()), "dad_backprop_delta")
    return D_out


def probe_mfma_loop(operands: torch.Tensor, iters: int = 20000) -> float:
    """dad_probe_mfma_loop: sustained TFLOP/s of a bare bf16 MFMA loop whose fragments come from `operands`."""
    sink = torch.zeros(1, dtype=torch.float32, device=operands.device)
    out = C.c_double(0.0)
    _check(lib().dad_probe_mfma_loop(operands.data_ptr(), operands.numel() * operands.element_size(), iters,
                                     sink.data_ptr(), _stream(), C.byref(out)), "dad_probe_mfma_loop")
    return out.value


def probe_read_stream(src: torch.Tensor) -> float:
    """dad_probe_read_stream: GB/s of one non-temporal pass over `src`."""
    sink = torch.zeros(1, dtype=torch.int32, device=src.device)
    out = C.c_double(0.0)
    _check(lib().dad_probe_read_stream(src.data_ptr(), src.numel() * src.element_size(), sink.data_ptr(), _stream(),
                                       C.byref(out)), "dad_probe_read_stream")
    return out.value


def poll_numeric_status(workspace) -> int:
    return lib().dad_poll_numeric_status(workspace.data_ptr(), _stream())


def profile_enable(on: bool):
    """dad_profile_enable: bracket every kernel launch with HIP events on its stream."""
    _check(lib().dad_profile_enable(1 if on else 0), "dad_profile_enable")


def profile_reset():
    _check(lib().dad_profile_reset(), "dad_profile_reset")


def profile_read() -> dict:
    """dad_profile_get for every kernel: {kernel name: (total ms, launches)} (zero-launch kernels omitted)."""
    L = lib()
    out = {}
    for i in range(L.dad_profile_kernel_count()):
        ms, n = C.c_double(0.0), C.c_int64(0)
        _check(L.dad_profile_get(i, C.byref(ms), C.byref(n)), "dad_profile_get")
        if n.value:
            out[L.dad_profile_kernel_name(i).decode()] = (ms.value, n.value)
    return out
