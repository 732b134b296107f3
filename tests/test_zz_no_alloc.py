"""dad_compress_rank_noalloc (the entry point that allocates nothing: its scratch is a static device
array) against dad_compress_rank on the same inputs, and against the fp64 oracle, through the C ABI.
Two calls in a row share the device's scratch array; the second is smaller than the first, and a
call that latched a numerical breakdown is followed by a healthy one."""
import numpy as np
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad
from paper_2102_09631_amd import workloads as W

pytestmark = pytest.mark.gpu


def _to_dev(x, dtype, dev):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def _one_call(w, layer, rows, dev, tol):
    _, h_in, h_out = w.all_layers()[layer]
    A_sites, D_sites = W.host_factors(w, layer, h_in, h_out, rows=rows)
    A_h, D_h = O.stack_factors(A_sites, D_sites)
    G0_h = W.host_start_matrix(w, layer, h_out)
    A, D, G0 = _to_dev(A_h, w.dtype, dev), _to_dev(D_h, w.dtype, dev), torch.from_numpy(G0_h).to(dev)
    r, n = w.rank, w.n_iter
    Pt_ws, Gt_ws = dad.compress_rank(A, D, r, n, G0, check=True)          # the existing entry point
    Pt = torch.full((r, h_in), float("nan"), dtype=torch.float32, device=dev)
    Gt = torch.full((r, h_out), float("nan"), dtype=torch.float32, device=dev)
    flag = torch.full((1,), 7, dtype=torch.int32, device=dev)
    torch.cuda.synchronize()
    before = torch.cuda.memory_allocated()
    dad.compress_rank_noalloc(A, D, r, n, G0, Pt, Gt, numeric_flag=flag)
    torch.cuda.synchronize()
    assert torch.cuda.memory_allocated() == before
    assert int(flag.item()) == 0
    # same kernels, same launch shapes, fixed summation orders: identical bits
    assert torch.equal(Pt, Pt_ws) and torch.equal(Gt, Gt_ws)
    Pt_ref, Gt_ref = O.block_spi(A_h, D_h, G0_h, n)
    e = O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), O.rank_r_grad(Pt_ref, Gt_ref))
    print(w.name, layer, A.shape, "noalloc vs oracle", e)
    assert e <= tol


def test_noalloc_two_calls_second_smaller(gpu):
    dad.init()
    # encoder layer, 4 x 4096 rows of bf16 (direct-to-LDS MFMA kernels), then the 64-row fp32 layer
    _one_call(W.WORKLOADS[2], 0, None, gpu, 2e-2)
    _one_call(W.WORKLOADS[0], 0, None, gpu, 1e-5)
    # and once more at a third size, bf16 with a ragged row count (register-staged kernels)
    _one_call(W.WORKLOADS[2], 1, 328, gpu, 2e-2)


def test_noalloc_flag_is_cleared_by_the_next_call(gpu):
    dev = gpu
    # Delta = 0: the iterate vanishes and the first Cholesky pivot is exactly zero
    A = torch.ones((64, 96), device=dev)
    D = torch.zeros((64, 80), device=dev)
    G0 = torch.from_numpy(W.host_start_matrix(W.WORKLOADS[0], 0, 80, r=4)).to(dev)
    Pt = torch.empty((4, 96), dtype=torch.float32, device=dev)
    Gt = torch.empty((4, 80), dtype=torch.float32, device=dev)
    flag = torch.zeros(1, dtype=torch.int32, device=dev)
    dad.compress_rank_noalloc(A, D, 4, 2, G0, Pt, Gt, numeric_flag=flag)
    torch.cuda.synchronize()
    assert int(flag.item()) == 1
    assert dad.poll_numeric_status(flag) == dad.DAD_ERR_NUMERIC
    _one_call(W.WORKLOADS[0], 0, None, dev, 1e-5)      # healthy call on the same scratch: flag back to 0
