"""Grouped entry points against the single-layer calls (bit for bit) and against the oracle."""
import numpy as np
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad

pytestmark = pytest.mark.gpu


def _pair(K, h_in, h_out, seed, dev, dtype=torch.float32):
    g = torch.Generator(device="cpu").manual_seed(seed)
    L = torch.randn(K, h_in, generator=g).to(dtype).to(dev)
    R = (0.1 * torch.randn(K, h_out, generator=g)).to(dtype).to(dev)
    return L, R


def _check_against_oracle(G, L, R, tol):
    ref = O.full_grad(L.float().cpu().numpy(), R.float().cpu().numpy())
    assert O.rel_fro(G.cpu().numpy(), ref) <= tol


RANK_SHAPES = [(4, 784, 128), (8, 1024, 10), (16, 768, 2304), (32, 1024, 4096), (64, 1280, 1280), (3, 53, 29),
               (1, 40, 24), (7, 130, 257)]


def test_grouped_rank_rebuild_equals_single_calls(gpu):
    """K = r pairs of every benchmark rank and ragged shapes: one grouped call against one call each."""
    pairs = [_pair(K, hi, ho, 10 + i, gpu) for i, (K, hi, ho) in enumerate(RANK_SHAPES)]
    single = [dad.reconstruct_grad(L, R) for L, R in pairs]
    grouped = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), a, b in zip(pairs, single, grouped):
        assert torch.equal(a, b)
        _check_against_oracle(b, L, R, 1e-5)


def test_grouped_rebuild_with_split_contraction_and_many_jobs(gpu):
    """40 jobs (two launches of the job table), among them fp32 full-gradient shapes whose
    contraction is split into slabs."""
    shapes = [(1024, 784, 1024), (1024, 1024, 1024), (2000, 96, 80), (64, 784, 128)] + [(5, 64 + i, 33 + 2 * i) for i in range(36)]
    pairs = [_pair(K, hi, ho, 100 + i, gpu) for i, (K, hi, ho) in enumerate(shapes)]
    assert dad.lib().dad_reconstruct_workspace_bytes(1024, 1024, 1024, dad.DAD_F32) > 0   # split
    single = [dad.reconstruct_grad(L, R) for L, R in pairs]
    grouped = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), a, b in zip(pairs, single, grouped):
        assert torch.equal(a, b)
        _check_against_oracle(b, L, R, 1e-5)


def test_grouped_rebuild_bf16_jobs(gpu):
    pairs = [_pair(4096, 512, 768, 7, gpu, torch.bfloat16), _pair(1000, 256, 264, 8, gpu, torch.bfloat16)]
    single = [dad.reconstruct_grad(L, R) for L, R in pairs]
    grouped = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), a, b in zip(pairs, single, grouped):
        assert torch.equal(a, b)
        _check_against_oracle(b, L, R, 1e-5)     # bf16 inputs are exact; only the fp32 sums differ


@pytest.mark.parametrize("K,h_in,h_out", [(64, 784, 128), (1024, 784, 1024), (1024, 1024, 10), (257, 129, 255),
                                          (9, 300, 520), (4097, 64, 96)])
def test_fp32_rebuild_on_the_matrix_instruction_matches_oracle(gpu, K, h_in, h_out):
    """Full fp32 gradients (the two MLP workloads' shapes and ragged ones, odd K included)."""
    L, R = _pair(K, h_in, h_out, K + h_in, gpu)
    G = dad.reconstruct_grad(L, R)
    _check_against_oracle(G, L, R, 1e-5)
    assert torch.equal(G, dad.reconstruct_grad(L, R))      # fixed summation order
