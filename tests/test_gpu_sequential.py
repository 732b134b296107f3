"""Parity of dad_compress_rank_sequential (Algorithm 2 one vector at a time, Eq. 5-7) with the
fp64 oracle's sequential_spi on the same seeded inputs.  The pair (Q, sG) is fixed by the
recurrence (no sign or basis freedom), so rows, singular values and the product are all compared:
relative Frobenius error <= 1e-5 for fp32 factors, <= 2e-2 for bf16 factors.
"""
import numpy as np
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad
from paper_2102_09631_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def to_dev(x, dtype, dev):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


def bf16_round(x):
    return W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.asarray(x, np.float32)))


def run(A, D, G0, r, n_iter, dtype, dev):
    Qt, sGt, sigma = dad.compress_rank_sequential(to_dev(A, dtype, dev), to_dev(D, dtype, dev), r, n_iter,
                                                  torch.from_numpy(G0).to(dev), check=True)
    G_r = dad.reconstruct_grad(Qt, sGt)
    torch.cuda.synchronize()
    Q_ref, sG_ref = O.sequential_spi(A, D, G0, n_iter)
    q = Qt.cpu().numpy().astype(np.float64)
    sg = sGt.cpu().numpy().astype(np.float64)
    return {
        "e_prod": O.rel_fro(G_r.cpu().numpy(), Q_ref.T @ sG_ref),
        "e_Q": O.rel_fro(q, Q_ref),
        "e_sG": O.rel_fro(sg, sG_ref),
        "e_sigma": float(np.abs(sigma.cpu().numpy() - np.linalg.norm(sG_ref, axis=1)).max()
                         / np.linalg.norm(sG_ref, axis=1).max()),
        "unit": float(np.abs(np.linalg.norm(q, axis=1) - 1.0).max()),
        "sigma_is_norm": float(np.abs(np.linalg.norm(sg, axis=1) - sigma.cpu().numpy()).max()
                               / np.linalg.norm(sg, axis=1).max()),
    }


def check(out, dtype, slack=0.0):
    tol = TOL[dtype] + slack
    assert out["e_prod"] <= tol, out
    assert out["e_Q"] <= tol and out["e_sG"] <= tol and out["e_sigma"] <= tol, out
    assert out["unit"] <= 1e-5 and out["sigma_is_norm"] <= 1e-5, out


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter", [(64, 784, 128, 4, 2), (37, 53, 29, 3, 3), (256, 300, 200, 8, 2),
                                                    (5, 17, 9, 1, 1), (1000, 96, 1031, 5, 2)])
def test_sequential_fp32_matches_oracle(gpu, N, h_in, h_out, r, n_iter):
    """Guarded fp32 kernels, ragged sizes included.  The rows of Delta decay gently so that the
    leading singular values are separated.  Peeling subtracts from M^T M g (size sigma_1^2) what the
    earlier pairs explain and keeps a remainder of size sigma_j^2, so the fp32 rounding of the four
    contractions of an iteration is magnified by (sigma_1/sigma_r)^2 in the last component: the bar
    is 1e-5 plus that term."""
    rng = np.random.default_rng([21, N, h_in, h_out])
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    D = (rng.standard_normal((N, h_out)) * (0.8 ** np.arange(N))[:, None]).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    out = run(A, D, G0, r, n_iter, "f32", gpu)
    sv = np.linalg.svd(A.astype(np.float64).T @ D.astype(np.float64), compute_uv=False)
    slack = 4 * np.finfo(np.float32).eps * (sv[0] / sv[r - 1]) ** 2
    print(N, h_in, h_out, r, n_iter, "slack", slack, out)
    check(out, "f32", slack)


def test_sequential_fp32_workload_factors(gpu):
    """The single-linear workload's own factors (no planted decay)."""
    w = W.WORKLOADS[0]
    A_s, D_s = W.host_factors(w, 0, 784, 128)
    A, D = O.stack_factors(A_s, D_s)
    G0 = W.host_start_matrix(w, 0, 128)
    out = run(A.astype(np.float32), D.astype(np.float32), G0, w.rank, w.n_iter, "f32", gpu)
    print(out)
    check(out, "f32")


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter,ratio", [(1024, 256, 512, 4, 2, 0.9), (4096, 768, 768, 3, 2, 0.97),
                                                          (1000, 256, 512, 2, 2, 0.9)])
def test_sequential_bf16_matches_oracle(gpu, N, h_in, h_out, r, n_iter, ratio):
    """bf16 factors: the MFMA thin kernels carry the vector as row 0 of an 8-row panel (first two
    cases) or, for a row count they do not take, the guarded kernels carry it alone (third case)."""
    rng = np.random.default_rng([22, N, h_in, h_out])
    A = bf16_round(rng.standard_normal((N, h_in)))
    D = bf16_round(rng.standard_normal((N, h_out)) * (ratio ** np.arange(N))[:, None])
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    out = run(A, D, G0, r, n_iter, "bf16", gpu)
    print(N, h_in, h_out, r, n_iter, out)
    check(out, "bf16")


def test_sequential_converges_to_truncated_svd(gpu):
    """With a planted gap and enough iterations the pairs are the leading singular triplets:
    the product equals the truncated SVD (Eckart-Young optimum) and sigma the singular values."""
    N, h_in, h_out, r = 48, 96, 80, 4
    rng = np.random.default_rng(23)
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    D = (rng.standard_normal((N, h_out)) * (0.5 ** np.arange(N))[:, None]).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    Qt, sGt, sigma = dad.compress_rank_sequential(to_dev(A, "f32", gpu), to_dev(D, "f32", gpu), r, 40,
                                                  torch.from_numpy(G0).to(gpu), check=True)
    M = O.full_grad(A, D)
    s = np.linalg.svd(M, compute_uv=False)
    assert np.abs(sigma.cpu().numpy() - s[:r]).max() <= 1e-4 * s[0]
    assert O.rel_fro(dad.reconstruct_grad(Qt, sGt).cpu().numpy(), O.truncated_svd(M, r)) <= 1e-4
    q = Qt.cpu().numpy().astype(np.float64)
    assert np.abs(q @ q.T - np.eye(r)).max() <= 1e-4          # left vectors come out orthonormal


def test_sequential_rank_exhausted_latches_numeric_status(gpu):
    """Delta = 0: every iterate vanishes; the call still ends and the status is latched."""
    N, h_in, h_out, r = 32, 40, 24, 2
    A = torch.ones((N, h_in), device=gpu)
    D = torch.zeros((N, h_out), device=gpu)
    G0 = torch.ones((r, h_out), device=gpu)
    ws = torch.empty(dad.lib().dad_compress_sequential_workspace_bytes(N, h_in, h_out, dad.DAD_F32), dtype=torch.uint8,
                     device=gpu)
    Qt, sGt, sigma = dad.compress_rank_sequential(A, D, r, 1, G0, workspace=ws)
    assert dad.poll_numeric_status(ws) == dad.DAD_ERR_NUMERIC
    assert torch.isfinite(Qt).all() and torch.isfinite(sGt).all() and float(sigma.abs().max()) == 0.0


def test_sequential_reruns_are_bit_identical(gpu):
    rng = np.random.default_rng(24)
    A = to_dev(bf16_round(rng.standard_normal((2048, 512))), "bf16", gpu)
    D = to_dev(bf16_round(rng.standard_normal((2048, 256))), "bf16", gpu)
    G0 = torch.from_numpy(rng.standard_normal((3, 256)).astype(np.float32)).to(gpu)
    a = dad.compress_rank_sequential(A, D, 3, 2, G0)
    b = dad.compress_rank_sequential(A, D, 3, 2, G0)
    for x, y in zip(a, b):
        assert torch.equal(x, y)


def test_sequential_replays_from_a_hip_graph(gpu):
    """The call records into a HIP graph (no memset, no host copy); every replay equals the eager result."""
    rng = np.random.default_rng(25)
    A = to_dev(bf16_round(rng.standard_normal((1024, 256))), "bf16", gpu)
    D = to_dev(bf16_round(rng.standard_normal((1024, 384))), "bf16", gpu)
    G0 = torch.from_numpy(rng.standard_normal((2, 384)).astype(np.float32)).to(gpu)
    ws = torch.empty(dad.lib().dad_compress_sequential_workspace_bytes(1024, 256, 384, dad.DAD_BF16), dtype=torch.uint8,
                     device=gpu)
    Qt, sGt, sig = dad.compress_rank_sequential(A, D, 2, 2, G0, workspace=ws)
    torch.cuda.synchronize()
    ref = [Qt.clone(), sGt.clone(), sig.clone()]
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            dad.compress_rank_sequential(A, D, 2, 2, G0, Qt=Qt, sGt=sGt, sigma=sig, workspace=ws)
    for _ in range(3):
        Qt.zero_(); sGt.zero_(); sig.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for x, y in zip((Qt, sGt, sig), ref):
            assert torch.equal(x, y)
