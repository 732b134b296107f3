"""dad_compress_rank_adaptive (the one-vector recurrence with the theta stop tests and the effective
rank) against the oracle's sequential_spi(theta=...) on the same seeded inputs.  The rank is an
integer decided by floating-point thresholds: the inputs have clear spectral gaps, so fp32 and fp64
decide alike; iteration counts may differ by one application."""
import numpy as np
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad

pytestmark = pytest.mark.gpu


def planted(rng, N, h_in, h_out, sigmas, noise=0.0):
    """Factors whose gradient has the given leading singular values (plus an optional flat tail)."""
    k = len(sigmas)
    U, _ = np.linalg.qr(rng.standard_normal((h_in, k)))
    V, _ = np.linalg.qr(rng.standard_normal((h_out, k)))
    W, _ = np.linalg.qr(rng.standard_normal((N, k)))
    A, D = W @ (U * np.sqrt(sigmas)).T, W @ (V * np.sqrt(sigmas)).T
    if noise:
        A = A + noise * rng.standard_normal(A.shape)
    return A.astype(np.float32), D.astype(np.float32)


def run(A, D, G0, r, max_iter, theta, dev, dtype=torch.float32):
    A_d, D_d = torch.from_numpy(A).to(dtype).to(dev), torch.from_numpy(D).to(dtype).to(dev)
    Qt, sGt, sigma, rank, iters = dad.compress_rank_adaptive(A_d, D_d, r, max_iter, theta, torch.from_numpy(G0).to(dev),
                                                             check=True)
    torch.cuda.synchronize()
    A_h, D_h = A_d.float().cpu().numpy().astype(np.float64), D_d.float().cpu().numpy().astype(np.float64)
    ref = O.sequential_spi(A_h, D_h, G0, max_iter, theta=theta)
    return (Qt.cpu().numpy(), sGt.cpu().numpy(), sigma.cpu().numpy(), int(rank.item()), iters.cpu().numpy()), ref, (A_h, D_h)


@pytest.mark.parametrize("k,N,h_in,h_out", [(1, 64, 96, 80), (2, 40, 784, 128), (3, 128, 300, 520), (5, 256, 1024, 256)])
def test_adaptive_finds_the_planted_rank(gpu, k, N, h_in, h_out):
    rng = np.random.default_rng(500 + k)
    theta, r = 1e-3, 8
    A, D = planted(rng, N, h_in, h_out, 2.0 * 0.5 ** np.arange(k))
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    (Qt, sGt, sigma, rank, iters), (Q_ref, sG_ref, rank_ref, iters_ref), (A_h, D_h) = run(A, D, G0, r, 60, theta, gpu)
    assert rank == rank_ref == k
    assert np.all(Qt[k:] == 0.0) and np.all(sGt[k:] == 0.0) and np.all(sigma[k:] == 0.0)
    M = O.full_grad(A_h, D_h)
    assert O.rel_fro(Qt.T.astype(np.float64) @ sGt, M) <= 5 * theta
    assert O.rel_fro(Qt.T.astype(np.float64) @ sGt, O.rank_r_grad(Q_ref, sG_ref)) <= 5 * theta
    assert np.allclose(sigma[:k], np.linalg.norm(sG_ref[:k], axis=1), rtol=5 * theta)
    assert np.all(np.abs(iters[:k] - np.array(iters_ref[:k])) <= 1), (iters, iters_ref)
    assert np.all(iters[k + 1:] == 0)            # nothing was spent after the rank was found exhausted


def test_adaptive_keeps_every_component_of_a_flat_spectrum_and_respects_the_cap(gpu):
    rng = np.random.default_rng(510)
    A = np.maximum(rng.standard_normal((512, 256)), 0.0).astype(np.float32)
    D = (0.1 * rng.standard_normal((512, 192))).astype(np.float32)
    G0 = rng.standard_normal((6, 192)).astype(np.float32)
    (Qt, sGt, sigma, rank, iters), (Q_ref, sG_ref, rank_ref, iters_ref), _ = run(A, D, G0, 6, 4, 1e-3, gpu)
    assert rank == rank_ref == 6
    assert list(iters) == list(iters_ref) == [4] * 6     # the flat bulk never meets theta: the cap decides
    # same fixed number of applications on both sides: the pairs themselves agree
    assert O.rel_fro(Qt.T.astype(np.float64) @ sGt, O.rank_r_grad(Q_ref, sG_ref)) <= 1e-4
    g = sGt / np.linalg.norm(sGt, axis=1, keepdims=True)
    assert np.abs(g @ g.T - np.eye(6)).max() <= 1e-5       # projector deflation keeps the right vectors orthogonal


def test_adaptive_bf16_factors_on_the_matrix_cores(gpu):
    """N = 1024 rows of bf16 factors (the thin MFMA kernels carry the single vector)."""
    rng = np.random.default_rng(520)
    A, D = planted(rng, 1024, 512, 384, np.array([4.0, 2.0, 1.0]))
    G0 = rng.standard_normal((8, 384)).astype(np.float32)
    (Qt, sGt, sigma, rank, iters), (Q_ref, sG_ref, rank_ref, iters_ref), (A_h, D_h) = run(A, D, G0, 8, 40, 1e-2, gpu,
                                                                                          torch.bfloat16)
    # bf16 rounding of the factors adds a full-rank tail of relative size ~2^-9 ~ 2e-3 < theta = 1e-2
    assert rank == rank_ref == 3
    assert O.rel_fro(Qt.T.astype(np.float64) @ sGt, O.rank_r_grad(Q_ref, sG_ref)) <= 2e-2


def test_adaptive_replays_from_a_hip_graph(gpu):
    dad.init()
    rng = np.random.default_rng(530)
    A, D = planted(rng, 64, 96, 80, np.array([2.0, 1.0]))
    A_d, D_d = torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu)
    G0 = torch.from_numpy(rng.standard_normal((4, 80)).astype(np.float32)).to(gpu)
    lib = dad.lib()
    ws = torch.zeros(lib.dad_compress_sequential_workspace_bytes(64, 96, 80, dad.DAD_F32), dtype=torch.uint8, device=gpu)
    Qt, sGt = torch.empty((4, 96), device=gpu), torch.empty((4, 80), device=gpu)
    sigma, rank, iters = torch.empty(4, device=gpu), torch.zeros(1, dtype=torch.int32, device=gpu), torch.zeros(4, dtype=torch.int32, device=gpu)

    def call():
        rc = lib.dad_compress_rank_adaptive(A_d.data_ptr(), D_d.data_ptr(), 64, 96, 80, dad.DAD_F32, 4, 30, 1e-3, G0.data_ptr(),
                                            Qt.data_ptr(), sGt.data_ptr(), sigma.data_ptr(), rank.data_ptr(), iters.data_ptr(),
                                            ws.data_ptr(), ws.numel(), torch.cuda.current_stream().cuda_stream)
        assert rc == dad.DAD_OK
    call()
    torch.cuda.synchronize()
    eager = (Qt.clone(), sGt.clone(), int(rank.item()), iters.clone())
    assert eager[2] == 2
    g = torch.cuda.CUDAGraph()
    with torch.cuda.graph(g):
        call()
    for _ in range(3):
        Qt.fill_(float("nan")); sGt.fill_(float("nan")); rank.zero_(); iters.zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        assert torch.equal(Qt, eager[0]) and torch.equal(sGt, eager[1]) and int(rank.item()) == 2 and torch.equal(iters, eager[3])
        _ = dad.reconstruct_grad(Qt, sGt)
        torch.cuda.synchronize()
