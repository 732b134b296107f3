"""Seeded sweep over small random shapes (ragged, tiny, r = 1, widths below a tile) for every entry
point against the fp64 oracle: the guarded kernels' bounds handling is what this exercises."""
import numpy as np
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad

pytestmark = pytest.mark.gpu


def shapes(seed, count, n_max, h_max, r_max):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        N = int(rng.integers(1, n_max + 1))
        h_in = int(rng.integers(1, h_max + 1))
        h_out = int(rng.integers(1, h_max + 1))
        r = int(rng.integers(1, min(N, h_in, h_out, r_max) + 1))
        out.append((N, h_in, h_out, r, int(rng.integers(1, 4))))
    return out


def factors(N, h_in, h_out, r, seed):
    rng = np.random.default_rng([seed, N, h_in, h_out, r])
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    # rows of Delta decay gently: separated singular values keep the comparison well posed
    D = (rng.standard_normal((N, h_out)) * (0.9 ** np.arange(N))[:, None]).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    return A, D, G0


def bound(A, D, r):
    """1e-5 plus the fp32 resolution of the weakest kept direction (see the steep-spectrum tests)."""
    s = np.linalg.svd(A.astype(np.float64).T @ D.astype(np.float64), compute_uv=False)
    return 1e-5 + 4 * np.finfo(np.float32).eps * s[0] / max(s[r - 1], 1e-300)


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter", shapes(101, 24, 300, 400, 48))
def test_random_shapes_block_route_and_rebuild(gpu, N, h_in, h_out, r, n_iter):
    A, D, G0 = factors(N, h_in, h_out, r, 1)
    a, d = torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu)
    G_full = dad.reconstruct_grad(a, d).cpu().numpy()
    assert O.rel_fro(G_full, O.full_grad(A, D)) <= 1e-5
    Pt, Gt = dad.compress_rank(a, d, r, n_iter, torch.from_numpy(G0).to(gpu), check=True)
    ref = O.rank_r_grad(*O.block_spi(A, D, G0, n_iter))
    err = O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), ref)
    assert err <= bound(A, D, r), (err, bound(A, D, r))
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-5


def flat_shapes(seed, count, n_max, h_max, r_max):
    """Shapes with enough rows and columns that a Gaussian gradient's spectrum is flat (no direction
    is weak): N, h >= 4 r."""
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(count):
        r = int(rng.integers(1, r_max + 1))
        N = int(rng.integers(4 * r, n_max + 1))
        h_in = int(rng.integers(4 * r, h_max + 1))
        h_out = int(rng.integers(4 * r, h_max + 1))
        out.append((N, h_in, h_out, r, int(rng.integers(1, 4))))
    return out


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter", flat_shapes(104, 24, 700, 600, 32))
def test_random_shapes_flat_spectrum_at_the_strict_bar(gpu, N, h_in, h_out, r, n_iter):
    """Gaussian factors without any planted decay (the spectra of the benchmark's own layers are flat):
    full and rank-r gradient at 1e-5 with no conditioning allowance, both compress routes."""
    rng = np.random.default_rng([4, N, h_in, h_out, r])
    A = np.maximum(rng.standard_normal((N, h_in)), 0.0).astype(np.float32)
    D = (0.1 * rng.standard_normal((N, h_out))).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    a, d, g0 = torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu), torch.from_numpy(G0).to(gpu)
    assert O.rel_fro(dad.reconstruct_grad(a, d).cpu().numpy(), O.full_grad(A, D)) <= 1e-5
    ref = O.rank_r_grad(*O.block_spi(A, D, G0, n_iter))
    Pt, Gt = dad.compress_rank(a, d, r, n_iter, g0, check=True)
    assert O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), ref) <= 1e-5
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-5
    Pt2, Gt2 = dad.compress_rank_gram(a, d, r, n_iter, g0, check=True)
    assert O.rel_fro(dad.reconstruct_grad(Pt2, Gt2).cpu().numpy(), ref) <= 1e-5


# fp32 shapes with r >= 16, which take the fp32 matrix-instruction thin kernels (narrower panels stay
# on the guarded kernels; the sweeps above mix both): ragged rows, widths that are not multiples of 4 (one-float staging), r on both sides of 32,
# column chunks for N << h, many row tiles.
BIG_F32 = [(1000, 1300, 2052, 33, 2), (777, 4096, 1024, 24, 2), (1024, 1280, 5120, 64, 2), (130, 8200, 9001, 64, 1),
           (4099, 515, 2049, 16, 3), (20000, 130, 420, 20, 2), (300, 97, 61, 17, 2)]


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter", BIG_F32)
def test_fp32_thin_contractions_on_the_matrix_instruction(gpu, N, h_in, h_out, r, n_iter):
    rng = np.random.default_rng([5, N, h_in, h_out, r])
    A = np.maximum(rng.standard_normal((N, h_in)), 0.0).astype(np.float32)
    D = (0.1 * rng.standard_normal((N, h_out))).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    a, d, g0 = torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu), torch.from_numpy(G0).to(gpu)
    ref = O.rank_r_grad(*O.block_spi(A, D, G0, n_iter))
    Pt, Gt = dad.compress_rank(a, d, r, n_iter, g0, check=True)
    assert O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), ref) <= 1e-5
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-5
    Pt2, Gt2 = dad.compress_rank(a, d, r, n_iter, g0)
    assert torch.equal(Pt, Pt2) and torch.equal(Gt, Gt2)            # fixed summation order


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter", shapes(102, 24, 300, 400, 48))
def test_random_shapes_gram_route(gpu, N, h_in, h_out, r, n_iter):
    A, D, G0 = factors(N, h_in, h_out, r, 2)
    ws = torch.empty(dad.compress_gram_workspace_bytes(N, h_in, h_out, r, torch.float32), dtype=torch.uint8, device=gpu)
    Pt, Gt = dad.compress_rank_gram(torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu), r, n_iter,
                                    torch.from_numpy(G0).to(gpu), workspace=ws)
    status = dad.poll_numeric_status(ws)
    s = np.linalg.svd(A.astype(np.float64).T @ D.astype(np.float64), compute_uv=False)
    if status != dad.DAD_OK:
        # only beyond its stated range (Gram matrix of the iterate outside fp64) may the route give up
        assert status == dad.DAD_ERR_NUMERIC and (s[0] / max(s[r - 1], 1e-300)) ** (2 * n_iter) > 1e12
        return
    ref = O.rank_r_grad(*O.block_spi(A, D, G0, n_iter))
    err = O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), ref)
    assert err <= bound(A, D, r), (err, bound(A, D, r))
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-5


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter", shapes(103, 12, 200, 300, 6))
def test_random_shapes_sequential_route(gpu, N, h_in, h_out, r, n_iter):
    A, D, G0 = factors(N, h_in, h_out, r, 3)
    Qt, sGt, sigma = dad.compress_rank_sequential(torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu), r, n_iter,
                                                  torch.from_numpy(G0).to(gpu), check=True)
    Q_ref, sG_ref = O.sequential_spi(A, D, G0, n_iter)
    s = np.linalg.svd(A.astype(np.float64).T @ D.astype(np.float64), compute_uv=False)
    tol = 1e-5 + 4 * np.finfo(np.float32).eps * (s[0] / max(s[r - 1], 1e-300)) ** 2   # peeling: squared ratio
    err = O.rel_fro(dad.reconstruct_grad(Qt, sGt).cpu().numpy(), Q_ref.T @ sG_ref)
    assert err <= tol, (err, tol)


@pytest.mark.parametrize("N,h,h_next,act", [(int(a), int(b), int(c), ["identity", "relu", "tanh", "sigmoid"][int(k)])
                                            for a, b, c, k in np.random.default_rng(104).integers(
                                                [1, 1, 1, 0], [300, 300, 300, 4], size=(16, 4))])
def test_random_shapes_backprop(gpu, N, h, h_next, act):
    rng = np.random.default_rng([105, N, h, h_next])
    Dn = rng.standard_normal((N, h_next)).astype(np.float32)
    Wn = rng.standard_normal((h, h_next)).astype(np.float32)
    Z = rng.standard_normal((N, h)).astype(np.float32)
    got = dad.backprop_delta(torch.from_numpy(Dn).to(gpu), torch.from_numpy(Wn).to(gpu), torch.from_numpy(Z).to(gpu),
                             act).cpu().numpy()
    assert O.rel_fro(got, O.backprop_delta(Dn, Wn, Z, act)) <= 1e-5


def bf16_cases():
    rng = np.random.default_rng(106)
    out = []
    for i in range(18):
        aligned = i % 3 != 2           # two of three: widths the MFMA kernels take (multiples of 128, r of 8)
        N = int(rng.integers(256, 1400)) if aligned else int(rng.integers(1, 700))
        if i % 6 == 0:
            N = 256 * int(rng.integers(1, 5))                      # the direct-to-LDS kernels' row counts
        if aligned:
            h_in, h_out = 128 * int(rng.integers(1, 6)), 128 * int(rng.integers(1, 6))
            r = 8 * int(rng.integers(1, 9))
        else:
            h_in, h_out = int(rng.integers(8, 500)), int(rng.integers(8, 500))
            r = int(rng.integers(1, min(N, h_in, h_out, 40) + 1))
        out.append((N, h_in, h_out, min(r, N)))
    return out


@pytest.mark.parametrize("N,h_in,h_out,r", bf16_cases())
def test_random_shapes_bf16(gpu, N, h_in, h_out, r):
    """bf16 factors on all three kernel families: direct-to-LDS MFMA (N a multiple of 256),
    register-staged MFMA (ragged N) and guarded kernels (ragged widths)."""
    from paper_2102_09631_amd import workloads as W
    rng = np.random.default_rng([107, N, h_in, h_out, r])
    rb = lambda x: W.bf16_bits_to_f32(W.f32_to_bf16_bits(x.astype(np.float32)))
    A, D = rb(rng.standard_normal((N, h_in))), rb(rng.standard_normal((N, h_out)) * 0.01)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    a = torch.from_numpy(A).to(gpu).to(torch.bfloat16)
    d = torch.from_numpy(D).to(gpu).to(torch.bfloat16)
    assert O.rel_fro(dad.reconstruct_grad(a, d).cpu().numpy(), O.full_grad(A, D)) <= 2e-2
    Pt, Gt = dad.compress_rank(a, d, r, 2, torch.from_numpy(G0).to(gpu), check=True)
    err = O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), O.rank_r_grad(*O.block_spi(A, D, G0, 2)))
    assert err <= 2e-2, err
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-4
