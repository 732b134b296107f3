"""Parity of the HIP path (through the C ABI) with the fp64 CPU oracle, element by
element on the same seeded inputs.  Bars: bit-exact for the stack (a copy);
relative Frobenius error <= 1e-5 for fp32 factors and <= 2e-2 for bf16 factors
with fp32 accumulation.
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


def run_layer(w, layer, h_in, h_out, dev, rows=None, sites=None, r=None, n_iter=None):
    """Stack -> full rebuild -> compress -> rank-r rebuild on the GPU, and the same in the oracle."""
    r = w.rank if r is None else r
    n_iter = w.n_iter if n_iter is None else n_iter
    A_sites, D_sites = W.host_factors(w, layer, h_in, h_out, rows=rows, sites=sites)
    G0 = W.host_start_matrix(w, layer, h_out, r=r)
    A, D = dad.stack_factors([to_dev(a, w.dtype, dev) for a in A_sites], [to_dev(d, w.dtype, dev) for d in D_sites])
    G_full = dad.reconstruct_grad(A, D)
    Pt, Gt = dad.compress_rank(A, D, r, n_iter, torch.from_numpy(G0).to(dev), check=True)
    G_r = dad.reconstruct_grad(Pt, Gt)
    torch.cuda.synchronize()
    A_ref, D_ref = O.stack_factors(A_sites, D_sites)
    out = {
        "stack_exact": bool(np.array_equal(A.float().cpu().numpy(), A_ref)
                            and np.array_equal(D.float().cpu().numpy(), D_ref)),
        "e_full": O.rel_fro(G_full.cpu().numpy(), O.full_grad(A_ref, D_ref)),
    }
    Pt_ref, Gt_ref = O.block_spi(A_ref, D_ref, G0, n_iter)
    out["e_rank"] = O.rel_fro(G_r.cpu().numpy(), O.rank_r_grad(Pt_ref, Gt_ref))
    Gt_h = Gt.cpu().numpy().astype(np.float64)
    out["orth"] = float(np.abs(Gt_h @ Gt_h.T - np.eye(r)).max())
    out["e_G"] = O.rel_fro(Gt_h, Gt_ref)           # diagnostic only: a basis is not unique in general
    out["shapes"] = (tuple(Pt.shape), tuple(Gt.shape), tuple(G_full.shape), tuple(G_r.shape))
    return out


def check(out, dtype, r, h_in, h_out):
    assert out["shapes"] == ((r, h_in), (r, h_out), (h_in, h_out), (h_in, h_out))
    assert out["stack_exact"]
    assert out["e_full"] <= TOL[dtype], out
    assert out["e_rank"] <= TOL[dtype], out
    assert out["orth"] <= (1e-5 if dtype == "f32" else 1e-4), out


def test_single_linear_784x128(gpu):
    w = W.WORKLOADS[0]
    out = run_layer(w, 0, 784, 128, gpu)
    print(out)
    check(out, "f32", 4, 784, 128)


@pytest.mark.parametrize("layer", [0, 1, 2])
def test_mlp_784_1024_1024_10(gpu, layer):
    w = W.WORKLOADS[1]
    _, h_in, h_out = w.all_layers()[layer]
    out = run_layer(w, layer, h_in, h_out, gpu)
    print(out)
    check(out, "f32", 8, h_in, h_out)


@pytest.mark.parametrize("layer", [0, 1, 2, 3])
def test_encoder_d768_reduced_rows(gpu, layer):
    """Encoder shapes with 4 sites x 640 rows: several row tiles and a K-split."""
    w = W.WORKLOADS[2]
    _, h_in, h_out = w.all_layers()[layer]
    out = run_layer(w, layer, h_in, h_out, gpu, rows=640)
    print(out)
    check(out, "bf16", 16, h_in, h_out)


@pytest.mark.parametrize("dtype_idx,N_rows,h_in,h_out,r", [
    (0, 37, 50, 23, 3),      # everything ragged, fp32
    (0, 1, 9, 5, 1),         # one sample per site
    (2, 77, 136, 72, 8),     # bf16, widths multiple of 8 only
    (2, 33, 65, 31, 5),      # bf16, odd widths (unaligned rows)
    (4, 200, 256, 384, 64),  # largest rank, GELU / Student-t draws
    (1, 300, 64, 64, 64),    # r equal to both widths
    (2, 100, 2050, 520, 16),  # bf16, few rows and wide: column-split guarded thin_nn, ragged last chunk
    (0, 20, 3000, 700, 4),    # fp32, N << h: many column chunks, finest row split
    (3, 512, 1024, 768, 32),  # direct-to-LDS kernels, 3 column strips, 2 row chunks (plain strip mapping)
    (3, 2048, 512, 2048, 32), # direct-to-LDS kernels, 8 row chunks (strips of a chunk share an XCD)
    (3, 600, 1024, 1024, 32), # N not a multiple of 256: register-staged MFMA kernels, ragged row tile
    (3, 256, 512, 256, 24),   # direct-to-LDS thin_nn with a padded panel (r < 32), register-staged thin_tn
    (4, 256, 256, 384, 48),   # the same with r between 32 and 64
    (2, 256, 384, 640, 8),    # smallest rank the MFMA kernels take; widths multiples of 128 only: 128-tile rebuild
    (3, 352, 640, 128, 16),   # 128-tile rebuild with a single column of tiles and K = 1056 (33 stages)
    (3, 256, 384, 640, 16),   # direct-to-LDS thin_tn with 128-column strips (widths not multiples of 256)
    (3, 256, 640, 384, 32),
])
def test_ragged_and_edge_shapes(gpu, dtype_idx, N_rows, h_in, h_out, r):
    w = W.WORKLOADS[dtype_idx]
    out = run_layer(w, 7, h_in, h_out, gpu, rows=N_rows, sites=3, r=r, n_iter=2)
    print(out)
    check(out, w.dtype, r, h_in, h_out)


def test_stack_with_empty_and_uneven_sites(gpu):
    rng = np.random.default_rng(5)
    rows = [5, 0, 17, 1, 64]
    for dtype, width in (("f32", (7, 3)), ("bf16", (9, 5)), ("bf16", (64, 128))):
        A_s = [rng.standard_normal((n, width[0])).astype(np.float32) for n in rows]
        D_s = [rng.standard_normal((n, width[1])).astype(np.float32) for n in rows]
        if dtype == "bf16":
            A_s = [W.bf16_bits_to_f32(W.f32_to_bf16_bits(a)).reshape(a.shape) for a in A_s]
            D_s = [W.bf16_bits_to_f32(W.f32_to_bf16_bits(d)).reshape(d.shape) for d in D_s]
        # each site block gets its own 16-byte aligned allocation
        A, D = dad.stack_factors([to_dev(a, dtype, gpu) for a in A_s], [to_dev(d, dtype, gpu) for d in D_s])
        A_ref, D_ref = O.stack_factors(A_s, D_s)
        assert A.shape == A_ref.shape and D.shape == D_ref.shape
        assert np.array_equal(A.float().cpu().numpy(), A_ref)
        assert np.array_equal(D.float().cpu().numpy(), D_ref)


def test_stack_of_forty_uneven_sites_takes_a_second_launch(gpu):
    """A copy launch holds 64 segments, i.e. the A and Delta blocks of 32 sites: 40 sites need two."""
    rng = np.random.default_rng(6)
    rows = [int(n) for n in rng.integers(0, 40, size=40)]
    rows[3] = 0
    for dtype, width in (("bf16", (33, 7)), ("f32", (24, 16))):     # odd bf16 widths: 2-byte tails and offsets
        A_s = [rng.standard_normal((n, width[0])).astype(np.float32) for n in rows]
        D_s = [rng.standard_normal((n, width[1])).astype(np.float32) for n in rows]
        if dtype == "bf16":
            A_s = [W.bf16_bits_to_f32(W.f32_to_bf16_bits(a)).reshape(a.shape) for a in A_s]
            D_s = [W.bf16_bits_to_f32(W.f32_to_bf16_bits(d)).reshape(d.shape) for d in D_s]
        A, D = dad.stack_factors([to_dev(a, dtype, gpu) for a in A_s], [to_dev(d, dtype, gpu) for d in D_s])
        A_ref, D_ref = O.stack_factors(A_s, D_s)
        assert np.array_equal(A.float().cpu().numpy(), A_ref) and np.array_equal(D.float().cpu().numpy(), D_ref)


def test_rank_budget_at_least_gradient_rank_recovers_gradient(gpu):
    """r = rank(M) = N: the rank-r gradient equals the full gradient and the truncated SVD."""
    w = W.WORKLOADS[0]
    A_sites, D_sites = W.host_factors(w, 3, 96, 48, rows=2, sites=2)      # N = 4
    G0 = W.host_start_matrix(w, 3, 48, r=4)
    A, D = dad.stack_factors([to_dev(a, "f32", gpu) for a in A_sites], [to_dev(d, "f32", gpu) for d in D_sites])
    Pt, Gt = dad.compress_rank(A, D, 4, 2, torch.from_numpy(G0).to(gpu), check=True)
    G_r = dad.reconstruct_grad(Pt, Gt).cpu().numpy()
    M = O.full_grad(*O.stack_factors(A_sites, D_sites))
    assert O.rel_fro(G_r, M) <= 1e-5
    assert O.rel_fro(G_r, O.truncated_svd(M, 4)) <= 1e-5


@pytest.mark.parametrize("ratio,N,h_in,h_out,r", [(0.8, 64, 96, 80, 8), (0.5, 64, 96, 80, 8), (0.3, 64, 96, 80, 8),
                                                   (0.5, 512, 256, 384, 16), (0.1, 64, 96, 80, 8)])
def test_steep_spectrum_keeps_orthonormality_and_degrades_gracefully(gpu, ratio, N, h_in, h_out, r):
    """Delta rows scaled geometrically: sigma_1/sigma_r up to 1e7.  The Cholesky orthonormalisation
    (fp64 Gram and factorisation) must not break down and G must stay orthonormal to fp32 accuracy.
    The fp32 contractions resolve a direction of relative size sigma_r/sigma_1 only to
    eps32 * sigma_1/sigma_r, which bounds the distance to the fp64 oracle."""
    rng = np.random.default_rng([11, int(ratio * 10), N])
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    D = (rng.standard_normal((N, h_out)) * (ratio ** np.arange(N))[:, None]).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    ws = torch.empty(dad.compress_workspace_bytes(N, h_in, h_out, r, torch.float32), dtype=torch.uint8, device=gpu)
    Pt, Gt = dad.compress_rank(torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu), r, 2,
                               torch.from_numpy(G0).to(gpu), workspace=ws)
    assert dad.poll_numeric_status(ws) == dad.DAD_OK
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-5
    s = np.linalg.svd(A.astype(np.float64).T @ D.astype(np.float64), compute_uv=False)
    bound = 1e-5 + np.finfo(np.float32).eps * s[0] / s[r - 1]
    err = O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), O.rank_r_grad(*O.block_spi(A, D, G0, 2)))
    print(ratio, N, r, "sigma_1/sigma_r", s[0] / s[r - 1], "err", err, "bound", bound)
    assert err <= bound


@pytest.mark.parametrize("ratio,r", [(0.9, 32), (0.8, 32), (0.5, 16)])
def test_steep_spectrum_bf16_path(gpu, ratio, r):
    """The same on the bf16 MFMA path (sigma_1/sigma_r from 3e1 to 3e4): the N x r intermediates and the
    panels are rounded to bf16, which puts a floor of about 2e-3 under the error but must not cost
    rank or orthonormality."""
    N, h_in, h_out = 1024, 256, 512
    rng = np.random.default_rng([12, int(ratio * 10), r])
    rnd = lambda x: W.bf16_bits_to_f32(W.f32_to_bf16_bits(x.astype(np.float32)))
    A = rnd(rng.standard_normal((N, h_in)))
    D = rnd(rng.standard_normal((N, h_out)) * (ratio ** np.arange(N))[:, None])
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    ws = torch.empty(dad.compress_workspace_bytes(N, h_in, h_out, r, torch.bfloat16), dtype=torch.uint8, device=gpu)
    Pt, Gt = dad.compress_rank(to_dev(A, "bf16", gpu), to_dev(D, "bf16", gpu), r, 2, torch.from_numpy(G0).to(gpu),
                               workspace=ws)
    assert dad.poll_numeric_status(ws) == dad.DAD_OK
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-4
    err = O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), O.rank_r_grad(*O.block_spi(A, D, G0, 2)))
    print(ratio, r, err)
    assert err <= TOL["bf16"]


def test_rank_pairs_restack_and_recompress(gpu):
    """Algorithm 1: per-site rank-r pairs are stacked (N' = S*r rows) and compressed again."""
    w = W.WORKLOADS[0]
    S, r = 3, 4
    A_sites, D_sites = W.host_factors(w, 5, 112, 80, rows=24, sites=S)
    G0s = [W.host_start_matrix(w, 10 + s, 80, r=r) for s in range(S)]
    G0agg = W.host_start_matrix(w, 20, 80, r=r)
    pairs_gpu, pairs_ref = [], []
    for s in range(S):
        a, d = to_dev(A_sites[s], "f32", gpu), to_dev(D_sites[s], "f32", gpu)
        pairs_gpu.append(dad.compress_rank(a, d, r, 2, torch.from_numpy(G0s[s]).to(gpu), check=True))
        pairs_ref.append(O.block_spi(A_sites[s], D_sites[s], G0s[s], 2))
    Pst, Gst = dad.stack_factors([p for p, _ in pairs_gpu], [g for _, g in pairs_gpu])
    assert tuple(Pst.shape) == (S * r, 112) and tuple(Gst.shape) == (S * r, 80)
    Pt, Gt = dad.compress_rank(Pst, Gst, r, 2, torch.from_numpy(G0agg).to(gpu), check=True)
    G_hat = dad.reconstruct_grad(Pt, Gt).cpu().numpy()
    Pst_ref, Gst_ref = O.stack_factors([p for p, _ in pairs_ref], [g for _, g in pairs_ref])
    ref = O.rank_r_grad(*O.block_spi(Pst_ref, Gst_ref, G0agg, 2))
    assert O.rel_fro(G_hat, ref) <= 1e-5


@pytest.mark.parametrize("route", ["block", "gram"])
def test_equal_pivots_do_not_hide_an_ill_conditioned_iterate(gpu, route):
    """A = Delta = I make M the identity, so with one application the iterate that is orthonormalised
    is the start matrix itself: Y = G0^T = Q R with R unit upper triangular and -1 above the diagonal.
    Every Cholesky pivot of Y^T Y is 1 although cond(R) grows like 2^r (here ~5e3): one fp32 round
    would leave G^T G - I at ~1e-4, so the decision to skip the second round must not be taken from the
    pivots.  span(Y) is the whole r-dimensional span of Q, hence P G^T = Q Q^T."""
    h, r = 64, 12
    rng = np.random.default_rng(77)
    Q, _ = np.linalg.qr(rng.standard_normal((h, r)))
    R = np.eye(r) - np.triu(np.ones((r, r)), 1)
    G0 = np.ascontiguousarray((Q @ R).T.astype(np.float32))   # r x h_out, row j = column j of Y
    eye = torch.eye(h, device=gpu)
    call = dad.compress_rank if route == "block" else dad.compress_rank_gram
    Pt, Gt = call(eye, eye.clone(), r, 1, torch.from_numpy(G0).to(gpu), check=True)
    g = Gt.cpu().numpy().astype(np.float64)
    assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-5
    ref = O.rank_r_grad(*O.block_spi(np.eye(h), np.eye(h), G0, 1))
    # Y R^-1 in fp32 resolves the span of Y only to eps32 * cond(Y), as on the steep spectra above
    tol = 1e-5 + np.finfo(np.float32).eps * np.linalg.cond(R)
    assert O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), ref) <= tol


def test_zero_deltas_latch_numeric_breakdown(gpu):
    A = torch.ones((16, 32), device=gpu)
    D = torch.zeros((16, 24), device=gpu)
    G0 = torch.from_numpy(W.host_start_matrix(W.WORKLOADS[0], 0, 24, r=2)).to(gpu)
    ws = torch.empty(dad.compress_workspace_bytes(16, 32, 24, 2, torch.float32), dtype=torch.uint8, device=gpu)
    dad.compress_rank(A, D, 2, 1, G0, workspace=ws)
    assert dad.poll_numeric_status(ws) == dad.DAD_ERR_NUMERIC
    # the flag is cleared by the next call on the same workspace
    D2 = torch.from_numpy(W.host_factors(W.WORKLOADS[0], 1, 32, 24, rows=16, sites=1)[1][0]).to(gpu)
    dad.compress_rank(A * torch.arange(1, 33, device=gpu), D2, 2, 1, G0, workspace=ws)
    assert dad.poll_numeric_status(ws) == dad.DAD_OK


def test_rerun_is_bit_identical(gpu):
    """Fixed-order reductions (no float atomics): two runs give the same bits."""
    w = W.WORKLOADS[1]
    A_sites, D_sites = W.host_factors(w, 1, 1024, 1024)
    A, D = dad.stack_factors([to_dev(a, "f32", gpu) for a in A_sites], [to_dev(d, "f32", gpu) for d in D_sites])
    G0 = torch.from_numpy(W.host_start_matrix(w, 1, 1024)).to(gpu)
    runs = []
    for _ in range(2):
        G = dad.reconstruct_grad(A, D)
        Pt, Gt = dad.compress_rank(A, D, 8, 2, G0, check=True)
        runs.append((G.clone(), Pt.clone(), Gt.clone()))
    for x, y in zip(*runs):
        assert torch.equal(x, y)


def test_calls_can_be_captured_in_a_hip_graph(gpu):
    """The entry points only enqueue kernels on the caller's stream (no allocation, no sync, no memset),
    so a caller may capture them; every replay must reproduce the eager result bit for bit."""
    w = W.WORKLOADS[2]
    A_sites, D_sites = W.host_factors(w, 1, 768, 768, rows=512)
    As = [to_dev(a, "bf16", gpu) for a in A_sites]
    Ds = [to_dev(d, "bf16", gpu) for d in D_sites]
    G0 = torch.from_numpy(W.host_start_matrix(w, 1, 768)).to(gpu)
    N = 4 * 512
    A = torch.empty((N, 768), dtype=torch.bfloat16, device=gpu)
    D = torch.empty((N, 768), dtype=torch.bfloat16, device=gpu)
    Pt = torch.empty((16, 768), device=gpu)
    Gt = torch.empty((16, 768), device=gpu)
    G = torch.empty((768, 768), device=gpu)
    Gr = torch.empty((768, 768), device=gpu)
    ws_c = torch.empty(dad.compress_workspace_bytes(N, 768, 768, 16, torch.bfloat16), dtype=torch.uint8, device=gpu)
    ws_r = torch.empty(max(16, dad.reconstruct_workspace_bytes(N, 768, 768, torch.bfloat16)), dtype=torch.uint8,
                       device=gpu)

    def path():
        dad.stack_factors(As, Ds, A_out=A, D_out=D)
        dad.compress_rank(A, D, 16, 2, G0, Pt=Pt, Gt=Gt, workspace=ws_c)
        dad.reconstruct_grad(A, D, G=G, workspace=ws_r)
        dad.reconstruct_grad(Pt, Gt, G=Gr)

    path()                      # eager: also performs the one-time kernel attribute set-up
    torch.cuda.synchronize()
    ref = [x.clone() for x in (A, D, Pt, Gt, G, Gr)]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        path()
    for rep in range(3):
        for x in (A, D, Pt, Gt, G, Gr):
            x.fill_(float(rep + 1))          # eager work between replays, and stale outputs to overwrite
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for x, y in zip((A, D, Pt, Gt, G, Gr), ref):
            assert torch.equal(x, y)
    assert dad.poll_numeric_status(ws_c) == dad.DAD_OK
