"""Parity of dad_compress_rank_gram (the few-rows form: the iteration runs on A A^T and
Delta Delta^T, Algorithm 2's precomputation) with the fp64 oracle.  The rank-r gradient
Pt^T Gt is unique given (A, Delta, G0, n_iter), so it is compared with block_spi's and with the
explicit-C route of the oracle; bars as for dad_compress_rank (1e-5 fp32, 2e-2 bf16).
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
    Pt, Gt = dad.compress_rank_gram(to_dev(A, dtype, dev), to_dev(D, dtype, dev), r, n_iter,
                                    torch.from_numpy(G0).to(dev), check=True)
    G_r = dad.reconstruct_grad(Pt, Gt).cpu().numpy()
    Pt_ref, Gt_ref = O.block_spi(A, D, G0, n_iter)
    g = Gt.cpu().numpy().astype(np.float64)
    return {
        "e_rank": O.rel_fro(G_r, O.rank_r_grad(Pt_ref, Gt_ref)),
        "orth": float(np.abs(g @ g.T - np.eye(r)).max()),
        "e_G": O.rel_fro(g, Gt_ref),
        "e_P": O.rel_fro(Pt.cpu().numpy().astype(np.float64), Pt_ref),
        "shapes": (tuple(Pt.shape), tuple(Gt.shape)),
    }


@pytest.mark.parametrize("N,h_in,h_out,r,n_iter", [
    (64, 784, 128, 4, 2),       # the single-linear workload's shape
    (12, 112, 80, 4, 2),        # an aggregator's stack of 3 rank-4 pairs
    (37, 53, 29, 3, 3),         # nothing divides anything
    (5, 17, 9, 5, 1),           # r = N
    (256, 1024, 4096, 32, 2),   # aggregator of the GPT-2-medium workload: 8 x rank 32
    (200, 300, 520, 17, 2),     # ragged rows and rank, 4 column chunks
    (1, 40, 24, 1, 2),          # one row: M is an outer product
    (130, 96, 1031, 33, 2),     # r > 32 takes the 4 x 4 ownership, odd width
])
def test_gram_route_fp32_matches_oracle(gpu, N, h_in, h_out, r, n_iter):
    rng = np.random.default_rng([31, N, h_in, h_out])
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    D = rng.standard_normal((N, h_out)).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    out = run(A, D, G0, r, n_iter, "f32", gpu)
    print(N, h_in, h_out, r, n_iter, out)
    assert out["shapes"] == ((r, h_in), (r, h_out))
    assert out["e_rank"] <= TOL["f32"], out
    assert out["orth"] <= 1e-5, out
    # both sides orthonormalise with a positive-diagonal triangular factor: the bases coincide too
    assert out["e_G"] <= 1e-4 and out["e_P"] <= 1e-4, out


def test_gram_route_largest_row_count(gpu):
    """N = DAD_GRAM_MAX_ROWS, r = 64: the ViT-large aggregator (16 sites x rank 64) at reduced width."""
    N, h_in, h_out, r = 1024, 640, 1280, 64
    rng = np.random.default_rng(32)
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    D = rng.standard_normal((N, h_out)).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    out = run(A, D, G0, r, 2, "f32", gpu)
    print(out)
    assert out["e_rank"] <= TOL["f32"] and out["orth"] <= 1e-5, out


@pytest.mark.parametrize("N,h_in,h_out,r", [(256, 768, 2304, 16), (100, 264, 520, 8), (64, 250, 130, 4)])
def test_gram_route_bf16_factors(gpu, N, h_in, h_out, r):
    """bf16 factors: their products are exact in the fp64 Gram matrices, so only the fp32 accumulation
    of the two projections separates the result from the oracle - far inside the bf16 bar, and G stays
    orthonormal to fp32 accuracy (nothing on this route is rounded to bf16).  The third shape has row
    lengths that 16-byte loads cannot take."""
    rng = np.random.default_rng([33, N, h_in, h_out])
    A = bf16_round(rng.standard_normal((N, h_in)))
    D = bf16_round(rng.standard_normal((N, h_out)) * 0.01)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    out = run(A, D, G0, r, 2, "bf16", gpu)
    print(N, h_in, h_out, r, out)
    assert out["e_rank"] <= TOL["bf16"] and out["e_rank"] <= 1e-4, out
    assert out["orth"] <= 1e-5, out


def test_gram_route_equals_block_route_on_the_gpu(gpu):
    """The two entry points give the same rank-r gradient (and, here, the same pair)."""
    w = W.WORKLOADS[1]
    A_s, D_s = W.host_factors(w, 1, 1024, 1024)
    A, D = O.stack_factors(A_s, D_s)                       # N = 1024 rows
    G0 = torch.from_numpy(W.host_start_matrix(w, 1, 1024)).to(gpu)
    a, d = to_dev(A.astype(np.float32), "f32", gpu), to_dev(D.astype(np.float32), "f32", gpu)
    Pb, Gb = dad.compress_rank(a, d, w.rank, w.n_iter, G0, check=True)
    Pg, Gg = dad.compress_rank_gram(a, d, w.rank, w.n_iter, G0, check=True)
    e = O.rel_fro(dad.reconstruct_grad(Pg, Gg).cpu().numpy(), dad.reconstruct_grad(Pb, Gb).cpu().numpy().astype(np.float64))
    print(e)
    assert e <= 1e-5
    assert O.rel_fro(Gg.cpu().numpy(), Gb.cpu().numpy().astype(np.float64)) <= 1e-4


@pytest.mark.parametrize("ratio", [0.8, 0.5, 0.3])
def test_gram_route_planted_spectrum(gpu, ratio):
    """Delta rows scaled geometrically (sigma_1/sigma_r = 5, 1e2 and 6e3): the Gram form squares the
    conditioning of the iterate but works in fp64; G stays orthonormal and the result stays at
    fp32 rounding distance from the oracle.  The steeper two take the second Cholesky round."""
    N, h_in, h_out, r = 64, 96, 80, 8
    rng = np.random.default_rng([34, int(ratio * 10)])
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    D = (rng.standard_normal((N, h_out)) * (ratio ** np.arange(N))[:, None]).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    out = run(A, D, G0, r, 2, "f32", gpu)
    print(ratio, out)
    assert out["e_rank"] <= TOL["f32"] and out["orth"] <= 1e-5, out


def test_gram_route_beyond_its_conditioning_range_says_so(gpu):
    """sigma_1/sigma_r = 1e7: the Gram matrix of the iterate (condition number 1e28) is beyond fp64.
    The call must either latch DAD_ERR_NUMERIC or deliver a valid pair - never a silent wrong answer -
    and the outputs stay finite."""
    N, h_in, h_out, r = 64, 96, 80, 8
    rng = np.random.default_rng([34, 1])
    A = rng.standard_normal((N, h_in)).astype(np.float32)
    D = (rng.standard_normal((N, h_out)) * (0.1 ** np.arange(N))[:, None]).astype(np.float32)
    G0 = rng.standard_normal((r, h_out)).astype(np.float32)
    ws = torch.empty(dad.compress_gram_workspace_bytes(N, h_in, h_out, r, torch.float32), dtype=torch.uint8, device=gpu)
    Pt, Gt = dad.compress_rank_gram(torch.from_numpy(A).to(gpu), torch.from_numpy(D).to(gpu), r, 2,
                                    torch.from_numpy(G0).to(gpu), workspace=ws)
    status = dad.poll_numeric_status(ws)
    assert torch.isfinite(Pt).all() and torch.isfinite(Gt).all()
    if status == dad.DAD_OK:
        g = Gt.cpu().numpy().astype(np.float64)
        assert np.abs(g @ g.T - np.eye(r)).max() <= 1e-5
        assert O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), O.rank_r_grad(*O.block_spi(A, D, G0, 2))) <= 1e-4
    else:
        assert status == dad.DAD_ERR_NUMERIC


def test_gram_route_rank_budget_equal_to_rank_recovers_gradient(gpu):
    """r = N = rank(M): the pair reproduces M and the truncated SVD."""
    rng = np.random.default_rng(35)
    A = rng.standard_normal((6, 96)).astype(np.float32)
    D = rng.standard_normal((6, 48)).astype(np.float32)
    G0 = rng.standard_normal((6, 48)).astype(np.float32)
    Pt, Gt = dad.compress_rank_gram(to_dev(A, "f32", gpu), to_dev(D, "f32", gpu), 6, 2, torch.from_numpy(G0).to(gpu),
                                    check=True)
    M = O.full_grad(A, D)
    G_r = dad.reconstruct_grad(Pt, Gt).cpu().numpy()
    assert O.rel_fro(G_r, M) <= 1e-5 and O.rel_fro(G_r, O.truncated_svd(M, 6)) <= 1e-5


def test_gram_route_two_level_aggregator(gpu):
    """Algorithm 1 with the aggregator's reduction on the Gram route, against the oracle's rank_dad."""
    w = W.WORKLOADS[0]
    S, r = 3, 4
    A_sites, D_sites = W.host_factors(w, 5, 112, 80, rows=24, sites=S)
    G0s = [W.host_start_matrix(w, 10 + s, 80, r=r) for s in range(S)]
    G0agg = W.host_start_matrix(w, 20, 80, r=r)
    pairs = [dad.compress_rank(to_dev(A_sites[s], "f32", gpu), to_dev(D_sites[s], "f32", gpu), r, 2,
                               torch.from_numpy(G0s[s]).to(gpu), check=True) for s in range(S)]
    Pst, Gst = dad.stack_factors([p for p, _ in pairs], [g for _, g in pairs])
    Pt, Gt = dad.compress_rank_gram(Pst, Gst, r, 2, torch.from_numpy(G0agg).to(gpu), check=True)
    Pt_ref, Gt_ref, _ = O.rank_dad(A_sites, D_sites, G0s, G0agg, 2)
    assert O.rel_fro(dad.reconstruct_grad(Pt, Gt).cpu().numpy(), O.rank_r_grad(Pt_ref, Gt_ref)) <= 1e-5


def test_gram_route_lost_rank_latches_numeric_status(gpu):
    """Delta = 0: the Gram matrix of the iterate vanishes, no pivot is positive; the call ends with
    finite outputs and the status latched, and the next call on the same workspace clears it."""
    rng = np.random.default_rng(36)
    A = torch.from_numpy(rng.standard_normal((32, 40)).astype(np.float32)).to(gpu)
    D = torch.from_numpy(rng.standard_normal((32, 24)).astype(np.float32)).to(gpu)
    G0 = torch.from_numpy(rng.standard_normal((2, 24)).astype(np.float32)).to(gpu)
    ws = torch.empty(dad.compress_gram_workspace_bytes(32, 40, 24, 2, torch.float32), dtype=torch.uint8, device=gpu)
    Pt, Gt = dad.compress_rank_gram(A, torch.zeros_like(D), 2, 1, G0, workspace=ws)
    assert dad.poll_numeric_status(ws) == dad.DAD_ERR_NUMERIC
    assert torch.isfinite(Pt).all() and torch.isfinite(Gt).all()
    dad.compress_rank_gram(A, D, 2, 1, G0, workspace=ws)
    assert dad.poll_numeric_status(ws) == dad.DAD_OK


def test_gram_route_reruns_are_bit_identical_and_graph_capturable(gpu):
    rng = np.random.default_rng(37)
    A = torch.from_numpy(rng.standard_normal((256, 1024)).astype(np.float32)).to(gpu)
    D = torch.from_numpy(rng.standard_normal((256, 512)).astype(np.float32)).to(gpu)
    G0 = torch.from_numpy(rng.standard_normal((16, 512)).astype(np.float32)).to(gpu)
    ws = torch.empty(dad.compress_gram_workspace_bytes(256, 1024, 512, 16, torch.float32), dtype=torch.uint8, device=gpu)
    Pt = torch.empty((16, 1024), device=gpu)
    Gt = torch.empty((16, 512), device=gpu)
    dad.compress_rank_gram(A, D, 16, 2, G0, Pt=Pt, Gt=Gt, workspace=ws)
    torch.cuda.synchronize()
    P0, G0ref = Pt.clone(), Gt.clone()
    dad.compress_rank_gram(A, D, 16, 2, G0, Pt=Pt, Gt=Gt, workspace=ws)
    torch.cuda.synchronize()
    assert torch.equal(Pt, P0) and torch.equal(Gt, G0ref)
    graph = torch.cuda.CUDAGraph()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        with torch.cuda.graph(graph, stream=side):
            dad.compress_rank_gram(A, D, 16, 2, G0, Pt=Pt, Gt=Gt, workspace=ws)
    for _ in range(3):
        Pt.zero_(); Gt.zero_()
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        assert torch.equal(Pt, P0) and torch.equal(Gt, G0ref)


def test_one_workspace_serves_all_compress_entry_points_in_turn(gpu):
    """The three compressions keep their flag and ticket words at the same place of the workspace and
    clear them at the start of every call: one buffer, used by one call after the other, gives each
    of them the result it gives on a fresh buffer, bit for bit."""
    rng = np.random.default_rng(38)
    mk = lambda *shape: torch.from_numpy(rng.standard_normal(shape).astype(np.float32)).to(gpu)
    A1, D1, G1 = mk(512, 256), mk(512, 384), mk(16, 384)        # block route (guarded kernels, fp32)
    A2, D2, G2 = mk(96, 200), mk(96, 136), mk(8, 136)           # Gram route
    A3, D3, G3 = mk(300, 64), mk(300, 80), mk(3, 80)            # sequential route
    A4 = mk(1024, 256).to(torch.bfloat16)                        # block route, bf16 MFMA kernels
    D4, G4 = mk(1024, 512).to(torch.bfloat16), mk(32, 512)
    calls = [
        (dad.compress_rank, (A1, D1, 16, 2, G1), dad.compress_workspace_bytes(512, 256, 384, 16, torch.float32)),
        (dad.compress_rank_gram, (A2, D2, 8, 2, G2), dad.compress_gram_workspace_bytes(96, 200, 136, 8, torch.float32)),
        (dad.compress_rank_sequential, (A3, D3, 3, 2, G3),
         dad.lib().dad_compress_sequential_workspace_bytes(300, 64, 80, dad.DAD_F32)),
        (dad.compress_rank, (A4, D4, 32, 2, G4), dad.compress_workspace_bytes(1024, 256, 512, 32, torch.bfloat16)),
    ]
    fresh = []
    for fn, args, nbytes in calls:
        ws = torch.full((nbytes,), 0xA5, dtype=torch.uint8, device=gpu)      # not zero on purpose
        fresh.append([x.clone() for x in fn(*args, workspace=ws)])
        assert dad.poll_numeric_status(ws) == dad.DAD_OK
    shared = torch.full((max(c[2] for c in calls),), 0x5A, dtype=torch.uint8, device=gpu)
    for rounds in range(2):
        for (fn, args, _), ref in zip(calls, fresh):
            out = fn(*args, workspace=shared)
            torch.cuda.synchronize()
            assert dad.poll_numeric_status(shared) == dad.DAD_OK
            for x, y in zip(out, ref):
                assert torch.equal(x, y)
