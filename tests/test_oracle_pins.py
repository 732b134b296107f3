"""Pins for the fp64 CPU oracle: each check ties an oracle function to something
other than itself (finite differences, brute force, numpy's SVD, closed forms,
invariants of orthogonal projections).  CPU only.
"""
import json
import os

import numpy as np
import pytest

from oracle import dad_oracle as O

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _tiny_mlp(rng, sizes=(5, 7, 6, 3), acts=("tanh", "sigmoid", "identity")):
    Ws = [rng.standard_normal((sizes[i], sizes[i + 1])) * 0.7 for i in range(len(sizes) - 1)]
    Bs = [rng.standard_normal(sizes[i + 1]) * 0.3 for i in range(len(sizes) - 1)]
    return Ws, Bs, list(acts)


# ---------------------------------------------------------------- Eq. 1-4 vs finite differences

@pytest.mark.parametrize("acts", [("tanh", "sigmoid", "identity"), ("relu", "tanh", "tanh")])
def test_factors_give_finite_difference_gradient(acts):
    """Eq. 4 with the factors of Eq. 2-3 is the derivative of the loss (check 1)."""
    rng = np.random.default_rng(7)
    Ws, Bs, acts = _tiny_mlp(rng, acts=acts)
    X = rng.standard_normal((9, 5))
    Y = rng.standard_normal((9, 3))
    factors = O.mlp_factors(Ws, Bs, acts, X, Y)
    eps = 1e-6
    for li, (A, D) in enumerate(factors):
        G = O.full_grad(A, D)
        assert G.shape == Ws[li].shape            # orientation h_{i-1} x h_i
        fd = np.zeros_like(G)
        for p in range(G.shape[0]):
            for q in range(G.shape[1]):
                Wp = [w.copy() for w in Ws]
                Wm = [w.copy() for w in Ws]
                Wp[li][p, q] += eps
                Wm[li][p, q] -= eps
                fd[p, q] = (O.mlp_loss(Wp, Bs, acts, X, Y) - O.mlp_loss(Wm, Bs, acts, X, Y)) / (2 * eps)
        assert np.linalg.norm(G - fd) / np.linalg.norm(fd) < 1e-7


def test_bias_gradient_is_column_sum_of_delta():
    """A ones column appended to A turns the bias into a weight row: its gradient is 1^T Delta."""
    rng = np.random.default_rng(8)
    Ws, Bs, acts = _tiny_mlp(rng)
    X = rng.standard_normal((4, 5))
    Y = rng.standard_normal((4, 3))
    A, D = O.mlp_factors(Ws, Bs, acts, X, Y)[1]
    eps = 1e-6
    fd = np.zeros(6)
    for q in range(6):
        Bp = [b.copy() for b in Bs]
        Bm = [b.copy() for b in Bs]
        Bp[1][q] += eps
        Bm[1][q] -= eps
        fd[q] = (O.mlp_loss(Ws, Bp, acts, X, Y) - O.mlp_loss(Ws, Bm, acts, X, Y)) / (2 * eps)
    A1 = np.concatenate([A, np.ones((4, 1))], axis=1)
    assert np.allclose(O.full_grad(A1, D)[-1], fd, rtol=1e-7, atol=1e-10)


# ---------------------------------------------------------------- dAD exactness (linearity)

def test_sites_sum_equals_stacked_equals_pooled():
    """Section 3.2: stacking the sites' factors gives the exact pooled gradient (check 2)."""
    rng = np.random.default_rng(11)
    Ws, Bs, acts = _tiny_mlp(rng)
    S, b = 3, 4
    Xs = [rng.standard_normal((b, 5)) for _ in range(S)]
    Ys = [rng.standard_normal((b, 3)) for _ in range(S)]
    per_site = [O.mlp_factors(Ws, Bs, acts, Xs[s], Ys[s], n_global=S * b) for s in range(S)]
    pooled = O.mlp_factors(Ws, Bs, acts, np.concatenate(Xs), np.concatenate(Ys))
    for li in range(3):
        A_st, D_st = O.stack_factors([per_site[s][li][0] for s in range(S)],
                                     [per_site[s][li][1] for s in range(S)])
        assert A_st.shape == (S * b, per_site[0][li][0].shape[1])
        # rows of site s sit at [s*b, (s+1)*b)
        assert np.array_equal(A_st[b:2 * b], per_site[1][li][0])
        assert np.array_equal(D_st[2 * b:], per_site[2][li][1])
        g_sum = sum(O.full_grad(*per_site[s][li]) for s in range(S))
        g_stack = O.full_grad(A_st, D_st)
        g_pool = O.full_grad(*pooled[li])
        assert np.allclose(g_sum, g_stack, rtol=1e-13, atol=1e-15)
        assert np.allclose(g_stack, g_pool, rtol=1e-13, atol=1e-15)


def test_full_grad_brute_force_and_special_cases():
    rng = np.random.default_rng(3)
    A = rng.standard_normal((6, 4))
    D = rng.standard_normal((6, 5))
    ref = np.zeros((4, 5))
    for p in range(4):
        for q in range(5):
            for n in range(6):
                ref[p, q] += A[n, p] * D[n, q]
    assert np.allclose(O.full_grad(A, D), ref, rtol=1e-14, atol=1e-15)
    # one sample: a plain outer product
    assert np.array_equal(O.full_grad(A[:1], D[:1]), np.outer(A[0], D[0]))
    # hand-worked 2x2 example stored as a text fixture
    with open(os.path.join(GOLDEN, "eq4_hand_example.json")) as f:
        ex = json.load(f)
    assert np.array_equal(O.full_grad(ex["A"], ex["Delta"]), np.array(ex["grad"], float))
    assert np.array_equal(O.rank_r_grad(ex["A"], ex["Delta"]), np.array(ex["grad"], float))


def test_gradient_rank_bounded_by_batch():
    """Section 3.1: the gradient's rank cannot exceed the batch size."""
    rng = np.random.default_rng(4)
    A = rng.standard_normal((3, 12))
    D = rng.standard_normal((3, 9))
    assert np.linalg.matrix_rank(O.full_grad(A, D)) == 3


# ---------------------------------------------------------------- structured power iteration

def test_structured_iterate_equals_plain_iterate():
    """Eq. 6 equals Eq. 5: B (Delta g) = M^T M g; sigma = sqrt(v^T C v) = ||A^T v||."""
    rng = np.random.default_rng(5)
    A = rng.standard_normal((7, 11))
    D = rng.standard_normal((7, 13))
    g = rng.standard_normal(13)
    M = O.full_grad(A, D)
    C = A @ A.T
    B = D.T @ C
    assert np.allclose(B @ (D @ g), M.T @ (M @ g), rtol=1e-12)
    v = D @ g
    assert np.isclose(np.sqrt(v @ C @ v), np.linalg.norm(A.T @ v), rtol=1e-13)
    assert np.allclose(A.T @ v, M @ g, rtol=1e-12)


@pytest.mark.parametrize("N,h_in,h_out,r,n", [(20, 33, 17, 5, 2), (64, 40, 50, 8, 3), (9, 30, 12, 4, 1)])
def test_three_routes_agree(N, h_in, h_out, r, n):
    rng = np.random.default_rng(N + r)
    A = np.maximum(rng.standard_normal((N, h_in)), 0)
    D = rng.standard_normal((N, h_out)) * 0.1
    G0 = rng.standard_normal((r, h_out))
    Pt, Gt = O.block_spi(A, D, G0, n)
    assert Pt.shape == (r, h_in) and Gt.shape == (r, h_out)
    Gh = O.rank_r_grad(Pt, Gt)
    assert Gh.shape == (h_in, h_out)
    dense = O.block_spi_dense(A, D, G0, n)
    Pt2, Gt2 = O.block_spi_precomputed(A, D, G0, n)
    assert O.rel_fro(Gh, dense) < 1e-11
    assert O.rel_fro(O.rank_r_grad(Pt2, Gt2), dense) < 1e-11
    assert np.allclose(Gt @ Gt.T, np.eye(r), atol=1e-12)


def test_full_rank_budget_recovers_gradient_and_truncated_svd():
    """r >= rank(M): the rank-r gradient is M itself and equals the truncated SVD (check 3a)."""
    rng = np.random.default_rng(21)
    # rank 3 through N = 3 samples
    A = rng.standard_normal((3, 14))
    D = rng.standard_normal((3, 10))
    G0 = rng.standard_normal((4, 10))
    M = O.full_grad(A, D)
    Gh = O.rank_r_grad(*O.block_spi(A, D, G0, 2))
    assert O.rel_fro(Gh, M) < 1e-12
    assert O.rel_fro(Gh, O.truncated_svd(M, 4)) < 1e-12
    assert O.rel_fro(O.block_spi_dense(A, D, G0, 2), M) < 1e-12
    # rank 4 through duplicated rows, r equal to the rank
    A4 = rng.standard_normal((4, 14))
    D4 = rng.standard_normal((4, 10))
    A = np.concatenate([A4, A4, A4])
    D = np.concatenate([D4, D4, D4])
    M = O.full_grad(A, D)
    assert np.linalg.matrix_rank(M) == 4
    Gh = O.rank_r_grad(*O.block_spi(A, D, G0, 2))
    assert O.rel_fro(Gh, M) < 1e-11
    assert O.rel_fro(Gh, O.truncated_svd(M, 4)) < 1e-11


def test_low_rank_budget_obeys_eckart_young_and_pythagoras():
    """r < rank(M): residual >= Eckart-Young bound, -> bound as n grows; projection identities (3b)."""
    rng = np.random.default_rng(22)
    N, h_in, h_out, r = 40, 30, 24, 5
    A = np.maximum(rng.standard_normal((N, h_in)), 0)
    D = rng.standard_normal((N, h_out)) * 0.03
    G0 = rng.standard_normal((r, h_out))
    M = O.full_grad(A, D)
    bound = O.eckart_young_residual(M, r)
    prev = np.inf
    for n in (1, 2, 4, 8, 64):
        Pt, Gt = O.block_spi(A, D, G0, n)
        Gh = O.rank_r_grad(Pt, Gt)
        res = np.linalg.norm(M - Gh)
        assert res >= bound * (1 - 1e-12)
        assert res <= prev * (1 + 1e-9)
        prev = res
        # orthogonal projection of M: ||M - Gh||^2 = ||M||^2 - ||Gh||^2
        assert np.isclose(res ** 2, np.linalg.norm(M) ** 2 - np.linalg.norm(Gh) ** 2, rtol=1e-10)
        assert np.allclose(Gt @ Gt.T, np.eye(r), atol=1e-12)
        # P = M G exactly
        assert np.allclose(Pt.T, M @ Gt.T, rtol=1e-10, atol=1e-14)
    assert prev / bound < 1.05


def test_converged_iteration_is_truncated_svd_and_sequential_route_agrees():
    """With a spectral gap and many iterations both the block and the one-vector-at-a-time
    (peeling, Eq. 7) routes reach numpy's truncated SVD."""
    rng = np.random.default_rng(23)
    N, h_in, h_out, r = 12, 40, 30, 4
    A = rng.standard_normal((N, h_in))
    D = rng.standard_normal((N, h_out)) * (0.5 ** np.arange(N))[:, None]
    M = O.full_grad(A, D)
    G0 = rng.standard_normal((r, h_out))
    tsvd = O.truncated_svd(M, r)
    assert O.rel_fro(O.rank_r_grad(*O.block_spi(A, D, G0, 60)), tsvd) < 1e-10
    Q, sG = O.sequential_spi(A, D, G0, 200)
    assert O.rel_fro(O.rank_r_grad(Q, sG), tsvd) < 1e-8
    # unit left vectors, singular values carried by the right rows
    assert np.allclose(np.linalg.norm(Q, axis=1), 1.0, atol=1e-12)
    s = np.linalg.svd(M, compute_uv=False)
    assert np.allclose(np.linalg.norm(sG, axis=1), s[:r], rtol=1e-8)


def test_sequential_route_with_the_printed_association_gives_the_same_pairs():
    """C = A A^T, B = Delta^T C as Algorithm 2 prints them against the iteration on M^T M."""
    rng = np.random.default_rng(31)
    A = rng.standard_normal((9, 20))
    D = rng.standard_normal((9, 14)) * (0.7 ** np.arange(9))[:, None]
    G0 = rng.standard_normal((3, 14))
    Q1, sG1 = O.sequential_spi(A, D, G0, 5)
    Q2, sG2 = O.sequential_spi_precomputed(A, D, G0, 5)
    assert np.allclose(Q1, Q2, rtol=1e-9, atol=1e-12) and np.allclose(sG1, sG2, rtol=1e-9, atol=1e-12)


def _planted(rng, N, h_in, h_out, sigmas):
    """Factors whose gradient A^T Delta has exactly the given non-zero singular values."""
    k = len(sigmas)
    U, _ = np.linalg.qr(rng.standard_normal((h_in, k)))
    V, _ = np.linalg.qr(rng.standard_normal((h_out, k)))
    W, _ = np.linalg.qr(rng.standard_normal((N, k)))
    return W @ (U * np.sqrt(sigmas)).T, W @ (V * np.sqrt(sigmas)).T     # A = W S^1/2 U^T, Delta = W S^1/2 V^T


@pytest.mark.parametrize("k", [1, 2, 3, 5])
def test_early_stop_finds_the_rank_of_a_planted_gradient(k):
    """Effective rank (Section 3.3.1, last paragraph; Algorithm 2's stop test): a gradient of exact
    rank k < r with a clear spectral gap yields k components, zero rows beyond, and the product
    equals the gradient to the convergence tolerance."""
    rng = np.random.default_rng(40 + k)
    theta, r = 1e-3, 6
    A, D = _planted(rng, 24, 30, 26, 2.0 * 0.5 ** np.arange(k))
    M = O.full_grad(A, D)
    G0 = rng.standard_normal((r, 26))
    Q, sG, rank, iters = O.sequential_spi(A, D, G0, 200, theta=theta)
    assert rank == k
    assert np.all(Q[k:] == 0.0) and np.all(sG[k:] == 0.0)
    assert O.rel_fro(O.rank_r_grad(Q, sG), M) < 5 * theta
    s = np.linalg.svd(M, compute_uv=False)
    assert np.allclose(np.linalg.norm(sG[:k], axis=1), s[:k], rtol=5 * theta)
    assert all(it < 200 for it in iters[:k])            # every live component stopped on the step test


def test_early_stop_keeps_every_component_of_a_flat_full_rank_spectrum():
    rng = np.random.default_rng(47)
    A = rng.standard_normal((64, 20))
    D = rng.standard_normal((64, 18))
    G0 = rng.standard_normal((5, 18))
    Q, sG, rank, iters = O.sequential_spi(A, D, G0, 30, theta=1e-3)
    assert rank == 5 and len(iters) == 5
    assert np.allclose(np.linalg.norm(Q, axis=1), 1.0, atol=1e-12)
    # the rows of sG are orthogonal (projector deflation), their norms are the singular-value estimates
    g = sG / np.linalg.norm(sG, axis=1, keepdims=True)
    assert np.allclose(g @ g.T, np.eye(5), atol=1e-10)


def test_early_stop_converges_to_the_truncated_svd_and_spends_less_for_a_larger_theta():
    rng = np.random.default_rng(48)
    A = rng.standard_normal((12, 40))
    D = rng.standard_normal((12, 30)) * (0.5 ** np.arange(12))[:, None]
    M = O.full_grad(A, D)
    G0 = rng.standard_normal((4, 30))
    Q, sG, rank, it_fine = O.sequential_spi(A, D, G0, 500, theta=1e-12)
    assert rank == 4 and O.rel_fro(O.rank_r_grad(Q, sG), O.truncated_svd(M, 4)) < 1e-8
    _, _, _, it_coarse = O.sequential_spi(A, D, G0, 500, theta=1e-3)
    _, _, _, it_coarser = O.sequential_spi(A, D, G0, 500, theta=1e-1)
    assert sum(it_coarser) < sum(it_coarse) < sum(it_fine)
    # with a cap below what theta asks for, the cap decides
    _, _, _, it_cap = O.sequential_spi(A, D, G0, 3, theta=1e-12)
    assert it_cap == [3, 3, 3, 3]


def test_subtraction_deflation_cannot_detect_an_exhausted_rank():
    """The finding behind the projector reading: with the subtraction of Eq. 7 and pairs converged
    only to theta, the next 'component' of an exactly rank-2 gradient has ||M g|| of the order of
    sigma_0, not of theta * sigma_0."""
    rng = np.random.default_rng(49)
    A, D = _planted(rng, 16, 22, 20, np.array([2.0, 1.0]))
    M = O.full_grad(A, D)
    T = M.T @ M
    Q, sG, rank, _ = O.sequential_spi(A, D, rng.standard_normal((2, 20)), 200, theta=1e-3)
    assert rank == 2
    sig = np.linalg.norm(sG, axis=1)
    gs = sG / sig[:, None]
    Tdef = T - sum(s ** 2 * np.outer(g, g) for s, g in zip(sig, gs))      # Eq. 7 by subtraction
    g = rng.standard_normal(20)
    for _ in range(500):
        g = Tdef @ g
        g /= np.linalg.norm(g)
    assert np.linalg.norm(M @ g) > 0.05 * sig[0]          # far above theta * sigma_0 = 2e-3
    P = np.eye(20) - gs.T @ gs                            # projector form: nothing is left to iterate on
    g = P @ rng.standard_normal(20)
    g /= np.linalg.norm(g)
    assert np.linalg.norm(P @ (T @ g)) < (1e-3 * sig[0]) ** 2
    assert np.linalg.norm(M @ g) < 1e-3 * sig[0]


def test_result_does_not_depend_on_basis_of_start_span():
    """Only span(G0) matters: mixing the start rows by an invertible matrix leaves P G^T unchanged."""
    rng = np.random.default_rng(24)
    A = rng.standard_normal((25, 18))
    D = rng.standard_normal((25, 16))
    G0 = rng.standard_normal((3, 16))
    T = rng.standard_normal((3, 3)) + 3 * np.eye(3)
    a = O.rank_r_grad(*O.block_spi(A, D, G0, 2))
    b = O.rank_r_grad(*O.block_spi(A, D, T @ G0, 2))
    assert O.rel_fro(a, b) < 1e-11


def test_stacked_rank_pairs_are_factors_again():
    """Algorithm 1: sum_s P_s G_s^T equals the gradient of the stacked r-row pairs."""
    rng = np.random.default_rng(25)
    pairs = []
    for s in range(3):
        A = rng.standard_normal((10, 12))
        D = rng.standard_normal((10, 9))
        pairs.append(O.block_spi(A, D, rng.standard_normal((2, 9)), 2))
    Pst, Gst = O.stack_factors([p for p, _ in pairs], [g for _, g in pairs])
    assert Pst.shape == (6, 12) and Gst.shape == (6, 9)
    assert np.allclose(O.full_grad(Pst, Gst), sum(O.rank_r_grad(p, g) for p, g in pairs), rtol=1e-12)


# ---------------------------------------------------------------- Algorithm 1 (two-level rank-dAD)

def _site_factors(rng, S, b, h_in, h_out, row_basis=None, col_basis=None):
    """Per-site factor pairs; with bases given, every site's gradient lives in their spans."""
    A_sites, D_sites = [], []
    for _ in range(S):
        A = rng.standard_normal((b, h_in))
        D = rng.standard_normal((b, h_out))
        if row_basis is not None:
            A = rng.standard_normal((b, row_basis.shape[0])) @ row_basis
        if col_basis is not None:
            D = rng.standard_normal((b, col_basis.shape[0])) @ col_basis
        A_sites.append(A)
        D_sites.append(D)
    return A_sites, D_sites


def test_rank_dad_is_exact_when_the_global_gradient_fits_both_budgets():
    """If every site's gradient, and their sum, has rank <= r, both reductions lose nothing and
    Algorithm 1 returns the pooled-batch gradient of Eq. 4 (computed here by brute force on the
    concatenated batch, without any of the oracle's iteration code)."""
    rng = np.random.default_rng(31)
    S, b, h_in, h_out, r = 4, 9, 14, 11, 3
    col_basis = rng.standard_normal((r, h_out))        # all deltas share a 3-dimensional row space
    A_sites, D_sites = _site_factors(rng, S, b, h_in, h_out, col_basis=col_basis)
    G0s = [rng.standard_normal((r, h_out)) for _ in range(S)]
    Pt, Gt, pairs = O.rank_dad(A_sites, D_sites, G0s, rng.standard_normal((r, h_out)), 2)
    assert Pt.shape == (r, h_in) and Gt.shape == (r, h_out) and len(pairs) == S
    A_all, D_all = np.vstack(A_sites), np.vstack(D_sites)
    M = np.einsum("np,nq->pq", A_all, D_all)
    assert np.linalg.matrix_rank(M) == r
    assert O.rel_fro(O.rank_r_grad(Pt, Gt), M) < 1e-10
    # each site's message is exact as well
    for (p, g), a, d in zip(pairs, A_sites, D_sites):
        assert O.rel_fro(O.rank_r_grad(p, g), a.T @ d) < 1e-10


def test_rank_dad_aggregator_with_full_budget_returns_sum_of_site_estimates():
    """An aggregator budget of S*r rows keeps everything the sites sent: the result is
    sum_s P_s G_s^T, whatever was lost at the sites; and that sum is what the sites lost
    relative to the true gradient, no more (triangle inequality on the residuals)."""
    rng = np.random.default_rng(32)
    S, b, h_in, h_out, r = 3, 12, 20, 16, 2
    A_sites, D_sites = _site_factors(rng, S, b, h_in, h_out)
    G0s = [rng.standard_normal((r, h_out)) for _ in range(S)]
    Pt, Gt, pairs = O.rank_dad(A_sites, D_sites, G0s, rng.standard_normal((S * r, h_out)), 2)
    site_sum = sum(p.T @ g for p, g in pairs)
    assert O.rel_fro(O.rank_r_grad(Pt, Gt), site_sum) < 1e-10
    M = sum(a.T @ d for a, d in zip(A_sites, D_sites))
    lost = sum(np.linalg.norm(a.T @ d - p.T @ g) for (p, g), a, d in zip(pairs, A_sites, D_sites))
    assert np.linalg.norm(M - site_sum) <= lost * (1 + 1e-12)


def test_rank_dad_converged_aggregator_is_truncated_svd_of_the_sites_sum():
    """With many iterations and a spectral gap the aggregator step is the best rank-r
    approximation (numpy SVD) of sum_s P_s G_s^T, and its residual is the Eckart-Young value."""
    rng = np.random.default_rng(33)
    S, b, h_in, h_out, r = 3, 10, 18, 15, 2
    A_sites, D_sites = [], []
    for _ in range(S):
        A_sites.append(rng.standard_normal((b, h_in)))
        D_sites.append(rng.standard_normal((b, h_out)) * (0.4 ** np.arange(b))[:, None])
    G0s = [rng.standard_normal((r, h_out)) for _ in range(S)]
    Pt, Gt, pairs = O.rank_dad(A_sites, D_sites, G0s, rng.standard_normal((r, h_out)), 80)
    site_sum = sum(p.T @ g for p, g in pairs)
    U, s, Vt = np.linalg.svd(site_sum)
    best = (U[:, :r] * s[:r]) @ Vt[:r]
    est = O.rank_r_grad(Pt, Gt)
    assert O.rel_fro(est, best) < 1e-8
    assert abs(np.linalg.norm(site_sum - est) - np.sqrt(np.sum(s[r:] ** 2))) < 1e-8 * s[0]
    assert np.allclose(Gt @ Gt.T, np.eye(r), atol=1e-12)


def test_rank_dad_single_site_full_budget_is_one_level():
    """S = 1 and an aggregator that keeps all r rows: the second reduction is the identity on
    the estimate, so the two-level result equals the one-level one."""
    rng = np.random.default_rng(34)
    A = rng.standard_normal((20, 13))
    D = rng.standard_normal((20, 10))
    G0 = rng.standard_normal((3, 10))
    Pt, Gt, _ = O.rank_dad([A], [D], [G0], rng.standard_normal((3, 10)), 2)
    assert O.rel_fro(O.rank_r_grad(Pt, Gt), O.rank_r_grad(*O.block_spi(A, D, G0, 2))) < 1e-10


# ---------------------------------------------------------------- Eq. 3, one step

@pytest.mark.parametrize("acts", [("tanh", "sigmoid", "identity"), ("relu", "tanh", "tanh")])
def test_backprop_delta_is_the_derivative_wrt_pre_activations(acts):
    """Delta_i of Eq. 3 is dLoss/dZ_i: perturb single entries of Z_i, run the tail of the
    network from the perturbed pre-activations, and compare central differences of the loss."""
    rng = np.random.default_rng(51)
    Ws, Bs, acts = _tiny_mlp(rng, acts=acts)
    X = rng.standard_normal((6, 5))
    Y = rng.standard_normal((6, 3))
    A, Z = O.mlp_forward(Ws, Bs, acts, X)
    L = len(Ws)

    def loss_from_Z(i, Zi):
        """Loss as a function of the pre-activations of layer i+1 (0-based i)."""
        a = O._ACT[acts[i]][0](Zi)
        for k in range(i + 1, L):
            a = O._ACT[acts[k]][0](a @ Ws[k] + Bs[k])
        return 0.5 * np.sum((a - Y) ** 2) / X.shape[0]

    # last layer's delta from the definition (Eq. 2), then walk down with the function under test
    delta = (A[L] - Y) / X.shape[0] * O._ACT[acts[L - 1]][1](Z[L - 1])
    eps = 1e-6
    for i in range(L - 2, -1, -1):
        delta = O.backprop_delta(delta, Ws[i + 1], Z[i], acts[i])
        fd = np.zeros_like(delta)
        for n in range(delta.shape[0]):
            for p in range(delta.shape[1]):
                Zp, Zm = Z[i].copy(), Z[i].copy()
                Zp[n, p] += eps
                Zm[n, p] -= eps
                fd[n, p] = (loss_from_Z(i, Zp) - loss_from_Z(i, Zm)) / (2 * eps)
        assert np.allclose(delta, fd, rtol=1e-5, atol=1e-9), i


def test_backprop_delta_special_cases():
    rng = np.random.default_rng(52)
    Dn = rng.standard_normal((7, 4))
    W = rng.standard_normal((5, 4))
    Z = rng.standard_normal((7, 5))
    brute = np.zeros((7, 5))
    for n in range(7):
        for p in range(5):
            brute[n, p] = sum(Dn[n, q] * W[p, q] for q in range(4))
    assert np.allclose(O.backprop_delta(Dn, W, Z, "identity"), brute, rtol=1e-13)
    assert np.allclose(O.backprop_delta(Dn, W, Z, "relu"), brute * (Z > 0), rtol=1e-13)
    # rows are independent: computing two row blocks separately and stacking them is the same
    both = O.backprop_delta(Dn, W, Z, "tanh")
    parts = np.vstack([O.backprop_delta(Dn[:3], W, Z[:3], "tanh"), O.backprop_delta(Dn[3:], W, Z[3:], "tanh")])
    assert np.array_equal(both, parts)
