"""Why the bf16 path carries W = A U as two bf16 terms: a numpy model of the path's roundings on
GELU activations (non-zero mean) and heavy-tailed deltas.  One bf16 rounding of W costs several times
more than every other rounding together; the value + remainder pair costs next to nothing.  CPU only;
the model shares no code with the library and is compared with the fp64 oracle."""
import math

import numpy as np

from oracle import dad_oracle as O
from paper_2102_09631_amd import workloads as W


def _bf16(x):
    return W.bf16_bits_to_f32(W.f32_to_bf16_bits(np.asarray(x, np.float32))).astype(np.float64)


def _two_terms(x):
    hi = _bf16(x)
    return hi + _bf16(x - hi)


def _ident(x):
    return x


def _model(A, D, G0t, n_iter, round_V, round_W, round_panels):
    """The block iteration of the library's bf16 path with its roundings switched on one by one."""
    G = G0t.T.astype(np.float64)
    for _ in range(n_iter):
        V = round_V(D @ round_panels(G))
        U = A.T @ V
        Wm = round_W(A @ round_panels(U))
        Y = D.T @ Wm
        Q, R = np.linalg.qr(Y)
        G = Q * np.sign(np.diag(R))
    P = A.T @ round_V(D @ round_panels(G))
    return P @ G.T


def test_one_rounding_of_W_dominates_and_two_terms_remove_it():
    rng = np.random.default_rng(20210209)
    N, h_in, h_out, r = 2048, 640, 160, 16
    z = rng.standard_normal((N, h_in))
    A = _bf16(0.5 * z * (1.0 + np.vectorize(math.erf)(z / math.sqrt(2.0))))          # GELU: mean 0.28, not centred
    D = _bf16(1e-3 * rng.standard_t(3, size=(N, h_out)))
    G0t = rng.standard_normal((r, h_out)).astype(np.float32)
    ref = O.rank_r_grad(*O.block_spi(A, D, G0t, 2))
    err = lambda **kw: O.rel_fro(_model(A, D, G0t, 2, **kw), ref)
    none = err(round_V=_ident, round_W=_ident, round_panels=_ident)
    only_W = err(round_V=_ident, round_W=_bf16, round_panels=_ident)
    others = err(round_V=_bf16, round_W=_ident, round_panels=_bf16)
    one_term = err(round_V=_bf16, round_W=_bf16, round_panels=_bf16)
    two_terms = err(round_V=_bf16, round_W=_two_terms, round_panels=_bf16)
    assert none < 1e-10
    assert only_W > 2.0 * others                  # the single rounding of W outweighs all the others together
    assert abs(two_terms - others) < 0.1 * others  # the remainder term removes W's share
    assert two_terms < 0.5 * one_term
    assert two_terms < 2e-2
