"""Parity of dad_backprop_delta (Eq. 3, one step) with the fp64 oracle, through the C ABI.

fp32: relative Frobenius error <= 1e-5.  bf16 inputs with fp32 accumulation and one rounding
of the result to bf16: <= 2e-2 (the result's own rounding contributes 2^-9 per element).
"""
import numpy as np
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad
from paper_2102_09631_amd import workloads as W

pytestmark = pytest.mark.gpu

TOL = {"f32": 1e-5, "bf16": 2e-2}


def draw(seed, N, h, hn, dtype):
    """Deltas of the next layer, weights and pre-activations with the scales of an MLP layer,
    already on the element type's grid so that both sides see the same numbers."""
    rng = np.random.default_rng([20210209, 77, seed])
    Dn = (rng.standard_normal((N, hn)) * 1e-2).astype(np.float32)
    Wn = (rng.standard_normal((h, hn)) / np.sqrt(hn)).astype(np.float32)
    Z = rng.standard_normal((N, h)).astype(np.float32)
    if dtype == "bf16":
        Dn, Wn, Z = (W.bf16_bits_to_f32(W.f32_to_bf16_bits(x)) for x in (Dn, Wn, Z))
    return Dn, Wn, Z


def to_dev(x, dtype, dev):
    t = torch.from_numpy(np.ascontiguousarray(x)).to(dev)
    return t.to(torch.bfloat16) if dtype == "bf16" else t


@pytest.mark.parametrize("dtype,N,h,hn,act", [
    ("f32", 37, 50, 23, "tanh"),          # everything ragged
    ("f32", 1, 9, 5, "sigmoid"),          # one sample
    ("f32", 130, 64, 200, "relu"),
    ("bf16", 77, 136, 72, "relu"),        # guarded kernel, bf16
    ("bf16", 33, 65, 31, "identity"),     # odd widths
    ("bf16", 256, 256, 32, "relu"),       # tile-aligned but h_next not a multiple of 64: guarded kernel
    ("bf16", 256, 256, 64, "relu"),       # one MFMA tile, one stage
    ("bf16", 512, 768, 192, "tanh"),      # 2 x 3 tiles, 3 stages
    ("bf16", 768, 512, 1024, "sigmoid"),  # 16 stages
    ("bf16", 256, 1024, 320, "identity"), # 5 stages (odd count)
    ("bf16", 512, 256, 3072, "relu"),     # long contraction
])
def test_backprop_delta_matches_oracle(gpu, dtype, N, h, hn, act):
    Dn, Wn, Z = draw(N + h + hn, N, h, hn, dtype)
    out = dad.backprop_delta(to_dev(Dn, dtype, gpu), to_dev(Wn, dtype, gpu), to_dev(Z, dtype, gpu), act)
    ref = O.backprop_delta(Dn, Wn, Z, act)
    got = out.float().cpu().numpy()
    assert got.shape == (N, h)
    err = O.rel_fro(got, ref)
    print(dtype, N, h, hn, act, err)
    assert err <= TOL[dtype]
    if act == "relu":      # the mask is exact: no value leaks where Z <= 0
        assert np.all(got[Z <= 0] == 0)


def test_backprop_delta_writes_sites_in_place_in_the_stacked_buffer(gpu):
    """Three sites write their rows at their offsets of one stacked buffer; the result is the
    delta of the stacked batch (rows are independent), and rows outside a call stay untouched."""
    h, hn, rows = 256, 64, (256, 512, 256)
    Dn, Wn, Z = draw(5, sum(rows), h, hn, "bf16")
    stacked = torch.full((sum(rows), h), 7.0, dtype=torch.bfloat16, device=gpu)
    Wd = to_dev(Wn, "bf16", gpu)
    off = 0
    for b in rows[:2]:
        dad.backprop_delta(to_dev(Dn[off:off + b], "bf16", gpu), Wd, to_dev(Z[off:off + b], "bf16", gpu), "relu",
                           D_out=stacked[off:off + b])
        off += b
    torch.cuda.synchronize()
    assert torch.all(stacked[off:] == 7.0)
    dad.backprop_delta(to_dev(Dn[off:], "bf16", gpu), Wd, to_dev(Z[off:], "bf16", gpu), "relu", D_out=stacked[off:])
    ref = O.backprop_delta(Dn, Wn, Z, "relu")
    assert O.rel_fro(stacked.float().cpu().numpy(), ref) <= TOL["bf16"]


def test_backprop_delta_feeds_the_gradient_rebuild(gpu):
    """Eq. 3 then Eq. 4 on the GPU against the oracle: the delta produced here is the factor
    dad_reconstruct_grad consumes."""
    N, h_prev, h, hn = 512, 256, 256, 128
    Dn, Wn, Z = draw(9, N, h, hn, "bf16")
    rng = np.random.default_rng(99)
    A_prev = W.bf16_bits_to_f32(W.f32_to_bf16_bits(rng.standard_normal((N, h_prev)).astype(np.float32)))
    D = dad.backprop_delta(to_dev(Dn, "bf16", gpu), to_dev(Wn, "bf16", gpu), to_dev(Z, "bf16", gpu), "tanh")
    G = dad.reconstruct_grad(to_dev(A_prev, "bf16", gpu), D).cpu().numpy()
    ref = O.full_grad(A_prev, O.backprop_delta(Dn, Wn, Z, "tanh"))
    assert O.rel_fro(G, ref) <= TOL["bf16"]


def test_backprop_delta_full_size_sampled(gpu):
    """GPT-2-medium FFN shape in the launch configuration the benchmark times (N = 65536 rows,
    4096 -> 1024 backwards: h = 4096, h_next = 1024): sampled rows against the oracle."""
    N, h, hn = 65536, 4096, 1024
    gen = torch.Generator(device=gpu)
    gen.manual_seed(20210209)
    Dn = (torch.randn(N, hn, generator=gen, device=gpu) * 1e-2).to(torch.bfloat16)
    Wn = (torch.randn(h, hn, generator=gen, device=gpu) / 32.0).to(torch.bfloat16)
    Z = torch.randn(N, h, generator=gen, device=gpu).to(torch.bfloat16)
    out = dad.backprop_delta(Dn, Wn, Z, "relu")
    rows = np.random.default_rng(3).choice(N, size=64, replace=False)
    ridx = torch.from_numpy(rows).to(gpu)
    ref = O.backprop_delta(Dn[ridx].float().cpu().numpy(), Wn.float().cpu().numpy(), Z[ridx].float().cpu().numpy(), "relu")
    err = O.rel_fro(out[ridx].float().cpu().numpy(), ref)
    print("full size sampled", err)
    assert err <= TOL["bf16"]
