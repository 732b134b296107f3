"""Host logic of the synthetic input generators (CPU only)."""
import numpy as np
import torch

from paper_2102_09631_amd import workloads as W


def test_bf16_rounding_matches_torch_rne():
    rng = np.random.default_rng(0)
    x = np.concatenate([rng.standard_normal(20000).astype(np.float32) * 3,
                        np.array([0.0, -0.0, 1.0, 1.00390625, 1.01171875, 3.3895314e38, 1e-40], np.float32)])
    bits = W.f32_to_bf16_bits(x)
    ref = torch.from_numpy(x).to(torch.bfloat16)
    assert np.array_equal(bits.view(np.int16), ref.view(torch.int16).numpy())
    assert np.array_equal(W.bf16_bits_to_f32(bits), ref.to(torch.float32).numpy())


def test_workload_table_matches_benchmark_configs():
    w = W.WORKLOADS
    assert [x.N for x in w] == [64, 1024, 16384, 65536, 262144]
    assert [x.rank for x in w] == [4, 8, 16, 32, 64]
    assert len(w[3].all_layers()) == 96 and len(w[4].all_layers()) == 128
    assert w[1].shapes == ((784, 1024), (1024, 1024), (1024, 10))


def test_host_draws_are_seeded_and_shaped():
    w = W.WORKLOADS[0]
    A1, D1 = W.host_factors(w, 0, 784, 128)
    A2, D2 = W.host_factors(w, 0, 784, 128)
    assert len(A1) == 2 and A1[0].shape == (32, 784) and D1[1].shape == (32, 128)
    assert all(np.array_equal(a, b) for a, b in zip(A1 + D1, A2 + D2))
    assert not np.array_equal(A1[0], A1[1])
    assert (np.concatenate(A1) >= 0).all()                       # ReLU
    assert abs(np.concatenate(D1).std() - 0.1) < 0.005            # variance 0.01
    G0 = W.host_start_matrix(w, 0, 128)
    assert G0.shape == (4, 128) and G0.dtype == np.float32
    # bf16 workloads come out on the bf16 grid
    w3 = W.WORKLOADS[2]
    A3, D3 = W.host_factors(w3, 1, 768, 768, rows=16, sites=2)
    for x in A3 + D3:
        assert np.array_equal(W.bf16_bits_to_f32(W.f32_to_bf16_bits(x)), x)
    w5 = W.WORKLOADS[4]
    A5, D5 = W.host_factors(w5, 0, 64, 32, rows=4000, sites=1)
    assert A5[0].min() > -0.2 and abs(A5[0].mean() - 0.2821) < 0.01   # GELU of N(0,1): mean 1/sqrt(4 pi)
