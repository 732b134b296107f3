"""Reduction and full rebuild on the sites' blocks (no stacked copy): bit for bit the result of
dad_stack_factors followed by the stacked call, and within the parity bar of the oracle."""
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad

pytestmark = pytest.mark.gpu


def _sites(rows, h_in, h_out, r, seed, dev, dtype):
    g = torch.Generator(device="cpu").manual_seed(seed)
    A = [torch.relu(torch.randn(n, h_in, generator=g)).to(dtype).to(dev) for n in rows]
    D = [(0.03 * torch.randn(n, h_out, generator=g)).to(dtype).to(dev) for n in rows]
    G0 = torch.randn(r, h_out, generator=g).to(dev)
    return A, D, G0


def _up(x):
    return (x + 255) // 256 * 256


def _in_place(rows, h_in, h_out, r, dtype):
    """True when the size query leaves no room for a stacked copy, i.e. the blocks are read in place."""
    N = sum(rows)
    import ctypes as C
    pr = (C.c_int64 * len(rows))(*rows)
    dt = dad.DAD_BF16 if dtype == torch.bfloat16 else dad.DAD_F32
    need = dad.lib().dad_compress_sites_workspace_bytes(len(rows), pr, h_in, h_out, r, dt)
    assert need > 0
    return need == _up(dad.compress_workspace_bytes(N, h_in, h_out, r, dtype))


# rows, h_in, h_out, r, dtype, read in place?
COMPRESS_CASES = [
    ([512, 1024, 256, 768], 256, 384, 32, torch.bfloat16, True),
    ([256, 0, 256, 1280, 0], 384, 128, 16, torch.bfloat16, True),       # empty sites, two-wave workgroups
    ([2048] * 8, 1024, 512, 64, torch.bfloat16, True),                  # row chunks of thin_tn span blocks
    ([256] * 32, 256, 256, 32, torch.bfloat16, True),                   # the most blocks a kernel takes
    ([65536 + 256, 256], 128, 128, 32, torch.bfloat16, True),           # 256-row workgroups
    ([256] * 33, 256, 256, 32, torch.bfloat16, False),                  # one block too many: stacked first
    ([500, 12, 1024], 256, 384, 32, torch.bfloat16, False),             # ragged sites
    ([512, 1024], 256, 384, 24, torch.bfloat16, False),                 # a rank without a direct-to-LDS kernel
    ([512, 1024], 200, 136, 8, torch.bfloat16, False),                  # widths the MFMA path does not take
    ([100, 0, 300, 57], 784, 128, 4, torch.float32, False),
    ([64] * 40, 96, 80, 8, torch.float32, False),                       # two launches of the stacking kernel
]


@pytest.mark.parametrize("rows,h_in,h_out,r,dtype,in_place", COMPRESS_CASES)
def test_compress_on_site_blocks_equals_stack_then_compress(gpu, rows, h_in, h_out, r, dtype, in_place):
    assert _in_place(rows, h_in, h_out, r, dtype) == in_place
    A_s, D_s, G0 = _sites(rows, h_in, h_out, r, sum(rows) + h_in + r, gpu, dtype)
    A, D = dad.stack_factors(A_s, D_s)
    Pt0, Gt0 = dad.compress_rank(A, D, r, 2, G0, check=True)
    Pt1, Gt1 = dad.compress_rank_sites(A_s, D_s, r, 2, G0, check=True)
    torch.cuda.synchronize()
    assert torch.equal(Pt0, Pt1) and torch.equal(Gt0, Gt1)
    # and against the oracle on the pooled factors (Section 3.2: the stacked product is the pooled gradient)
    ref = O.rank_r_grad(*O.block_spi(A.float().cpu().numpy(), D.float().cpu().numpy(), G0.cpu().numpy(), 2))
    got = Pt1.double().cpu().numpy().T @ Gt1.double().cpu().numpy()
    tol = 2e-2 if dtype == torch.bfloat16 else 1e-5
    assert O.rel_fro(got, ref) <= tol


REBUILD_CASES = [
    ([512, 1024, 256, 768], 256, 512, torch.bfloat16, True),
    ([4096, 0, 8192, 256], 512, 256, torch.bfloat16, True),            # several K chunks, blocks inside chunks
    ([256] * 32, 384, 128, torch.bfloat16, True),                      # 128-tiles
    ([1000, 1048], 256, 256, torch.bfloat16, False),
    ([512, 512], 200, 136, torch.bfloat16, False),
    ([100, 0, 300, 57], 784, 128, torch.float32, False),
]


@pytest.mark.parametrize("rows,h_in,h_out,dtype,in_place", REBUILD_CASES)
def test_full_rebuild_on_site_blocks_equals_stack_then_rebuild(gpu, rows, h_in, h_out, dtype, in_place):
    N = sum(rows)
    need = dad.reconstruct_sites_workspace_bytes(rows, h_in, h_out, dtype)
    assert (need == _up(dad.reconstruct_workspace_bytes(N, h_in, h_out, dtype))) == in_place
    A_s, D_s, _ = _sites(rows, h_in, h_out, 1, N + h_out, gpu, dtype)
    A, D = dad.stack_factors(A_s, D_s)
    G0 = dad.reconstruct_grad(A, D)
    G1 = dad.reconstruct_grad_sites(A_s, D_s)
    torch.cuda.synchronize()
    assert torch.equal(G0, G1)
    ref = O.full_grad(A.float().cpu().numpy(), D.float().cpu().numpy())
    assert O.rel_fro(G1.cpu().numpy(), ref) <= 1e-5       # bf16 inputs are exact; only the fp32 sums differ


def test_grouped_compress_mixes_stacked_layers_and_site_layers(gpu):
    """One grouped call, three lanes: a stacked layer, a layer on blocks read in place and a ragged one."""
    r = 32
    specs = [([512, 1024, 256], 256, 384), ([768, 768], 384, 256), ([300, 212, 512], 256, 128), ([1024, 1024], 512, 256)]
    layers, single = [], []
    for i, (rows, h_in, h_out) in enumerate(specs):
        A_s, D_s, G0 = _sites(rows, h_in, h_out, r, 40 + i, gpu, torch.bfloat16)
        A, D = dad.stack_factors(A_s, D_s)
        single.append(dad.compress_rank(A, D, r, 2, G0, check=True))
        layers.append((A, D, G0) if i == 0 else (A_s, D_s, G0))
    group = dad.CompressGroup(layers, r, 2, lanes=3)
    for _ in range(2):                                    # the second run re-uses the lanes' regions
        Pts, Gts = group.run(check=True)
        torch.cuda.synchronize()
        for (Pt0, Gt0), Pt1, Gt1 in zip(single, Pts, Gts):
            assert torch.equal(Pt0, Pt1) and torch.equal(Gt0, Gt1)


def test_site_calls_at_benchmark_size(gpu):
    """One GPT-2-medium MLP layer as its 8 sites of 8192 rows: reduction and full gradient read the
    sites in place and return the stacked calls' bits."""
    from paper_2102_09631_amd import workloads as W
    w = W.by_name("gpt2_medium_stack")
    h_in, h_out = 1024, 4096
    A_s, D_s = W.device_factors(w, 2, h_in, h_out)          # one tensor per site
    G0 = W.device_start_matrix(w, 2, h_out)
    b = w.rows_per_site
    A, D = dad.stack_factors(A_s, D_s)
    assert _in_place([b] * w.sites, h_in, h_out, w.rank, torch.bfloat16)
    Pt0, Gt0 = dad.compress_rank(A, D, w.rank, w.n_iter, G0, check=True)
    Pt1, Gt1 = dad.compress_rank_sites(A_s, D_s, w.rank, w.n_iter, G0, check=True)
    G_full0 = dad.reconstruct_grad(A, D)
    G_full1 = dad.reconstruct_grad_sites(A_s, D_s)
    torch.cuda.synchronize()
    assert torch.equal(Pt0, Pt1) and torch.equal(Gt0, Gt1) and torch.equal(G_full0, G_full1)
