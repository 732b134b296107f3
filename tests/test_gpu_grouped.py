"""Grouped entry points against the single-layer calls (bit for bit) and against the oracle."""
import pytest
import torch

from oracle import dad_oracle as O
from paper_2102_09631_amd import binding as dad

pytestmark = pytest.mark.gpu


def _pair(K, h_in, h_out, seed, dev, dtype=torch.float32):
    g = torch.Generator(device="cpu").manual_seed(seed)
    L = torch.randn(K, h_in, generator=g).to(dtype).to(dev)
    R = (0.1 * torch.randn(K, h_out, generator=g)).to(dtype).to(dev)
    return L, R


def _check_against_oracle(G, L, R, tol):
    ref = O.full_grad(L.float().cpu().numpy(), R.float().cpu().numpy())
    assert O.rel_fro(G.cpu().numpy(), ref) <= tol


RANK_SHAPES = [(4, 784, 128), (8, 1024, 10), (16, 768, 2304), (32, 1024, 4096), (64, 1280, 1280), (3, 53, 29),
               (1, 40, 24), (7, 130, 257)]


def test_grouped_rank_rebuild_equals_single_calls(gpu):
    """K = r pairs of every benchmark rank and ragged shapes: one grouped call against one call each."""
    pairs = [_pair(K, hi, ho, 10 + i, gpu) for i, (K, hi, ho) in enumerate(RANK_SHAPES)]
    single = [dad.reconstruct_grad(L, R) for L, R in pairs]
    grouped = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), a, b in zip(pairs, single, grouped):
        assert torch.equal(a, b)
        _check_against_oracle(b, L, R, 1e-5)


def test_grouped_rebuild_with_split_contraction_and_many_jobs(gpu):
    """40 jobs (two launches of the job table), among them fp32 full-gradient shapes whose
    contraction is split into slabs."""
    shapes = [(1024, 784, 1024), (1024, 1024, 1024), (2000, 96, 80), (64, 784, 128)] + [(5, 64 + i, 33 + 2 * i) for i in range(36)]
    pairs = [_pair(K, hi, ho, 100 + i, gpu) for i, (K, hi, ho) in enumerate(shapes)]
    assert dad.lib().dad_reconstruct_workspace_bytes(1024, 1024, 1024, dad.DAD_F32) > 0   # split
    single = [dad.reconstruct_grad(L, R) for L, R in pairs]
    grouped = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), a, b in zip(pairs, single, grouped):
        assert torch.equal(a, b)
        _check_against_oracle(b, L, R, 1e-5)


def test_grouped_rebuild_bf16_jobs(gpu):
    pairs = [_pair(4096, 512, 768, 7, gpu, torch.bfloat16), _pair(1000, 256, 264, 8, gpu, torch.bfloat16)]
    single = [dad.reconstruct_grad(L, R) for L, R in pairs]
    grouped = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), a, b in zip(pairs, single, grouped):
        assert torch.equal(a, b)
        _check_against_oracle(b, L, R, 1e-5)     # bf16 inputs are exact; only the fp32 sums differ


@pytest.mark.parametrize("K,h_in,h_out", [(64, 784, 128), (1024, 784, 1024), (1024, 1024, 10), (257, 129, 255),
                                          (9, 300, 520), (4097, 64, 96)])
def test_fp32_rebuild_on_the_matrix_instruction_matches_oracle(gpu, K, h_in, h_out):
    """Full fp32 gradients (the two MLP workloads' shapes and ragged ones, odd K included)."""
    L, R = _pair(K, h_in, h_out, K + h_in, gpu)
    G = dad.reconstruct_grad(L, R)
    _check_against_oracle(G, L, R, 1e-5)
    assert torch.equal(G, dad.reconstruct_grad(L, R))      # fixed summation order


# ---------------------------------------------------------------- grouped compress

def _layer(N, h_in, h_out, r, seed, dev, dtype):
    g = torch.Generator(device="cpu").manual_seed(seed)
    A = torch.relu(torch.randn(N, h_in, generator=g)).to(dtype).to(dev)
    D = (0.03 * torch.randn(N, h_out, generator=g)).to(dtype).to(dev)
    G0 = torch.randn(r, h_out, generator=g).to(dev)
    return A, D, G0


BF16_LAYERS = [(1024, 768, 2304), (1024, 768, 768), (512, 256, 512), (1000, 384, 128), (2048, 1024, 256)]
F32_LAYERS = [(64, 784, 128), (300, 96, 80), (1024, 1024, 10), (37, 53, 29)]


@pytest.mark.parametrize("lanes", [1, 2, 3, 8])
@pytest.mark.parametrize("kind", ["bf16", "f32"])
def test_grouped_compress_equals_single_calls(gpu, kind, lanes):
    dtype, shapes, r, tol = (torch.bfloat16, BF16_LAYERS, 16, 2e-2) if kind == "bf16" else (torch.float32, F32_LAYERS, 4, 1e-5)
    layers = [_layer(N, hi, ho, r, 40 + i, gpu, dtype) for i, (N, hi, ho) in enumerate(shapes)]
    single = [dad.compress_rank(A, D, r, 2, G0, check=True) for A, D, G0 in layers]
    grp = dad.CompressGroup(layers, r, 2, lanes=lanes)
    Pts, Gts = grp.run(check=True)
    torch.cuda.synchronize()
    for (A, D, G0), (p1, g1), p2, g2 in zip(layers, single, Pts, Gts):
        assert torch.equal(p1, p2) and torch.equal(g1, g2)
    A, D, G0 = layers[0]
    ref = O.rank_r_grad(*O.block_spi(A.float().cpu().numpy(), D.float().cpu().numpy(), G0.cpu().numpy(), 2))
    assert O.rel_fro(dad.reconstruct_grad(Pts[0], Gts[0]).cpu().numpy(), ref) <= tol


def test_grouped_compress_reports_a_breakdown_of_any_layer(gpu):
    layers = [_layer(N, hi, ho, 4, 60 + i, gpu, torch.float32) for i, (N, hi, ho) in enumerate(F32_LAYERS)]
    broken = list(layers)
    A, D, G0 = broken[1]
    broken[1] = (A, torch.zeros_like(D), G0)          # Delta = 0: the first Cholesky pivot of that layer is zero
    grp = dad.CompressGroup(broken, 4, 2, lanes=2)
    grp.run()
    assert dad.poll_numeric_status(grp.workspace) == dad.DAD_ERR_NUMERIC
    healthy = dad.CompressGroup(layers, 4, 2, lanes=2, workspace=grp.workspace)
    healthy.run()
    assert dad.poll_numeric_status(grp.workspace) == dad.DAD_OK


def test_grouped_compress_replays_from_a_hip_graph(gpu):
    dad.init()
    layers = [_layer(N, hi, ho, 16, 80 + i, gpu, torch.bfloat16) for i, (N, hi, ho) in enumerate(BF16_LAYERS[:4])]
    grp = dad.CompressGroup(layers, 16, 2, lanes=3)
    eager = [(p.clone(), g.clone()) for p, g in zip(*grp.run(check=True))]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        grp.run()
    for rep in range(3):
        for p, g in zip(grp.Pt, grp.Gt):
            p.fill_(float("nan"))
            g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (p1, g1), p2, g2 in zip(eager, grp.Pt, grp.Gt):
            assert torch.equal(p1, p2) and torch.equal(g1, g2), rep
        _ = dad.reconstruct_grad(grp.Pt[0], grp.Gt[0])    # eager work between the replays
        torch.cuda.synchronize()


# ---------------------------------------------------------------- batches: runs of equal layers share their launches

# (rows, h_in, h_out, r): runs of equal shapes, as lists of layer counts per run
BATCH_CASES = [
    ((2048, 256, 384, 32), [5, 1, 3]),        # a batch of 5, a layer of another shape, a batch of 3
    ((256, 128, 128, 16), [33]),              # more jobs than one batch takes: 32 + 1
    ((8192, 1024, 512, 64), [4]),             # a site reduction's size: single-wave workgroups, row chunks
    ((1024, 384, 128, 16), [2, 2]),
]


@pytest.mark.parametrize("lanes", [1, 3])
@pytest.mark.parametrize("shape,runs", BATCH_CASES)
def test_batched_layers_equal_single_calls(gpu, shape, runs, lanes):
    """Runs of equal layers (the S site reductions of Algorithm 1) go through merged launches; every
    layer's pair must be what a call of its own returns, bit for bit, whatever batch it lands in."""
    N, hi, ho, r = shape
    layers = []
    for k, count in enumerate(runs):
        n, a, b = (N, hi, ho) if k % 2 == 0 else (N // 2, ho, hi)     # odd runs: another shape
        layers += [_layer(n, a, b, r, 300 + 17 * k + i, gpu, torch.bfloat16) for i in range(count)]
    single = [dad.compress_rank(A, D, r, 2, G0, check=True) for A, D, G0 in layers]
    grp = dad.CompressGroup(layers, r, 2, lanes=lanes)
    for _ in range(2):                                                  # the second run re-uses the regions
        for p, g in zip(grp.Pt, grp.Gt):
            p.fill_(float("nan"))
            g.fill_(float("nan"))
        Pts, Gts = grp.run(check=True)
        torch.cuda.synchronize()
        for (p1, g1), p2, g2 in zip(single, Pts, Gts):
            assert torch.equal(p1, p2) and torch.equal(g1, g2)
    for i in (0, len(layers) - 1):
        A, D, G0 = layers[i]
        ref = O.rank_r_grad(*O.block_spi(A.float().cpu().numpy(), D.float().cpu().numpy(), G0.cpu().numpy(), 2))
        assert O.rel_fro(dad.reconstruct_grad(Pts[i], Gts[i]).cpu().numpy(), ref) <= 2e-2


def test_batch_reports_a_breakdown_of_one_job(gpu):
    layers = [_layer(1024, 256, 256, 16, 500 + i, gpu, torch.bfloat16) for i in range(4)]
    broken = list(layers)
    A, D, G0 = broken[2]
    broken[2] = (A, torch.zeros_like(D), G0)
    grp = dad.CompressGroup(broken, 16, 2, lanes=2)
    grp.run()
    assert dad.poll_numeric_status(grp.workspace) == dad.DAD_ERR_NUMERIC
    healthy = dad.CompressGroup(layers, 16, 2, lanes=2, workspace=grp.workspace)
    Pts, Gts = healthy.run()
    assert dad.poll_numeric_status(grp.workspace) == dad.DAD_OK
    for (A, D, G0), p, g in zip(layers, Pts, Gts):
        p1, g1 = dad.compress_rank(A, D, 16, 2, G0)
        assert torch.equal(p1, p) and torch.equal(g1, g)


def test_batch_replays_from_a_hip_graph(gpu):
    dad.init()
    layers = [_layer(2048, 256, 512, 32, 600 + i, gpu, torch.bfloat16) for i in range(6)]
    grp = dad.CompressGroup(layers, 32, 2, lanes=2)
    eager = [(p.clone(), g.clone()) for p, g in zip(*grp.run(check=True))]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        grp.run()
    for rep in range(3):
        for p, g in zip(grp.Pt, grp.Gt):
            p.fill_(float("nan"))
            g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (p1, g1), p2, g2 in zip(eager, grp.Pt, grp.Gt):
            assert torch.equal(p1, p2) and torch.equal(g1, g2), rep
        _ = dad.reconstruct_grad(grp.Pt[0], grp.Gt[0])    # eager work between the replays
        torch.cuda.synchronize()


def test_grouped_rebuild_of_bf16_runs_shares_launches(gpu):
    """A block's full gradients in one call: the four encoder-sized shapes run as one launch with a
    common K split, a ragged job in between runs on its own; every result within the a5 bar of the
    oracle and identical from run to run."""
    shapes = [(4096, 768, 2304), (4096, 768, 768), (4096, 768, 3072), (4096, 3072, 768), (1000, 256, 264),
              (2048, 256, 512), (2048, 512, 256)]
    pairs = [_pair(K, hi, ho, 700 + i, gpu, torch.bfloat16) for i, (K, hi, ho) in enumerate(shapes)]
    first = [g.clone() for g in dad.reconstruct_grad_grouped(pairs)]
    again = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), a, b in zip(pairs, first, again):
        assert torch.equal(a, b)
        _check_against_oracle(b, L, R, 1e-5)
    # the ragged job is planned as a call of its own
    assert torch.equal(first[4], dad.reconstruct_grad(*pairs[4]))


def test_grouped_rebuild_of_many_bf16_jobs(gpu):
    """More jobs than one launch takes (16), at a benchmark K with several chunks."""
    pairs = [_pair(8192, 256, 256 if i % 2 else 512, 800 + i, gpu, torch.bfloat16) for i in range(19)]
    got = dad.reconstruct_grad_grouped(pairs)
    torch.cuda.synchronize()
    for (L, R), G in zip(pairs, got):
        _check_against_oracle(G, L, R, 1e-5)


# layers of equal N whose widths differ (all multiples of 256) share launches too
MIXED_WIDTH_CASES = [
    (4096, 16, [(768, 2304), (768, 768), (768, 3072), (3072, 768)]),                    # an encoder block
    (2048, 32, [(256, 512), (512, 256), (768, 1024), (256, 512), (256, 512)]),          # equal and unequal neighbours
    (1024, 64, [(1280, 256), (256, 1280), (512, 512)]),
    (2048, 32, [(256, 512), (384, 128), (256, 256), (512, 256), (256, 384), (512, 512)]),  # 384 / 128 wide layers break the runs
]


@pytest.mark.parametrize("lanes", [1, 2])
@pytest.mark.parametrize("N,r,widths", MIXED_WIDTH_CASES)
def test_batched_layers_of_different_widths_equal_single_calls(gpu, N, r, widths, lanes):
    layers = [_layer(N, hi, ho, r, 900 + 13 * i, gpu, torch.bfloat16) for i, (hi, ho) in enumerate(widths)]
    single = [dad.compress_rank(A, D, r, 2, G0, check=True) for A, D, G0 in layers]
    grp = dad.CompressGroup(layers, r, 2, lanes=lanes)
    for _ in range(2):
        for p, g in zip(grp.Pt, grp.Gt):
            p.fill_(float("nan"))
            g.fill_(float("nan"))
        Pts, Gts = grp.run(check=True)
        torch.cuda.synchronize()
        for i, ((p1, g1), p2, g2) in enumerate(zip(single, Pts, Gts)):
            assert torch.equal(p1, p2) and torch.equal(g1, g2), i
    A, D, G0 = layers[-1]
    ref = O.rank_r_grad(*O.block_spi(A.float().cpu().numpy(), D.float().cpu().numpy(), G0.cpu().numpy(), 2))
    assert O.rel_fro(dad.reconstruct_grad(Pts[-1], Gts[-1]).cpu().numpy(), ref) <= 2e-2


def test_mixed_width_batch_reports_a_breakdown_and_replays_from_a_graph(gpu):
    dad.init()
    widths = [(768, 2304), (768, 768), (768, 3072), (3072, 768)]
    layers = [_layer(4096, hi, ho, 16, 950 + i, gpu, torch.bfloat16) for i, (hi, ho) in enumerate(widths)]
    broken = list(layers)
    A, D, G0 = broken[1]
    broken[1] = (A, torch.zeros_like(D), G0)
    bad = dad.CompressGroup(broken, 16, 2, lanes=2)
    bad.run()
    assert dad.poll_numeric_status(bad.workspace) == dad.DAD_ERR_NUMERIC
    grp = dad.CompressGroup(layers, 16, 2, lanes=2, workspace=bad.workspace)
    eager = [(p.clone(), g.clone()) for p, g in zip(*grp.run(check=True))]
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        grp.run()
    for rep in range(3):
        for p, g in zip(grp.Pt, grp.Gt):
            p.fill_(float("nan"))
            g.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for (p1, g1), p2, g2 in zip(eager, grp.Pt, grp.Gt):
            assert torch.equal(p1, p2) and torch.equal(g1, g2), rep
        _ = dad.reconstruct_grad(grp.Pt[0], grp.Gt[0])
        torch.cuda.synchronize()


def test_a_whole_step_replays_from_one_hip_graph(gpu):
    """stack -> full gradients (one joined launch) -> grouped reduction on four lanes -> grouped rank-r
    gradients, recorded into ONE graph (the lanes fork and join inside the capture) and replayed with
    eager work in between; every replay must give the eager bits."""
    dad.init()
    r, S, b = 16, 4, 1024
    widths = [(768, 2304), (768, 768), (768, 3072), (3072, 768)]
    g = torch.Generator(device="cpu").manual_seed(4242)
    sites = [([torch.randn(b, hi, generator=g).to(torch.bfloat16).to(gpu) for _ in range(S)],
              [(0.03 * torch.randn(b, ho, generator=g)).to(torch.bfloat16).to(gpu) for _ in range(S)]) for hi, ho in widths]
    G0 = [torch.randn(r, ho, generator=g).to(gpu) for _, ho in widths]
    stacked = [(torch.empty((S * b, hi), dtype=torch.bfloat16, device=gpu), torch.empty((S * b, ho), dtype=torch.bfloat16, device=gpu))
               for hi, ho in widths]
    full = dad.RebuildGroup(stacked)
    comp = dad.CompressGroup([(A, D, g0) for (A, D), g0 in zip(stacked, G0)], r, 2, lanes=4)
    rank = dad.RebuildGroup(list(zip(comp.Pt, comp.Gt)))

    def step():
        for (As, Ds), (A, D) in zip(sites, stacked):
            dad.stack_factors(As, Ds, A_out=A, D_out=D)
        full.run()
        comp.run()
        rank.run()

    step()
    torch.cuda.synchronize()
    assert dad.poll_numeric_status(comp.workspace) == dad.DAD_OK
    outputs = full.G + comp.Pt + comp.Gt + rank.G
    eager = [t.clone() for t in outputs]
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        step()
    for rep in range(3):
        for t in outputs + [x for pair in stacked for x in pair]:
            t.fill_(float("nan"))
        torch.cuda.synchronize()
        graph.replay()
        torch.cuda.synchronize()
        for a, b_ in zip(eager, outputs):
            assert torch.equal(a, b_), rep
        _ = dad.reconstruct_grad(stacked[0][0], stacked[0][1])     # eager work between the replays
        torch.cuda.synchronize()
    ref = O.full_grad(stacked[2][0].float().cpu().numpy(), stacked[2][1].float().cpu().numpy())
    assert O.rel_fro(full.G[2].cpu().numpy(), ref) <= 1e-5
