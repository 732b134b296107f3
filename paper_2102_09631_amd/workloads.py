"""Seeded synthetic factor generators (inputs only: none of the method's arithmetic).

Every workload is a list of linear layers (h_in -> h_out) whose factor pairs
A (N x h_in) and Delta (N x h_out) are drawn from the value distributions of
the five benchmark configurations.  Rows [s*b, (s+1)*b) belong to simulated
site s.  The same arrays are handed to the HIP library and to the CPU checker.

Host generators use numpy's PCG64 keyed by (base, config, layer, stream);
device generators use a seeded torch.Generator and exist for the sizes that are
too large to draw on the host.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

SEED_BASE = 20210209
STREAM_A, STREAM_DELTA, STREAM_G0 = 0, 1, 2


@dataclass(frozen=True)
class Workload:
    name: str
    index: int                 # position in the benchmark's config list
    shapes: tuple              # distinct (h_in, h_out) linears of one block
    blocks: int                # how many times the block repeats in the stack
    sites: int                 # S
    rows_per_site: int         # b
    dtype: str                 # "f32" or "bf16"
    act: str                   # distribution of A: "relu", "normal", "gelu"
    delta: str                 # distribution of Delta: "normal" or "student3"
    delta_scale: float         # standard deviation (normal) or multiplier (t)
    rank: int                  # r
    n_iter: int                # power iterations
    layers: tuple = field(default=())

    @property
    def N(self) -> int:
        return self.sites * self.rows_per_site

    def all_layers(self):
        """(layer_index, h_in, h_out) over the whole stack."""
        out = []
        for blk in range(self.blocks):
            for j, (hi, ho) in enumerate(self.shapes):
                out.append((blk * len(self.shapes) + j, hi, ho))
        return out


WORKLOADS = (
    Workload("linear_784x128", 0, ((784, 128),), 1, 2, 32, "f32",
             "relu", "normal", math.sqrt(0.01), 4, 2),
    Workload("mlp_784_1024_1024_10", 1, ((784, 1024), (1024, 1024), (1024, 10)), 1, 4, 256, "f32",
             "relu", "normal", math.sqrt(1e-3), 8, 2),
    Workload("encoder_d768", 2, ((768, 2304), (768, 768), (768, 3072), (3072, 768)), 1, 4, 4096,
             "bf16", "normal", "normal", math.sqrt(1e-4), 16, 2),
    Workload("gpt2_medium_stack", 3, ((1024, 3072), (1024, 1024), (1024, 4096), (4096, 1024)), 24,
             8, 8192, "bf16", "normal", "normal", math.sqrt(1e-4), 32, 2),
    Workload("vit_large_stack", 4, ((1280, 3840), (1280, 1280), (1280, 5120), (5120, 1280)), 32,
             16, 16384, "bf16", "gelu", "student3", 1e-3, 64, 2),
)


def by_name(name: str) -> Workload:
    for w in WORKLOADS:
        if w.name == name:
            return w
    raise KeyError(name)


# ---------------------------------------------------------------- bf16 <-> f32

def f32_to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (nearest, ties to even); returns uint16 bit patterns."""
    u = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    rounded = u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))
    return (rounded >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    """Exact widening of bfloat16 bit patterns to float32."""
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


# ---------------------------------------------------------------- host draws

def _rng(cfg_index: int, layer: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64([SEED_BASE, cfg_index, layer, stream]))


def _erf(x: np.ndarray) -> np.ndarray:
    from scipy.special import erf
    return erf(x)


def _draw_A(rng, kind, shape):
    z = rng.standard_normal(shape)
    if kind == "relu":
        return np.maximum(z, 0.0)
    if kind == "gelu":                     # exact (erf) GELU
        return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))
    return z


def _draw_delta(rng, kind, scale, shape):
    if kind == "student3":
        return scale * rng.standard_t(3.0, size=shape)
    return scale * rng.standard_normal(shape)


def host_factors(w: Workload, layer: int, h_in: int, h_out: int, rows: int | None = None,
                 sites: int | None = None):
    """Per-site factor pairs of one layer as float32 arrays already on the dtype's grid.

    Returns (A_sites, D_sites): lists of S arrays (b x h_in), (b x h_out) float32.
    For a bf16 workload the values are rounded to bfloat16 once, here, so both
    the library and the checker consume exactly the same numbers.
    `rows`/`sites` override b and S to make reduced-size cases of the same recipe.
    """
    S = w.sites if sites is None else sites
    b = w.rows_per_site if rows is None else rows
    ra, rd = _rng(w.index, layer, STREAM_A), _rng(w.index, layer, STREAM_DELTA)
    A_sites, D_sites = [], []
    for _ in range(S):
        a = _draw_A(ra, w.act, (b, h_in)).astype(np.float32)
        d = _draw_delta(rd, w.delta, w.delta_scale, (b, h_out)).astype(np.float32)
        if w.dtype == "bf16":
            a = bf16_bits_to_f32(f32_to_bf16_bits(a))
            d = bf16_bits_to_f32(f32_to_bf16_bits(d))
        A_sites.append(a)
        D_sites.append(d)
    return A_sites, D_sites


def host_start_matrix(w: Workload, layer: int, h_out: int, r: int | None = None) -> np.ndarray:
    """Seeded Gaussian power-iteration start matrix, r x h_out float32, row j = g_0^j."""
    r = w.rank if r is None else r
    return _rng(w.index, layer, STREAM_G0).standard_normal((r, h_out)).astype(np.float32)


# ---------------------------------------------------------------- device draws

def device_factors(w: Workload, layer: int, h_in: int, h_out: int, device="cuda"):
    """Same distributions drawn on the device, one (b x h) tensor per site.

    Used where the stack is too large to draw on the host.  Returns lists of
    torch tensors in the workload's dtype.
    """
    import torch

    gen = torch.Generator(device=device)
    gen.manual_seed(SEED_BASE + 1000 * w.index + layer)
    tdt = torch.bfloat16 if w.dtype == "bf16" else torch.float32
    A_sites, D_sites = [], []
    for _ in range(w.sites):
        z = torch.randn(w.rows_per_site, h_in, generator=gen, device=device, dtype=torch.float32)
        if w.act == "relu":
            z = torch.relu_(z)
        elif w.act == "gelu":
            z = torch.nn.functional.gelu(z)
        A_sites.append(z.to(tdt))
        del z
        d = torch.randn(w.rows_per_site, h_out, generator=gen, device=device, dtype=torch.float32)
        if w.delta == "student3":
            # t(3) = normal / sqrt(chi2(3)/3)
            c = torch.randn(3, w.rows_per_site, h_out, generator=gen, device=device,
                            dtype=torch.float32).square_().sum(0).div_(3.0).sqrt_()
            d = d / c
            del c
        D_sites.append((d * w.delta_scale).to(tdt))
        del d
    return A_sites, D_sites


def device_start_matrix(w: Workload, layer: int, h_out: int, device="cuda"):
    import torch

    g = torch.from_numpy(host_start_matrix(w, layer, h_out))
    return g.to(device)
