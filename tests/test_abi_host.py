"""The C-ABI library loads without a GPU, exports every symbol the header declares,
and rejects bad arguments on the host before anything is enqueued (CPU only)."""
import ctypes as C
import os
import re

import pytest

from paper_2102_09631_amd import binding as dad

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(dad.LIB_PATH):
        from paper_2102_09631_amd.build import build_library
        build_library(verbose=False)
    return dad.lib()


def test_every_declared_symbol_is_exported(lib):
    text = open(os.path.join(ROOT, "include", "dad.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = set(re.findall(r"\b(dad_[a-z_]+)\s*\(", text))
    assert {"dad_stack_factors", "dad_compress_rank", "dad_reconstruct_grad", "dad_backprop_delta", "dad_compress_workspace_bytes",
            "dad_reconstruct_workspace_bytes", "dad_poll_numeric_status", "dad_status_string"} <= names
    for n in names:
        assert hasattr(lib, n), n


def test_status_strings(lib):
    seen = set()
    for s in range(8):
        txt = lib.dad_status_string(s).decode()
        assert txt and txt not in seen
        seen.add(txt)
    assert "unknown" in lib.dad_status_string(99).decode()


def test_workspace_queries(lib):
    assert lib.dad_compress_workspace_bytes(64, 784, 128, 4, dad.DAD_F32) > 64 * 4 * 4
    assert lib.dad_compress_workspace_bytes(64, 784, 128, 0, dad.DAD_F32) == 0
    assert lib.dad_compress_workspace_bytes(64, 784, 128, 65, dad.DAD_F32) == 0
    assert lib.dad_compress_workspace_bytes(3, 784, 128, 4, dad.DAD_F32) == 0      # r > N
    assert lib.dad_compress_workspace_bytes(64, 784, 128, 4, 7) == 0
    big = lib.dad_compress_workspace_bytes(262144, 1280, 5120, 64, dad.DAD_BF16)
    assert 262144 * 64 * 2 <= big < (1 << 30)
    assert lib.dad_reconstruct_workspace_bytes(4, 784, 128, dad.DAD_F32) == 0     # no split for K = r
    assert lib.dad_reconstruct_workspace_bytes(0, 784, 128, dad.DAD_F32) == 0


def test_compress_rejects_bad_arguments_on_host(lib):
    p = 0x1000  # fake, aligned, never dereferenced: every call below must fail before a launch
    ws = 1 << 30

    def call(A=p, D=p, N=64, hi=784, ho=128, dt=dad.DAD_F32, r=4, n=2, G0=p, Pt=p, Gt=p, w=p, wb=ws):
        return lib.dad_compress_rank(A, D, N, hi, ho, dt, r, n, G0, Pt, Gt, w, wb, None)

    assert call(A=None) == dad.DAD_ERR_NULL
    assert call(G0=None) == dad.DAD_ERR_NULL
    assert call(w=None) == dad.DAD_ERR_NULL
    assert call(dt=5) == dad.DAD_ERR_DTYPE
    assert call(r=0) == dad.DAD_ERR_SHAPE
    assert call(r=65) == dad.DAD_ERR_SHAPE
    assert call(N=3) == dad.DAD_ERR_SHAPE          # r > N
    assert call(ho=2) == dad.DAD_ERR_SHAPE         # r > h_out
    assert call(n=0) == dad.DAD_ERR_SHAPE
    assert call(N=0) == dad.DAD_ERR_SHAPE
    assert call(N=(1 << 36) + 1) == dad.DAD_ERR_SHAPE      # beyond what the launch grids hold
    assert call(hi=(1 << 21) + 1) == dad.DAD_ERR_SHAPE
    assert call(ho=(1 << 21) + 1) == dad.DAD_ERR_SHAPE
    assert call(D=p + 4) == dad.DAD_ERR_ALIGN
    assert call(wb=128) == dad.DAD_ERR_WORKSPACE


def test_noalloc_rejects_bad_arguments_and_oversize_on_host(lib):
    p = 0x1000  # never dereferenced: every call below must fail before a launch

    def call(A=p, D=p, N=64, hi=784, ho=128, dt=dad.DAD_F32, r=4, n=2, G0=p, Pt=p, Gt=p, flag=None):
        return lib.dad_compress_rank_noalloc(A, D, N, hi, ho, dt, r, n, G0, Pt, Gt, flag, None)

    assert call(D=None) == dad.DAD_ERR_NULL
    assert call(dt=3) == dad.DAD_ERR_DTYPE
    assert call(r=65) == dad.DAD_ERR_SHAPE
    assert call(Gt=p + 4) == dad.DAD_ERR_ALIGN
    assert call(flag=p + 2) == dad.DAD_ERR_ALIGN
    # the static scratch holds DAD_STATIC_SCRATCH_BYTES: the largest benchmark shape does not fit
    big = dict(N=262144, hi=1280, ho=5120, dt=dad.DAD_BF16, r=64)
    assert lib.dad_compress_workspace_bytes(262144, 1280, 5120, 64, dad.DAD_BF16) > dad.DAD_STATIC_SCRATCH_BYTES
    assert call(**big) == dad.DAD_ERR_WORKSPACE
    assert lib.dad_compress_workspace_bytes(65536, 1024, 4096, 32, dad.DAD_BF16) <= dad.DAD_STATIC_SCRATCH_BYTES


def test_reconstruct_and_stack_reject_bad_arguments_on_host(lib):
    p = 0x1000
    assert lib.dad_reconstruct_grad(None, p, 4, 8, 8, 0, p, None, 0, None) == dad.DAD_ERR_NULL
    assert lib.dad_reconstruct_grad(p, p, 0, 8, 8, 0, p, None, 0, None) == dad.DAD_ERR_SHAPE
    assert lib.dad_reconstruct_grad(p, p, 4, (1 << 21) + 1, 8, 0, p, None, 0, None) == dad.DAD_ERR_SHAPE
    assert lib.dad_reconstruct_grad(p, p, 4, 8, 8, 9, p, None, 0, None) == dad.DAD_ERR_DTYPE
    assert lib.dad_reconstruct_grad(p, p + 2, 4, 8, 8, 0, p, None, 0, None) == dad.DAD_ERR_ALIGN
    need = lib.dad_reconstruct_workspace_bytes(65536, 1024, 1024, dad.DAD_BF16)
    if need:
        assert lib.dad_reconstruct_grad(p, p, 65536, 1024, 1024, 1, p, None, 0, None) == dad.DAD_ERR_NULL
        assert lib.dad_reconstruct_grad(p, p, 65536, 1024, 1024, 1, p, p, need - 1, None) == dad.DAD_ERR_WORKSPACE
    ptrs = (C.c_void_p * 2)(p, p)
    rows = (C.c_int64 * 2)(4, 4)
    bad_rows = (C.c_int64 * 2)(4, -1)
    assert lib.dad_stack_factors(0, ptrs, ptrs, rows, 8, 8, 0, p, p, None) == dad.DAD_ERR_SHAPE
    assert lib.dad_stack_factors(2, ptrs, ptrs, bad_rows, 8, 8, 0, p, p, None) == dad.DAD_ERR_SHAPE
    assert lib.dad_stack_factors(2, None, ptrs, rows, 8, 8, 0, p, p, None) == dad.DAD_ERR_NULL
    assert lib.dad_stack_factors(2, ptrs, ptrs, rows, 8, 8, 0, p + 8, p, None) == dad.DAD_ERR_ALIGN
    assert lib.dad_stack_factors(2, ptrs, ptrs, rows, 8, 8, 3, p, p, None) == dad.DAD_ERR_DTYPE
    nullp = (C.c_void_p * 2)(p, None)
    assert lib.dad_stack_factors(2, nullp, ptrs, rows, 8, 8, 0, p, p, None) == dad.DAD_ERR_NULL


def test_grouped_rebuild_rejects_bad_arguments_on_host(lib):
    p = 0x1000
    D = dad.RebuildDesc
    good = (D * 2)(D(p, p, p, 4, 8, 8), D(p, p, p, 8, 16, 24))
    assert lib.dad_reconstruct_grad_grouped(2, None, 0, None, 0, None) == dad.DAD_ERR_NULL
    assert lib.dad_reconstruct_grad_grouped(0, good, 0, None, 0, None) == dad.DAD_ERR_SHAPE
    assert lib.dad_reconstruct_grad_grouped(4097, good, 0, None, 0, None) == dad.DAD_ERR_SHAPE
    assert lib.dad_reconstruct_grad_grouped(2, good, 6, None, 0, None) == dad.DAD_ERR_DTYPE
    bad = (D * 2)(D(p, p, p, 4, 8, 8), D(p, None, p, 8, 16, 24))
    assert lib.dad_reconstruct_grad_grouped(2, bad, 0, None, 0, None) == dad.DAD_ERR_NULL
    bad = (D * 2)(D(p, p, p, 4, 8, 8), D(p, p, p, 0, 16, 24))
    assert lib.dad_reconstruct_grad_grouped(2, bad, 0, None, 0, None) == dad.DAD_ERR_SHAPE
    bad = (D * 2)(D(p, p, p + 4, 4, 8, 8), D(p, p, p, 8, 16, 24))
    assert lib.dad_reconstruct_grad_grouped(2, bad, 0, None, 0, None) == dad.DAD_ERR_ALIGN
    big = (D * 2)(D(p, p, p, 1024, 1024, 1024), D(p, p, p, 1024, 1024, 1024))
    need = lib.dad_reconstruct_grouped_workspace_bytes(2, big, dad.DAD_F32)
    assert need >= 2 * lib.dad_reconstruct_workspace_bytes(1024, 1024, 1024, dad.DAD_F32) > 0
    assert lib.dad_reconstruct_grad_grouped(2, big, 0, None, 0, None) == dad.DAD_ERR_NULL
    assert lib.dad_reconstruct_grad_grouped(2, big, 0, p, need - 1, None) == dad.DAD_ERR_WORKSPACE
    assert lib.dad_reconstruct_grouped_workspace_bytes(2, good, dad.DAD_F32) == 0


def test_grouped_compress_rejects_bad_arguments_on_host(lib):
    p = 0x1000
    D = dad.CompressDesc
    good = (D * 2)(D(p, p, p, p, p, 64, 784, 128), D(p, p, p, p, p, 256, 128, 96))
    ws = 1 << 30

    def call(n=2, descs=good, dt=dad.DAD_F32, r=4, it=2, lanes=2, w=p, wb=ws):
        return lib.dad_compress_rank_grouped(n, descs, dt, r, it, lanes, w, wb, None)

    assert call(descs=None) == dad.DAD_ERR_NULL
    assert call(w=None) == dad.DAD_ERR_NULL
    assert call(dt=4) == dad.DAD_ERR_DTYPE
    assert call(n=0) == dad.DAD_ERR_SHAPE
    assert call(lanes=0) == dad.DAD_ERR_SHAPE
    assert call(lanes=9) == dad.DAD_ERR_SHAPE
    assert call(r=65) == dad.DAD_ERR_SHAPE
    assert call(it=0) == dad.DAD_ERR_SHAPE
    bad = (D * 2)(D(p, p, p, p, p, 64, 784, 128), D(p, p, p, None, p, 256, 128, 96))
    assert call(descs=bad) == dad.DAD_ERR_NULL
    bad = (D * 2)(D(p, p, p, p, p, 64, 784, 128), D(p, p, p, p, p, 3, 128, 96))      # r > N
    assert call(descs=bad) == dad.DAD_ERR_SHAPE
    bad = (D * 2)(D(p, p + 8, p, p, p, 64, 784, 128), D(p, p, p, p, p, 256, 128, 96))
    assert call(descs=bad) == dad.DAD_ERR_ALIGN
    need = lib.dad_compress_grouped_workspace_bytes(2, good, dad.DAD_F32, 4, 2)
    one = max(lib.dad_compress_workspace_bytes(64, 784, 128, 4, dad.DAD_F32),
              lib.dad_compress_workspace_bytes(256, 128, 96, 4, dad.DAD_F32))
    assert need >= 256 + 2 * one
    assert lib.dad_compress_grouped_workspace_bytes(2, good, dad.DAD_F32, 4, 1) < need
    assert call(wb=need - 1) == dad.DAD_ERR_WORKSPACE
    assert lib.dad_compress_grouped_workspace_bytes(2, good, dad.DAD_F32, 4, 9) == 0


def test_site_calls_reject_bad_arguments_and_size_their_workspace_on_host(lib):
    p = 0x1000
    vp, i64 = C.c_void_p, C.c_int64

    def tables(rows, ptr=p):
        S = len(rows)
        return S, (vp * S)(*[ptr if n else None for n in rows]), (vp * S)(*[ptr if n else None for n in rows]), \
            (i64 * S)(*rows)

    def compress(rows, hi=256, ho=384, dt=dad.DAD_BF16, r=32, it=2, G0=p, Pt=p, Gt=p, w=p, wb=1 << 40, ptr=p):
        S, pa, pd, pr = tables(rows, ptr)
        return lib.dad_compress_rank_sites(S, pa, pd, pr, hi, ho, dt, r, it, G0, Pt, Gt, w, wb, None)

    def rebuild(rows, hi=256, ho=384, dt=dad.DAD_BF16, G=p, w=p, wb=1 << 40, ptr=p):
        S, pa, pd, pr = tables(rows, ptr)
        return lib.dad_reconstruct_grad_sites(S, pa, pd, pr, hi, ho, dt, G, w, wb, None)

    rows = [512, 0, 1024]
    assert compress(rows, w=None) == dad.DAD_ERR_NULL
    assert compress(rows, G0=None) == dad.DAD_ERR_NULL
    assert compress(rows, dt=9) == dad.DAD_ERR_DTYPE
    assert compress(rows, r=65) == dad.DAD_ERR_SHAPE
    assert compress(rows, it=0) == dad.DAD_ERR_SHAPE
    assert compress([0, 0]) == dad.DAD_ERR_SHAPE                       # no rows at all
    assert compress([512, -1]) == dad.DAD_ERR_SHAPE
    assert compress(rows, ptr=p + 8) == dad.DAD_ERR_ALIGN
    assert lib.dad_compress_rank_sites(0, None, None, None, 256, 384, dad.DAD_BF16, 32, 2, p, p, p, p, 1 << 40,
                                       None) == dad.DAD_ERR_SHAPE
    S, pa, pd, pr = tables(rows)
    assert lib.dad_compress_rank_sites(S, None, pd, pr, 256, 384, dad.DAD_BF16, 32, 2, p, p, p, p, 1 << 40,
                                       None) == dad.DAD_ERR_NULL
    assert rebuild(rows, G=None) == dad.DAD_ERR_NULL
    assert rebuild(rows, dt=9) == dad.DAD_ERR_DTYPE
    assert rebuild([0]) == dad.DAD_ERR_SHAPE
    assert rebuild(rows, ptr=p + 4) == dad.DAD_ERR_ALIGN

    def cbytes(rows, hi=256, ho=384, r=32, dt=dad.DAD_BF16):
        return lib.dad_compress_sites_workspace_bytes(len(rows), (i64 * len(rows))(*rows), hi, ho, r, dt)

    def rbytes(rows, hi=256, ho=384, dt=dad.DAD_BF16):
        return lib.dad_reconstruct_sites_workspace_bytes(len(rows), (i64 * len(rows))(*rows), hi, ho, dt)

    def up(x):
        return (x + 255) // 256 * 256

    # blocks of whole 256-row multiples on the direct-to-LDS path: no room for a stacked copy
    assert cbytes(rows) == up(lib.dad_compress_workspace_bytes(1536, 256, 384, 32, dad.DAD_BF16))
    assert rbytes([4096, 4096]) == up(lib.dad_reconstruct_workspace_bytes(8192, 256, 384, dad.DAD_BF16))
    # a ragged site, a rank the direct-to-LDS kernel is not built for, fp32, or too many sites: stacked copy included
    stacked = 1536 * (256 + 384) * 2
    assert cbytes([500, 12, 1024]) == up(lib.dad_compress_workspace_bytes(1536, 256, 384, 32, dad.DAD_BF16)) + stacked
    assert cbytes(rows, r=24) == up(lib.dad_compress_workspace_bytes(1536, 256, 384, 24, dad.DAD_BF16)) + stacked
    assert cbytes(rows, dt=dad.DAD_F32) == up(lib.dad_compress_workspace_bytes(1536, 256, 384, 32, dad.DAD_F32)) + 2 * stacked
    many = [256] * 40
    assert cbytes(many) == up(lib.dad_compress_workspace_bytes(10240, 256, 384, 32, dad.DAD_BF16)) + 10240 * 640 * 2
    assert rbytes([4000, 4192]) == up(lib.dad_reconstruct_workspace_bytes(8192, 256, 384, dad.DAD_BF16)) + 8192 * 640 * 2
    assert cbytes([0, 0]) == 0 and rbytes([0]) == 0 and cbytes(rows, r=0) == 0
    need = cbytes(rows)
    assert compress(rows, wb=need - 1) == dad.DAD_ERR_WORKSPACE
    assert rebuild([4000, 4192], wb=rbytes([4000, 4192]) - 1) == dad.DAD_ERR_WORKSPACE

    # a grouped layer given as sites is checked and sized the same way
    D = dad.CompressDesc
    S, pa, pd, pr = tables(rows)
    descs = (D * 2)(D(p, p, p, p, p, 512, 256, 384), D(None, None, p, p, p, 0, 256, 384, S, pa, pd, pr))
    need = lib.dad_compress_grouped_workspace_bytes(2, descs, dad.DAD_BF16, 32, 2)
    assert need == 256 + 2 * cbytes(rows)
    assert lib.dad_compress_rank_grouped(2, descs, dad.DAD_BF16, 32, 2, 2, p, need - 1, None) == dad.DAD_ERR_WORKSPACE
    bad = (D * 1)(D(None, None, p, p, p, 0, 256, 384, S, None, pd, pr))
    assert lib.dad_compress_rank_grouped(1, bad, dad.DAD_BF16, 32, 2, 1, p, 1 << 40, None) == dad.DAD_ERR_NULL
    bad = (D * 1)(D(p, p, p, p, p, 512, 256, 384, -1, pa, pd, pr))
    assert lib.dad_compress_rank_grouped(1, bad, dad.DAD_BF16, 32, 2, 1, p, 1 << 40, None) == dad.DAD_ERR_SHAPE


def test_backprop_rejects_bad_arguments_on_host(lib):
    p = 0x1000  # never dereferenced: every call below must fail before a launch

    def call(Dn=p, Wn=p, Z=p, N=256, h=256, hn=64, dt=dad.DAD_BF16, act=1, out=p):
        return lib.dad_backprop_delta(Dn, Wn, Z, N, h, hn, dt, act, out, None)

    assert call(Dn=None) == dad.DAD_ERR_NULL
    assert call(out=None) == dad.DAD_ERR_NULL
    assert call(dt=4) == dad.DAD_ERR_DTYPE
    assert call(act=4) == dad.DAD_ERR_SHAPE
    assert call(act=-1) == dad.DAD_ERR_SHAPE
    assert call(N=0) == dad.DAD_ERR_SHAPE
    assert call(hn=0) == dad.DAD_ERR_SHAPE
    assert call(h=(1 << 24) + 1) == dad.DAD_ERR_SHAPE
    assert call(Z=p + 2) == dad.DAD_ERR_ALIGN      # shape served by the MFMA kernel


def test_gram_route_rejects_bad_arguments_on_host(lib):
    p = 0x1000  # never dereferenced: every call below must fail before a launch
    ws = 1 << 30

    def call(A=p, D=p, N=64, hi=784, ho=128, dt=dad.DAD_F32, r=4, n=2, G0=p, Pt=p, Gt=p, w=p, wb=ws):
        return lib.dad_compress_rank_gram(A, D, N, hi, ho, dt, r, n, G0, Pt, Gt, w, wb, None)

    assert call(D=None) == dad.DAD_ERR_NULL
    assert call(Gt=None) == dad.DAD_ERR_NULL
    assert call(dt=5) == dad.DAD_ERR_DTYPE
    assert call(N=dad.DAD_GRAM_MAX_ROWS + 1) == dad.DAD_ERR_SHAPE
    assert call(N=0) == dad.DAD_ERR_SHAPE
    assert call(r=65) == dad.DAD_ERR_SHAPE
    assert call(N=3) == dad.DAD_ERR_SHAPE          # r > N
    assert call(n=0) == dad.DAD_ERR_SHAPE
    assert call(Pt=p + 8) == dad.DAD_ERR_ALIGN
    need = lib.dad_compress_gram_workspace_bytes(64, 784, 128, 4, dad.DAD_F32)
    assert need > 2 * 64 * 64 * 8 and call(wb=need - 1) == dad.DAD_ERR_WORKSPACE
    assert lib.dad_compress_gram_workspace_bytes(dad.DAD_GRAM_MAX_ROWS + 1, 784, 128, 4, dad.DAD_F32) == 0
    assert lib.dad_compress_gram_workspace_bytes(64, 784, 128, 4, 3) == 0
    assert lib.dad_compress_gram_workspace_bytes(1024, 1280, 5120, 64, dad.DAD_F32) < (1 << 27)


def test_sequential_rejects_bad_arguments_on_host(lib):
    p = 0x1000  # never dereferenced: every call below must fail before a launch
    ws = 1 << 30

    def call(A=p, D=p, N=64, hi=784, ho=128, dt=dad.DAD_F32, r=4, n=2, G0=p, Q=p, sG=p, sig=p, w=p, wb=ws):
        return lib.dad_compress_rank_sequential(A, D, N, hi, ho, dt, r, n, G0, Q, sG, sig, w, wb, None)

    assert call(A=None) == dad.DAD_ERR_NULL
    assert call(Q=None) == dad.DAD_ERR_NULL
    assert call(w=None) == dad.DAD_ERR_NULL
    assert call(dt=2) == dad.DAD_ERR_DTYPE
    assert call(r=0) == dad.DAD_ERR_SHAPE
    assert call(r=65) == dad.DAD_ERR_SHAPE
    assert call(N=3) == dad.DAD_ERR_SHAPE          # r > N
    assert call(n=0) == dad.DAD_ERR_SHAPE
    assert call(G0=p + 4) == dad.DAD_ERR_ALIGN
    assert call(wb=16) == dad.DAD_ERR_WORKSPACE
    need = lib.dad_compress_sequential_workspace_bytes(64, 784, 128, dad.DAD_F32)
    assert need > 64 * 4 and call(wb=need - 1) == dad.DAD_ERR_WORKSPACE
    assert lib.dad_compress_sequential_workspace_bytes(0, 784, 128, dad.DAD_F32) == 0
    assert lib.dad_compress_sequential_workspace_bytes(64, 784, 128, 9) == 0


def test_adaptive_rejects_bad_arguments_on_host(lib):
    p = 0x1000  # never dereferenced: every call below must fail before a launch
    ws = 1 << 30

    def call(A=p, N=64, dt=dad.DAD_F32, r=4, n=20, theta=1e-3, G0=p, rank=p, iters=None, wb=ws):
        return lib.dad_compress_rank_adaptive(A, p, N, 784, 128, dt, r, n, theta, G0, p, p, p, rank, iters, p, wb, None)

    assert call(A=None) == dad.DAD_ERR_NULL
    assert call(rank=None) == dad.DAD_ERR_NULL
    assert call(dt=2) == dad.DAD_ERR_DTYPE
    assert call(r=65) == dad.DAD_ERR_SHAPE
    assert call(n=0) == dad.DAD_ERR_SHAPE
    assert call(theta=-1e-3) == dad.DAD_ERR_SHAPE
    assert call(theta=1.0) == dad.DAD_ERR_SHAPE
    assert call(theta=float("nan")) == dad.DAD_ERR_SHAPE
    assert call(G0=p + 4) == dad.DAD_ERR_ALIGN
    assert call(rank=p + 2) == dad.DAD_ERR_ALIGN
    assert call(iters=p + 2) == dad.DAD_ERR_ALIGN
    assert call(wb=16) == dad.DAD_ERR_WORKSPACE


def test_binding_fails_loudly_without_library(monkeypatch, tmp_path):
    monkeypatch.setattr(dad, "_lib", None)
    monkeypatch.setattr(dad, "LIB_PATH", str(tmp_path / "libdad.so"))
    with pytest.raises(RuntimeError, match="missing"):
        dad.lib()


def test_binding_constants_match_the_header():
    text = open(os.path.join(ROOT, "include", "dad.h")).read()

    def macro(name):
        m = re.search(r"#define\s+" + name + r"\s+(.+)", text)
        assert m, name
        expr = re.sub(r"/\*.*?\*/", "", m.group(1)).strip()
        expr = expr.replace("(int64_t)", "").replace("u", "")
        return int(eval(expr, {"__builtins__": {}}))

    assert macro("DAD_MAX_LANES") == dad.DAD_MAX_LANES
    assert macro("DAD_STATIC_SCRATCH_BYTES") == dad.DAD_STATIC_SCRATCH_BYTES
    for name in ("DAD_OK", "DAD_ERR_NULL", "DAD_ERR_SHAPE", "DAD_ERR_ALIGN", "DAD_ERR_WORKSPACE", "DAD_ERR_DTYPE",
                 "DAD_ERR_NUMERIC", "DAD_ERR_HIP"):
        m = re.search(name + r"\s*=\s*(\d+)", text)
        assert m and int(m.group(1)) == getattr(dad, name), name
    assert re.search(r"DAD_F32\s*=\s*0", text) and dad.DAD_F32 == 0
    assert re.search(r"DAD_BF16\s*=\s*1", text) and dad.DAD_BF16 == 1


def test_grouped_compress_workspace_reflects_how_layers_are_batched(lib):
    """The size query shows the units a grouped call forms: a batch needs one region per job on ONE lane,
    layers that are not batched need one region per lane."""
    p = 0x1000
    D = dad.CompressDesc

    def up(x):
        return (x + 255) // 256 * 256

    def single(N, hi, ho, r):
        return up(lib.dad_compress_workspace_bytes(N, hi, ho, r, dad.DAD_BF16))

    def grouped(shapes, r, lanes):
        descs = (D * len(shapes))(*[D(p, p, p, p, p, N, hi, ho) for N, hi, ho in shapes])
        return lib.dad_compress_grouped_workspace_bytes(len(shapes), descs, dad.DAD_BF16, r, lanes)

    site = (8192, 1024, 512)
    # eight equal site-sized layers: one batch, one lane, eight regions
    assert grouped([site] * 8, 32, 4) == 256 + 8 * single(*site, 32)
    # 33 of them: a batch of 32 and a single layer, two units on two lanes, each lane sized for the batch
    assert grouped([site] * 33, 32, 4) == 256 + 2 * 32 * single(*site, 32)
    # a layer of another shape (384 wide: not a multiple of 256) splits the run: units of 5, 1, 3 on three lanes
    other = (8192, 384, 128)
    need = grouped([site] * 5 + [other] + [site] * 3, 32, 4)
    assert need == 256 + 3 * max(5 * single(*site, 32), single(*other, 32))
    # benchmark-sized layers (537 MB of factors each) are not batched: one region per lane
    big = (65536, 1024, 3072)
    assert grouped([big] * 4, 32, 2) == 256 + 2 * single(*big, 32)
    # small layers of unequal widths (multiples of 256) form one batch whose regions are sized for the widest job
    mixed = [(4096, 768, 2304), (4096, 768, 768), (4096, 768, 3072), (4096, 3072, 768)]
    need = grouped(mixed, 16, 4)
    assert need >= 256 + 4 * max(single(*m, 16) for m in mixed)
    assert need <= 256 + 4 * (single(4096, 3072, 3072, 16) + (1 << 20))
    # the same widths at the encoder's own row count (100-126 MB per layer) stay separate layers
    enc = [(16384, hi, ho) for _, hi, ho in mixed]
    assert grouped(enc, 16, 4) == 256 + 4 * max(single(*m, 16) for m in enc)
    # fp32 layers are never batched
    descs = (D * 3)(*[D(p, p, p, p, p, 1024, 1024, 1024) for _ in range(3)])
    assert lib.dad_compress_grouped_workspace_bytes(3, descs, dad.DAD_F32, 8, 2) == \
        256 + 2 * up(lib.dad_compress_workspace_bytes(1024, 1024, 1024, 8, dad.DAD_F32))
