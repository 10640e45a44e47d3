"""The fast build of the large-tile GEMM kernels against the checking build (libaxe_hip_paranoid.so: a full wait after
every load into LDS and every store, a full wait and a workgroup barrier after every row of MFMAs).  Same arithmetic in
the same order, so the two must agree bit for bit; a difference means that the fast build's counted waits, asm-issued
loads and stores or single barrier per K-step let something be read before it had arrived."""
import contextlib
import os

import numpy as np
import pytest
import torch

from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W

pytestmark = pytest.mark.gpu

PARANOID = os.path.join(os.path.dirname(B.LIB_PATH), "libaxe_hip_paranoid.so")


@contextlib.contextmanager
def library(path):
    B.lib()
    old = B._lib
    B._lib = B.load(path)
    try:
        yield
    finally:
        B._lib = old


def dev(a):
    a = np.ascontiguousarray(a)
    return torch.from_numpy(a.view({1: np.uint8, 2: np.int16, 4: np.int32}[a.dtype.itemsize])).cuda()


def dense_case(which):
    rows = 0
    if which == "config4":
        g, kw = W.config4(), dict(device_axis=True)
    elif which == "bf16_chained_17x16":
        g, kw = W.gemm_bf16(4352, 4096, 512, 91), {}
    elif which == "bf16_ragged":
        g, kw = W.gemm_bf16(1000, 1288, 512, 92), {}
    elif which == "fp8_f32_scales":
        g, kw = W.gemm_fp8(4352, 4096, 1024, 95, scaled=True), {}
    elif which == "fp8_e8m0":
        g, kw = W.gemm_fp8(4352, 4096, 1024, 96, scaled="e8m0"), {}
    else:                                                  # one E8M0 code per row of A
        g, kw = W.gemm_fp8(4352, 4096, 2048, 97, scaled="e8m0"), {}
        g.scale_a = np.random.default_rng(5).integers(122, 133, (g.M, g.K // 128)).astype(np.uint8)
        rows = 1
    As, Bs, Cs = W.gemm_specs(g, shard=3, **kw)
    axes = ["m", "gpuid"]
    sa = torch.from_numpy(g.scale_a).cuda() if g.scale_a is not None else None
    sb = torch.from_numpy(g.scale_b).cuda() if g.scale_b is not None else None
    desc = B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16 if g.dtype == "bf16" else B.AXE_FP8_E4M3, B.AXE_BF16,
                      B.Layout(As, axes), B.Layout(Bs, axes), B.Layout(Cs, axes), g.M * g.K, g.N * g.K, g.M * g.N, sa, sb,
                      scale_dtype=B.AXE_SCALE_E8M0 if g.scale_dtype == "e8m0" else B.AXE_SCALE_F32, scale_a_rows=rows,
                      tile_hint=B.AXE_TILE_256x256x64 if which == "bf16_ragged" else B.AXE_TILE_AUTO)
    return g, desc, dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))


@pytest.mark.parametrize("which", ["config4", "bf16_chained_17x16", "bf16_ragged", "fp8_f32_scales", "fp8_e8m0", "fp8_e8m0_rows"])
def test_dense_gemm_fast_build_equals_checking_build(which):
    g, desc, dA, dB = dense_case(which)
    assert B.axe_gemm_tile(desc) in (B.AXE_TILE_256x256x64, B.AXE_TILE_256x224x64)
    out = []
    for path in (B.LIB_PATH, PARANOID):
        with library(path):
            dC = torch.zeros(g.M * g.N, dtype=torch.int16, device="cuda")
            B.axe_gemm(desc, dA, dB, dC)
            torch.cuda.synchronize()
            out.append(dC)
    assert torch.equal(out[0], out[1]), f"{(out[0] != out[1]).sum().item()} elements differ"


@pytest.mark.parametrize("kernel,gated", [(B.AXE_GROUPED_TILES_256, False), (B.AXE_GROUPED_TILES_128, False), (B.AXE_GROUPED_TILES_128, True)])
def test_grouped_gemm_fast_build_equals_checking_build(kernel, gated):
    rng = np.random.default_rng(17)
    off = np.concatenate([[0], np.cumsum(rng.integers(0, 400, 40))]).astype(np.int32)
    N, K = 1536, 512
    g = W.gemm_grouped_bf16(off, N, K, 98, std_b=2.0 * K ** -0.5)
    NC = N // 2 if gated else N
    plain = B.Layout(W.grouped_gemm_specs(g)[1])
    dA, dB, dR = dev(g.a_mk.reshape(-1)), dev(g.b_gnk.reshape(-1)), torch.from_numpy(g.group_rows).cuda()
    useL = plain
    if gated:                                              # gate and up rows interleaved, packed by axe_relayout
        useL = B.Layout(W.gated_b_spec(K, N, g.G, True))
        packed = torch.empty_like(dB)
        B.axe_relayout(plain, useL, (g.G, K, N), dB, packed)
        dB = packed
    desc = B.GroupedGemmDesc(g.M, N, K, g.G, B.Layout(W.row_major_spec(g.M, K)), useL, B.Layout(W.row_major_spec(g.M, NC)),
                             g.M * K, g.b_gnk.size, g.M * NC, epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, kernel_hint=kernel)
    out = []
    for path in (B.LIB_PATH, PARANOID):
        with library(path):
            dC = torch.zeros(g.M * NC, dtype=torch.int16, device="cuda")
            B.axe_gemm_grouped(desc, dA, dB, dC, dR)
            torch.cuda.synchronize()
            out.append(dC)
    assert torch.equal(out[0], out[1]), f"{(out[0] != out[1]).sum().item()} elements differ"


@pytest.mark.parametrize("tiles", [B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128])
@pytest.mark.parametrize("gated", [False, True])
def test_fp8_grouped_tile_kernel_fast_build_equals_checking_build(gated, tiles):
    rng = np.random.default_rng(23)
    off = np.concatenate([[0], np.cumsum(rng.integers(0, 500, 24))]).astype(np.int32)
    N, K = 1024, 768
    g = W.gemm_grouped_fp8(off, N, K, 99, scale_dtype="e8m0")
    NC = N // 2 if gated else N
    plain = B.Layout(W.grouped_gemm_specs(g)[1])
    dA, dB, dR = dev(g.a_mk.reshape(-1)), dev(g.b_gnk.reshape(-1)), torch.from_numpy(g.group_rows).cuda()
    useL = plain
    if gated:
        useL = B.Layout(W.gated_b_spec(K, N, g.G))
        packed = torch.empty_like(dB)
        B.axe_relayout(plain, useL, (g.G, K, N), dB, packed)
        dB = packed
    sa, sb = torch.from_numpy(g.scale_a).cuda(), torch.from_numpy(g.scale_b).cuda()
    desc = B.GroupedGemmDesc(g.M, N, K, g.G, B.Layout(W.row_major_spec(g.M, K)), useL, B.Layout(W.row_major_spec(g.M, NC)),
                             g.M * K, g.b_gnk.size, g.M * NC, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_BF16,
                             epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, kernel_hint=tiles,
                             scale_a=sa, scale_b=sb, scale_dtype=B.AXE_SCALE_E8M0)
    out = []
    for path in (B.LIB_PATH, PARANOID):
        with library(path):
            dC = torch.zeros(g.M * NC, dtype=torch.int16, device="cuda")
            B.axe_gemm_grouped(desc, dA, dB, dC, dR)
            torch.cuda.synchronize()
            out.append(dC)
    assert torch.equal(out[0], out[1]), f"{(out[0] != out[1]).sum().item()} elements differ"


@pytest.mark.parametrize("kernel", [B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128])
def test_grouped_pair_fast_build_equals_checking_build(kernel):
    """Both grouped GEMMs of a layer in one launch (tile-level hand-over through counters): H and C of the two builds."""
    rng = np.random.default_rng(29)
    off = np.concatenate([[0], np.cumsum(rng.integers(0, 400, 40))]).astype(np.int32)
    K1, I, N2 = 512, 384, 768
    g = W.gemm_grouped_bf16(off, 2 * I, K1, 101, std_b=2.0 * K1 ** -0.5)
    M, G = g.M, g.G
    w2 = W.to_bf16_bits(W.normal(102, (G, N2, I), I ** -0.5))
    plain1, gated1 = B.Layout(W.grouped_gemm_specs(g)[1]), B.Layout(W.gated_b_spec(K1, 2 * I, G, True))
    plain2, blocked2 = B.Layout(W.spec([(G, N2 * I, "m"), (I, 1, "m"), (N2, I, "m")])), B.Layout(W.blocked_b_spec(I, N2, G=G))
    dA, dW1, dW2, dR = dev(g.a_mk.reshape(-1)), dev(g.b_gnk.reshape(-1)), dev(w2.reshape(-1)), torch.from_numpy(g.group_rows).cuda()
    dW1p, dW2p = torch.empty_like(dW1), torch.empty_like(dW2)
    B.axe_relayout(plain1, gated1, (G, K1, 2 * I), dW1, dW1p)
    B.axe_relayout(plain2, blocked2, (G, I, N2), dW2, dW2p)
    d1 = B.GroupedGemmDesc(M, 2 * I, K1, G, B.Layout(W.row_major_spec(M, K1)), gated1, B.Layout(W.row_major_spec(M, I)),
                           M * K1, dW1.numel(), M * I, epilogue=B.AXE_EPI_SWIGLU, kernel_hint=kernel)
    d2 = B.GroupedGemmDesc(M, N2, I, G, B.Layout(W.row_major_spec(M, I)), blocked2, B.Layout(W.row_major_spec(M, N2)),
                           M * I, dW2.numel(), M * N2, kernel_hint=kernel)
    assert B.axe_gemm_grouped_pair_fused(d1, d2)
    out = []
    for path in (B.LIB_PATH, PARANOID):
        with library(path):
            dH = torch.zeros(M * I, dtype=torch.int16, device="cuda")
            dC = torch.zeros(M * N2, dtype=torch.int16, device="cuda")
            sync = torch.zeros(M + 1, dtype=torch.int32, device="cuda")
            B.axe_gemm_grouped_pair(d1, d2, dA, dW1p, dH, dW2p, dC, dR, sync)
            B.axe_gemm_grouped_pair_status(sync, M)
            out.append((dH, dC))
    assert torch.equal(out[0][0], out[1][0]) and torch.equal(out[0][1], out[1][1])
