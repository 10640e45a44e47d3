"""The C-ABI boundary without a GPU: the shared library loads, exports every symbol include/axe.h
declares, and turns malformed arguments into error codes before anything is launched."""
import ctypes as C
import os
import re

import pytest

from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def declared_functions():
    text = open(os.path.join(ROOT, "include", "axe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    return sorted(set(re.findall(r"\b(axe_[a-z_0-9]+)\s*\(", text)))


def test_library_exports_every_declared_symbol():
    L = B.lib()
    names = declared_functions()
    assert set(names) == set(B.EXPORTS)
    for n in names:
        assert getattr(L, n) is not None
    assert B.version() >= 10300
    assert b"shape" in L.axe_strerror(B.AXE_ESHAPE)


def test_probe_library_exports_what_its_header_declares():
    """libaxe_probe.so (measurement aids, loaded by the benchmark only) against include/axe_probe.h."""
    text = open(os.path.join(ROOT, "include", "axe_probe.h")).read()
    text = re.sub(r"/\*.*?\*/", "", text, flags=re.S)
    names = sorted(set(re.findall(r"\b(axe_[a-z_0-9]+)\s*\(", text)))
    assert names == ["axe_probe_mfma", "axe_probe_mfma_fragment", "axe_probe_mfma_walk", "axe_probe_stream"]
    P = C.CDLL(os.path.join(os.path.dirname(B.LIB_PATH), "libaxe_probe.so"))
    for n in names:
        assert getattr(P, n) is not None


def _eval_rc(spec, shape, n=None, axes=None):
    L = B.Layout(spec, axes)
    shp = (C.c_int64 * len(shape))(*shape)
    n = 1 if n is None else n
    # device pointers are never touched when validation fails; pass a dummy non-NULL address
    return B.lib().axe_layout_eval(C.byref(L.c), len(shape), shp, n, None, 0x1000, None)


def test_layout_eval_rejects_bad_layouts():
    ok = W.spec([(4, 1, "m")])
    assert _eval_rc(W.spec([(0, 1, "m")]), (1,)) == B.AXE_EINVAL            # extent must be > 0
    assert _eval_rc(W.spec([(-3, 1, "m")]), (1,)) == B.AXE_EINVAL
    assert _eval_rc(W.spec([(4, 0, "m")]), (4,)) == B.AXE_EINVAL            # stride must be != 0
    assert _eval_rc(W.spec([(4, 1, "m")], R=[(2, 0, "m")]), (4,)) == B.AXE_EINVAL
    assert _eval_rc(W.spec([]), (1,)) == B.AXE_EINVAL                       # n_D >= 1
    assert _eval_rc(ok, (5,)) == B.AXE_ESHAPE                               # shape not admitted
    assert _eval_rc(ok, (2, 3)) == B.AXE_ESHAPE
    assert _eval_rc(ok, (4,), n=5) == B.AXE_ERANGE                          # implicit indices beyond E_D
    assert _eval_rc(ok, (4,), n=-1) == B.AXE_EINVAL
    assert _eval_rc(W.spec([(4, 1, "m")], swizzle=("m", 3, 2, 4)), (4,)) == B.AXE_EINVAL   # base+bits > shift
    assert "swizzle" in B.lib().axe_last_error().decode()
    # axis index out of range
    L = B.Layout(ok)
    L._d[0].axis = 3
    shp = (C.c_int64 * 1)(4)
    assert B.lib().axe_layout_eval(C.byref(L.c), 1, shp, 1, None, 0x1000, None) == B.AXE_EINVAL
    # overflowing extents
    big = W.spec([(2 ** 40, 1, "m"), (2 ** 40, 1, "m")])
    assert _eval_rc(big, (1,)) == B.AXE_ERANGE
    # n = 0 is a no-op that needs no device
    assert _eval_rc(ok, (4,), n=0) == B.AXE_OK


def _relayout_rc(src, dst, shape, eb=2, s_elems=None, d_elems=None, sp=0x10000, dp=0x9000000, axes=("m", "gpuid")):
    Ls, Ld = B.Layout(src, axes), B.Layout(dst, axes)
    n = 1
    for s in shape:
        n *= s
    shp = (C.c_int64 * len(shape))(*shape)
    return B.lib().axe_relayout(C.byref(Ls.c), C.byref(Ld.c), len(shape), shp, eb, 0, sp,
                                n if s_elems is None else s_elems, dp, n if d_elems is None else d_elems, None)


def test_relayout_rejects_before_launch():
    rm = W.row_major_spec(8, 8)
    assert _relayout_rc(rm, W.row_major_spec(4, 8), (8, 8)) == B.AXE_ESHAPE
    assert _relayout_rc(rm, rm, (8, 8), eb=3) == B.AXE_EINVAL
    # destination where two logical elements share an address
    alias = W.spec([(8, 4, "m"), (8, 1, "m")])
    assert _relayout_rc(rm, alias, (8, 8)) == B.AXE_EALIAS
    # ... or a replica of one element lands on another element: element 0 writes {0, 2}, element 2 writes {2, 4}
    rep_alias = W.spec([(4, 1, "m")], R=[(2, 2, "m")])
    assert _relayout_rc(W.spec([(4, 1, "m")]), rep_alias, (4,), d_elems=6) == B.AXE_EALIAS
    # a sharded axis of extent > 1 cannot live on one GPU
    sharded = W.spec([(2, 1, "gpuid"), (4, 8, "m"), (8, 1, "m")])
    assert _relayout_rc(sharded, rm, (8, 8)) == B.AXE_EALIAS
    # addresses beyond the declared buffers
    assert _relayout_rc(rm, rm, (8, 8), d_elems=63) == B.AXE_ERANGE
    assert _relayout_rc(rm, W.spec([(8, 8, "m"), (8, 1, "m")], O={"m": -1}), (8, 8)) == B.AXE_ERANGE
    assert _relayout_rc(W.spec([(8, -8, "m"), (8, 1, "m")]), rm, (8, 8)) == B.AXE_ERANGE   # negative stride, no offset
    # overlapping / misaligned / NULL buffers
    assert _relayout_rc(rm, rm, (8, 8), sp=0x10000, dp=0x10040) == B.AXE_EINVAL
    assert _relayout_rc(rm, rm, (8, 8), sp=0x10001) == B.AXE_EINVAL
    assert _relayout_rc(rm, rm, (8, 8), sp=0) == B.AXE_EINVAL
    # swizzle on a negative coordinate
    neg = W.spec([(8, 8, "m"), (8, 1, "m")], O={"m": -64}, swizzle=("m", 1, 0, 3))
    assert _relayout_rc(rm, neg, (8, 8)) == B.AXE_ERANGE


def _gemm_desc(M=256, N=256, K=256, A=None, Bs=None, Cs=None, in_dtype=B.AXE_BF16, out_dtype=B.AXE_BF16,
               tile=B.AXE_TILE_AUTO, a_elems=None, axes=("m", "gpuid")):
    A = A or W.row_major_spec(M, K)
    Bs = Bs or W.col_major_spec(K, N)
    Cs = Cs or W.row_major_spec(M, N)
    return B.GemmDesc(M, N, K, in_dtype, out_dtype, B.Layout(A, axes), B.Layout(Bs, axes), B.Layout(Cs, axes),
                      M * K if a_elems is None else a_elems, N * K, M * N, tile_hint=tile)


def _tile_rc(desc):
    return B.lib().axe_gemm_tile(C.byref(desc.c))


def test_gemm_family_matching_and_errors():
    BIG = B.AXE_TILE_256x256x64
    # 16-bit inputs: problems of less than 5 x 2^20 elements of C go to the 64 x 64 tiles by themselves (a single
    # large tile takes longer than all the small ones together); the large tile can be asked for
    assert _tile_rc(_gemm_desc()) == B.AXE_TILE_64x64x32
    assert _tile_rc(_gemm_desc(tile=BIG)) == BIG
    assert _tile_rc(_gemm_desc(M=4096, N=4096)) == BIG
    assert _tile_rc(_gemm_desc(M=200)) == B.AXE_TILE_64x64x32
    # an fp32 output on the large tile: 16-bit inputs only, whole tiles
    assert _tile_rc(_gemm_desc(out_dtype=B.AXE_F32)) == B.AXE_TILE_64x64x32
    assert _tile_rc(_gemm_desc(out_dtype=B.AXE_F32, tile=BIG)) == BIG
    assert _tile_rc(_gemm_desc(M=4096, N=4096, out_dtype=B.AXE_F32)) == BIG
    assert _tile_rc(_gemm_desc(M=4096, N=4096, in_dtype=B.AXE_F16, out_dtype=B.AXE_F32)) == BIG
    assert _tile_rc(_gemm_desc(M=4096, N=4096, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_F32)) == B.AXE_TILE_64x64x32
    assert _tile_rc(_gemm_desc(M=4096, N=4096, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_F32, tile=BIG)) == B.AXE_EUNSUPPORTED
    assert _tile_rc(_gemm_desc(M=4000, N=4100, out_dtype=B.AXE_F32, tile=BIG)) == BIG                   # ragged edges as well
    assert _tile_rc(_gemm_desc(M=4000, N=4098, out_dtype=B.AXE_F32, tile=BIG)) == B.AXE_EUNSUPPORTED
    # 16-bit inputs: the large tile takes ragged edges (any M, N a multiple of 8) -- on request, and by itself once
    # the problem is a few tiles large; fp8 and odd N stay with whole tiles / the small tile
    assert _tile_rc(_gemm_desc(M=200, tile=B.AXE_TILE_256x256x64)) == B.AXE_TILE_256x256x64
    assert _tile_rc(_gemm_desc(M=1000, N=1000)) == B.AXE_TILE_64x64x32
    assert _tile_rc(_gemm_desc(M=3000, N=3000)) == B.AXE_TILE_256x256x64
    assert _tile_rc(_gemm_desc(M=3000, N=3000, in_dtype=B.AXE_F16, out_dtype=B.AXE_F16)) == B.AXE_TILE_256x256x64
    assert _tile_rc(_gemm_desc(M=3000, N=3001)) == B.AXE_TILE_64x64x32
    assert _tile_rc(_gemm_desc(M=3000, N=3004, tile=B.AXE_TILE_256x256x64)) == B.AXE_EUNSUPPORTED
    assert _tile_rc(_gemm_desc(M=3000, N=3000, out_dtype=B.AXE_F32)) == B.AXE_TILE_256x256x64    # fp32: N a multiple of 4
    assert _tile_rc(_gemm_desc(M=3000, N=3002, out_dtype=B.AXE_F32)) == B.AXE_TILE_64x64x32
    assert _tile_rc(_gemm_desc(M=200, in_dtype=B.AXE_FP8_E4M3, tile=B.AXE_TILE_256x256x64)) == B.AXE_EUNSUPPORTED
    assert _tile_rc(_gemm_desc(M=3000, N=3000, in_dtype=B.AXE_FP8_E4M3)) == B.AXE_TILE_64x64x32
    # the shard of a column-parallel layer: extent-1 device iter + device offset are dropped (rule D0)
    g = W.gemm_bf16(256, 512, 256, 1)
    _, Bshard, _ = W.gemm_specs(g, device_axis=True, shard=5)
    assert _tile_rc(_gemm_desc(N=512, Bs=Bshard, tile=BIG)) == BIG
    # a weight still spread over 8 GPUs is not one GPU's tensor
    spread = W.spec([(256, 1, "m"), (8, 1, "gpuid"), (64, 256, "m")])
    assert _tile_rc(_gemm_desc(N=512, Bs=spread)) == B.AXE_EALIAS
    # wrong shapes, wrong families
    assert _tile_rc(_gemm_desc(A=W.row_major_spec(256, 128))) == B.AXE_ESHAPE
    assert _tile_rc(_gemm_desc(A=W.col_major_spec(256, 256))) == B.AXE_EUNSUPPORTED     # A not K-contiguous
    assert _tile_rc(_gemm_desc(Bs=W.row_major_spec(256, 256))) == B.AXE_EUNSUPPORTED    # B not K-contiguous
    assert _tile_rc(_gemm_desc(K=250, A=W.row_major_spec(256, 250), Bs=W.col_major_spec(250, 256))) == B.AXE_EUNSUPPORTED
    assert _tile_rc(_gemm_desc(a_elems=100)) == B.AXE_ERANGE
    assert _tile_rc(_gemm_desc(in_dtype=7)) == B.AXE_EINVAL
    # fp16 inputs go with an fp16 (or fp32) output, bf16 inputs with bf16 (or fp32)
    assert _tile_rc(_gemm_desc(in_dtype=B.AXE_F16, out_dtype=B.AXE_F16, tile=BIG)) == BIG
    assert _tile_rc(_gemm_desc(in_dtype=B.AXE_F16, out_dtype=B.AXE_F32)) == B.AXE_TILE_64x64x32
    assert _tile_rc(_gemm_desc(in_dtype=B.AXE_F16, out_dtype=B.AXE_BF16)) == B.AXE_EUNSUPPORTED
    assert _tile_rc(_gemm_desc(in_dtype=B.AXE_BF16, out_dtype=B.AXE_F16)) == B.AXE_EUNSUPPORTED
    assert _tile_rc(_gemm_desc(M=0)) == B.AXE_EINVAL
    # pitched operands (leading dimension larger than the row) are in the family
    pitched = W.spec([(256, 264, "m"), (256, 1, "m")])
    assert _tile_rc(_gemm_desc(A=pitched, a_elems=256 * 264, tile=BIG)) == BIG
    # NULL device pointers are refused by axe_gemm itself
    d = _gemm_desc()
    assert B.lib().axe_gemm(C.byref(d.c), None, None, None, None) == B.AXE_EINVAL


def test_gemm_row_scaled_activations_kernel_choice():
    import numpy as np
    g = W.gemm_fp8(256, 256, 256, 3)
    As, Bs, Cs = W.gemm_specs(g)
    class FakeTensor:                                     # plan only: nothing is launched, any non-NULL pointer will do
        def data_ptr(self):
            return 4096
    def desc(rows, tile=B.AXE_TILE_AUTO, dt=B.AXE_FP8_E4M3):
        return B.GemmDesc(256, 256, 256, dt, B.AXE_BF16, B.Layout(As), B.Layout(Bs), B.Layout(Cs), 256 * 256, 256 * 256, 256 * 256,
                          FakeTensor(), FakeTensor(), tile_hint=tile, scale_a_rows=rows)
    BIG = B.AXE_TILE_256x256x64
    assert _tile_rc(desc(0, tile=BIG)) == BIG and _tile_rc(desc(128, tile=BIG)) == BIG
    assert _tile_rc(desc(0)) == B.AXE_TILE_64x64x32          # a problem this small takes the 64 x 64 tiles by itself
    assert _tile_rc(desc(1)) == B.AXE_TILE_64x64x32
    assert _tile_rc(desc(1, tile=B.AXE_TILE_256x256x64)) == B.AXE_EUNSUPPORTED      # fp32 row scales: the 64 x 64 kernel only
    assert _tile_rc(desc(64)) == B.AXE_EINVAL
    # E8M0 row codes ride on the 256 x 256 scale-path kernel when K is a multiple of 1024
    def desc_e8(K, M=2048, tile=B.AXE_TILE_AUTO):
        return B.GemmDesc(M, 2048, K, B.AXE_FP8_E4M3, B.AXE_BF16, B.Layout(W.row_major_spec(M, K)), B.Layout(W.col_major_spec(K, 2048)),
                          B.Layout(W.row_major_spec(M, 2048)), M * K, 2048 * K, M * 2048, FakeTensor(), FakeTensor(), tile_hint=tile,
                          scale_a_rows=1, scale_dtype=B.AXE_SCALE_E8M0)
    assert _tile_rc(desc_e8(2048)) == BIG and _tile_rc(desc_e8(1024, tile=BIG)) == BIG
    assert _tile_rc(desc_e8(1536)) == BIG and _tile_rc(desc_e8(768, tile=BIG)) == BIG     # any K that is a multiple of 128
    assert _tile_rc(desc_e8(1088)) == B.AXE_TILE_64x64x32 and _tile_rc(desc_e8(1088, tile=BIG)) == B.AXE_EUNSUPPORTED
    assert _tile_rc(desc_e8(2048, M=2000)) == B.AXE_TILE_64x64x32
    assert _tile_rc(desc_e8(2048, tile=B.AXE_TILE_256x224x64)) == B.AXE_EUNSUPPORTED


def test_gemm_accepts_blocked_operands():
    """Operands stored as contiguous 256 x 64 blocks (a tile product, Sec. 3.3) are in the family of the
    bf16 256 x 256 kernel; the same layouts are refused where no kernel reads them."""
    M = N = 512
    K = 256
    blkA, blkB = W.blocked_a_spec(M, K), W.blocked_b_spec(K, N)
    kw = dict(M=M, N=N, K=K)
    plainA, plainB = W.row_major_spec(M, K), W.col_major_spec(K, N)
    assert _tile_rc(_gemm_desc(A=blkA, Bs=blkB, **kw)) == B.AXE_TILE_256x256x64
    assert _tile_rc(_gemm_desc(A=plainA, Bs=blkB, **kw)) == B.AXE_TILE_256x256x64
    assert _tile_rc(_gemm_desc(A=blkA, Bs=plainB, **kw)) == B.AXE_TILE_256x256x64
    assert _tile_rc(_gemm_desc(A=blkA, Bs=blkB, tile=B.AXE_TILE_64x64x32, **kw)) == B.AXE_EUNSUPPORTED
    assert _tile_rc(_gemm_desc(A=blkA, Bs=blkB, out_dtype=B.AXE_F32, **kw)) == B.AXE_TILE_256x256x64   # fp32 output as well
    # row blocks of 128 rows are not a multiple of the tile
    r, k = W.blocked_iters(M, K, rb=128)
    assert _tile_rc(_gemm_desc(A=W.spec(r + k), Bs=plainB, **kw)) == B.AXE_EUNSUPPORTED
    # K-tiles of 32 are not the kernel's K step
    r, k = W.blocked_iters(M, K, kb=32)
    assert _tile_rc(_gemm_desc(A=W.spec(r + k), Bs=plainB, **kw)) == B.AXE_EUNSUPPORTED
    # blocked along k only (rows pitched): a legal mixture
    mixed = W.spec([(M, 64, "m"), (K // 64, M * 64, "m"), (64, 1, "m")])
    assert _tile_rc(_gemm_desc(A=mixed, Bs=plainB, **kw)) == B.AXE_TILE_256x256x64
    # grouped: blocked right-hand sides
    chk = lambda d: B.lib().axe_gemm_grouped_check(C.byref(d.c))
    assert chk(_grouped_desc(Bs=W.blocked_b_spec(256, 512, G=4))) == B.AXE_OK


def _grouped_desc(M=1000, N=512, K=256, G=4, A=None, Bs=None, Cs=None, in_dtype=B.AXE_BF16, out_dtype=B.AXE_BF16,
                  b_elems=None):
    A = A or W.row_major_spec(M, K)
    Bs = Bs or W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")])
    Cs = Cs or W.row_major_spec(M, N)
    return B.GroupedGemmDesc(M, N, K, G, B.Layout(A), B.Layout(Bs), B.Layout(Cs), M * K + 64,
                             b_elems if b_elems is not None else 2 * G * N * K, M * N + 64, in_dtype, out_dtype)


def test_grouped_gemm_family_matching_and_errors():
    chk = lambda d: B.lib().axe_gemm_grouped_check(C.byref(d.c))
    assert chk(_grouped_desc()) == B.AXE_OK
    assert chk(_grouped_desc(M=7)) == B.AXE_OK                                          # M is free: ragged groups are the point
    # contiguous groups fuse with the column digit under rule D1; the grouped form (Alg. 1) still has one iter per block
    assert chk(_grouped_desc(G=1)) == B.AXE_OK
    # pitched B: rows of K + 8, groups 64 elements apart from dense packing
    assert chk(_grouped_desc(Bs=W.spec([(4, 512 * 264 + 64, "m"), (256, 1, "m"), (512, 264, "m")]))) == B.AXE_OK
    # groups stored in two banks: no single stride between groups
    two = W.spec([(2, 10 ** 6, "m"), (2, 512 * 256, "m"), (256, 1, "m"), (512, 256, "m")])
    assert chk(_grouped_desc(Bs=two, b_elems=4 * 10 ** 6)) == B.AXE_EUNSUPPORTED
    # each B[e] row-major (unit stride along n) is outside the family
    assert chk(_grouped_desc(Bs=W.spec([(4, 512 * 256, "m"), (256, 512, "m"), (512, 1, "m")]))) == B.AXE_EUNSUPPORTED
    assert chk(_grouped_desc(N=500, Bs=W.spec([(4, 500 * 256, "m"), (256, 1, "m"), (500, 256, "m")]))) == B.AXE_EUNSUPPORTED
    assert chk(_grouped_desc(K=96, A=W.row_major_spec(1000, 96), Bs=W.spec([(4, 512 * 96, "m"), (96, 1, "m"), (512, 96, "m")]))) \
        == B.AXE_EUNSUPPORTED
    assert chk(_grouped_desc(in_dtype=B.AXE_F16, out_dtype=B.AXE_F16)) == B.AXE_OK
    assert chk(_grouped_desc(in_dtype=B.AXE_F16)) == B.AXE_EUNSUPPORTED                 # fp16 in, bf16 out
    assert chk(_grouped_desc(in_dtype=B.AXE_FP8_E4M3)) == B.AXE_OK                      # fp8 in, bf16 out: the streaming kernel
    assert chk(_grouped_desc(in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_F32)) == B.AXE_EUNSUPPORTED
    assert chk(_grouped_desc(out_dtype=B.AXE_F32)) == B.AXE_EUNSUPPORTED
    assert chk(_grouped_desc(in_dtype=9)) == B.AXE_EINVAL
    assert chk(_grouped_desc(G=0, Bs=W.spec([(1, 1, "m"), (256, 1, "m"), (512, 256, "m")]))) == B.AXE_EINVAL
    assert chk(_grouped_desc(A=W.row_major_spec(1000, 128))) == B.AXE_ESHAPE
    assert chk(_grouped_desc(b_elems=1000)) == B.AXE_ERANGE
    d = _grouped_desc()
    assert B.lib().axe_gemm_grouped(C.byref(d.c), None, None, None, None, None) == B.AXE_EINVAL


def test_grouped_gemm_gated_epilogue_needs_interleaved_gate_and_up():
    M, N, K, G = 1000, 512, 256, 4
    chk = lambda d: B.lib().axe_gemm_grouped_check(C.byref(d.c))
    def desc(Bs, Cn=N // 2, epi=B.AXE_EPI_SWIGLU):
        return B.GroupedGemmDesc(M, N, K, G, B.Layout(W.row_major_spec(M, K)), B.Layout(Bs), B.Layout(W.row_major_spec(M, Cn)),
                                 M * K, G * N * K, M * Cn, epilogue=epi)
    assert chk(desc(W.gated_b_spec(K, N, G))) == B.AXE_OK
    assert chk(desc(W.gated_b_spec(K, N, G, blocked=True))) == B.AXE_OK
    # gate and up side by side (the plain matrix) cannot feed the fused epilogue
    assert chk(desc(W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")]))) == B.AXE_EUNSUPPORTED
    # runs of 32 instead of 16
    assert chk(desc(W.spec([(G, N * K, "m"), (K, 1, "m"), (2, 32 * K, "m"), (N // 64, 64 * K, "m"), (32, K, "m")]))) == B.AXE_EUNSUPPORTED
    # C must be N / 2 wide
    assert chk(desc(W.gated_b_spec(K, N, G), Cn=N)) == B.AXE_ESHAPE
    assert chk(desc(W.gated_b_spec(K, N, G), epi=7)) == B.AXE_EINVAL
    # without the epilogue the interleaved layout is just a permutation of columns nobody asked for
    assert chk(desc(W.gated_b_spec(K, N, G), Cn=N, epi=B.AXE_EPI_NONE)) == B.AXE_EUNSUPPORTED


def test_grouped_pair_checks_and_choice():
    """axe_gemm_grouped_pair: the second problem must read exactly what the first writes; which pairs share a launch."""
    fused = lambda a, b: B.lib().axe_gemm_grouped_pair_fused(C.byref(a.c), C.byref(b.c))
    def pair(M=4000, K1=512, I=256, N2=512, G=8, dt=B.AXE_BF16, hint=B.AXE_GROUPED_TILES, M2=None, K2=None, G2=None, dt2=None, a2_pitch=None,
             epi=B.AXE_EPI_SWIGLU, h_pitch=None):
        M2, K2, G2, dt2 = M2 or M, K2 or I, G2 or G, dt2 or dt
        N1 = 2 * I if epi == B.AXE_EPI_SWIGLU else I
        b1 = W.gated_b_spec(K1, N1, G, True) if epi == B.AXE_EPI_SWIGLU else W.blocked_b_spec(K1, N1, G=G)
        a2_pitch = a2_pitch or h_pitch
        c1 = W.row_major_spec(M, I) if h_pitch is None else W.spec([(M, h_pitch, "m"), (I, 1, "m")])
        d1 = B.GroupedGemmDesc(M, N1, K1, G, B.Layout(W.row_major_spec(M, K1)), B.Layout(b1),
                               B.Layout(c1), M * K1, G * N1 * K1, M * (h_pitch or I), in_dtype=dt, out_dtype=dt,
                               epilogue=epi, kernel_hint=hint)
        a2 = W.row_major_spec(M2, K2) if a2_pitch is None else W.spec([(M2, a2_pitch, "m"), (K2, 1, "m")])
        d2 = B.GroupedGemmDesc(M2, N2, K2, G2, B.Layout(a2), B.Layout(W.blocked_b_spec(K2, N2, G=G2)),
                               B.Layout(W.row_major_spec(M2, N2)), M2 * (a2_pitch or K2), G2 * N2 * K2, M2 * N2, in_dtype=dt2, out_dtype=dt2,
                               kernel_hint=hint)
        return d1, d2
    assert fused(*pair()) == 1
    assert fused(*pair(dt=B.AXE_F16)) == 1
    assert fused(*pair(hint=B.AXE_GROUPED_TILES_128)) == 1 and fused(*pair(hint=B.AXE_GROUPED_TILES_256)) == 1
    # not one launch: the streaming kernel on either side, fewer than four or an odd number of K-steps, an ungated first
    # problem, more tiles than one workgroup per compute unit can hold (64 each)
    assert fused(*pair(M=32, hint=B.AXE_GROUPED_AUTO)) == 0
    assert fused(*pair(I=128)) == 0
    assert fused(*pair(K1=320)) == 0
    assert fused(*pair(epi=B.AXE_EPI_NONE)) == 0
    assert fused(*pair(h_pitch=320)) == 1 and fused(*pair(h_pitch=264)) == 0          # rows of H on 128-byte lines, or not
    assert fused(*pair(M=256 * 2000, N2=2048, hint=B.AXE_GROUPED_TILES_128)) == 0
    # the second problem's A is not the first problem's C
    assert fused(*pair(M2=4096)) == B.AXE_EINVAL
    assert fused(*pair(K2=512)) == B.AXE_EINVAL
    assert fused(*pair(G2=4)) == B.AXE_EINVAL
    assert fused(*pair(dt2=B.AXE_F16)) == B.AXE_EINVAL
    assert fused(*pair(a2_pitch=264)) == B.AXE_EINVAL
    # errors of either problem come through
    d1, d2 = pair()
    L = B.lib()
    d2.c.kernel_hint = 77
    assert fused(d1, d2) == L.axe_gemm_grouped_check(C.byref(d2.c)) == B.AXE_EINVAL
    d1, d2 = pair()
    assert L.axe_gemm_grouped_pair(C.byref(d1.c), C.byref(d2.c), None, None, None, None, None, None, None, 0, None) == B.AXE_EINVAL
    # aliasing (refused before anything is launched; the addresses are placeholders): H and C disjoint from each
    # other and from every input, the workspace disjoint from all of them
    far = {k: (i + 1) << 32 for i, k in enumerate(["A", "B1", "H", "B2", "C", "rows", "sync"])}
    def call(**kw):
        a = {**far, **kw}
        return L.axe_gemm_grouped_pair(C.byref(d1.c), C.byref(d2.c), a["A"], a["B1"], a["H"], a["B2"], a["C"], a["rows"], a["sync"],
                                       d1.c.M + 1, None)
    assert call(C=far["H"]) == B.AXE_EINVAL and call(C=far["A"]) == B.AXE_EINVAL and call(C=far["B1"] + 64) == B.AXE_EINVAL
    assert call(H=far["B2"]) == B.AXE_EINVAL and call(H=far["rows"] - 16) == B.AXE_EINVAL
    assert call(sync=far["C"] + 1024) == B.AXE_EINVAL and call(sync=far["A"]) == B.AXE_EINVAL
    assert "overlap" in L.axe_last_error().decode()
    assert L.axe_gemm_grouped_pair(C.byref(d1.c), C.byref(d2.c), far["A"], far["B1"], far["H"], far["B2"], far["C"], far["rows"],
                                   far["sync"], d1.c.M, None) == B.AXE_EINVAL                       # workspace one word short
    assert L.axe_gemm_grouped_pair_status(None, 0, None) == B.AXE_EINVAL
    assert L.axe_gemm_grouped_pair_status(None, (1 << 20) + 1, None) == B.AXE_EINVAL     # beyond the library's own workspace
    big = pair(M=(1 << 20) + 8)
    assert L.axe_gemm_grouped_pair_static(C.byref(big[0].c), C.byref(big[1].c), None, None, None, None, None, None, None) == B.AXE_EUNSUPPORTED


def test_grouped_gemm_fp8_goes_to_the_streaming_kernel_only():
    class Fake:
        def data_ptr(self):
            return 4096
    chk = lambda d: B.lib().axe_gemm_grouped_check(C.byref(d.c))
    def desc(M=100, N=512, K=256, G=64, hint=B.AXE_GROUPED_AUTO, scales=True, out=B.AXE_BF16, Bs=None, sd=B.AXE_SCALE_F32):
        Bs = Bs or W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")])
        return B.GroupedGemmDesc(M, N, K, G, B.Layout(W.row_major_spec(M, K)), B.Layout(Bs), B.Layout(W.row_major_spec(M, N)),
                                 M * K, G * N * K, M * N, in_dtype=B.AXE_FP8_E4M3, out_dtype=out, kernel_hint=hint,
                                 scale_a=Fake() if scales else None, scale_b=Fake() if scales else None, scale_dtype=sd)
    assert chk(desc()) == B.AXE_OK and chk(desc(scales=False)) == B.AXE_OK and chk(desc(sd=B.AXE_SCALE_E8M0)) == B.AXE_OK
    assert chk(desc(M=4000)) == B.AXE_OK                                                  # large groups stream too (in passes of 64 rows)
    assert chk(desc(M=4000, hint=B.AXE_GROUPED_STREAM)) == B.AXE_OK
    assert chk(desc(hint=B.AXE_GROUPED_TILES)) == B.AXE_EUNSUPPORTED                       # fp32 scales: no tile kernel
    for hint in (B.AXE_GROUPED_TILES, B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128):   # E8M0 scales or none: tiles of either height
        assert chk(desc(hint=hint, sd=B.AXE_SCALE_E8M0)) == B.AXE_OK and chk(desc(hint=hint, scales=False)) == B.AXE_OK
    assert chk(desc(K=192, Bs=W.spec([(64, 512 * 192, "m"), (192, 1, "m"), (512, 192, "m")]))) == B.AXE_EUNSUPPORTED   # K no multiple of 128
    assert chk(desc(out=B.AXE_F16)) == B.AXE_EUNSUPPORTED
    assert chk(desc(sd=5)) == B.AXE_EINVAL
    d = desc()
    d.c.d_scale_b = None
    assert chk(d) == B.AXE_EINVAL                                                          # scales come in pairs
    bf = B.GroupedGemmDesc(100, 512, 256, 64, B.Layout(W.row_major_spec(100, 256)), B.Layout(W.spec([(64, 512 * 256, "m"), (256, 1, "m"), (512, 256, "m")])),
                           B.Layout(W.row_major_spec(100, 512)), 100 * 256, 64 * 512 * 256, 100 * 512, scale_a=Fake(), scale_b=Fake())
    assert chk(bf) == B.AXE_EINVAL                                                         # scales with bf16 inputs


def test_python_binding_raises_axe_error():
    with pytest.raises(B.AxeError) as e:
        B._check(B.AXE_EALIAS)
    assert e.value.code == B.AXE_EALIAS


C_PROGRAM = r"""
#include "axe.h"
#include "axe_probe.h"
#include <stdio.h>
int main(void) {
  axe_iter_t d[2] = {{4, 8, 0}, {8, 1, 0}};
  const char* names[1] = {"m"};
  int64_t off[1] = {3};
  int64_t span[1];
  axe_layout_t L;
  L.n_axes = 1; L.axis_names = names; L.n_d = 2; L.d = d; L.n_r = 0; L.r = 0; L.offset = off;
  L.swz_axis = -1; L.swz_bits = 0; L.swz_base = 0; L.swz_shift = 0;
  if (axe_layout_span(&L, span) != AXE_OK) return 1;                 /* (4, 8)(8, 1): 1 + 3 * 8 + 7 * 1 */
  if (axe_relayout(&L, &L, 1, 0, 2, 0, 0, 0, 0, 0, 0) == AXE_OK) return 3;   /* NULL arguments are refused, nothing is launched */
  printf("%d %lld %s\n", (int)axe_version(), (long long)span[0], axe_strerror(AXE_ETIMEOUT));
  return span[0] == 32 ? 0 : 2;
}
"""


@pytest.mark.parametrize("compiler,std", [("gcc", "-std=c99"), ("g++", "-std=c++11")])
def test_headers_are_plain_c_and_a_c_program_links_against_the_library(tmp_path, compiler, std):
    """The boundary is a C ABI: include/*.h compile as strict C99 (and as C++) without warnings, and a program with no
    Python and no torch in it links against the shared library and calls it."""
    import subprocess
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    libdir = os.path.dirname(B.LIB_PATH)
    src = tmp_path / ("prog.c" if compiler == "gcc" else "prog.cpp")
    src.write_text(C_PROGRAM)
    exe = tmp_path / "prog"
    subprocess.check_call([compiler, std, "-pedantic", "-Wall", "-Wextra", "-Werror", "-I", os.path.join(root, "include"), str(src), "-o",
                           str(exe), "-L", libdir, "-laxe_hip", "-Wl,-rpath," + libdir])
    out = subprocess.run([str(exe)], capture_output=True, text=True)
    assert out.returncode == 0, out.stdout + out.stderr
    version, span, msg = out.stdout.split(None, 2)
    assert int(version) == B.lib().axe_version() and int(span) == 32 and "wait" in msg
