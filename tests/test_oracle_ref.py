"""Pins for the array side of the oracle (relayout, number formats, GEMM).  CPU only.

Each pin comes from something other than the function under test: NumPy reshape/transpose for
the blocked layout, torch's dtype views for the number formats, BLAS fp64 matmul and hand
arithmetic for the GEMM, brute force for the block-scaled form."""
import itertools
from math import prod

import numpy as np
import pytest
import torch

from oracle import axe_layout as ax
from oracle import axe_ref as R
from oracle.axe_layout import Layout, Swizzle
from paper_2601_19092_amd import workloads as W


# ----------------------------------------------------------------------------- relayout
def blocked_by_numpy(src2d: np.ndarray, tr=128, tc=64, swizzle=True) -> np.ndarray:
    """The destination image derived without the evaluator: reshape to
    [tile-row, r, tile-col, chunk, e], move tile-col outward, XOR the chunk index with r & 7."""
    rows, cols = src2d.shape
    v = src2d.reshape(rows // tr, tr, cols // tc, tc // 8, 8).transpose(0, 2, 1, 3, 4).copy()
    if swizzle:
        out = np.empty_like(v)
        r = np.arange(tr)
        for c in range(tc // 8):
            out[:, :, r, c ^ (r & 7), :] = v[:, :, r, c, :]
        v = out
    return v.reshape(-1)


@pytest.mark.parametrize("rows,cols", [(128, 64), (256, 192), (1024, 512)])
@pytest.mark.parametrize("kind", ["uniform", "index"])
def test_blocked_swizzled_relayout_matches_numpy_closed_form(rows, cols, kind):
    words = W.relayout_words(rows, cols, 7, kind)
    src_L = Layout.from_spec(W.row_major_spec(rows, cols))
    dst_L = Layout.from_spec(W.blocked_swizzled_spec(rows, cols))
    dst = np.full(rows * cols, 0xDEAD, dtype=np.uint16)
    R.relayout_ref(src_L, dst_L, (rows, cols), words.reshape(-1), dst)
    assert np.array_equal(dst, blocked_by_numpy(words))
    # round trip restores the source bit for bit
    back = np.zeros(rows * cols, dtype=np.uint16)
    R.relayout_ref(dst_L, src_L, (rows, cols), dst, back)
    assert np.array_equal(back, words.reshape(-1))


def test_blocked_spec_is_tile_of_grid_and_tile():
    # the literal strides in the workload description equal (grid) (x) (tile) built by the oracle
    for rows, cols in ((256, 192), (8192, 8192)):
        grid = ax.row_major((rows // 128, cols // 64))
        tile_ = ax.row_major((128, 64))
        T, ST = ax.tile(grid, (rows // 128, cols // 64), tile_, (128, 64))
        spec = Layout.from_spec(W.blocked_swizzled_spec(rows, cols, swizzle=False))
        assert T.D == spec.D and ST == (rows // 128, 128, cols // 64, 64)
    full = Layout.from_spec(W.blocked_swizzled_spec(8192, 8192))
    assert [(i.extent, i.stride) for i in full.D] == [(64, 1048576), (128, 64), (128, 8192), (64, 1)]
    assert full.swizzle == Swizzle("m", 3, 3, 6)


def test_blocked_destination_is_a_permutation():
    rows, cols = 512, 256
    L = Layout.from_spec(W.blocked_swizzled_spec(rows, cols))
    addr = R.evaluate_np(L, np.arange(rows * cols), ["m"])[:, 0, 0]
    assert np.array_equal(np.sort(addr), np.arange(rows * cols))
    # tile bases are multiples of 512 elements, so the swizzle acts inside each tile
    plain = R.evaluate_np(L.with_(swizzle=None), np.arange(rows * cols), ["m"])[:, 0, 0]
    assert np.array_equal(addr // 512, plain // 512)


def test_relayout_identity_composition_and_replicas():
    rng = np.random.default_rng(5)
    shape = (6, 4, 5)
    n = prod(shape)
    src = rng.integers(0, 2 ** 32, n, dtype=np.uint32)
    A = ax.row_major(shape)
    B = Layout.make(shape, (1, 6, 24))                        # column-major
    C = Layout.make((6, 4, 5), (5, 30, 1))                    # a permuted-axes layout
    # L -> L is a memcpy
    out = np.zeros(n, dtype=np.uint32)
    assert np.array_equal(R.relayout_ref(A, A, shape, src, out), src)
    # A -> B equals numpy's transpose to Fortran order
    ab = R.relayout_ref(A, B, shape, src, np.zeros(n, dtype=np.uint32)).copy()
    assert np.array_equal(ab, src.reshape(shape).ravel(order="F"))
    # A -> B -> A is the identity; (A -> B) then (B -> C) equals A -> C
    assert np.array_equal(R.relayout_ref(B, A, shape, ab, np.zeros(n, dtype=np.uint32)), src)
    bc = R.relayout_ref(B, C, shape, ab, np.zeros(n, dtype=np.uint32))
    ac = R.relayout_ref(A, C, shape, src, np.zeros(n, dtype=np.uint32))
    assert np.array_equal(bc, ac)
    # replicated destination: every replica is written; untouched words keep their contents
    D = Layout.make((4, 3), (3, 1), R=((2,), (20,)), O={"m": 2})
    dst = np.full(40, 99, dtype=np.uint32)
    R.relayout_ref(ax.row_major((4, 3)), D, (4, 3), src[:12], dst)
    want = np.full(40, 99, dtype=np.uint32)
    want[2:14] = src[:12]
    want[22:34] = src[:12]
    assert np.array_equal(dst, want)
    # out-of-buffer addresses are errors, not silent wraps
    with pytest.raises(IndexError):
        R.relayout_ref(ax.row_major((4, 3)), D, (4, 3), src[:12], np.zeros(30, dtype=np.uint32))


def test_relayout_ignores_non_memory_axes_of_one_device():
    # the shard of config 4: an extent-1 device iter and a device offset do not move any address
    g = W.gemm_bf16(8, 6, 4, 1)
    _, Bspec, _ = W.gemm_specs(g, device_axis=True, shard=5)
    Lb = Layout.from_spec(Bspec)
    plain = Layout.from_spec(W.col_major_spec(4, 6))
    xs = np.arange(24)
    assert np.array_equal(R.evaluate_np(Lb, xs, ["m", "gpuid"])[:, 0, 0], R.evaluate_np(plain, xs, ["m"])[:, 0, 0])
    assert set(R.evaluate_np(Lb, xs, ["m", "gpuid"])[:, 0, 1]) == {5}
    assert ax.canon_D(Lb.D) == ax.canon_D(plain.D)


# ----------------------------------------------------------------------------- number formats
def test_bf16_decode_matches_torch_for_all_codes():
    codes = np.arange(65536, dtype=np.uint16)
    want = torch.from_numpy(codes.view(np.int16).copy()).view(torch.bfloat16).to(torch.float64).numpy()
    got = R.bf16_to_f64(codes)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert got[0x3F80] == 1.0 and got[0xC000] == -2.0 and got[0x3DCD] == pytest.approx(0.1, rel=4e-3)


def test_f16_decode_matches_numpy_for_all_codes_in_python_and_c():
    codes = np.arange(65536, dtype=np.uint16)
    want = codes.view(np.float16).astype(np.float64)
    got = R.f16_to_f64(codes)
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok]) and np.array_equal(np.signbit(got[ok]), np.signbit(want[ok]))
    # format facts: largest finite value, smallest subnormal, one
    assert R.f16_to_f64(np.array([0x7BFF, 0x0001, 0x3C00], dtype=np.uint16)).tolist() == [65504.0, 2.0 ** -24, 1.0]
    # the C decoder: a 1 x K by K x 1 product with b = 1 sums the decoded values of a
    fin = codes[np.isfinite(want)]
    for chunk in np.array_split(fin, 64):
        a = chunk.reshape(1, -1)
        ones = np.full((a.shape[1], 1), 0x3C00, dtype=np.uint16)
        assert R.gemm_ref(a, ones, R.AXE_F16)[0, 0] == np.sum(want[chunk.astype(np.int64)], dtype=np.float64)
    # single codes, so that no two decoding mistakes can cancel in a sum
    for c in (0x0001, 0x03FF, 0x0400, 0x3555, 0x7BFF, 0x8001, 0xC000, 0xFBFF):
        one = np.array([[c]], dtype=np.uint16)
        assert R.gemm_ref(one, np.array([[0x3C00]], dtype=np.uint16), R.AXE_F16)[0, 0] == want[c]
    # RNE cast of the generator: ties go to the even code
    assert W.to_f16_bits(np.array([1.0 + 2.0 ** -11, 1.0 + 3 * 2.0 ** -11], dtype=np.float32)).tolist() == [0x3C00, 0x3C02]


def test_e4m3_decode_matches_torch_and_format_facts():
    codes = np.arange(256, dtype=np.uint8)
    want = torch.from_numpy(codes.copy()).view(torch.float8_e4m3fn).to(torch.float64).numpy()
    got = R.e4m3_table()
    assert np.array_equal(np.isnan(got), np.isnan(want))
    ok = ~np.isnan(want)
    assert np.array_equal(got[ok], want[ok])
    assert list(np.where(np.isnan(got))[0]) == [0x7F, 0xFF]
    assert np.nanmax(got) == 448.0 and got[0x7E] == 448.0 and got[0x01] == 2.0 ** -9 and got[0x38] == 1.0
    assert not np.isinf(got).any()


def test_e8m0_decode_format_facts():
    """E8M0 (OCP microscaling): value 2^(code - 127), bias 127, 255 is NaN, no zero, no sign; torch's
    float8_e8m0fnu view, where this build of torch has it, must agree on every code."""
    v = R.e8m0_decode(np.arange(256, dtype=np.uint8))
    assert v[127] == 1.0 and v[128] == 2.0 and v[126] == 0.5 and v[0] == 2.0 ** -127 and v[254] == 2.0 ** 127
    assert np.isnan(v[255]) and np.all(v[:255] > 0)
    assert np.all(v[1:255] == 2.0 * v[0:254])                       # each code doubles the one before
    assert np.array_equal(v[1:255].astype(np.float32).astype(np.float64), v[1:255])     # exact in fp32 (normal numbers)
    import torch
    if hasattr(torch, "float8_e8m0fnu"):
        t = torch.arange(256, dtype=torch.uint8).view(torch.float8_e8m0fnu).to(torch.float64).numpy()
        assert np.array_equal(np.isnan(t), np.isnan(v)) and np.array_equal(t[:255], v[:255])
    # a GEMM with E8M0 scales is the fp32-scaled GEMM on the decoded scales
    g = W.gemm_fp8(128, 256, 384, 5, scaled="e8m0")
    assert g.scale_a.dtype == np.uint8 and g.scale_a.min() >= 124 and g.scale_a.max() <= 130
    sa, sb = R.e8m0_decode(g.scale_a).astype(np.float32), R.e8m0_decode(g.scale_b).astype(np.float32)
    c = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, sa, sb)
    want = R.gemm_ref_numpy(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, sa, sb)
    assert np.allclose(c, want, rtol=1e-12, atol=1e-12)
    # power-of-two scales commute with rounding: scaling the block sums equals scaling the decoded inputs
    A, Bm = R.decode(g.a_mk, R.AXE_FP8_E4M3), R.decode(g.b_nk, R.AXE_FP8_E4M3)
    As = A * np.repeat(np.repeat(sa.astype(np.float64), 128, 0), 128, 1)[:128, :384]
    Bs = Bm * np.repeat(np.repeat(sb.astype(np.float64), 128, 0), 128, 1)[:256, :384]
    assert np.allclose(As @ Bs.T, c, rtol=1e-12, atol=1e-12)


def test_input_quantisation_is_round_to_nearest_even():
    x = W.normal(3, (4096,), 1.0)
    # bf16: decoded value is the nearest representable; spacing is 2^-7 relative at most
    d = R.bf16_to_f64(W.to_bf16_bits(x))
    assert np.all(np.abs(d - x) <= np.abs(x.astype(np.float64)) * 2.0 ** -8)
    assert R.bf16_to_f64(W.to_bf16_bits(np.array([1.0 + 2.0 ** -8], np.float32)))[0] == 1.0            # tie -> even
    assert R.bf16_to_f64(W.to_bf16_bits(np.array([1.0 + 3 * 2.0 ** -8], np.float32)))[0] == 1.0 + 2.0 ** -6
    # e4m3: nearest of the 254 finite codes, ties to even mantissa, clip at 448
    table = R.e4m3_table()
    finite = np.sort(table[~np.isnan(table)])
    e = R.e4m3_to_f64(W.to_e4m3_bits(x * 3))
    nearest = np.min(np.abs(finite[None, :] - (x * 3).astype(np.float64)[:, None]), axis=1)
    assert np.allclose(np.abs(e - (x * 3).astype(np.float64)), nearest, rtol=0, atol=0)
    assert list(R.e4m3_to_f64(W.to_e4m3_bits(np.array([1000.0, -1000.0, 1.0625, 1.1875], np.float32)))) == [448.0, -448.0, 1.0, 1.25]


# ----------------------------------------------------------------------------- GEMM
def test_gemm_hand_case():
    # exact small integers: A = [[1,2],[3,4],[5,6]] (3x2), B = [[1,0,2,-1],[0.5,1,0,4]] (2x4)
    a = W.to_bf16_bits(np.array([[1, 2], [3, 4], [5, 6]], np.float32))
    b_kn = np.array([[1, 0, 2, -1], [0.5, 1, 0, 4]], np.float32)
    b = W.to_bf16_bits(b_kn.T.copy())            # memory image (N, K)
    want = np.array([[2, 2, 2, 7], [5, 4, 6, 13], [8, 6, 10, 19]], np.float64)
    assert np.array_equal(R.gemm_ref(a, b.T, R.AXE_BF16), want)
    assert np.array_equal(R.gemm_ref_numpy(a, b.T, R.AXE_BF16), want)


@pytest.mark.parametrize("M,N,K", [(33, 17, 65), (128, 96, 256), (200, 120, 512)])
def test_gemm_c_loop_agrees_with_blas_fp64(M, N, K):
    g = W.gemm_bf16(M, N, K, 11)
    c = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_BF16)
    blas = R.bf16_to_f64(g.a_mk) @ R.bf16_to_f64(g.b_nk).T
    assert R.rel_frobenius(c, blas) <= 1e-12
    assert np.max(np.abs(c - blas)) <= 1e-11 * np.max(np.abs(blas))
    # a row/column subset is the same numbers
    rows, cols = np.array([0, 5, M - 1]), np.array([N - 1, 2])
    assert np.array_equal(R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_BF16, rows=rows, cols=cols), c[np.ix_(rows, cols)])


def test_gemm_identity_returns_b_exactly():
    K = N = 64
    g = W.gemm_bf16(K, N, K, 12)
    eye = W.to_bf16_bits(np.eye(K, dtype=np.float32))
    c = R.gemm_ref(eye, g.b_nk.T, R.AXE_BF16)
    assert np.array_equal(c, R.bf16_to_f64(g.b_nk).T)


def test_gemm_fp8_scaled_form():
    M, N, K = 256, 384, 512
    g = W.gemm_fp8(M, N, K, 13)
    c = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, g.scale_a, g.scale_b)
    A = R.e4m3_to_f64(g.a_mk)
    B = R.e4m3_to_f64(g.b_nk).T
    # brute force from the definition, block by block, with numpy fp64
    want = np.zeros((M, N))
    for ib, jb, kb in itertools.product(range(M // 128), range(N // 128), range(K // 128)):
        blk = A[ib * 128:(ib + 1) * 128, kb * 128:(kb + 1) * 128] @ B[kb * 128:(kb + 1) * 128, jb * 128:(jb + 1) * 128]
        want[ib * 128:(ib + 1) * 128, jb * 128:(jb + 1) * 128] += float(g.scale_a[ib, kb]) * float(g.scale_b[jb, kb]) * blk
    assert R.rel_frobenius(c, want) <= 1e-12
    assert R.rel_frobenius(R.gemm_ref_numpy(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, g.scale_a, g.scale_b), want) <= 1e-12
    # all scales = 1 reduces to the unscaled GEMM; a scale that is wrong for one block is seen
    one_a, one_b = np.ones_like(g.scale_a), np.ones_like(g.scale_b)
    c1 = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, one_a, one_b)
    assert R.rel_frobenius(c1, A @ B) <= 1e-12
    bad = g.scale_a.copy()
    bad[1, 2] *= 2
    cb = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, bad, g.scale_b)
    assert R.rel_frobenius(cb[128:], want[128:]) > 1e-2 and np.array_equal(cb[:128], c[:128])
    # swapping which scale table indexes rows and which columns is seen (M != N)
    assert g.scale_a.shape != g.scale_b.shape


def test_gemm_fp8_row_scaled_activations():
    """One scale per row of A and 128-wide k block (weights keep 128 x 128 blocks): brute force from the
    definition; repeating a block's scale over its 128 rows gives back the block-scaled form."""
    M, N, K = 130, 256, 384
    g = W.gemm_fp8(M, N, K, 14)
    rng = np.random.default_rng(2)
    sa_rows = rng.uniform(0.5, 2.0, (M, K // 128)).astype(np.float32)
    A, Bm = R.e4m3_to_f64(g.a_mk), R.e4m3_to_f64(g.b_nk).T
    want = np.zeros((M, N))
    for i in range(M):
        for kb in range(K // 128):
            ks = slice(kb * 128, (kb + 1) * 128)
            want[i] += float(sa_rows[i, kb]) * (A[i, ks] @ Bm[ks]) * np.repeat(g.scale_b[:, kb].astype(np.float64), 128)[:N]
    c = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, sa_rows, g.scale_b, block_m_a=1)
    assert R.rel_frobenius(c, want) <= 1e-12
    assert R.rel_frobenius(R.gemm_ref_numpy(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, sa_rows, g.scale_b, block_m_a=1), want) <= 1e-12
    rep = np.repeat(g.scale_a, 128, axis=0)[:M]
    np.testing.assert_array_equal(R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, rep, g.scale_b, block_m_a=1),
                                  R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, g.scale_a, g.scale_b))
    # one row's scale changed: that row changes, no other
    bad = sa_rows.copy()
    bad[77, 1] *= 2
    cb = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, bad, g.scale_b, block_m_a=1)
    assert np.array_equal(np.delete(cb, 77, axis=0), np.delete(c, 77, axis=0)) and R.rel_frobenius(cb[77], c[77]) > 1e-2
    with pytest.raises(ValueError):
        R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, g.scale_a, g.scale_b, block_m_a=1)      # wrong shape for per-row scales


def test_gemm_operand_orientation_is_checked_by_shape():
    # K-contiguous B handed over as (K, N) view: a transposed operand changes the result
    g = W.gemm_bf16(8, 8, 8, 14)
    c = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_BF16)
    wrong = R.gemm_ref(g.a_mk, g.b_nk, R.AXE_BF16)
    assert R.rel_frobenius(wrong, c) > 0.1
    with pytest.raises(ValueError):
        R.gemm_ref(g.a_mk, g.b_nk[:4].T[:3], R.AXE_BF16)


def test_workload_seeds_and_statistics():
    g1 = W.config1()
    assert (g1.M, g1.N, g1.K, g1.out_dtype) == (256, 256, 256, "f32")
    assert np.array_equal(g1.a_mk, W.config1().a_mk)                     # reproducible
    a = R.bf16_to_f64(g1.a_mk)
    assert abs(a.mean()) < 0.02 and abs(a.std() - 1.0) < 0.02
    g3 = W.config3(256, 128, 1024)
    assert abs(R.bf16_to_f64(g3.a_mk).std() - 1024 ** -0.5) < 1e-3
    g4 = W.config4(128, 64, 256)
    assert abs(R.bf16_to_f64(g4.b_nk).std() - 0.02) < 1e-3
    g5 = W.config5(256, 256, 256)
    assert g5.scale_a.min() >= 0.5 and g5.scale_a.max() <= 2.0 and g5.scale_a.dtype == np.float32
    v = R.e4m3_to_f64(g5.a_mk)
    assert not np.isnan(v).any() and np.abs(v).max() <= 448
    w = W.config2("uniform", 128, 64)
    assert np.abs(R.bf16_to_f64(w)).max() <= 1.0
    idx = W.config2("index", 128, 64)
    assert idx[0, 1] == 40503 and idx[1, 0] == (64 * 40503) % 65536


# ----------------------------------------------------------------------------- grouped GEMM (MoE)
def _grouped_case(seed, off, N, K, M=None):
    g = W.gemm_grouped_bf16(off, N, K, seed, M=M)
    return g, g.a_mk, g.b_gnk.transpose(0, 2, 1)          # logical (G, K, N) view of the (G, N, K) image


def test_grouped_gemm_equals_block_diagonal_dense_product():
    """Independent construction: place group g's rows of A in column block g of a (M, G K) matrix and
    stack the B[g] vertically; one dense fp64 product (BLAS) then is the grouped GEMM."""
    off = [0, 5, 5, 19, 40]                              # an empty group, ragged sizes
    g, a, b = _grouped_case(3, off, N=24, K=32)
    A = R.decode(a, R.AXE_BF16)
    B = R.decode(np.ascontiguousarray(b), R.AXE_BF16)
    G, K, N = B.shape
    wide = np.zeros((g.M, G * K))
    for e in range(G):
        wide[off[e]:off[e + 1], e * K:(e + 1) * K] = A[off[e]:off[e + 1]]
    want = wide @ B.reshape(G * K, N)
    got = R.gemm_grouped_ref(a, b, off, R.AXE_BF16)
    assert not np.isnan(got).any()
    np.testing.assert_allclose(got, want, rtol=1e-12, atol=1e-12)


def test_grouped_gemm_brute_force_and_undefined_rows():
    off = [2, 3, 7]                                      # rows 0, 1 and 7.. belong to no group
    g, a, b = _grouped_case(4, off, N=5, K=16, M=9)
    A = R.decode(a, R.AXE_BF16)
    B = R.decode(np.ascontiguousarray(b), R.AXE_BF16)
    got = R.gemm_grouped_ref(a, b, off, R.AXE_BF16)
    for r in range(9):
        owner = [e for e in range(2) if off[e] <= r < off[e + 1]]
        for j in range(5):
            if not owner:
                assert np.isnan(got[r, j])
            else:
                want = sum(A[r, k] * B[owner[0], k, j] for k in range(16))
                assert abs(got[r, j] - want) <= 1e-12 * max(1.0, abs(want))


def test_grouped_gemm_special_cases():
    # one group = the plain GEMM; sampled rows / columns = the same entries of the full result
    g, a, b = _grouped_case(5, [0, 33], N=17, K=48)
    full = R.gemm_grouped_ref(a, b, [0, 33], R.AXE_BF16)
    np.testing.assert_array_equal(full, R.gemm_ref(a, b[0], R.AXE_BF16))
    rows, cols = np.array([32, 0, 7]), np.array([16, 3])
    np.testing.assert_array_equal(R.gemm_grouped_ref(a, b, [0, 33], R.AXE_BF16, rows=rows, cols=cols), full[np.ix_(rows, cols)])
    # swapping two groups (rows and right-hand sides together) swaps their output rows
    off = [0, 4, 10]
    g, a, b = _grouped_case(6, off, N=8, K=16)
    c = R.gemm_grouped_ref(a, b, off, R.AXE_BF16)
    a2 = np.concatenate([a[4:10], a[0:4]])
    c2 = R.gemm_grouped_ref(a2, b[::-1], [0, 6, 10], R.AXE_BF16)
    np.testing.assert_array_equal(c2, np.concatenate([c[4:10], c[0:4]]))
    with pytest.raises(ValueError):
        R.gemm_grouped_ref(a, b, [0, 11, 10], R.AXE_BF16)


def test_moe_routing_recipe():
    """tokens x topk rows in all, every token in topk distinct experts, fixed by the seed."""
    off = W.moe_group_rows(512, 128, 8, W.SEED_BASE)
    assert off.dtype == np.int32 and off.size == 129 and off[0] == 0 and off[-1] == 512 * 8
    assert (np.diff(off) >= 0).all() and np.diff(off).max() <= 512          # an expert sees a token at most once
    np.testing.assert_array_equal(off, W.moe_group_rows(512, 128, 8, W.SEED_BASE))
    assert (W.moe_group_rows(512, 128, 8, W.SEED_BASE + 1) != off).any()
    g1, g2 = W.moe_gemm1(64), W.moe_gemm2(64)
    assert (g1.M, g1.N, g1.K, g1.G) == (512, 1536, 2048, 128) and (g2.N, g2.K) == (2048, 768)
    np.testing.assert_array_equal(g1.group_rows, g2.group_rows)


def test_swiglu_closed_forms_and_library_routine():
    x = np.array([[0.0, 1.0, -1.0, 30.0, -30.0, -800.0, 2.0, 3.0, 5.0, -7.0, 0.5, 1.0]])     # gate | up, I = 6
    h = R.swiglu_ref(x)
    e = np.e
    assert h[0, 0] == 0.0                                               # silu(0) = 0
    assert abs(h[0, 1] - (1 / (1 + 1 / e)) * 3.0) < 1e-15               # silu(1) = e / (1 + e)
    assert abs(h[0, 2] - (-1 / (1 + e)) * 5.0) < 1e-15                  # silu(-1) = -1 / (1 + e)
    assert abs(h[0, 3] - 30.0 * -7.0) < 1e-9                            # silu(x) -> x
    assert abs(h[0, 4]) < 1e-11 and h[0, 5] == 0.0                      # silu(-x) -> 0, also where exp overflows
    # silu(x) - silu(-x) = x  (from sigma(x) + sigma(-x) = 1)
    g = np.linspace(-9, 9, 181)[None, :]
    both = R.swiglu_ref(np.concatenate([g, np.ones_like(g)], axis=1)) - R.swiglu_ref(np.concatenate([-g, np.ones_like(g)], axis=1))
    np.testing.assert_allclose(both, g, atol=1e-14)
    # against the library's SiLU in fp64, and the gate / up halves are not swapped (silu is not symmetric)
    p = np.random.default_rng(1).standard_normal((7, 10)) * 3
    want = torch.nn.functional.silu(torch.from_numpy(p[:, :5])).numpy() * p[:, 5:]
    np.testing.assert_allclose(R.swiglu_ref(p), want, rtol=1e-14, atol=1e-300)
    assert not np.allclose(R.swiglu_ref(p), R.swiglu_ref(np.concatenate([p[:, 5:], p[:, :5]], axis=1)))
    assert np.isnan(R.swiglu_ref(np.full((1, 4), np.nan))).all()


def test_grouped_gemm_block_scaled_fp8():
    """Row scales for A, 128 x 128 block scales per group for B: brute force from the definition; all scales one gives
    the unscaled grouped GEMM."""
    off = [0, 3, 3, 140, 150]
    g = W.gemm_grouped_fp8(off, 256, 384, 15)
    A, Bm = R.e4m3_to_f64(g.a_mk), R.e4m3_to_f64(g.b_gnk)                   # (M, K), (G, N, K)
    want = np.full((g.M, g.N), np.nan)
    for e in range(g.G):
        for r in range(off[e], off[e + 1]):
            acc = np.zeros(g.N)
            for kb in range(3):
                ks = slice(kb * 128, (kb + 1) * 128)
                acc += float(g.scale_a[r, kb]) * (Bm[e][:, ks] @ A[r, ks]) * np.repeat(g.scale_b[e, :, kb].astype(np.float64), 128)
            want[r] = acc
    got = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_FP8_E4M3, scale_a=g.scale_a, scale_b=g.scale_b)
    assert not np.isnan(got).any() and R.rel_frobenius(got, want) <= 1e-12
    ones = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_FP8_E4M3,
                              scale_a=np.ones_like(g.scale_a), scale_b=np.ones_like(g.scale_b))
    np.testing.assert_allclose(ones, R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_FP8_E4M3), rtol=1e-13)
    # a scale of group 2 does not touch group 0
    bad = g.scale_b.copy()
    bad[2, 1, 0] *= 2
    other = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_FP8_E4M3, scale_a=g.scale_a, scale_b=bad)
    assert np.array_equal(other[:3], got[:3]) and np.array_equal(other[3:140, :128], got[3:140, :128])
    assert R.rel_frobenius(other[3:140, 128:], got[3:140, 128:]) > 1e-2
