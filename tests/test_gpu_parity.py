"""Parity of the HIP path (through the C ABI) with the CPU oracle, element by element.

Bars: layout evaluation and relayout bit-exact; GEMM relative Frobenius error <= 5e-3 (bf16
inputs) / 3e-2 (fp8 inputs) against the fp64 oracle on the same quantised inputs, for the whole
matrix and for every 128 x 128 tile of it (a single wrong tile cannot hide in the global norm)."""
import ctypes as C
import itertools
import random
from math import prod

import numpy as np
import pytest
import torch

from oracle import axe_layout as ax
from oracle import axe_ref as R
from oracle.axe_layout import Iter, Layout, Swizzle
from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W
from packing import pack_blocked, pack_gate_up

pytestmark = pytest.mark.gpu

BF16_TOL, FP8_TOL = 5e-3, 3e-2


def dev(a: np.ndarray) -> torch.Tensor:
    """Raw words -> CUDA tensor of the same bit width."""
    a = np.ascontiguousarray(a)
    view = {1: np.uint8, 2: np.int16, 4: np.int32, 8: np.int64}[a.dtype.itemsize] if a.dtype.kind in "ui" else a.dtype
    return torch.from_numpy(a.view(view).copy()).cuda()


def host_words(t: torch.Tensor, dtype) -> np.ndarray:
    return t.cpu().numpy().view(dtype)


def spec_of(L: Layout) -> dict:
    z = L.swizzle
    return W.spec([(i.extent, i.stride, i.axis) for i in L.D], [(i.extent, i.stride, i.axis) for i in L.R],
                  dict(L.O), (z.axis, z.bits, z.base, z.shift) if z else None)


# ----------------------------------------------------------------------------- layout evaluation
def eval_both(L: Layout, shape, idx=None):
    axes = L.axes()
    bl = B.Layout(spec_of(L), axes)
    n = L.E_D if idx is None else len(idx)
    didx = None if idx is None else torch.from_numpy(np.asarray(idx, dtype=np.int64)).cuda()
    got = B.axe_layout_eval(bl, shape, n, didx).cpu().numpy()
    xs = np.arange(n) if idx is None else np.asarray(idx)
    want = R.evaluate_np(L, xs, axes)
    return got, want


def test_eval_paper_examples(golden):
    cases = []
    g = golden["tensor_core_tile"]
    cases.append((Layout.make(g["D"]["extents"], g["D"]["strides"], R=(g["R"]["extents"], g["R"]["strides"]), O=g["O"]), g["shape"]))
    g = golden["mesh_fully_sharded"]
    cases.append((Layout.make(g["D"]["extents"], g["D"]["strides"]), g["shape"]))
    g = golden["mesh_shard_replica"]
    cases.append((Layout.make(g["D"]["extents"], g["D"]["strides"], R=(g["R"]["extents"], g["R"]["strides"])), g["shape"]))
    g = golden["cute_partition"]
    cases.append((Layout.make(g["D"]["extents"], g["D"]["strides"], O=g["O"]), (16, 64)))
    g = golden["triton_local"]
    cases.append((Layout.make(g["D"]["extents"], g["D"]["strides"]), (16, 64)))
    g = golden["tile_example"]
    cases.append((Layout.make(g["T"]["extents"], g["T"]["strides"]), (16, 24)))
    cases.append((Layout.make((24, 24), (1, 24)), (24, 24)))
    for L, shape in cases:
        got, want = eval_both(L, shape)
        assert got.shape == want.shape and np.array_equal(got, want), repr(L)
        # and against the scalar definition for a few points
        for x in (0, L.E_D // 3, L.E_D - 1):
            assert [tuple(r) for r in got[x]] == ax.evaluate(L, x, L.axes())


def test_eval_random_layouts_and_explicit_indices():
    rng = random.Random(21)
    axes = ["m", "lane", "reg", "gpuid"]
    for trial in range(40):
        D = tuple(Iter(rng.randint(1, 7), rng.choice([1, 2, 3, 5, 8, 64, -4, -1, 1000003]), rng.choice(axes))
                  for _ in range(rng.randint(1, 6)))
        Rr = tuple(Iter(rng.randint(1, 3), rng.choice([1, 7, -2, 4096]), rng.choice(axes)) for _ in range(rng.randint(0, 2)))
        O = {a: rng.randint(-9, 9) for a in axes if rng.random() < 0.5}
        L = Layout(D, Rr, ax._norm_offset(O))
        if trial % 3 == 0:
            lo = int(R.evaluate_np(L, np.arange(L.E_D), L.axes())[:, :, L.axes().index(D[0].axis)].min())
            L = L.with_(O={**L.offset, D[0].axis: L.offset.get(D[0].axis, 0) - min(lo, 0)}, swizzle=Swizzle(D[0].axis, 2, 1, 4))
        got, want = eval_both(L, (L.E_D,))
        assert np.array_equal(got, want), repr(L)
        idx = [rng.randrange(L.E_D) for _ in range(17)]
        got, want = eval_both(L, (L.E_D,), idx)
        assert np.array_equal(got, want)
    # out-of-range explicit indices give INT64_MIN, in-range neighbours are unaffected
    L = Layout.make((4, 4), (4, 1))
    bl = B.Layout(spec_of(L))
    idx = torch.tensor([3, 16, -1, 15], dtype=torch.int64).cuda()
    got = B.axe_layout_eval(bl, (4, 4), 4, idx).cpu().numpy().reshape(-1)
    assert list(got) == [3, np.iinfo(np.int64).min, np.iinfo(np.int64).min, 15]


@pytest.mark.parametrize("axes", [["m"], ["m", "lane"], ["m", "lane", "reg"], ["m", "lane", "reg", "gpuid"], ["m", "a", "b", "c", "d"]])
def test_eval_without_replicas_every_axis_count(axes):
    """Layouts without replicas take a specialised kernel per number of axes (five axes: the general one); odd
    point counts, extents that are no powers of two, negative strides, explicit indices with some out of range."""
    rng = random.Random(len(axes))
    for trial in range(6):
        ext = [rng.choice([2, 3, 4, 5, 7, 8, 16]) for _ in range(rng.randint(1, 5))]
        D = [Iter(e, rng.choice([1, 2, 3, 17, 64, -5]) * rng.choice([1, 9]), rng.choice(axes)) for e in ext]
        L = Layout(tuple(D), (), ax._norm_offset({a: rng.randint(0, 9) for a in axes}))
        E = L.E_D
        bl = B.Layout(spec_of(L), axes)
        got = B.axe_layout_eval(bl, (E,), E).cpu().numpy()                       # implicit indices, E odd or even
        want = R.evaluate_np(L, np.arange(E), axes)
        assert np.array_equal(got, want), repr(L)
        idx = np.array([E - 1, 0, -1, E, E // 2, 2 ** 40, 1 % E], dtype=np.int64)  # 7 indices: an odd count
        got = B.axe_layout_eval(bl, (E,), len(idx), torch.from_numpy(idx).cuda()).cpu().numpy()
        ok = (idx >= 0) & (idx < E)
        assert np.array_equal(got[ok], R.evaluate_np(L, idx[ok], axes)), repr(L)
        assert (got[~ok] == np.iinfo(np.int64).min).all()


def test_eval_large_blocked_swizzled_layout():
    # the config-2 destination at full size: 2^26 points, compared on a strided sample plus both ends,
    # and as a permutation (every address exactly once) on the device result
    rows = cols = 8192
    L = Layout.from_spec(W.blocked_swizzled_spec(rows, cols))
    bl = B.Layout(W.blocked_swizzled_spec(rows, cols))
    n = rows * cols
    got = B.axe_layout_eval(bl, (rows, cols), n)
    sample = np.concatenate([np.arange(0, 70000), np.arange(0, n, 9973), np.arange(n - 70000, n)])
    want = R.evaluate_np(L, sample, ["m"])[:, 0, 0]
    assert np.array_equal(got.reshape(-1)[torch.from_numpy(sample).cuda()].cpu().numpy(), want)
    srt = torch.sort(got.reshape(-1)).values
    assert bool((srt == torch.arange(n, device="cuda")).all())
    # a layout whose E_D exceeds 2^31 takes the 64-bit digit path
    big = Layout.make((1 << 20, 1 << 13), (1 << 13, 1))
    idx = np.array([0, 1, (1 << 33) - 1, (1 << 32) + 12345, 123456789012 % (1 << 33)], dtype=np.int64)
    g2 = B.axe_layout_eval(B.Layout(spec_of(big)), (1 << 20, 1 << 13), len(idx), torch.from_numpy(idx).cuda()).cpu().numpy()
    assert np.array_equal(g2, R.evaluate_np(big, idx, ["m"]))


# ----------------------------------------------------------------------------- relayout
def relayout_both(src_L: Layout, dst_L: Layout, shape, src_words: np.ndarray, dst_len: int, fill=0xA5):
    want = np.zeros(dst_len, dtype=src_words.dtype)
    want.view(np.uint8)[:] = fill
    R.relayout_ref(src_L, dst_L, shape, src_words, want)
    d_dst = torch.full((dst_len * src_words.dtype.itemsize,), fill, dtype=torch.uint8).cuda()
    d_src = dev(src_words.view(np.uint8))
    B.axe_relayout(B.Layout(spec_of(src_L), ["m", "gpuid"]), B.Layout(spec_of(dst_L), ["m", "gpuid"]), shape, d_src, d_dst,
                   elem_bytes=src_words.dtype.itemsize)
    got = d_dst.cpu().numpy().view(src_words.dtype)
    return got, want


@pytest.mark.parametrize("rows,cols", [(128, 64), (256, 192), (1152, 704)])
def test_relayout_blocked_swizzled_small(rows, cols):
    words = W.relayout_words(rows, cols, 31, "index").reshape(-1)
    src_L = Layout.from_spec(W.row_major_spec(rows, cols))
    dst_L = Layout.from_spec(W.blocked_swizzled_spec(rows, cols))
    got, want = relayout_both(src_L, dst_L, (rows, cols), words, rows * cols)
    assert np.array_equal(got, want)
    back, want_back = relayout_both(dst_L, src_L, (rows, cols), got, rows * cols)
    assert np.array_equal(back, want_back) and np.array_equal(back, words)


@pytest.mark.parametrize("eb", [1, 2, 4, 8, 16])
def test_relayout_element_sizes_transposes_and_ragged(eb):
    rng = np.random.default_rng(eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64, 16: np.dtype((np.void, 16))}[eb]
    for shape in ((24, 24), (37, 53), (6, 4, 5), (96, 40), (3, 128, 7)):
        n = prod(shape)
        src = rng.integers(0, 256, n * eb, dtype=np.uint8).view(dt)
        A = ax.row_major(shape)
        strides_f = [prod(shape[:i]) for i in range(len(shape))]
        Bf = Layout.make(shape, strides_f)                                  # column-major
        for s_L, d_L in ((A, Bf), (Bf, A), (A, A)):
            got, want = relayout_both(s_L, d_L, shape, src, n)
            assert got.tobytes() == want.tobytes(), (shape, eb)
    # destination with a pitch, an offset and two replicas; untouched words keep the fill pattern
    shape = (10, 12)
    src = rng.integers(0, 256, 120 * eb, dtype=np.uint8).view(dt)
    D = Layout.make(shape, (16, 1), R=((2,), (200,)), O={"m": 5})
    got, want = relayout_both(ax.row_major(shape), D, shape, src, 400)
    assert got.tobytes() == want.tobytes()
    # negative stride (reversed rows) with the offset that keeps addresses non-negative
    Rv = Layout.make(shape, (-12, 1), O={"m": 108})
    got, want = relayout_both(ax.row_major(shape), Rv, shape, src, 120)
    assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_relayout_transposing_path(eb):
    """Source and destination contiguous along different digits: tiles through LDS.  Whole and clipped
    tiles, a batch digit, pitched rows and offsets on both sides, both directions."""
    rng = np.random.default_rng(100 + eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]
    ce = 16 // eb
    T = {1: 128, 2: 128, 4: 128, 8: 64}[eb]
    cases = [((T, T), None), ((2 * T + ce, 3 * T - ce), None), ((ce * 5, 4 * T), None),
             ((3, T + 2 * ce, 2 * T), "batch"), ((T + ce, T - ce), "pitched"), ((5 * T, 7 * T + 3 * ce), None)]
    for shape, kind in cases:
        rows, cols = shape[-2], shape[-1]
        if kind == "batch":
            s_L, d_L = ax.row_major(shape), Layout.make(shape, (rows * cols, 1, rows))
            n_src = n_dst = prod(shape)
        elif kind == "pitched":
            ps, pd = cols + 3 * ce, rows + 2 * ce
            s_L, d_L = Layout.make(shape, (ps, 1), O={"m": ce}), Layout.make(shape, (1, pd), O={"m": 2 * ce})
            n_src, n_dst = ce + rows * ps, 2 * ce + cols * pd
        else:
            s_L, d_L = ax.row_major(shape), Layout.make(shape, (1, rows))
            n_src = n_dst = prod(shape)
        src = rng.integers(0, 256, n_src * eb, dtype=np.uint8).view(dt)
        got, want = relayout_both(s_L, d_L, shape, src, n_dst)
        assert got.tobytes() == want.tobytes(), (shape, kind)
        back, wb = relayout_both(d_L, s_L, shape, got, n_src)
        assert back.tobytes() == wb.tobytes(), (shape, kind)


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_relayout_transposing_path_replicas_and_swizzles(eb):
    """The tiled path with a replicated destination and with swizzle stages that move whole 16-byte chunks."""
    rng = np.random.default_rng(300 + eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]
    ce = 16 // eb
    T = {1: 128, 2: 128, 4: 128, 8: 64}[eb]
    lg = ce.bit_length() - 1
    for shape in [(T, T), (2 * T, T + ce), (T + 3 * ce, 2 * T), (4 * T, 6 * T)]:
        rows, cols = shape
        n = rows * cols
        size = 1 << (n - 1).bit_length()
        src = rng.integers(0, 256, n * eb, dtype=np.uint8).view(dt)
        row, col = ax.row_major(shape), Layout.make(shape, (1, rows))
        for R_, span in [(((2,), (n,)), 2 * n), (((2, 3), (3 * (n + ce), n + ce)), 6 * (n + ce))]:
            got, want = relayout_both(row, Layout.make(shape, (1, rows), R=R_), shape, src, span)
            assert got.tobytes() == want.tobytes(), (shape, R_)
        sw_d = Swizzle("m", 3, lg, lg + 5)
        sw_s = Swizzle("m", 2, lg + 1, lg + 4)
        for s_L, d_L in [(row, col.with_(swizzle=sw_d)), (row.with_(swizzle=sw_s), col),
                         (row.with_(swizzle=sw_s), col.with_(swizzle=sw_d)),
                         (col.with_(swizzle=sw_d), row.with_(swizzle=sw_s))]:
            src_p = rng.integers(0, 256, size * eb, dtype=np.uint8).view(dt)
            got, want = relayout_both(s_L, d_L, shape, src_p, size)
            assert got.tobytes() == want.tobytes(), (shape, s_L, d_L)
        d_L = Layout.make(shape, (1, rows), R=((2,), (size,))).with_(swizzle=sw_d)
        got, want = relayout_both(row, d_L, shape, src, 2 * size)
        assert got.tobytes() == want.tobytes(), shape


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_relayout_transposing_path_element_by_element(eb):
    """Transposing pairs whose rows are not whole 16-byte chunks: odd extents, pitches, offsets and replica
    strides, swizzles inside a chunk; several tiles with clipped edges, a batch digit; both directions."""
    rng = np.random.default_rng(400 + eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]
    w = max(64 // eb, 2)
    cases = []
    for shape in [(w + 1, 2 * w + 3), (129, 67 + w), (64, 64 + w + 1), (3, w + 5, 70 + w), (301, 515), (1000, 37 + w)]:
        rows, cols = shape[-2], shape[-1]
        n = prod(shape)
        if len(shape) == 3:
            s_L, d_L = ax.row_major(shape), Layout.make(shape, (rows * cols, 1, rows))
        else:
            s_L, d_L = ax.row_major(shape), Layout.make(shape, (1, rows))
        cases.append((shape, s_L, d_L, n, n))
    rows, cols = w + 2, 2 * w + 1
    shape = (rows, cols)
    cases.append((shape, Layout.make(shape, (cols + 3, 1), O={"m": 1}), Layout.make(shape, (1, rows + 5), O={"m": 3}),
                  1 + rows * (cols + 3), 3 + cols * (rows + 5)))
    rows, cols = 2 * w, 2 * w
    shape = (rows, cols)
    n = rows * cols
    cases.append((shape, ax.row_major(shape), Layout.make(shape, (1, rows), R=((3,), (n + 1,))), n, 3 * (n + 1)))
    cases.append((shape, ax.row_major(shape).with_(swizzle=Swizzle("m", 2, 0, 7)),
                  Layout.make(shape, (1, rows)).with_(swizzle=Swizzle("m", 3, 1, 8)), n, n))
    for shape, s_L, d_L, n_src, n_dst in cases:
        src = rng.integers(0, 256, n_src * eb, dtype=np.uint8).view(dt)
        got, want = relayout_both(s_L, d_L, shape, src, n_dst)
        assert got.tobytes() == want.tobytes(), (shape, s_L, d_L)
        if not d_L.R:
            back, wb = relayout_both(d_L, s_L, shape, got, n_src)
            assert back.tobytes() == wb.tobytes(), (shape, "back")


def operand_image_layouts(M, K, which=None):
    """(source spec, destination spec, 4-D shape, destination elements, axes): a row-major (M, K) bf16 matrix, and the
    memory image [tile][wave][lane][reg] of the MFMA operand registers of the 256 x 256 kernel -- the operand layout
    axe_gemm_describe reports for one (256, 64) tile, tiled over the matrix (axe_layout_tile) and folded onto the
    memory axis (axe_layout_flatten)."""
    which = B.AXE_DESC_A_OPERAND if which is None else which
    desc = B.GemmDesc(M, 256, K, B.AXE_BF16, B.AXE_BF16, B.Layout(W.row_major_spec(M, K)), B.Layout(W.col_major_spec(K, 256)),
                      B.Layout(W.row_major_spec(M, 256)), M * K, 256 * K, M * 256, tile_hint=B.AXE_TILE_256x256x64)
    spec, tshape = B.axe_gemm_describe(desc, which)
    assert tshape == (256, 64)
    axes = ["m", "lds", "wg", "wave", "lane", "reg"]
    op = B.Layout(spec, axes)
    gm, gk = M // 256, K // 64
    grid = B.Layout(W.spec([(gm, gk, "wg"), (gk, 1, "wg")]), axes)
    tiled, shape = B.layout_tile(grid, (gm, gk), op, tshape)
    span = B.layout_span(B.Layout(tiled, axes))
    regs, lanes, waves = span["reg"], span["lane"], span["wave"]
    assert (lanes, waves) == (64, 4)
    pitch = {"reg": 1, "lane": regs, "wave": lanes * regs, "wg": waves * lanes * regs}
    dst = B.layout_flatten(B.Layout(tiled, axes), pitch, "m")
    src = W.spec([(gm, 256 * K, "m"), (256, K, "m"), (gk, 64, "m"), (64, 1, "m")])
    return src, dst, shape, gm * gk * waves * lanes * regs, axes


def test_relayout_into_the_mfma_operand_register_order():
    """A register layout as the target of a relayout (Sec. 3.2: copy between layouts of different scopes; thread axes
    of Sec. 2.2): the rows of A in the order the lanes of the 256 x 256 kernel hold them, each wave's copy written
    (the layout is replicated over the wave columns).  Checked against the oracle's relayout of the same two layouts."""
    M, K = 768, 320
    src_spec, dst_spec, shape, n_dst, axes = operand_image_layouts(M, K)
    assert shape == (M // 256, 256, K // 64, 64)
    words = W.to_bf16_bits(W.normal(131, (M, K))).reshape(-1)
    want = np.full(n_dst, 0xA5A5, dtype=np.uint16)
    R.relayout_ref(Layout.from_spec(src_spec), Layout.from_spec(dst_spec), shape, words, want)
    assert not (want == 0xA5A5).all() and n_dst == 2 * M * K              # two wave columns: every element lands twice
    d_dst = torch.full((n_dst,), -23131, dtype=torch.int16, device="cuda")          # 0xA5A5
    B.axe_relayout(B.Layout(src_spec, axes), B.Layout(dst_spec, axes), shape, dev(words), d_dst)
    got = host_words(d_dst, np.uint16)
    assert np.array_equal(got, want)
    # every 16-byte chunk of the image is an aligned run of 8 consecutive k of one row of A: a lane fetches its operand
    # fragment from this image with one 16-byte load
    void = np.dtype((np.void, 16))
    assert np.isin(got.reshape(-1, 8).view(void).ravel(), words.reshape(-1, 8).view(void).ravel()).all()


@pytest.mark.parametrize("rows,cols,dtype", [(8192, 8192, np.uint16), (4096, 12288, np.uint16), (8192, 8192, np.uint32)])
def test_relayout_transpose_full_size(rows, cols, dtype):
    """Row-major -> column-major of a matrix of the workload's size against the definition written with
    NumPy (a transposed view made contiguous), bit for bit; and back."""
    rng = np.random.default_rng(rows + cols)
    src = rng.integers(0, np.iinfo(dtype).max, rows * cols, dtype=dtype)
    d_src = dev(src.view(np.uint8))
    d_dst = torch.zeros(rows * cols * src.itemsize, dtype=torch.uint8, device="cuda")
    Ls, Ld = B.Layout(W.row_major_spec(rows, cols)), B.Layout(W.col_major_spec(rows, cols))
    B.axe_relayout(Ls, Ld, (rows, cols), d_src, d_dst, elem_bytes=src.itemsize)
    got = d_dst.cpu().numpy().view(dtype)
    assert np.array_equal(got, np.ascontiguousarray(src.reshape(rows, cols).T).reshape(-1))
    d_back = torch.zeros_like(d_dst)
    B.axe_relayout(Ld, Ls, (rows, cols), d_dst, d_back, elem_bytes=src.itemsize)
    assert np.array_equal(d_back.cpu().numpy().view(dtype), src)


def test_relayout_without_common_refinement_uses_generic_path():
    # source digits (6, 4), destination digits (4, 6) over the same 24 elements: no joint loop nest
    rng = np.random.default_rng(3)
    src = rng.integers(0, 2 ** 16, 24, dtype=np.uint16)
    s_L = Layout.make((6, 4), (1, 6))
    d_L = Layout.make((4, 6), (1, 4))
    got, want = relayout_both(s_L, d_L, (24,), src, 24)
    assert np.array_equal(got, want)
    s_L = Layout.make((9, 10), (10, 1))
    d_L = Layout.make((6, 15), (1, 6))
    src = rng.integers(0, 2 ** 16, 90, dtype=np.uint16)
    got, want = relayout_both(s_L, d_L, (90,), src, 90)
    assert np.array_equal(got, want)


def test_relayout_composition():
    rng = np.random.default_rng(4)
    shape = (64, 48)
    src = rng.integers(0, 2 ** 32, prod(shape), dtype=np.uint32)
    A, Bc = ax.row_major(shape), Layout.make(shape, (1, 64))
    Cb, _ = ax.tile(ax.row_major((4, 3)), (4, 3), ax.row_major((16, 16)), (16, 16))
    ab, _ = relayout_both(A, Bc, shape, src, prod(shape))
    bc, _ = relayout_both(Bc, Cb, shape, ab, prod(shape))
    ac, want = relayout_both(A, Cb, shape, src, prod(shape))
    assert np.array_equal(bc, ac) and np.array_equal(ac, want)


@pytest.mark.parametrize("kind", ["uniform", "index"])
def test_relayout_config2_full_size(kind):
    rows = cols = 8192
    words = W.config2(kind).reshape(-1)
    src_spec, dst_spec = W.row_major_spec(rows, cols), W.blocked_swizzled_spec(rows, cols)
    d_src = dev(words)
    d_dst = torch.zeros(rows * cols, dtype=torch.int16, device="cuda")
    Ls, Ld = B.Layout(src_spec), B.Layout(dst_spec)
    B.axe_relayout(Ls, Ld, (rows, cols), d_src, d_dst)
    got = host_words(d_dst, np.uint16)
    want = np.zeros(rows * cols, dtype=np.uint16)
    R.relayout_ref(Layout.from_spec(src_spec), Layout.from_spec(dst_spec), (rows, cols), words, want)
    assert np.array_equal(got, want)
    d_back = torch.zeros(rows * cols, dtype=torch.int16, device="cuda")
    B.axe_relayout(Ld, Ls, (rows, cols), d_dst, d_back)
    assert np.array_equal(host_words(d_back, np.uint16), words)          # bit-exact round trip


# ----------------------------------------------------------------------------- GEMM
IN_DT = {"bf16": B.AXE_BF16, "f16": B.AXE_F16, "fp8": B.AXE_FP8_E4M3}
OUT_DT = {"f32": B.AXE_F32, "bf16": B.AXE_BF16, "f16": B.AXE_F16}
ORACLE_DT = {"bf16": R.AXE_BF16, "f16": R.AXE_F16, "fp8": R.AXE_FP8_E4M3}


def decode16(words: np.ndarray, dtype: str) -> np.ndarray:
    return R.f16_to_f64(words) if dtype == "f16" else R.bf16_to_f64(words)


def run_gemm(g: W.GemmInputs, tile=B.AXE_TILE_AUTO, device_axis=False, lda=None, ldb=None, ldc=None):
    """Launches axe_gemm on the inputs; returns C decoded to fp64 (M, N)."""
    As, Bs, Cs = W.gemm_specs(g, device_axis=device_axis, shard=3)
    a, b = g.a_mk, g.b_nk
    if lda:
        As = W.spec([(g.M, lda, "m"), (g.K, 1, "m")])
        a = np.zeros((g.M, lda), dtype=a.dtype); a[:, :g.K] = g.a_mk
    if ldb:
        Bs = W.spec([(g.K, 1, "m"), (g.N, ldb, "m")])
        b = np.zeros((g.N, ldb), dtype=b.dtype); b[:, :g.K] = g.b_nk
    ldc_ = ldc or g.N
    if ldc:
        Cs = W.spec([(g.M, ldc, "m"), (g.N, 1, "m")])
    axes = ["m", "gpuid"]
    dA, dB = dev(a.reshape(-1)), dev(b.reshape(-1))
    out_t = torch.float32 if g.out_dtype == "f32" else torch.int16
    dC = torch.zeros(g.M * ldc_, dtype=out_t, device="cuda")
    sa = torch.from_numpy(g.scale_a).cuda() if g.scale_a is not None else None
    sb = torch.from_numpy(g.scale_b).cuda() if g.scale_b is not None else None
    desc = B.GemmDesc(g.M, g.N, g.K, IN_DT[g.dtype], OUT_DT[g.out_dtype],
                      B.Layout(As, axes), B.Layout(Bs, axes), B.Layout(Cs, axes),
                      a.size, b.size, g.M * ldc_, sa, sb, tile_hint=tile,
                      scale_dtype=B.AXE_SCALE_E8M0 if g.scale_dtype == "e8m0" else B.AXE_SCALE_F32)
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    c = dC.cpu().numpy().reshape(g.M, ldc_)[:, :g.N]
    return c.astype(np.float64) if g.out_dtype == "f32" else decode16(c.view(np.uint16), g.out_dtype)


def gemm_desc_only(g: W.GemmInputs, tile=B.AXE_TILE_AUTO):
    """Descriptor of the plain problem (no device buffers): for questions to the host side."""
    As, Bs, Cs = W.gemm_specs(g)
    return B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16 if g.dtype == "bf16" else B.AXE_FP8_E4M3,
                      B.AXE_F32 if g.out_dtype == "f32" else B.AXE_BF16,
                      B.Layout(As), B.Layout(Bs), B.Layout(Cs), g.M * g.K, g.N * g.K, g.M * g.N, tile_hint=tile)


def oracle_scales(g: W.GemmInputs):
    """The scale arrays as the oracle takes them (fp32); E8M0 codes are decoded by the oracle's own rule."""
    if g.scale_a is None or g.scale_dtype != "e8m0":
        return g.scale_a, g.scale_b
    return R.e8m0_decode(g.scale_a).astype(np.float32), R.e8m0_decode(g.scale_b).astype(np.float32)


def oracle_gemm(g: W.GemmInputs, rows=None, cols=None):
    sa, sb = oracle_scales(g)
    return R.gemm_ref(g.a_mk, g.b_nk.T, ORACLE_DT[g.dtype], sa, sb, rows=rows, cols=cols)


def check_gemm(c, ref, tol, tile=128):
    assert np.isfinite(c).all()
    err = R.rel_frobenius(c, ref)
    assert err <= tol, f"global relative Frobenius error {err:.3e} > {tol}"
    M, N = ref.shape
    worst = 0.0
    for i in range(0, M, tile):
        for j in range(0, N, tile):
            worst = max(worst, R.rel_frobenius(c[i:i + tile, j:j + tile], ref[i:i + tile, j:j + tile]))
    assert worst <= tol, f"worst {tile}x{tile} tile error {worst:.3e} > {tol}"
    return err


def test_gemm_config1_bf16_256_fp32_out():
    g = W.config1()
    c = run_gemm(g)
    err = check_gemm(c, oracle_gemm(g), BF16_TOL)
    assert err < 1e-5            # fp32 output: only accumulation order differs from the fp64 sum


@pytest.mark.parametrize("M,N,K", [(64, 64, 32), (200, 136, 96), (65, 63, 8), (1, 1, 8), (300, 70, 520)])
@pytest.mark.parametrize("out", ["f32", "bf16"])
def test_gemm_bf16_small_tile_ragged(M, N, K, out):
    g = W.gemm_bf16(M, N, K, 40 + M, out_dtype=out)
    c = run_gemm(g, tile=B.AXE_TILE_64x64x32)
    check_gemm(c, oracle_gemm(g), BF16_TOL, tile=64)


# Short K and few whole tiles: the 64 x 64 kernel's burst variant (all K-tiles requested up front, one block of LDS per
# K-tile).  nkt = 1, 2, 4, 7, 8 K-tiles; 1, 6, 16 and 60 tiles; bf16 and fp16, fp32 and 16-bit output; pitched A, B, C.
# K = 576 (9 K-tiles) and 17 x 16 tiles (more tiles than compute units) take the regular variant: same answers.
@pytest.mark.parametrize("M,N,K", [(64, 64, 64), (128, 192, 128), (256, 256, 256), (384, 640, 448), (64, 128, 512),
                                   (128, 128, 576), (1088, 1024, 256)])
@pytest.mark.parametrize("dtype,out", [("bf16", "f32"), ("bf16", "bf16"), ("f16", "f16")])
def test_gemm_small_tile_short_k(M, N, K, dtype, out):
    g = (W.gemm_bf16 if dtype == "bf16" else W.gemm_f16)(M, N, K, 30 + K, std_b=K ** -0.5, out_dtype=out)
    tol = 1e-5 if out == "f32" else (F16_TOL if dtype == "f16" else BF16_TOL)
    c = run_gemm(g, tile=B.AXE_TILE_64x64x32)
    check_gemm(c, oracle_gemm(g), tol, tile=64)
    c = run_gemm(g, tile=B.AXE_TILE_64x64x32, lda=K + 8, ldb=K + 24, ldc=N + 4)
    check_gemm(c, oracle_gemm(g), tol, tile=64)


def test_gemm_identity_and_pitched_operands():
    K = N = 128
    g = W.gemm_bf16(K, N, K, 50, out_dtype="f32")
    g.a_mk = W.to_bf16_bits(np.eye(K, dtype=np.float32))
    c = run_gemm(g, lda=K + 24, ldb=K + 8, ldc=N + 4)
    assert np.array_equal(c, R.bf16_to_f64(g.b_nk).T)       # A = I returns B exactly


def test_gemm_device_axis_of_extent_one():
    g = W.config4(128, 192, 256)
    g.out_dtype = "f32"
    c = run_gemm(g, device_axis=True)
    check_gemm(c, oracle_gemm(g), BF16_TOL, tile=64)


def test_gemm_fp8_small_tile_e8m0():
    for M, N, K in ((128, 256, 384), (200, 72, 272), (64, 64, 128)):
        g = W.gemm_fp8(M, N, K, 60 + K, scaled="e8m0")
        c = run_gemm(g, tile=B.AXE_TILE_64x64x32)
        check_gemm(c, oracle_gemm(g), FP8_TOL, tile=64)


@pytest.mark.parametrize("M,N,K,scaled", [(128, 128, 128, False), (128, 256, 384, True), (200, 72, 272, True),
                                          (64, 64, 16, False)])
def test_gemm_fp8_small_tile(M, N, K, scaled):
    g = W.gemm_fp8(M, N, K, 60 + K, scaled=scaled)
    c = run_gemm(g, tile=B.AXE_TILE_64x64x32)
    check_gemm(c, oracle_gemm(g), FP8_TOL, tile=64)
    g.out_dtype = "f32"
    c = run_gemm(g, tile=B.AXE_TILE_64x64x32)
    err = check_gemm(c, oracle_gemm(g), FP8_TOL, tile=64)
    assert err < 3e-5            # fp32 output: the MFMA adds the 128 products of an instruction in an aligned adder (about 17 bits): 1.3 - 1.5e-5 measured, whatever K


# ----------------------------------------------------------------------------- large tile (256 x 256)
# K = 64 nk: nk = 1, 2, 3 (shorter than the pipeline), 16, 11 and 9 (odd numbers of K-steps); several tiles
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (256, 256, 128), (512, 768, 192), (768, 256, 1024),
                                   (512, 768, 704), (768, 512, 576)])
def test_gemm_bf16_large_tile(M, N, K):
    g = W.gemm_bf16(M, N, K, 70 + K)
    c = run_gemm(g, tile=B.AXE_TILE_256x256x64)
    check_gemm(c, oracle_gemm(g), BF16_TOL)
    # bf16 output of the large tile equals the small tile's up to the last rounding (different k order)
    c_small = run_gemm(g, tile=B.AXE_TILE_64x64x32)
    assert R.rel_frobenius(c, c_small) < 2e-3


# Left to itself the library takes the 64 x 64 tiles for problems of less than 5 x 2^20 elements of C (fp8: 2^20) and the
# large tile beyond -- with whole tiles, ragged edges or an fp32 output alike; either way the result is the oracle's.
@pytest.mark.parametrize("M,N,K,dtype,out,want", [(768, 768, 256, "bf16", "bf16", B.AXE_TILE_64x64x32),
                                                  (2304, 2304, 128, "bf16", "bf16", B.AXE_TILE_256x256x64),
                                                  (2300, 2312, 128, "f16", "f16", B.AXE_TILE_256x256x64),
                                                  (2304, 2304, 128, "bf16", "f32", B.AXE_TILE_256x256x64),
                                                  (512, 512, 256, "fp8", "bf16", B.AXE_TILE_64x64x32),
                                                  (1024, 1024, 256, "fp8", "bf16", B.AXE_TILE_256x256x64)])
def test_gemm_kernel_chosen_by_problem_size(M, N, K, dtype, out, want):
    if dtype == "fp8":
        g = W.gemm_fp8(M, N, K, 490 + M, scaled=True)
    else:
        g = (W.gemm_bf16 if dtype == "bf16" else W.gemm_f16)(M, N, K, 490 + M, std_b=K ** -0.5, out_dtype=out)
    As, Bs, Cs = W.gemm_specs(g)
    class _Fake:
        def data_ptr(self):
            return 0x1000
    scales = dict(scale_a=_Fake(), scale_b=_Fake()) if dtype == "fp8" else {}
    desc = B.GemmDesc(M, N, K, IN_DT[dtype], OUT_DT[out], B.Layout(As), B.Layout(Bs), B.Layout(Cs), M * K, N * K, M * N, **scales)
    assert B.axe_gemm_tile(desc) == want
    c = run_gemm(g)
    tol = FP8_TOL if dtype == "fp8" else (1e-5 if out == "f32" else (F16_TOL if dtype == "f16" else BF16_TOL))
    check_gemm(c, oracle_gemm(g), tol)


# fp32 output of the large tile (16-bit inputs): the accumulators as they are -- only the order of the K sum differs
# from the oracle's fp64 sum.  nk = 1, 3, 9, and 8 with 17 x 16 tiles chained; pitched C with a guard pattern.
@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (512, 768, 192), (768, 512, 576), (4352, 4096, 512),
                                   (1000, 1004, 256), (257, 260, 128), (300, 4, 64)])            # and ragged edges (N a multiple of 4)
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_gemm_large_tile_fp32_output(M, N, K, dtype):
    g = (W.gemm_bf16 if dtype == "bf16" else W.gemm_f16)(M, N, K, 470 + K, std_b=K ** -0.5, out_dtype="f32")
    ldc, fill = N + 12, 12345.0
    dA, dB = dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))
    dC = torch.full((M * ldc,), fill, dtype=torch.float32, device="cuda")
    dt = B.AXE_BF16 if dtype == "bf16" else B.AXE_F16
    desc = B.GemmDesc(M, N, K, dt, B.AXE_F32, B.Layout(W.row_major_spec(M, K)), B.Layout(W.col_major_spec(K, N)),
                      B.Layout(W.spec([(M, ldc, "m"), (N, 1, "m")])), M * K, N * K, M * ldc, tile_hint=B.AXE_TILE_256x256x64)
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy().reshape(M, ldc)
    assert (raw[:, N:] == fill).all(), "the kernel wrote outside the M x N result"
    c = raw[:, :N].astype(np.float64)
    check_gemm(c, oracle_gemm(g), 1e-5)                     # whole matrix and every 128 x 128 tile, also for the chained launch


def test_gemm_large_tile_fp32_output_blocked_operands():
    g = W.gemm_bf16(512, 768, 256, 481, std_b=1 / 16, out_dtype="f32")
    dA, dB = dev(pack_blocked(g.a_mk)), dev(pack_blocked(g.b_nk))
    dC = torch.zeros(g.M * g.N, dtype=torch.float32, device="cuda")
    desc = B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16, B.AXE_F32, B.Layout(W.blocked_a_spec(g.M, g.K)), B.Layout(W.blocked_b_spec(g.K, g.N)),
                      B.Layout(W.row_major_spec(g.M, g.N)), g.M * g.K, g.N * g.K, g.M * g.N)
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    c = dC.cpu().numpy().reshape(g.M, g.N).astype(np.float64)
    assert R.rel_frobenius(c, oracle_gemm(g)) < 1e-5


# Ragged edges on the large tile (16-bit inputs): any M, N a multiple of 8.  C is pitched and followed by guard rows,
# all filled with a pattern beforehand: nothing outside the M x N result may change.  K = 64 nk with nk = 1, 2, 3
# (shorter than the pipeline), 4 and 8 (several tiles chained per workgroup), 11 (odd).
@pytest.mark.parametrize("M,N,K", [(200, 136, 64), (257, 264, 128), (1000, 1000, 256), (513, 8, 192), (300, 520, 704),
                                   (1, 256, 64), (777, 1288, 512), (255, 248, 256)])
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_gemm_large_tile_ragged_edges(M, N, K, dtype):
    g = (W.gemm_bf16 if dtype == "bf16" else W.gemm_f16)(M, N, K, 370 + M, std_b=K ** -0.5)
    ldc, guard, fill = N + 24, 3, 0x1234
    dA, dB = dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))
    dC = torch.full(((M + guard) * ldc,), fill, dtype=torch.int16, device="cuda")
    dt = B.AXE_BF16 if dtype == "bf16" else B.AXE_F16
    desc = B.GemmDesc(M, N, K, dt, dt, B.Layout(W.row_major_spec(M, K)), B.Layout(W.col_major_spec(K, N)),
                      B.Layout(W.spec([(M, ldc, "m"), (N, 1, "m")])), M * K, N * K, (M + guard) * ldc,
                      tile_hint=B.AXE_TILE_256x256x64)
    assert B.lib().axe_gemm_tile(C.byref(desc.c)) == B.AXE_TILE_256x256x64
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy().view(np.uint16).reshape(M + guard, ldc)
    assert (raw[:M, N:] == fill).all() and (raw[M:] == fill).all(), "the kernel wrote outside the M x N result"
    c = decode16(raw[:M, :N], dtype)
    check_gemm(c, oracle_gemm(g), BF16_TOL if dtype == "bf16" else F16_TOL, tile=64)
    g.out_dtype = dtype
    c_small = run_gemm(g, tile=B.AXE_TILE_64x64x32)
    assert R.rel_frobenius(c, c_small) < (2e-3 if dtype == "bf16" else 3e-4)


def test_gemm_large_tile_ragged_edges_many_tiles_per_workgroup():
    # 37 x 35 tiles, the last of each ragged: more tiles than compute units, chained through the pipeline
    g = W.gemm_bf16(9300, 8808, 256, 391, std_b=1 / 16)
    c = run_gemm(g)
    check_gemm(c, oracle_gemm(g), BF16_TOL)                 # whole matrix, every 128 x 128 tile (the ragged last ones included)


# 224 columns per tile (7 fragments per wave along N): same K cases, N a multiple of 224
@pytest.mark.parametrize("M,N,K", [(256, 224, 64), (256, 448, 128), (512, 672, 192), (768, 224, 1024), (512, 448, 704)])
def test_gemm_bf16_large_tile_224_columns(M, N, K):
    g = W.gemm_bf16(M, N, K, 170 + K)
    c = run_gemm(g, tile=B.AXE_TILE_256x224x64)
    check_gemm(c, oracle_gemm(g), BF16_TOL, tile=32)
    c_small = run_gemm(g, tile=B.AXE_TILE_64x64x32)
    assert R.rel_frobenius(c, c_small) < 2e-3


def test_gemm_bf16_large_tile_identity_pitched_and_device_axis():
    K = N = 256
    g = W.gemm_bf16(K, N, K, 71)
    g.a_mk = W.to_bf16_bits(np.eye(K, dtype=np.float32))
    c = run_gemm(g, tile=B.AXE_TILE_256x256x64, lda=K + 64, ldb=K + 8, ldc=N + 8, device_axis=False)
    assert np.array_equal(c, R.bf16_to_f64(g.b_nk).T)       # exact: bf16 values survive fp32 and the final rounding
    g4 = W.config4(512, 256, 512)
    c = run_gemm(g4, tile=B.AXE_TILE_256x256x64, device_axis=True)
    check_gemm(c, oracle_gemm(g4), BF16_TOL)


@pytest.mark.parametrize("M,N,K,scaled", [(256, 256, 128, False), (256, 512, 384, True), (512, 256, 256, True),
                                          (512, 768, 1408, True), (768, 512, 2048, False), (256, 256, 8960, True),
                                          (256, 256, 128, "e8m0"), (256, 512, 384, "e8m0"), (512, 768, 1408, "e8m0"),
                                          (768, 512, 2048, "e8m0"), (256, 256, 8960, "e8m0"), (512, 256, 17152, "e8m0")])
def test_gemm_fp8_large_tile(M, N, K, scaled):
    g = W.gemm_fp8(M, N, K, 80 + K, scaled=scaled)
    c = run_gemm(g, tile=B.AXE_TILE_256x256x64)
    check_gemm(c, oracle_gemm(g), FP8_TOL)


# ----------------------------------------------------------------------------- full-size configurations
# Whole C on the GPU in the launch configuration the benchmark times, against the whole fp64 C of the oracle:
# the bound on every 128 x 128 tile (hence on the whole matrix: the squared errors of the tiles add up).  The oracle's
# plain triple loop takes one to two minutes for an 8192^3 problem, so a case is checked in bands of rows, one test
# each: the GPU result is computed once per case and kept for its bands.
FULL_CASES = {
    # name: (inputs, keywords of run_gemm, tolerance, bands)
    "config3": (lambda: W.config3(), {}, BF16_TOL, 8),
    "config4": (lambda: W.config4(), dict(device_axis=True), BF16_TOL, 2),
    "config5": (lambda: W.config5(), {}, FP8_TOL, 8),
    # configuration 5's shape with power-of-two (E8M0) block scales, and fp8 without scales: the matrix cores' scale path
    "config5_e8m0": (lambda: W.gemm_fp8(8192, 8192, 8192, 19097, scaled="e8m0"), {}, FP8_TOL, 8),
    "e8m0_17x16_tiles_66_ksteps": (lambda: W.gemm_fp8(4352, 4096, 8448, 96, scaled="e8m0"), {}, FP8_TOL, 2),   # code registers refilled
    "fp8_unscaled_4096": (lambda: W.gemm_fp8(4096, 4096, 4096, 97, scaled=False), {}, FP8_TOL, 1),
    # more tiles than compute units, so every workgroup walks two tiles as one pipeline, on a tile grid that is not made
    # of 16 x 16 blocks (the other workgroup -> tile order); the last 16 workgroups get a second tile, the others do not
    "chained_17x16_bf16": (lambda: W.gemm_bf16(4352, 4096, 512, 91), {}, BF16_TOL, 1),
    # 224-column tiles, 17 x 16 of them (left to itself the library takes 17 x 14 tiles of 256 x 256 here)
    "chained_17x16_bf16_224": (lambda: W.gemm_bf16(4352, 3584, 512, 93), dict(tile=B.AXE_TILE_256x224x64), BF16_TOL, 1),
    # fp8 with fp32 scales, 66 K-steps: the register of block scales is refilled inside each chained tile
    "chained_17x16_fp8": (lambda: W.gemm_fp8(4352, 4096, 8448, 92, scaled=True), {}, FP8_TOL, 2),
}
_FULL = {}


def full_size_case(name):
    """(inputs, C of the GPU decoded to fp64) of one case; one case is held at a time."""
    if name not in _FULL:
        _FULL.clear()
        make, kw, _, _ = FULL_CASES[name]
        g = make()
        _FULL[name] = (g, run_gemm(g, **kw))
    return _FULL[name]


def band_rows(M, band, nbands):
    per = -(-(M // 128) // nbands) * 128                       # whole 128-row tile rows per band
    return np.arange(band * per, min(M, (band + 1) * per))


@pytest.mark.parametrize("name,band", [(n, b) for n, c in FULL_CASES.items() for b in range(c[3])])
def test_gemm_full_size_every_tile_against_the_oracle(name, band):
    g, c = full_size_case(name)
    _, _, tol, nbands = FULL_CASES[name]
    if name == "config4":
        # 16 x 16 tiles of 256 x 224 fill the 256 compute units; 16 x 14 tiles of 256 x 256 would leave 32 idle
        assert B.axe_gemm_tile(gemm_desc_only(g)) == B.AXE_TILE_256x224x64
    if name == "chained_17x16_bf16_224":
        assert B.axe_gemm_tile(gemm_desc_only(g)) == B.AXE_TILE_256x256x64
    rows = band_rows(g.M, band, nbands)
    assert len(rows) > 0
    check_gemm(c[rows], oracle_gemm(g, rows, None), tol)


@pytest.mark.parametrize("name", ["config3", "config4", "config5"])
def test_gemm_full_size_projections(name):
    """An extra that does not go through the oracle's C: two randomised projections (C v and u^T C, computed in fp64
    from the inputs with NumPy), every 256-row and 256-column block of the full matrix."""
    g, c = full_size_case(name)
    tol = FULL_CASES[name][2]
    rng = np.random.default_rng(3)
    M, N = g.M, g.N
    dt = R.AXE_BF16 if g.dtype == "bf16" else R.AXE_FP8_E4M3
    A, Bm = R.decode(g.a_mk, dt), R.decode(g.b_nk, dt)          # (M,K), (N,K)
    v, u = rng.choice([-1.0, 1.0], N), rng.choice([-1.0, 1.0], M)
    if g.scale_a is None:
        y_ref, z_ref = A @ (Bm.T @ v), (u @ A) @ Bm.T
    else:
        y_ref, z_ref = np.zeros(M), np.zeros(N)
        fa, fb = oracle_scales(g)
        sa = np.repeat(fa.astype(np.float64), 128, axis=0)[:M]             # (M, nkb)
        sb = np.repeat(fb.astype(np.float64), 128, axis=0)[:N]             # (N, nkb)
        for kb in range(g.scale_a.shape[1]):
            ks = slice(kb * 128, (kb + 1) * 128)
            y_ref += sa[:, kb] * (A[:, ks] @ (Bm[:, ks].T @ (sb[:, kb] * v)))
            z_ref += sb[:, kb] * (((u * sa[:, kb]) @ A[:, ks]) @ Bm[:, ks].T)
    y, z = c @ v, u @ c
    for blk in range(0, M, 256):
        assert np.linalg.norm(y[blk:blk + 256] - y_ref[blk:blk + 256]) <= tol * np.linalg.norm(c[blk:blk + 256])
    for blk in range(0, N, 256):
        assert np.linalg.norm(z[blk:blk + 256] - z_ref[blk:blk + 256]) <= tol * np.linalg.norm(c[:, blk:blk + 256])
    # (with random signs the rounding errors of a row add in quadrature, so the projection error of a
    #  correct result is about the element-wise relative error times the block's Frobenius norm)
    assert np.linalg.norm(y - y_ref) <= tol / 2 * np.linalg.norm(c)


@pytest.mark.parametrize("which", ["config4", "chained_256", "fp8"])
def test_gemm_is_bitwise_repeatable(which):
    """The kernels are deterministic: many launches on the same buffers give the same bits every time
    (each launch into a cleared C).  Guards the padding of the asm-issued buffer instructions: without it
    a store now and then used a stale scalar offset and landed on a neighbouring fragment."""
    if which == "config4":
        g, kw = W.config4(), dict(device_axis=True)
    elif which == "chained_256":
        g, kw = W.gemm_bf16(4352, 4096, 512, 91), {}
    else:
        g, kw = W.gemm_fp8(4352, 4096, 1024, 95, scaled=True), {}
    As, Bs, Cs = W.gemm_specs(g, shard=3, **kw)
    axes = ["m", "gpuid"]
    dA, dB = dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))
    dC = torch.zeros(g.M * g.N, dtype=torch.int16, device="cuda")
    sa = torch.from_numpy(g.scale_a).cuda() if g.scale_a is not None else None
    sb = torch.from_numpy(g.scale_b).cuda() if g.scale_b is not None else None
    desc = B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16 if g.dtype == "bf16" else B.AXE_FP8_E4M3, B.AXE_BF16,
                      B.Layout(As, axes), B.Layout(Bs, axes), B.Layout(Cs, axes), g.M * g.K, g.N * g.K, g.M * g.N, sa, sb)
    first = None
    for it in range(40):
        dC.zero_()
        B.axe_gemm(desc, dA, dB, dC)
        if first is None:
            first = dC.clone()
        else:
            assert torch.equal(first, dC), f"launch {it} differs from launch 0 in {(first != dC).sum().item()} elements"


# ----------------------------------------------------------------------------- grouped GEMM (MoE)
SENTINEL = 0x7FC1          # a NaN pattern in bf16 and in binary16: rows of C that belong to no group must keep it


def run_grouped(g: W.GroupedGemmInputs, lda=None, ldb=None, ldg=None, ldc=None, rows_on_device=None, kernel=B.AXE_GROUPED_TILES_256):
    """Launches axe_gemm_grouped; returns (C decoded to fp64, raw C words), both (M, N)."""
    lda_, ldb_, ldc_ = lda or g.K, ldb or g.K, ldc or g.N
    ldg_ = ldg or g.N * ldb_
    As, Bs, Cs = W.grouped_gemm_specs(g, lda_, ldb_, ldg_, ldc_)
    a = np.zeros((g.M, lda_), dtype=np.uint16); a[:, :g.K] = g.a_mk
    b = np.zeros((g.G, ldg_), dtype=np.uint16)
    bv = np.zeros((g.G, g.N, ldb_), dtype=np.uint16); bv[:, :, :g.K] = g.b_gnk
    b[:, :g.N * ldb_] = bv.reshape(g.G, -1)
    dA, dB = dev(a.reshape(-1)), dev(b.reshape(-1))
    dC = torch.full((g.M * ldc_,), SENTINEL, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(np.ascontiguousarray(g.group_rows if rows_on_device is None else rows_on_device, dtype=np.int32)).cuda()
    desc = B.GroupedGemmDesc(g.M, g.N, g.K, g.G, B.Layout(As), B.Layout(Bs), B.Layout(Cs), a.size, b.size, g.M * ldc_,
                             in_dtype=IN_DT[g.dtype], out_dtype=OUT_DT[g.dtype], kernel_hint=kernel)
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy().view(np.uint16).reshape(g.M, ldc_)
    if ldc_ > g.N:
        assert (raw[:, g.N:] == SENTINEL).all(), "the padding of C was written"
    raw = raw[:, :g.N]
    return decode16(raw, g.dtype), raw


def check_grouped(g: W.GroupedGemmInputs, c, raw, ref):
    """ref: the oracle's (M, N) with NaN rows where no group owns the row."""
    owned = ~np.isnan(ref[:, 0])
    assert (raw[~owned] == SENTINEL).all(), "a row outside every group was written"
    assert np.isfinite(c[owned]).all()
    if not owned.any():
        return
    assert R.rel_frobenius(c[owned], ref[owned]) <= BF16_TOL
    off = g.group_rows
    for e in range(g.G):                                   # every group, every 128 x 128 block of it: no tile can hide
        for i in range(off[e], off[e + 1], 128):
            for j in range(0, g.N, 128):
                blk = (slice(i, min(i + 128, off[e + 1])), slice(j, j + 128))
                err = R.rel_frobenius(c[blk], ref[blk])
                assert err <= BF16_TOL, f"group {e} rows {i} columns {j}: {err:.3e}"


GROUPED_CASES = [
    # (group_rows, N, K, M)   M None = group_rows[-1]
    ([0, 256], 256, 64, None),                             # one full tile, one K-step
    ([0, 1], 256, 128, None),                              # a single row
    ([0, 100, 100, 357, 400], 512, 192, None),             # an empty group, ragged sizes, odd number of K-steps
    ([3, 130, 700, 701], 256, 256, 720),                   # rows below the first and above the last group stay untouched
    ([0, 0, 0], 256, 64, 8),                               # nothing to do at all
    ([0, 300, 520, 1300, 1301, 2000], 768, 512, None),     # chained launch (8 K-steps), several tiles per group
]


KERNELS = [B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128, B.AXE_GROUPED_STREAM]


@pytest.mark.parametrize("kernel", KERNELS)
@pytest.mark.parametrize("off,N,K,M", GROUPED_CASES)
def test_gemm_grouped_small_cases(off, N, K, M, kernel):
    g = W.gemm_grouped_bf16(off, N, K, 77, M=M)
    c, raw = run_grouped(g, kernel=kernel)
    ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16)
    check_grouped(g, c, raw, ref)


@pytest.mark.parametrize("kernel", KERNELS)
def test_gemm_grouped_pitched_operands_and_many_groups(kernel):
    rng = np.random.default_rng(5)
    sizes = rng.integers(0, 90, 150)                       # 150 groups: three 64-group chunks in the kernel's tile search
    off = np.concatenate([[0], np.cumsum(sizes)])
    g = W.gemm_grouped_bf16(off, 256, 128, 78)
    c, raw = run_grouped(g, lda=136, ldb=144, ldg=256 * 144 + 64, ldc=264, kernel=kernel)
    ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16)
    check_grouped(g, c, raw, ref)


def test_gemm_grouped_offsets_out_of_range_are_clamped():
    """Whatever the device-side offsets hold, nothing outside the buffers is touched: entries are clamped to
    [0, M].  With clamped values that still increase, the result is that of the clamped offsets."""
    off_dev = [-5, 100, 300, 10 ** 6]
    off_eff = [0, 100, 300, 400]
    g = W.gemm_grouped_bf16(off_eff, 256, 128, 79)
    for kernel in KERNELS:
        c, raw = run_grouped(g, rows_on_device=off_dev, kernel=kernel)
        check_grouped(g, c, raw, R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off_eff, R.AXE_BF16))
    c, raw = run_grouped(g, rows_on_device=off_dev)
    ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off_eff, R.AXE_BF16)
    check_grouped(g, c, raw, ref)


_MOE_FULL = {}


def moe_full_size_case(which):
    """Inputs and the oracle's whole result for one grouped GEMM of the layer at 4096 tokens (computed once per session)."""
    if which not in _MOE_FULL:
        g = (W.moe_gemm1 if which == "gemm1" else W.moe_gemm2)(4096)
        _MOE_FULL[which] = (g, R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), g.group_rows, R.AXE_BF16))
    return _MOE_FULL[which]


@pytest.mark.parametrize("kernel", [B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128])
@pytest.mark.parametrize("which", ["gemm1", "gemm2"])
def test_gemm_grouped_moe_layer_shapes_full_size(which, kernel):
    """The two grouped GEMMs of the MoE layer at 4096 tokens (32768 routed rows, 128 experts), in the launch
    configuration the benchmark times, against the oracle's whole result: every group, every 128-column block."""
    g, ref = moe_full_size_case(which)
    c, raw = run_grouped(g, kernel=kernel)
    check_grouped(g, c, raw, ref)


# ----------------------------------------------------------------------------- blocked (pre-tiled) operands
def run_gemm_blocked(g: W.GemmInputs, a_blocked: bool, b_blocked: bool):
    """bf16 GEMM whose operands are stored as contiguous 256 x 64 blocks (images built with NumPy
    reshape / transpose, layouts stated as tile products); returns C decoded to fp64."""
    As = W.blocked_a_spec(g.M, g.K) if a_blocked else W.row_major_spec(g.M, g.K)
    Bs = W.blocked_b_spec(g.K, g.N) if b_blocked else W.col_major_spec(g.K, g.N)
    a = pack_blocked(g.a_mk) if a_blocked else g.a_mk.reshape(-1)
    b = pack_blocked(g.b_nk) if b_blocked else g.b_nk.reshape(-1)
    dA, dB = dev(a), dev(b)
    dC = torch.zeros(g.M * g.N, dtype=torch.int16, device="cuda")
    desc = B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16, B.AXE_BF16, B.Layout(As), B.Layout(Bs), B.Layout(W.row_major_spec(g.M, g.N)),
                      a.size, b.size, g.M * g.N, tile_hint=B.AXE_TILE_256x256x64)
    assert B.axe_gemm_tile(desc) == B.AXE_TILE_256x256x64
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    return R.bf16_to_f64(dC.cpu().numpy().view(np.uint16).reshape(g.M, g.N))


@pytest.mark.parametrize("M,N,K", [(256, 256, 64), (512, 768, 192), (768, 256, 1024), (4352, 4096, 512)])
@pytest.mark.parametrize("a_blocked,b_blocked", [(True, True), (True, False), (False, True)])
def test_gemm_bf16_blocked_operands(M, N, K, a_blocked, b_blocked):
    g = W.gemm_bf16(M, N, K, 91, std_b=K ** -0.5)
    c = run_gemm_blocked(g, a_blocked, b_blocked)
    check_gemm(c, oracle_gemm(g), BF16_TOL)
    if M * N * K > 1 << 28:                                 # the chained launch (17 x 16 tiles): also bit-identical to the plain layout
        assert np.array_equal(c, run_gemm(g))


def test_gemm_grouped_blocked_right_hand_sides():
    off = [0, 300, 520, 1300, 1301, 2000]
    g = W.gemm_grouped_bf16(off, 768, 512, 92)
    As, _, Cs = W.grouped_gemm_specs(g)
    b = pack_blocked(g.b_gnk)                              # (G, N * K): each group's image, one after the other
    dA, dB = dev(g.a_mk.reshape(-1)), dev(b.reshape(-1))
    dC = torch.full((g.M * g.N,), SENTINEL, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(g.group_rows).cuda()
    desc = B.GroupedGemmDesc(g.M, g.N, g.K, g.G, B.Layout(As), B.Layout(W.blocked_b_spec(g.K, g.N, G=g.G)), B.Layout(Cs),
                             g.a_mk.size, b.size, g.M * g.N)
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy().view(np.uint16).reshape(g.M, g.N)
    ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16)
    check_grouped(g, R.bf16_to_f64(raw), raw, ref)
    # and bit-identical to the launch on the plain layout (same kernel, same order of operations)
    _, raw_plain = run_grouped(g)
    assert np.array_equal(raw, raw_plain)


def test_relayout_produces_the_blocked_operand_layout():
    """The blocked image the GEMM reads is what axe_relayout writes from the plain one (weight pre-packing)."""
    K, N = 512, 768
    b_nk = W.to_bf16_bits(W.normal(93, (N, K)))
    Ls, Ld = B.Layout(W.col_major_spec(K, N)), B.Layout(W.blocked_b_spec(K, N))
    src, dst = dev(b_nk.reshape(-1)), torch.zeros(N * K, dtype=torch.int16, device="cuda")
    B.axe_relayout(Ls, Ld, (K, N), src, dst)
    torch.cuda.synchronize()
    assert np.array_equal(dst.cpu().numpy().view(np.uint16), pack_blocked(b_nk))


@pytest.mark.parametrize("eb,blocked", [(2, False), (2, True), (1, False)])
def test_relayout_produces_the_gate_up_interleaved_layouts(eb, blocked):
    """What the gated epilogue reads -- each group's gate and up rows interleaved in runs of 16, plain or in 256 x 64
    blocks -- is what axe_relayout writes from the plain (G, K, N) image, for 2-byte and 1-byte (fp8) elements."""
    G, K, N = 3, 256, 512
    rng = np.random.default_rng(95)
    b_gnk = rng.integers(0, 256 ** eb, (G, N, K)).astype(np.uint16 if eb == 2 else np.uint8)
    Ls = B.Layout(W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")]))
    Ld = B.Layout(W.gated_b_spec(K, N, G, blocked))
    src = dev(b_gnk.reshape(-1))
    dst = torch.zeros_like(src)
    B.axe_relayout(Ls, Ld, (G, K, N), src, dst)
    torch.cuda.synchronize()
    img = pack_gate_up(b_gnk)
    img = pack_blocked(img) if blocked else img
    assert np.array_equal(dst.cpu().numpy().view(b_gnk.dtype), img.reshape(-1))


@pytest.mark.parametrize("kernel", [B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128])
@pytest.mark.parametrize("blocked", [False, True])
@pytest.mark.parametrize("off,N,K", [([0, 300, 520, 1300, 1301, 2000], 768, 512), ([5, 6, 6, 270], 256, 192)])
def test_gemm_grouped_gated_epilogue(off, N, K, blocked, kernel):
    """First group GEMM of the MoE layer with the gated activation fused: C = silu(A Wg) * (A Wu), (M, N / 2)."""
    M = off[-1] + 3
    g = W.gemm_grouped_bf16(off, N, K, 94, M=M, std_b=2.0 * K ** -0.5)      # products of a few units: silu is well off its linear part
    img = pack_gate_up(g.b_gnk)
    img = pack_blocked(img) if blocked else img
    dA, dB = dev(g.a_mk.reshape(-1)), dev(img.reshape(-1))
    dC = torch.full((M * (N // 2),), SENTINEL, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(g.group_rows).cuda()
    desc = B.GroupedGemmDesc(M, N, K, g.G, B.Layout(W.row_major_spec(M, K)), B.Layout(W.gated_b_spec(K, N, g.G, blocked)),
                             B.Layout(W.row_major_spec(M, N // 2)), M * K, img.size, M * (N // 2), epilogue=B.AXE_EPI_SWIGLU,
                             kernel_hint=kernel)
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy().view(np.uint16).reshape(M, N // 2)
    ref = R.swiglu_ref(R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16))
    g_half = W.GroupedGemmInputs(M, N // 2, K, g.G, g.a_mk, g.b_gnk, g.group_rows)
    check_grouped(g_half, R.bf16_to_f64(raw), raw, ref)


def test_gemm_grouped_gated_moe_layer_full_size():
    """gemm1 of the layer at 4096 tokens with the fused activation, blocked weights (what the benchmark times);
    the oracle computes sampled groups and the rows at group borders."""
    g = W.moe_gemm1(4096)
    I = g.N // 2
    img = pack_blocked(pack_gate_up(g.b_gnk))
    dA, dB = dev(g.a_mk.reshape(-1)), dev(img.reshape(-1))
    dC = torch.full((g.M * I,), SENTINEL, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(g.group_rows).cuda()
    desc = B.GroupedGemmDesc(g.M, g.N, g.K, g.G, B.Layout(W.row_major_spec(g.M, g.K)), B.Layout(W.gated_b_spec(g.K, g.N, g.G, True)),
                             B.Layout(W.row_major_spec(g.M, I)), g.M * g.K, img.size, g.M * I, epilogue=B.AXE_EPI_SWIGLU)
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    c = R.bf16_to_f64(dC.cpu().numpy().view(np.uint16).reshape(g.M, I))
    assert np.isfinite(c).all()
    off, bl = g.group_rows, g.b_gnk.transpose(0, 2, 1)
    sizes = np.diff(off)
    rng = np.random.default_rng(12)
    for e in sorted({int(np.argmax(sizes)), int(np.argmin(sizes)), 0, g.G - 1, int(rng.integers(g.G))}):
        rows = np.arange(off[e], off[e + 1])[:300]
        j = int(rng.integers(I // 64)) * 64
        cols = np.concatenate([np.arange(j, j + 64), I + np.arange(j, j + 64)])        # the gate and up columns of 64 outputs
        ref = R.swiglu_ref(R.gemm_ref(g.a_mk, bl[e], R.AXE_BF16, rows=rows, cols=cols))
        err = R.rel_frobenius(c[np.ix_(rows, np.arange(j, j + 64))], ref)
        assert err <= BF16_TOL, f"group {e} columns {j}: {err:.3e}"
    edge = np.unique(np.concatenate([off[:-1][sizes > 0], off[1:][sizes > 0] - 1]))
    ref = R.swiglu_ref(R.gemm_grouped_ref(g.a_mk, bl, off, R.AXE_BF16, rows=edge))
    assert R.rel_frobenius(c[edge], ref) <= BF16_TOL
    # every 256-row block of every group against a cheap fp64 bound: |h| <= |gate| |up| is no check of values,
    # so instead compare one random column per block with the oracle
    cols1 = np.array([int(rng.integers(I))])
    for e in range(0, g.G, 7):
        if sizes[e]:
            rows = np.arange(off[e], off[e + 1])
            ref = R.swiglu_ref(R.gemm_ref(g.a_mk, bl[e], R.AXE_BF16, rows=rows, cols=np.array([cols1[0], I + cols1[0]])))
            assert R.rel_frobenius(c[np.ix_(rows, cols1)], ref) <= 2 * BF16_TOL, e


# ----------------------------------------------------------------------------- HIP graph capture
def test_entry_points_can_be_captured_in_a_hip_graph():
    """A serving loop records its launches once and replays them.  The library allocates nothing, clears
    nothing with memset and never synchronises, so a chain relayout -> grouped GEMM (gated) -> grouped GEMM ->
    dense GEMM can be captured; every replay must reproduce the eager result bit for bit, with the program's own
    eager work and synchronisations in between and with the inputs (group sizes included) changed between replays."""
    tokens_rows = [[0, 300, 520, 1300, 1301, 2000], [0, 0, 700, 701, 1500, 1800]]
    N1, K1, N2 = 512, 256, 256                                  # expert: K1 -> N1 / 2 (gated) -> N2
    G, M = 5, 2000
    g1 = W.gemm_grouped_bf16(tokens_rows[0], N1, K1, 95)
    w2 = W.to_bf16_bits(W.normal(96, (G, N2, N1 // 2), (N1 // 2) ** -0.5))
    dense_b = W.to_bf16_bits(W.normal(97, (256, N2), N2 ** -0.5))            # (N, K) image of a 256-column dense GEMM
    dA = dev(g1.a_mk.reshape(-1))
    dW1 = dev(g1.b_gnk.reshape(-1))
    dW1p = torch.zeros_like(dW1)
    dW2 = dev(w2.reshape(-1))
    dBd = dev(dense_b.reshape(-1))
    dR = torch.from_numpy(g1.group_rows).cuda()
    dH = torch.zeros(M * (N1 // 2), dtype=torch.int16, device="cuda")
    dY = torch.zeros(M * N2, dtype=torch.int16, device="cuda")
    Mp = 2048                                                   # the dense GEMM reads Y padded to a multiple of 256 rows
    dYp = torch.zeros(Mp * N2, dtype=torch.int16, device="cuda")
    dZ = torch.zeros(Mp * 256, dtype=torch.int16, device="cuda")
    plain1 = B.Layout(W.spec([(G, N1 * K1, "m"), (K1, 1, "m"), (N1, K1, "m")]))
    gated1 = B.Layout(W.gated_b_spec(K1, N1, G, blocked=True))
    d1 = B.GroupedGemmDesc(M, N1, K1, G, B.Layout(W.row_major_spec(M, K1)), gated1, B.Layout(W.row_major_spec(M, N1 // 2)),
                           M * K1, dW1.numel(), M * (N1 // 2), epilogue=B.AXE_EPI_SWIGLU)
    g2 = W.GroupedGemmInputs(M, N2, N1 // 2, G, None, w2, g1.group_rows)
    As2, Bs2, Cs2 = W.grouped_gemm_specs(g2)
    d2 = B.GroupedGemmDesc(M, N2, N1 // 2, G, B.Layout(As2), B.Layout(Bs2), B.Layout(Cs2), M * (N1 // 2), dW2.numel(), M * N2)
    d3 = B.GemmDesc(Mp, 256, N2, B.AXE_BF16, B.AXE_BF16, B.Layout(W.row_major_spec(Mp, N2)), B.Layout(W.col_major_spec(N2, 256)),
                    B.Layout(W.row_major_spec(Mp, 256)), Mp * N2, dBd.numel(), Mp * 256)

    def chain():
        B.axe_relayout(plain1, gated1, (G, K1, N1), dW1, dW1p)
        B.axe_gemm_grouped(d1, dA, dW1p, dH, dR)
        B.axe_gemm_grouped(d2, dH, dW2, dY, dR)
        dYp[:M * N2].copy_(dY)
        B.axe_gemm(d3, dYp, dBd, dZ)

    def eager(rows, a_words):
        dR.copy_(torch.from_numpy(np.asarray(rows, dtype=np.int32)))
        dA.copy_(dev(a_words.reshape(-1)))
        for t in (dH, dY, dYp, dZ, dW1p):
            t.zero_()
        chain()
        torch.cuda.synchronize()
        return dH.clone(), dY.clone(), dZ.clone()

    inputs = [(tokens_rows[0], g1.a_mk), (tokens_rows[1], np.roll(g1.a_mk, 17, axis=0)), (tokens_rows[0], np.roll(g1.a_mk, 5, axis=1))]
    want = [eager(r, a) for r, a in inputs]
    assert not torch.equal(want[0][1], want[1][1])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                               # warm-up on the capture stream, as torch asks for
        chain()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        chain()
    for rep in range(2):
        for (rows, a_words), (h, y, z) in zip(inputs, want):
            dR.copy_(torch.from_numpy(np.asarray(rows, dtype=np.int32)))
            dA.copy_(dev(a_words.reshape(-1)))
            for t in (dH, dY, dYp, dZ, dW1p):
                t.zero_()
            scratch = torch.randn(1 << 20, device="cuda").sum().item()       # eager work and a synchronisation between replays
            graph.replay()
            torch.cuda.synchronize()
            assert torch.equal(dH, h) and torch.equal(dY, y) and torch.equal(dZ, z), (rep, rows)


# ----------------------------------------------------------------------------- IEEE binary16 (the paper's MoE layer is an FP16 layer)
F16_TOL = 2e-3            # output rounding 2^-12 / sqrt(3) dominates (bf16: 2^-9 / sqrt(3)); a correct kernel lands near 2e-4


@pytest.mark.parametrize("M,N,K,out", [(64, 64, 32, "f16"), (200, 136, 96, "f32"), (65, 63, 8, "f16"), (256, 256, 64, "f16"),
                                       (512, 768, 192, "f16"), (768, 256, 1024, "f16")])
def test_gemm_f16(M, N, K, out):
    g = W.gemm_f16(M, N, K, 98, std_b=K ** -0.5, out_dtype=out)
    c = run_gemm(g)
    check_gemm(c, oracle_gemm(g), F16_TOL)


def test_gemm_f16_chained_and_blocked():
    g = W.gemm_f16(4352, 4096, 512, 99, std_b=512 ** -0.5)
    c = run_gemm(g)
    rows = np.array([0, 255, 256, 4351])
    assert R.rel_frobenius(c[rows], oracle_gemm(g, rows, None)) <= F16_TOL
    cols = np.array([0, 4095])
    assert R.rel_frobenius(c[:, cols], oracle_gemm(g, None, cols)) <= F16_TOL
    # blocked operands: same kernel, same order of operations, same bits
    dA, dB = dev(pack_blocked(g.a_mk)), dev(pack_blocked(g.b_nk))
    dC = torch.zeros(g.M * g.N, dtype=torch.int16, device="cuda")
    desc = B.GemmDesc(g.M, g.N, g.K, B.AXE_F16, B.AXE_F16, B.Layout(W.blocked_a_spec(g.M, g.K)), B.Layout(W.blocked_b_spec(g.K, g.N)),
                      B.Layout(W.row_major_spec(g.M, g.N)), g.M * g.K, g.N * g.K, g.M * g.N)
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    assert np.array_equal(R.f16_to_f64(dC.cpu().numpy().view(np.uint16).reshape(g.M, g.N)), c)


def test_gemm_grouped_f16_plain_and_gated():
    off = [0, 300, 520, 1300, 1301, 2000]
    N, K = 768, 512
    g = W.gemm_grouped_bf16(off, N, K, 100, std_b=2.0 * K ** -0.5, dtype="f16")
    bl = g.b_gnk.transpose(0, 2, 1)
    P = R.gemm_grouped_ref(g.a_mk, bl, off, R.AXE_F16)
    owned = ~np.isnan(P[:, 0])
    for kernel in KERNELS:
        c, raw = run_grouped(g, kernel=kernel)
        assert R.rel_frobenius(c[owned], P[owned]) <= F16_TOL, kernel
        check_grouped(g, c, raw, P)
    # gated
    img = pack_blocked(pack_gate_up(g.b_gnk))
    dA, dB = dev(g.a_mk.reshape(-1)), dev(img.reshape(-1))
    dC = torch.full((g.M * (N // 2),), SENTINEL, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(g.group_rows).cuda()
    desc = B.GroupedGemmDesc(g.M, N, K, g.G, B.Layout(W.row_major_spec(g.M, K)), B.Layout(W.gated_b_spec(K, N, g.G, True)),
                             B.Layout(W.row_major_spec(g.M, N // 2)), g.M * K, img.size, g.M * (N // 2),
                             in_dtype=B.AXE_F16, out_dtype=B.AXE_F16, epilogue=B.AXE_EPI_SWIGLU)
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    h = R.f16_to_f64(dC.cpu().numpy().view(np.uint16).reshape(g.M, N // 2))
    assert R.rel_frobenius(h[owned], R.swiglu_ref(P)[owned]) <= F16_TOL


# ----------------------------------------------------------------------------- grouped GEMM, few rows per group (decode)
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
@pytest.mark.parametrize("gated,blocked", [(False, False), (False, True), (True, False), (True, True)])
@pytest.mark.parametrize("sizes", [[1, 0, 16, 17, 33, 64, 65, 70, 3, 48],                  # 64 rows per pass
                                   [1, 0, 16, 17, 33, 9, 40, 0, 3, 20, 2, 12]])            # a dozen per group: 32 per pass, K split
def test_gemm_grouped_stream_kernel_variants(dtype, gated, blocked, sizes):
    """The streaming kernel on ragged small groups (1 .. 70 rows: up to two passes of 64 rows, or of 32, every number
    of row fragments), plain and gated, plain and blocked weights, bf16 and fp16."""
    off = np.concatenate([[0], np.cumsum(sizes)])
    N, K = 512, 320
    g = W.gemm_grouped_bf16(off, N, K, 101, M=int(off[-1]) + 2, std_b=2.0 * K ** -0.5, dtype=dtype)
    odt, tol = ORACLE_DT[dtype], (F16_TOL if dtype == "f16" else BF16_TOL)
    ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, odt)
    img = pack_gate_up(g.b_gnk) if gated else g.b_gnk
    Kp = 384                                                 # K = 320 is no multiple of the K-tile: pad with zeros
    a_words = np.zeros((g.M, Kp), dtype=np.uint16); a_words[:, :K] = g.a_mk
    b_p = np.zeros((g.G, N, Kp), dtype=np.uint16); b_p[:, :, :K] = img
    img = pack_blocked(b_p) if blocked else b_p
    if gated:
        Bs = W.gated_b_spec(Kp, N, g.G, blocked)
    else:
        Bs = W.blocked_b_spec(Kp, N, G=g.G) if blocked else W.spec([(g.G, N * Kp, "m"), (Kp, 1, "m"), (N, Kp, "m")])
    NC = N // 2 if gated else N
    dA, dB = dev(a_words.reshape(-1)), dev(img.reshape(-1))
    dC = torch.full((g.M * NC,), SENTINEL, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(g.group_rows).cuda()
    desc = B.GroupedGemmDesc(g.M, N, Kp, g.G, B.Layout(W.row_major_spec(g.M, Kp)), B.Layout(Bs), B.Layout(W.row_major_spec(g.M, NC)),
                             a_words.size, img.size, g.M * NC, in_dtype=IN_DT[dtype], out_dtype=OUT_DT[dtype],
                             epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, kernel_hint=B.AXE_GROUPED_STREAM)
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy().view(np.uint16).reshape(g.M, NC)
    want = R.swiglu_ref(ref) if gated else ref
    owned = ~np.isnan(want[:, 0])
    assert (raw[~owned] == SENTINEL).all()
    c = decode16(raw, dtype)
    assert np.isfinite(c[owned]).all()
    assert R.rel_frobenius(c[owned], want[owned]) <= tol
    for e in range(g.G):
        if sizes[e]:
            for j in range(0, NC, 64):
                blk = (slice(off[e], off[e + 1]), slice(j, j + 64))
                assert R.rel_frobenius(c[blk], want[blk]) <= tol, (e, j)


@pytest.mark.parametrize("tokens", [1, 8, 64])
def test_gemm_grouped_moe_layer_at_decode_sizes(tokens):
    """Both grouped GEMMs of the layer at decode batch sizes through the kernel the library picks itself (streaming),
    blocked weights, gated first GEMM: the whole result against the oracle."""
    g1, g2 = W.moe_gemm1(tokens), W.moe_gemm2(tokens)
    I = g1.N // 2
    for g, gated in ((g1, True), (g2, False)):
        img = pack_blocked(pack_gate_up(g.b_gnk) if gated else g.b_gnk)
        NC = I if gated else g.N
        Bs = W.gated_b_spec(g.K, g.N, g.G, True) if gated else W.blocked_b_spec(g.K, g.N, G=g.G)
        dA, dB = dev(g.a_mk.reshape(-1)), dev(img.reshape(-1))
        dC = torch.full((g.M * NC,), SENTINEL, dtype=torch.int16, device="cuda")
        dR = torch.from_numpy(g.group_rows).cuda()
        desc = B.GroupedGemmDesc(g.M, g.N, g.K, g.G, B.Layout(W.row_major_spec(g.M, g.K)), B.Layout(Bs), B.Layout(W.row_major_spec(g.M, NC)),
                                 g.M * g.K, img.size, g.M * NC, epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE)
        B.axe_gemm_grouped(desc, dA, dB, dC, dR)
        torch.cuda.synchronize()
        c = R.bf16_to_f64(dC.cpu().numpy().view(np.uint16).reshape(g.M, NC))
        ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), g.group_rows, R.AXE_BF16)
        ref = R.swiglu_ref(ref) if gated else ref
        assert np.isfinite(c).all() and not np.isnan(ref).any()
        assert R.rel_frobenius(c, ref) <= BF16_TOL
        for r in range(0, g.M, 16):
            assert R.rel_frobenius(c[r:r + 16], ref[r:r + 16]) <= BF16_TOL, r


def test_gemm_grouped_stream_kernel_many_empty_groups_and_passes_of_16_rows():
    """Few rows in all (M <= 4 G): the variant that takes a group 16 rows at a time; groups of 40 and 17 rows need
    several passes, most groups are empty."""
    sizes = np.zeros(40, dtype=np.int64)
    sizes[[0, 7, 8, 31, 39]] = [40, 17, 1, 16, 3]
    off = np.concatenate([[0], np.cumsum(sizes)])
    g = W.gemm_grouped_bf16(off, 512, 448, 102)
    assert g.M <= 4 * g.G
    c, raw = run_grouped(g, kernel=B.AXE_GROUPED_STREAM)
    check_grouped(g, c, raw, R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16))


@pytest.mark.parametrize("scale_dtype", ["f32", "e8m0"])
@pytest.mark.parametrize("M,N,K", [(130, 256, 384), (256, 128, 1024), (70, 72, 272)])
def test_gemm_fp8_row_scaled_activations(M, N, K, scale_dtype):
    """One scale per row of A and 128-wide k block (the usual choice for activations), 128 x 128 blocks for B."""
    g = W.gemm_fp8(M, N, K, 103, scaled="e8m0" if scale_dtype == "e8m0" else True)
    rng = np.random.default_rng(3)
    nkb = (K + 127) // 128
    if scale_dtype == "e8m0":
        sa_rows = rng.integers(124, 131, (M, nkb)).astype(np.uint8)
        sa_oracle, sb_oracle = R.e8m0_decode(sa_rows).astype(np.float32), R.e8m0_decode(g.scale_b).astype(np.float32)
    else:
        sa_rows = rng.uniform(0.5, 2.0, (M, nkb)).astype(np.float32)
        sa_oracle, sb_oracle = sa_rows, g.scale_b
    As, Bs, Cs = W.gemm_specs(g)
    dA, dB = dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))
    dC = torch.zeros(M * N, dtype=torch.int16, device="cuda")
    sa, sb = torch.from_numpy(sa_rows).cuda(), torch.from_numpy(g.scale_b).cuda()
    desc = B.GemmDesc(M, N, K, B.AXE_FP8_E4M3, B.AXE_BF16, B.Layout(As), B.Layout(Bs), B.Layout(Cs), M * K, N * K, M * N, sa, sb,
                      scale_dtype=B.AXE_SCALE_E8M0 if scale_dtype == "e8m0" else B.AXE_SCALE_F32, scale_a_rows=1)
    assert B.axe_gemm_tile(desc) == B.AXE_TILE_64x64x32
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    c = R.bf16_to_f64(dC.cpu().numpy().view(np.uint16).reshape(M, N))
    ref = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, sa_oracle, sb_oracle, block_m_a=1)
    assert R.rel_frobenius(c, ref) <= FP8_TOL
    for i in range(0, M, 16):                                # per 16 rows: a scale applied to the wrong row cannot hide
        assert R.rel_frobenius(c[i:i + 16], ref[i:i + 16]) <= FP8_TOL, i


# One E8M0 code per row of A on the 256 x 256 tile (the matrix cores' scale path): K = 1024 nw with nw = 1 (a single
# window of 8 K-tiles), 2, 3 (odd), 9 (more than 64 K-steps: B's code registers are refilled as well); one tile, several
# tiles, and 17 x 16 tiles (chained: the next tile's first window is fetched across the tile
# boundary).  The row codes differ from row to row and from k block to k block over a range of 2^11.
# K = 128, 768 and 1152: 1, 6 and 9 K-tiles -- a partial window of row codes only (its 8-byte reads run on into the next
# row and, for the last rows, start early at the end of the array), and a full window followed by a partial one.
# 8192 x 8192 x 2048: the tile grid and launch of configuration 5 (32 x 32 tiles, four chained per workgroup), two windows of codes.
@pytest.mark.parametrize("M,N,K", [(256, 256, 1024), (512, 768, 2048), (768, 512, 3072), (256, 512, 9216), (4352, 4096, 2048),
                                   (256, 256, 128), (512, 256, 768), (256, 512, 1152), (8192, 8192, 2048)])
def test_gemm_fp8_row_scaled_activations_large_tile(M, N, K):
    g = W.gemm_fp8(M, N, K, 107, scaled="e8m0")
    rng = np.random.default_rng(M + K)
    nkb = K // 128
    sa_rows = rng.integers(122, 133, (M, nkb)).astype(np.uint8)
    As, Bs, Cs = W.gemm_specs(g)
    dA, dB = dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))
    dC = torch.zeros(M * N, dtype=torch.int16, device="cuda")
    sa, sb = torch.from_numpy(sa_rows).cuda(), torch.from_numpy(g.scale_b).cuda()
    desc = B.GemmDesc(M, N, K, B.AXE_FP8_E4M3, B.AXE_BF16, B.Layout(As), B.Layout(Bs), B.Layout(Cs), M * K, N * K, M * N, sa, sb,
                      scale_dtype=B.AXE_SCALE_E8M0, scale_a_rows=1, tile_hint=B.AXE_TILE_256x256x64)
    assert B.axe_gemm_tile(desc) == B.AXE_TILE_256x256x64
    B.axe_gemm(desc, dA, dB, dC)
    torch.cuda.synchronize()
    c = R.bf16_to_f64(dC.cpu().numpy().view(np.uint16).reshape(M, N))
    ref = R.gemm_ref(g.a_mk, g.b_nk.T, R.AXE_FP8_E4M3, R.e8m0_decode(sa_rows).astype(np.float32),
                     R.e8m0_decode(g.scale_b).astype(np.float32), block_m_a=1)
    check_gemm(c, ref, FP8_TOL)
    for i in range(0, M, 16):                                # per 16 rows: a code applied to the wrong row cannot hide
        assert R.rel_frobenius(c[i:i + 16], ref[i:i + 16]) <= FP8_TOL, i
    # the same problem through the 64 x 64 kernel, which folds the row scales per lane: same result up to the last rounding
    desc2 = B.GemmDesc(M, N, K, B.AXE_FP8_E4M3, B.AXE_BF16, B.Layout(As), B.Layout(Bs), B.Layout(Cs), M * K, N * K, M * N, sa, sb,
                       scale_dtype=B.AXE_SCALE_E8M0, scale_a_rows=1, tile_hint=B.AXE_TILE_64x64x32)
    dC2 = torch.zeros(M * N, dtype=torch.int16, device="cuda")
    B.axe_gemm(desc2, dA, dB, dC2)
    torch.cuda.synchronize()
    assert R.rel_frobenius(R.bf16_to_f64(dC2.cpu().numpy().view(np.uint16).reshape(M, N)), c) < 4e-3


@pytest.mark.parametrize("kernel", KERNELS)
def test_gemm_grouped_largest_group_count(kernel):
    """4096 groups (the limit of the tile table's packing), most of them empty, a few large ones."""
    G = 4096
    rng = np.random.default_rng(6)
    sizes = np.zeros(G, dtype=np.int64)
    hot = rng.choice(G, 300, replace=False)
    sizes[hot] = rng.integers(1, 40, 300)
    sizes[[0, G - 1, 2047]] = [130, 257, 64]
    off = np.concatenate([[0], np.cumsum(sizes)])
    M, N, K = int(off[-1]), 256, 64
    a = W.to_bf16_bits(W.normal(104, (M, K)))
    base = W.to_bf16_bits(W.normal(105, (64, N, K), K ** -0.5))
    b = base[np.arange(G) % 64] ^ (np.arange(G, dtype=np.uint16) % 2 * 0x8000)[:, None, None]     # 64 distinct matrices, sign flipped per parity
    g = W.GroupedGemmInputs(M, N, K, G, a, np.ascontiguousarray(b), off.astype(np.int32))
    c, raw = run_grouped(g, kernel=kernel)
    ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16)
    assert np.isfinite(c).all() and R.rel_frobenius(c, ref) <= BF16_TOL
    for e in np.nonzero(sizes)[0]:
        assert R.rel_frobenius(c[off[e]:off[e + 1]], ref[off[e]:off[e + 1]]) <= BF16_TOL, e


def test_gemm_grouped_fewer_rows_than_groups():
    """Fewer rows than groups: the streaming kernel's launch has one workgroup row per possible non-empty group and
    finds the group by counting; groups at both ends, in different 64-group blocks, and a run of empty ones."""
    sizes = np.zeros(200, dtype=np.int64)
    sizes[[0, 63, 64, 77, 199]] = [1, 2, 1, 3, 1]
    off = np.concatenate([[0], np.cumsum(sizes)])
    g = W.gemm_grouped_bf16(off, 256, 192, 106)
    assert g.M < g.G
    for kernel in KERNELS:
        c, raw = run_grouped(g, kernel=kernel)
        check_grouped(g, c, raw, R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16))


# ----------------------------------------------------------------------------- fp8 grouped GEMM (decode sizes)
@pytest.mark.parametrize("scale_dtype", ["f32", "e8m0", None])
@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("sizes,hint", [([1, 0, 3, 16, 2, 0, 7, 1] * 4, B.AXE_GROUPED_AUTO),           # M <= 8 G: the split-K variant
                                        ([40, 0, 9, 33, 1, 17, 20, 0], B.AXE_GROUPED_STREAM),            # a dozen rows per group: split K, passes of 32 rows
                                        ([70, 0, 33, 64, 17], B.AXE_GROUPED_STREAM)])                    # passes of 64 rows
def test_gemm_grouped_fp8_block_scaled(sizes, hint, gated, scale_dtype):
    """e4m3 operands, one scale per row of A and k block, one per 128 x 128 block of each group's B (fp32 or E8M0), or none;
    plain and gated epilogue; both variants of the streaming kernel."""
    off = np.concatenate([[0], np.cumsum(sizes)])
    N, K = 512, 384
    g = W.gemm_grouped_fp8(off, N, K, 107, M=int(off[-1]) + 1, scale_dtype=scale_dtype or "f32")
    if scale_dtype is None:
        sa_o = sb_o = None
    elif scale_dtype == "e8m0":
        sa_o, sb_o = R.e8m0_decode(g.scale_a).astype(np.float32), R.e8m0_decode(g.scale_b).astype(np.float32)
    else:
        sa_o, sb_o = g.scale_a, g.scale_b
    ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_FP8_E4M3, scale_a=sa_o, scale_b=sb_o)
    if gated:
        ref = R.swiglu_ref(ref)
    img = pack_gate_up(g.b_gnk) if gated else g.b_gnk
    Bs = W.gated_b_spec(K, N, g.G) if gated else W.spec([(g.G, N * K, "m"), (K, 1, "m"), (N, K, "m")])
    NC = N // 2 if gated else N
    dA, dB = dev(g.a_mk.reshape(-1)), dev(img.reshape(-1))
    dC = torch.full((g.M * NC,), SENTINEL, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(g.group_rows).cuda()
    sa = torch.from_numpy(g.scale_a).cuda() if scale_dtype else None
    sb = torch.from_numpy(g.scale_b).cuda() if scale_dtype else None
    desc = B.GroupedGemmDesc(g.M, N, K, g.G, B.Layout(W.row_major_spec(g.M, K)), B.Layout(Bs), B.Layout(W.row_major_spec(g.M, NC)),
                             g.a_mk.size, img.size, g.M * NC, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_BF16,
                             epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, kernel_hint=hint, scale_a=sa, scale_b=sb,
                             scale_dtype=B.AXE_SCALE_E8M0 if scale_dtype == "e8m0" else B.AXE_SCALE_F32)
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    raw = dC.cpu().numpy().view(np.uint16).reshape(g.M, NC)
    owned = ~np.isnan(ref[:, 0])
    assert (raw[~owned] == SENTINEL).all()
    c = R.bf16_to_f64(raw)
    assert np.isfinite(c[owned]).all()
    assert R.rel_frobenius(c[owned], ref[owned]) <= FP8_TOL
    for e in range(g.G):
        if sizes[e]:
            for j in range(0, NC, 64):
                blk = (slice(off[e], off[e + 1]), slice(j, j + 64))
                assert R.rel_frobenius(c[blk], ref[blk]) <= FP8_TOL, (e, j)


# fp8 on the grouped TILE kernel (the matrix cores' scale path, tiles of 256 and of 128 rows): E8M0 scales (per row of A, per
# 128 x 128 block of each group's B) or none; plain and gated epilogue.  K = 768 (6 K-tiles: no full window of row codes,
# the row codes of a window end before 8 bytes are up -- also at the very end of the code array), 1152 (9: a full window
# and a partial one; odd, so one tile per workgroup), 2048 (16: two windows, chained tiles); groups from 1 to 700
# rows, empty groups, rows outside every group.
@pytest.mark.parametrize("tiles", [B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128])
@pytest.mark.parametrize("scale_dtype", ["e8m0", None])
@pytest.mark.parametrize("gated", [False, True])
@pytest.mark.parametrize("sizes,N,K", [([300, 0, 33, 256, 257, 1], 512, 768), ([70, 700, 5], 768, 1152), ([130, 512, 64, 0, 300, 2], 512, 2048)])
def test_gemm_grouped_fp8_tile_kernel(sizes, N, K, gated, scale_dtype, tiles):
    off = np.concatenate([[0], np.cumsum(sizes)])
    for M in (int(off[-1]) + 3, int(off[-1])):             # with and without rows behind the last group (the last row's codes end the array)
        g = W.gemm_grouped_fp8(off, N, K, 108 + K, M=M, scale_dtype=scale_dtype or "e8m0")
        if scale_dtype:
            g.scale_a = np.random.default_rng(K).integers(121, 134, g.scale_a.shape).astype(np.uint8)   # codes over a range of 2^12
        sa_o = R.e8m0_decode(g.scale_a).astype(np.float32) if scale_dtype else None
        sb_o = R.e8m0_decode(g.scale_b).astype(np.float32) if scale_dtype else None
        ref = R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_FP8_E4M3, scale_a=sa_o, scale_b=sb_o)
        if gated:
            ref = R.swiglu_ref(ref)
        img = pack_gate_up(g.b_gnk) if gated else g.b_gnk
        Bs = W.gated_b_spec(K, N, g.G) if gated else W.spec([(g.G, N * K, "m"), (K, 1, "m"), (N, K, "m")])
        NC = N // 2 if gated else N
        dA, dB = dev(g.a_mk.reshape(-1)), dev(img.reshape(-1))
        dC = torch.full((g.M * NC,), SENTINEL, dtype=torch.int16, device="cuda")
        dR = torch.from_numpy(g.group_rows).cuda()
        sa = torch.from_numpy(g.scale_a).cuda() if scale_dtype else None
        sb = torch.from_numpy(g.scale_b).cuda() if scale_dtype else None
        desc = B.GroupedGemmDesc(g.M, N, K, g.G, B.Layout(W.row_major_spec(g.M, K)), B.Layout(Bs), B.Layout(W.row_major_spec(g.M, NC)),
                                 g.a_mk.size, img.size, g.M * NC, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_BF16,
                                 epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, kernel_hint=tiles,
                                 scale_a=sa, scale_b=sb, scale_dtype=B.AXE_SCALE_E8M0)
        assert B.axe_gemm_grouped_kernel(desc) == tiles
        B.axe_gemm_grouped(desc, dA, dB, dC, dR)
        torch.cuda.synchronize()
        raw = dC.cpu().numpy().view(np.uint16).reshape(g.M, NC)
        owned = ~np.isnan(ref[:, 0])
        assert (raw[~owned] == SENTINEL).all(), "a row outside every group was written"
        c = R.bf16_to_f64(raw)
        assert np.isfinite(c[owned]).all()
        assert R.rel_frobenius(c[owned], ref[owned]) <= FP8_TOL
        for e in range(g.G):                                   # every group, every 16-row band and 64-column block of it
            for i in range(off[e], off[e + 1], 16):
                for j in range(0, NC, 64):
                    blk = (slice(i, min(i + 16, off[e + 1])), slice(j, j + 64))
                    assert R.rel_frobenius(c[blk], ref[blk]) <= FP8_TOL, (e, i, j)
        # the streaming kernel on the same problem: the same result up to the last rounding
        desc2 = B.GroupedGemmDesc(g.M, N, K, g.G, B.Layout(W.row_major_spec(g.M, K)), B.Layout(Bs), B.Layout(W.row_major_spec(g.M, NC)),
                                  g.a_mk.size, img.size, g.M * NC, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_BF16,
                                  epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, kernel_hint=B.AXE_GROUPED_STREAM,
                                  scale_a=sa, scale_b=sb, scale_dtype=B.AXE_SCALE_E8M0)
        dC2 = torch.full((g.M * NC,), SENTINEL, dtype=torch.int16, device="cuda")
        B.axe_gemm_grouped(desc2, dA, dB, dC2, dR)
        torch.cuda.synchronize()
        c2 = R.bf16_to_f64(dC2.cpu().numpy().view(np.uint16).reshape(g.M, NC))
        assert R.rel_frobenius(c2[owned], c[owned]) < 5e-3


@pytest.mark.parametrize("kernel,gated", [(B.AXE_GROUPED_TILES_256, False), (B.AXE_GROUPED_TILES_128, False), (B.AXE_GROUPED_TILES_128, True),
                                          (B.AXE_GROUPED_STREAM, False)])
def test_gemm_grouped_is_bitwise_repeatable(kernel, gated):
    """As for the dense kernels: 40 launches of the layer's first GEMM at 512 tokens give the same bits (the 128-row
    tile has its own schedule of asm-issued loads and counted waits; the streaming kernel adds partial sums in a fixed order)."""
    g = W.moe_gemm1(512)
    NC = g.N // 2 if gated else g.N
    img = pack_gate_up(g.b_gnk) if gated else g.b_gnk
    Bs = W.gated_b_spec(g.K, g.N, g.G) if gated else W.grouped_gemm_specs(g)[1]
    dA, dB = dev(g.a_mk.reshape(-1)), dev(img.reshape(-1))
    dC = torch.zeros(g.M * NC, dtype=torch.int16, device="cuda")
    dR = torch.from_numpy(g.group_rows).cuda()
    desc = B.GroupedGemmDesc(g.M, g.N, g.K, g.G, B.Layout(W.row_major_spec(g.M, g.K)), B.Layout(Bs), B.Layout(W.row_major_spec(g.M, NC)),
                             g.M * g.K, img.size, g.M * NC, epilogue=B.AXE_EPI_SWIGLU if gated else B.AXE_EPI_NONE, kernel_hint=kernel)
    first = None
    for it in range(40):
        dC.zero_()
        B.axe_gemm_grouped(desc, dA, dB, dC, dR)
        if first is None:
            first = dC.clone()
        else:
            assert torch.equal(first, dC), f"launch {it} differs from launch 0 in {(first != dC).sum().item()} elements"
    # and the result is the right one (one group, against the oracle)
    e = int(np.argmax(np.diff(g.group_rows)))
    rows = np.arange(g.group_rows[e], g.group_rows[e + 1])
    ref = R.gemm_ref(g.a_mk, g.b_gnk[e].T, R.AXE_BF16, rows=rows)
    ref = R.swiglu_ref(ref) if gated else ref
    c = R.bf16_to_f64(first.cpu().numpy().view(np.uint16).reshape(g.M, NC))[rows]
    assert R.rel_frobenius(c, ref) <= BF16_TOL


@pytest.mark.parametrize("dtype", ["f16", "fp8"])
def test_gated_grouped_gemm_keeps_its_bits_beside_a_busy_copy_stream(dtype):
    """The layer's first GEMM at 4096 tokens with the gated activation, launched while a large device copy of another
    stream saturates the memory pipeline: every launch gives the bits of the quiet launch.  (Regression: the gated
    epilogue computed the next fragment into the registers of the 16-byte store it had just issued as an asm statement;
    with the memory pipeline backed up the store now and then read four lanes of the new values.  Every asm-issued
    store is followed by wait states since.)"""
    rows = W.moe_group_rows(4096, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
    M, N, K, G = int(rows[-1]), 2 * W.MOE_INTER, W.MOE_HIDDEN, W.MOE_EXPERTS
    dR = torch.from_numpy(rows).cuda()
    if dtype == "f16":
        g = W.moe_gemm1(4096, dtype="f16")
        dA = dev(g.a_mk[:M].reshape(-1))
        dB = dev(pack_blocked(pack_gate_up(g.b_gnk)).reshape(-1))
        desc = B.GroupedGemmDesc(M, N, K, G, B.Layout(W.row_major_spec(M, K)), B.Layout(W.gated_b_spec(K, N, G, True)),
                                 B.Layout(W.row_major_spec(M, N // 2)), M * K, G * N * K, M * (N // 2), in_dtype=B.AXE_F16, out_dtype=B.AXE_F16,
                                 epilogue=B.AXE_EPI_SWIGLU)
    else:
        f = W.gemm_grouped_fp8(rows, N, K, W.SEED_BASE + 22, scale_dtype="e8m0")
        dA, dB = dev(f.a_mk[:M].reshape(-1)), dev(pack_gate_up(f.b_gnk).reshape(-1))
        sa, sb = torch.from_numpy(f.scale_a[:M]).cuda(), torch.from_numpy(f.scale_b).cuda()
        desc = B.GroupedGemmDesc(M, N, K, G, B.Layout(W.row_major_spec(M, K)), B.Layout(W.gated_b_spec(K, N, G)),
                                 B.Layout(W.row_major_spec(M, N // 2)), M * K, G * N * K, M * (N // 2), in_dtype=B.AXE_FP8_E4M3,
                                 out_dtype=B.AXE_BF16, epilogue=B.AXE_EPI_SWIGLU, scale_a=sa, scale_b=sb, scale_dtype=B.AXE_SCALE_E8M0)
    dC = torch.zeros(M * (N // 2), dtype=torch.int16, device="cuda")
    B.axe_gemm_grouped(desc, dA, dB, dC, dR)
    torch.cuda.synchronize()
    quiet = dC.clone()
    side = torch.cuda.Stream()
    big_a = torch.empty(1 << 28, dtype=torch.uint8, device="cuda")
    big_b = torch.empty_like(big_a)
    for it in range(60):
        dC.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(side):
            big_b.copy_(big_a)
        B.axe_gemm_grouped(desc, dA, dB, dC, dR)
        torch.cuda.synchronize()
        assert torch.equal(dC, quiet), f"launch {it}: {(dC != quiet).sum().item()} elements differ from the quiet launch"


@pytest.mark.parametrize("G,N,lo,hi", [(2, 512, 40, 71),      # few groups: K split over waves, 64 rows per pass
                                       (1, 256, 17, 18),      # one group = a dense GEMM with few rows
                                       (300, 256, 0, 41)])    # many groups of a few dozen rows: whole-K waves
def test_gemm_grouped_stream_kernel_choice_by_launch_size(G, N, lo, hi):
    rng = np.random.default_rng(G)
    sizes = rng.integers(lo, hi, G)
    off = np.concatenate([[0], np.cumsum(sizes)])
    g = W.gemm_grouped_bf16(off, N, 320 if G < 300 else 64, 108)
    assert g.M > 8 * g.G
    Kp = 384 if G < 300 else 64
    a = np.zeros((g.M, Kp), dtype=np.uint16); a[:, :g.K] = g.a_mk
    b = np.zeros((g.G, N, Kp), dtype=np.uint16); b[:, :, :g.K] = g.b_gnk
    gp = W.GroupedGemmInputs(g.M, N, Kp, g.G, a, b, g.group_rows)
    c, raw = run_grouped(gp, kernel=B.AXE_GROUPED_STREAM)
    check_grouped(gp, c, raw, R.gemm_grouped_ref(g.a_mk, g.b_gnk.transpose(0, 2, 1), off, R.AXE_BF16))


def test_hot_path_replayed_from_a_hip_graph():
    """The path a launch-bound caller would record once: relayout of an operand into blocks, two dense GEMMs (64 x 64
    tiles and the chained 256 x 256 pipeline) and a layout evaluation, captured into one HIP graph.  No entry point
    allocates, synchronises or records a memset, so the capture takes them as they are; every replay -- with eager
    work and synchronisations in between, and other input bits in the same buffers -- must equal the eager bits."""
    gs = [W.gemm_bf16(256, 256, 256, 301), W.gemm_bf16(4352, 4096, 512, 302)]
    alt = [W.gemm_bf16(256, 256, 256, 303), W.gemm_bf16(4352, 4096, 512, 304)]
    bufs, descs = [], []
    for g in gs:
        As, Bs, Cs = W.gemm_specs(g)
        descs.append(B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16, B.AXE_BF16, B.Layout(As), B.Layout(Bs), B.Layout(Cs),
                                g.M * g.K, g.N * g.K, g.M * g.N))
        bufs.append((dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1)), torch.zeros(g.M * g.N, dtype=torch.int16, device="cuda")))
    rows, cols = 512, 384
    Ls, Ld = B.Layout(W.row_major_spec(rows, cols)), B.Layout(W.blocked_swizzled_spec(rows, cols))
    src = torch.randint(-30000, 30000, (rows * cols,), dtype=torch.int16, device="cuda")
    dst = torch.zeros(rows * cols, dtype=torch.int16, device="cuda")
    pts = torch.zeros((rows * cols, Ld.E_R, len(Ld.axes)), dtype=torch.int64, device="cuda")

    def path():
        B.axe_relayout(Ls, Ld, (rows, cols), src, dst)
        for d, (a, b, c) in zip(descs, bufs):
            B.axe_gemm(d, a, b, c)
        B.axe_layout_eval(Ld, (rows, cols), rows * cols, out=pts)

    def results():
        torch.cuda.synchronize()
        return [dst.cpu().numpy().copy(), pts.cpu().numpy().copy()] + [c.cpu().numpy().copy() for _, _, c in bufs]

    def load(inputs, seed):
        for (a, b, _), g in zip(bufs, inputs):
            a.copy_(dev(g.a_mk.reshape(-1)))
            b.copy_(dev(g.b_nk.reshape(-1)))
        src.copy_(torch.from_numpy(np.random.default_rng(seed).integers(-30000, 30000, rows * cols, dtype=np.int16)).cuda())

    want = []
    for k, inputs in enumerate((gs, alt)):
        load(inputs, k)
        path()
        want.append(results())
    assert not np.array_equal(want[0][2], want[1][2])
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        path()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        path()
    for rep in range(3):
        for k, inputs in enumerate((gs, alt)):
            load(inputs, k)
            for t in [dst, pts] + [c for _, _, c in bufs]:
                t.fill_(-1)
            torch.randn(1 << 20, device="cuda").sum().item()        # eager work and a synchronisation between replays
            graph.replay()
            got = results()
            for x, y in zip(got, want[k]):
                assert np.array_equal(x, y), (rep, k)
