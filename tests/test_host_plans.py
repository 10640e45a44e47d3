"""Host logic without a GPU: the plans axe_layout_eval / axe_relayout build (canonicalisation,
common refinement, vector width, loop order, unroll digit) are executed by host-memory stand-ins
of the integer kernels (libaxe_hostcheck.so) that refuse any address outside the declared
buffers; results must equal the oracle bit for bit.  This is what is checked before a plan is
ever run on the GPU."""
import ctypes as C
import os
import random
from math import prod

import numpy as np
import pytest

from oracle import axe_layout as ax
from oracle import axe_ref as R
from oracle.axe_layout import Iter, Layout, Swizzle
from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W

HOSTCHECK = os.environ.get("AXE_TEST_HOST_LIB") or os.path.join(os.path.dirname(B.LIB_PATH), "libaxe_hostcheck.so")


@pytest.fixture(scope="module")
def hc():
    if not os.path.exists(HOSTCHECK):
        from paper_2601_19092_amd.build import build_hostcheck
        build_hostcheck()
    L = C.CDLL(HOSTCHECK)
    LP = C.POINTER(B.axe_layout_t)
    L.axe_layout_eval.argtypes = [LP, C.c_int32, C.POINTER(C.c_int64), C.c_int64, C.c_void_p, C.c_void_p, C.c_void_p]
    L.axe_relayout.argtypes = [LP, LP, C.c_int32, C.POINTER(C.c_int64), C.c_int32, C.c_int32, C.c_void_p, C.c_int64,
                               C.c_void_p, C.c_int64, C.c_void_p]
    L.axe_hostcheck_set_buffers.argtypes = [C.c_int64, C.c_int64]
    L.axe_last_error.restype = C.c_char_p
    return L


def spec_of(L: Layout) -> dict:
    z = L.swizzle
    return W.spec([(i.extent, i.stride, i.axis) for i in L.D], [(i.extent, i.stride, i.axis) for i in L.R],
                  dict(L.O), (z.axis, z.bits, z.base, z.shift) if z else None)


def host_relayout(hc, src_L, dst_L, shape, src, dst_len, fill=0xA5, env=None):
    eb = src.dtype.itemsize
    dst = np.zeros(dst_len, dtype=src.dtype)
    dst.view(np.uint8)[:] = fill
    want = dst.copy()
    R.relayout_ref(src_L, dst_L, shape, src, want)
    ls, ld = B.Layout(spec_of(src_L), ["m", "gpuid"]), B.Layout(spec_of(dst_L), ["m", "gpuid"])
    shp = (C.c_int64 * len(shape))(*shape)
    hc.axe_hostcheck_set_buffers(src.nbytes, dst.nbytes)
    old = {}
    for k, v in (env or {}).items():
        old[k] = os.environ.get(k)
        os.environ[k] = str(v)
    try:
        rc = hc.axe_relayout(C.byref(ls.c), C.byref(ld.c), len(shape), shp, eb, 0, src.ctypes.data, src.size,
                             dst.ctypes.data, dst.size, None)
    finally:
        for k, v in old.items():
            if v is None:
                del os.environ[k]
            else:
                os.environ[k] = v
    assert rc == 0, hc.axe_last_error().decode()
    assert hc.axe_hostcheck_violations() == 0
    return dst, want


@pytest.mark.parametrize("rows,cols", [(128, 64), (256, 192), (1152, 704)])
@pytest.mark.parametrize("unroll", [1, 2, 4, 8])
def test_plan_blocked_swizzled(hc, rows, cols, unroll):
    words = W.relayout_words(rows, cols, 31, "index").reshape(-1)
    src_L = Layout.from_spec(W.row_major_spec(rows, cols))
    dst_L = Layout.from_spec(W.blocked_swizzled_spec(rows, cols))
    got, want = host_relayout(hc, src_L, dst_L, (rows, cols), words, rows * cols, env={"AXE_RELAYOUT_UNROLL": unroll})
    assert np.array_equal(got, want)
    back, wb = host_relayout(hc, dst_L, src_L, (rows, cols), got, rows * cols, env={"AXE_RELAYOUT_UNROLL": unroll})
    assert np.array_equal(back, wb) and np.array_equal(back, words)


@pytest.mark.parametrize("eb", [1, 2, 4, 8, 16])
def test_plan_element_sizes_transposes_replicas(hc, eb):
    rng = np.random.default_rng(eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64, 16: np.dtype((np.void, 16))}[eb]
    for shape in ((24, 24), (37, 53), (6, 4, 5), (96, 40), (3, 128, 7), (1,), (1, 1), (16,)):
        n = prod(shape)
        src = rng.integers(0, 256, n * eb, dtype=np.uint8).view(dt)
        A = ax.row_major(shape)
        Bf = Layout.make(shape, [prod(shape[:i]) for i in range(len(shape))])
        for s_L, d_L in ((A, Bf), (Bf, A), (A, A)):
            got, want = host_relayout(hc, s_L, d_L, shape, src, n)
            assert got.tobytes() == want.tobytes(), (shape, eb)
    shape = (10, 12)
    src = rng.integers(0, 256, 120 * eb, dtype=np.uint8).view(dt)
    D = Layout.make(shape, (16, 1), R=((2,), (200,)), O={"m": 5})
    got, want = host_relayout(hc, ax.row_major(shape), D, shape, src, 400)
    assert got.tobytes() == want.tobytes()
    D8 = Layout.make(shape, (16, 1), R=((2, 2), (200, 400)), O={"m": 8})
    got, want = host_relayout(hc, ax.row_major(shape), D8, shape, src, 808)
    assert got.tobytes() == want.tobytes()
    Rv = Layout.make(shape, (-12, 1), O={"m": 108})
    got, want = host_relayout(hc, ax.row_major(shape), Rv, shape, src, 120)
    assert got.tobytes() == want.tobytes()


@pytest.mark.parametrize("diag", [0, 1, 3])
def test_plan_transposing_tile_walks(hc, diag, monkeypatch):
    """The order in which the tiles are walked (row by row, or diagonally with a step of 1 or 3 tiles, so that
    concurrent workgroups spread their writes over the memory channels) is a bijection of the tile grid for any
    grid: every element arrives, none twice.  Grids of 5 x 3, 3 x 5 and 1 x 4 tiles with clipped edges, a batch."""
    monkeypatch.setenv("AXE_TRANSPOSE_DIAG", str(diag))
    rng = np.random.default_rng(300 + diag)
    T, ce = 128, 8
    for shape in ((4 * T + ce, 3 * T), (3 * T - ce, 5 * T), (4 * ce, 4 * T), (2, 2 * T + ce, 3 * T)):
        rows, cols = shape[-2], shape[-1]
        s_L = ax.row_major(shape)
        d_L = Layout.make(shape, (1, rows) if len(shape) == 2 else (rows * cols, 1, rows))
        src = rng.integers(0, 65536, prod(shape), dtype=np.uint16)
        got, want = host_relayout(hc, s_L, d_L, shape, src, prod(shape))
        assert hc.axe_hostcheck_transposes() == 1, shape
        assert got.tobytes() == want.tobytes(), shape


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_plan_transposing_path(hc, eb):
    """Source and destination contiguous along different digits: the tiled path through LDS.  Whole
    and clipped tiles, a batch digit, pitched rows on both sides, an offset; the stand-in kernel checks
    every 16-byte access against the buffers and that nothing is stored that was not loaded."""
    rng = np.random.default_rng(100 + eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]
    ce = 16 // eb
    T = {1: 128, 2: 128, 4: 128, 8: 64}[eb]
    cases = [((T, T), None), ((2 * T + ce, 3 * T - ce), None), ((ce * 5, 4 * T), None),
             ((3, T + 2 * ce, 2 * T), "batch"), ((T + ce, T - ce), "pitched")]
    for shape, kind in cases:
        rows, cols = shape[-2], shape[-1]
        if kind == "batch":
            # (b, r, c): source row-major, destination transposes the last two dimensions inside each batch
            s_L = ax.row_major(shape)
            d_L = Layout.make(shape, (rows * cols, 1, rows))
            n_src = n_dst = prod(shape)
        elif kind == "pitched":
            ps, pd = cols + 3 * ce, rows + 2 * ce                          # row pitches, multiples of a chunk
            s_L = Layout.make(shape, (ps, 1), O={"m": ce})
            d_L = Layout.make(shape, (1, pd), O={"m": 2 * ce})
            n_src, n_dst = ce + rows * ps, 2 * ce + cols * pd
        else:
            s_L = ax.row_major(shape)
            d_L = Layout.make(shape, (1, rows))
            n_src = n_dst = prod(shape)
        src = rng.integers(0, 256, n_src * eb, dtype=np.uint8).view(dt)
        got, want = host_relayout(hc, s_L, d_L, shape, src, n_dst)
        assert hc.axe_hostcheck_transposes() == 1, (shape, kind)
        assert got.tobytes() == want.tobytes(), (shape, kind)
        back, wb = host_relayout(hc, d_L, s_L, shape, got, n_src)           # and the other way round
        assert hc.axe_hostcheck_transposes() == 1 and back.tobytes() == wb.tobytes()
    assert hc.axe_hostcheck_transposes_elementwise() == 0


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_plan_transposing_path_replicas_and_swizzles(hc, eb):
    """The 16-byte tiled path also serves a replicated destination (every replica written from the same LDS
    tile) and a swizzle stage on either side that moves whole chunks."""
    rng = np.random.default_rng(300 + eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]
    ce = 16 // eb
    T = {1: 128, 2: 128, 4: 128, 8: 64}[eb]
    lg = ce.bit_length() - 1
    for shape in [(T, T), (2 * T, T + ce), (T + 3 * ce, 2 * T)]:
        rows, cols = shape
        n = rows * cols
        size = 1 << (n - 1).bit_length()                                   # a swizzle permutes a power-of-two span
        src = rng.integers(0, 256, n * eb, dtype=np.uint8).view(dt)
        row, col = ax.row_major(shape), Layout.make(shape, (1, rows))
        # two and 2 x 3 replicas of a transposed destination, strides multiples of a chunk
        for R_, span in [(((2,), (n,)), 2 * n), (((2, 3), (3 * (n + ce), n + ce)), 6 * (n + ce))]:
            got, want = host_relayout(hc, row, Layout.make(shape, (1, rows), R=R_), shape, src, span)
            assert hc.axe_hostcheck_transposes() == 1 and hc.axe_hostcheck_transposes_elementwise() == 0
            assert got.tobytes() == want.tobytes(), (shape, R_)
        # swizzled destination, swizzled source, both; XOR target bits at or above a chunk
        sw_d = Swizzle("m", 3, lg, lg + 5)
        sw_s = Swizzle("m", 2, lg + 1, lg + 4)
        for s_L, d_L in [(row, col.with_(swizzle=sw_d)), (row.with_(swizzle=sw_s), col),
                         (row.with_(swizzle=sw_s), col.with_(swizzle=sw_d)),
                         (col.with_(swizzle=sw_d), row.with_(swizzle=sw_s))]:
            src_p = rng.integers(0, 256, size * eb, dtype=np.uint8).view(dt)
            got, want = host_relayout(hc, s_L, d_L, shape, src_p, size)
            assert hc.axe_hostcheck_transposes() == 1 and hc.axe_hostcheck_transposes_elementwise() == 0
            assert got.tobytes() == want.tobytes(), (shape, s_L, d_L)
        # replicas and a swizzle together
        d_L = Layout.make(shape, (1, rows), R=((2,), (size,))).with_(swizzle=sw_d)
        got, want = host_relayout(hc, row, d_L, shape, src, 2 * size)
        assert hc.axe_hostcheck_transposes() == 1 and got.tobytes() == want.tobytes()


@pytest.mark.parametrize("eb", [1, 2, 4, 8])
def test_plan_transposing_path_element_by_element(hc, eb):
    """Rows that are not whole 16-byte chunks (odd extents, odd pitches, odd offsets, odd replica strides, a swizzle
    inside a chunk): 64 x 64 tiles through LDS, element by element; the stand-in checks every access."""
    rng = np.random.default_rng(400 + eb)
    dt = {1: np.uint8, 2: np.uint16, 4: np.uint32, 8: np.uint64}[eb]
    ce = 16 // eb
    w = max(64 // eb, 2)                                                   # shortest row the path takes
    cases = []
    for shape in [(w + 1, 2 * w + 3), (129, 67 + w), (64, 64 + w + 1), (3, w + 5, 70 + w)]:
        rows, cols = shape[-2], shape[-1]
        lead = shape[:-2]
        n = prod(shape)
        if lead:
            s_L = ax.row_major(shape)
            d_L = Layout.make(shape, (rows * cols, 1, rows))
        else:
            s_L, d_L = ax.row_major(shape), Layout.make(shape, (1, rows))
        cases.append((shape, s_L, d_L, n, n))
    rows, cols = w + 2, 2 * w + 1
    shape = (rows, cols)
    cases.append((shape, Layout.make(shape, (cols + 3, 1), O={"m": 1}), Layout.make(shape, (1, rows + 5), O={"m": 3}),
                  1 + rows * (cols + 3), 3 + cols * (rows + 5)))           # odd pitches and offsets
    rows, cols = 2 * w, 2 * w
    shape = (rows, cols)
    n = rows * cols
    cases.append((shape, ax.row_major(shape), Layout.make(shape, (1, rows), R=((3,), (n + 1,))), n, 3 * (n + 1)))
    cases.append((shape, ax.row_major(shape).with_(swizzle=Swizzle("m", 2, 0, 7)),
                  Layout.make(shape, (1, rows)).with_(swizzle=Swizzle("m", 3, 1, 8)), n, n))
    for shape, s_L, d_L, n_src, n_dst in cases:
        src = rng.integers(0, 256, n_src * eb, dtype=np.uint8).view(dt)
        got, want = host_relayout(hc, s_L, d_L, shape, src, n_dst)
        assert hc.axe_hostcheck_transposes() == 1 and hc.axe_hostcheck_transposes_elementwise() == 1, (shape, s_L, d_L)
        assert got.tobytes() == want.tobytes(), (shape, s_L, d_L)
    # rows shorter than 64 bytes on either side stay on the loop-nest paths
    shape = (w // 2, 4 * w)
    src = rng.integers(0, 256, prod(shape) * eb, dtype=np.uint8).view(dt)
    got, want = host_relayout(hc, ax.row_major(shape), Layout.make(shape, (1, shape[0])), shape, src, prod(shape))
    assert hc.axe_hostcheck_transposes() == 0 and got.tobytes() == want.tobytes()


def test_plan_random_layout_pairs(hc):
    """Random pairs of injective layouts over the same element count: permuted / split /
    padded strides on both sides, with and without swizzles; joint and generic paths."""
    rng = random.Random(77)
    done = 0
    while done < 150:
        # random mixed-radix factorisation for each side, random nesting order of strides
        E = rng.choice([24, 36, 48, 64, 96, 120, 128, 256, 360, 512])
        def rand_layout():
            ext, rest = [], E
            while rest > 1 and len(ext) < 5:
                f = rng.choice([d for d in range(2, rest + 1) if rest % d == 0])
                ext.append(f)
                rest //= f
            order = list(range(len(ext)))
            rng.shuffle(order)
            strides, acc = [0] * len(ext), 1
            pad = rng.choice([0, 0, 1, 8])
            for k in order:
                strides[k] = acc
                acc = acc * ext[k] + (pad if rng.random() < 0.3 else 0)
            size = sum((e - 1) * s for e, s in zip(ext, strides)) + 1
            L = Layout(tuple(Iter(e, s, "m") for e, s in zip(ext, strides)))
            if rng.random() < 0.3:
                bits, base = rng.choice([(1, 0), (2, 1), (3, 3)])
                shift = base + bits + rng.randint(0, 2)
                L = L.with_(swizzle=Swizzle("m", bits, base, shift))
                size = ((size - 1) | ((1 << (bits + base)) - 1)) + 1
            return L, size
        (s_L, s_size), (d_L, d_size) = rand_layout(), rand_layout()
        if not s_L.D or not d_L.D:
            continue
        src = np.array([rng.randrange(65536) for _ in range(s_size)], dtype=np.uint16)
        got, want = host_relayout(hc, s_L, d_L, (E,), src, d_size)
        assert np.array_equal(got, want), (s_L, d_L)
        done += 1


def test_plan_eval_matches_oracle(hc):
    rng = random.Random(5)
    axes = ["m", "lane", "reg", "gpuid"]
    for _ in range(60):
        D = tuple(Iter(rng.randint(1, 6), rng.choice([1, 2, 3, 8, -4, 1000003]), rng.choice(axes)) for _ in range(rng.randint(1, 6)))
        Rr = tuple(Iter(rng.randint(1, 3), rng.choice([1, 7, -2]), rng.choice(axes)) for _ in range(rng.randint(0, 2)))
        L = Layout(D, Rr, ax._norm_offset({a: rng.randint(-3, 3) for a in axes if rng.random() < 0.5}))
        bl = B.Layout(spec_of(L), L.axes())
        n = L.E_D
        out = np.zeros((n, L.E_R, len(L.axes())), dtype=np.int64)
        shp = (C.c_int64 * 1)(n)
        assert hc.axe_layout_eval(C.byref(bl.c), 1, shp, n, None, out.ctypes.data, None) == 0
        assert np.array_equal(out, R.evaluate_np(L, np.arange(n), L.axes()))


def test_plan_replicated_destination_whose_replicas_step_over_the_shard_part(hc):
    """Replica strides that nest with the shard strides are accepted and every replica is written (the aliasing
    test looks at shard and replica iters together; the overlapping case is refused in test_boundary)."""
    src_L = Layout.make((4,), (1,))
    dst_L = Layout.make((4,), (1,), R=((2,), (4,)))
    words = np.array([11, 22, 33, 44], dtype=np.uint16)
    got, want = host_relayout(hc, src_L, dst_L, (4,), words, 8)
    assert np.array_equal(got, want) and list(got) == [11, 22, 33, 44, 11, 22, 33, 44]


@pytest.mark.parametrize("eb,blocked", [(2, False), (2, True), (1, False)])
def test_plan_gate_up_interleaved_weight_packing(hc, eb, blocked):
    """The images the gated grouped GEMM reads, from the plain (G, K, N) one: against the oracle and against the NumPy
    reshape / transpose construction."""
    from packing import pack_blocked, pack_gate_up
    G, K, N = 2, 128, 512
    rng = np.random.default_rng(7 + eb)
    b_gnk = rng.integers(0, 256 ** eb, (G, N, K)).astype(np.uint16 if eb == 2 else np.uint8)
    s_L = Layout.from_spec(W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")]))
    d_L = Layout.from_spec(W.gated_b_spec(K, N, G, blocked))
    got, want = host_relayout(hc, s_L, d_L, (G, K, N), b_gnk.reshape(-1), b_gnk.size)
    img = pack_gate_up(b_gnk)
    img = pack_blocked(img) if blocked else img
    assert np.array_equal(got, want) and np.array_equal(got, img.reshape(-1))


def test_gemm_plan_is_reused_only_for_an_identical_descriptor(hc):
    """axe_gemm keeps the plan of the last descriptor a thread launched.  A descriptor that differs in any word must be
    planned afresh: after a successful plan, the same descriptor with a changed stride, shape or dtype has to be judged
    on its own (the host-check library's GEMM launch stand-ins return 'not supported', so a plan that passes ends
    in AXE_EHIP and nothing is launched)."""
    hc.axe_gemm.argtypes = [C.POINTER(B.axe_gemm_desc_t), C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    M = N = K = 256
    def desc(lda=None, K_=K, dt=B.AXE_BF16):
        lda = lda or K_
        return B.GemmDesc(M, N, K_, dt, B.AXE_F32, B.Layout(W.spec([(M, lda, "m"), (K_, 1, "m")])), B.Layout(W.col_major_spec(K_, N)),
                          B.Layout(W.row_major_spec(M, N)), M * lda, N * K_, M * N)
    def call(d, pa=0x10000, pb=0x200000, pc=0x400000):
        return hc.axe_gemm(C.byref(d.c), pa, pb, pc, None)
    good = desc()
    assert call(good) == B.AXE_EHIP and call(good) == B.AXE_EHIP            # planned, then reused
    assert call(desc(lda=K + 3)) == B.AXE_EUNSUPPORTED                      # pitch no multiple of 16 bytes: not the cached plan
    assert call(good) == B.AXE_EHIP
    assert call(desc(K_=K + 4)) == B.AXE_EUNSUPPORTED
    assert call(desc(dt=99)) == B.AXE_EINVAL
    assert call(good, pa=0x10001) == B.AXE_EINVAL                           # pointer checks run on a reused plan as well
    assert call(good, pc=0x10000) == B.AXE_EINVAL                           # C overlaps A
    assert call(good) == B.AXE_EHIP


def test_plan_relayout_into_a_register_layout_image(hc):
    """Destination = the MFMA operand layout of the 256 x 256 kernel (as axe_gemm_describe reports it), tiled over the
    matrix and folded onto memory [tile][wave][lane][reg] by the layout operators; source row-major.  The plan the host
    makes for it (16-byte units, a replicated destination) is executed on host memory against the oracle."""
    M, K = 512, 192
    desc = B.GemmDesc(M, 256, K, B.AXE_BF16, B.AXE_BF16, B.Layout(W.row_major_spec(M, K)), B.Layout(W.col_major_spec(K, 256)),
                      B.Layout(W.row_major_spec(M, 256)), M * K, 256 * K, M * 256, tile_hint=B.AXE_TILE_256x256x64)
    axes = ["m", "lds", "wg", "wave", "lane", "reg"]
    for which in (B.AXE_DESC_A_OPERAND, B.AXE_DESC_B_OPERAND):
        spec, tshape = B.axe_gemm_describe(desc, which)
        rows = M if which == B.AXE_DESC_A_OPERAND else 256
        # B's tile is (k, n): the matrix image B[n][k] is row-major in n, so its logical (k, n) view has strides (1, K)
        gr, gk = rows // 256, K // 64
        if which == B.AXE_DESC_A_OPERAND:
            grid, gshape = W.spec([(gr, gk, "wg"), (gk, 1, "wg")]), (gr, gk)
            src = W.spec([(gr, 256 * K, "m"), (256, K, "m"), (gk, 64, "m"), (64, 1, "m")])
        else:
            grid, gshape = W.spec([(gk, 1, "wg"), (gr, gk, "wg")]), (gk, gr)
            src = W.spec([(gk, 64, "m"), (64, 1, "m"), (gr, 256 * K, "m"), (256, K, "m")])
        tiled, shape = B.layout_tile(B.Layout(grid, axes), gshape, B.Layout(spec, axes), tshape)
        span = B.layout_span(B.Layout(tiled, axes))
        regs = span["reg"]
        pitch = {"reg": 1, "lane": regs, "wave": 64 * regs, "wg": span["wave"] * 64 * regs}
        dst = B.layout_flatten(B.Layout(tiled, axes), pitch, "m")
        n_dst = gr * gk * span["wave"] * 64 * regs
        words = np.random.default_rng(7).integers(0, 1 << 16, rows * K, dtype=np.uint16)
        want = np.full(n_dst, 0xA5A5, dtype=np.uint16)
        R.relayout_ref(Layout.from_spec(src), Layout.from_spec(dst), shape, words, want)
        got = np.full(n_dst, 0xA5A5, dtype=np.uint16)
        ls, ld = B.Layout(src, axes), B.Layout(dst, axes)
        hc.axe_hostcheck_set_buffers(words.nbytes, got.nbytes)
        rc = hc.axe_relayout(C.byref(ls.c), C.byref(ld.c), len(shape), (C.c_int64 * len(shape))(*shape), 2, 0, words.ctypes.data,
                             words.size, got.ctypes.data, got.size, None)
        assert rc == 0, hc.axe_last_error().decode()
        assert hc.axe_hostcheck_violations() == 0 and np.array_equal(got, want), which
        assert n_dst == 2 * rows * K                               # each operand is replicated over the other wave dimension
