"""The layouts axe_gemm_describe reports for every tile movement, evaluated with the oracle: they
must be bijections onto the hardware boxes they claim, compose as tile products (Sec. 3.3), keep the
direct-to-LDS loads linear in the lane id, and give bank-conflict-free operand reads on a 64-bank LDS.
CPU only (describe is host code)."""
import itertools
from math import prod

import numpy as np
import pytest

from oracle import axe_layout as ax
from oracle import axe_ref as R
from oracle.axe_layout import Layout
from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W

AXES = ["m", "lds", "wg", "wave", "lane", "reg"]


def desc_for(kind):
    if kind == "small_bf16":
        M, N, K, dt, out, tile = 256, 256, 256, B.AXE_BF16, B.AXE_F32, B.AXE_TILE_AUTO
    elif kind == "small_fp8":
        M, N, K, dt, out, tile = 128, 192, 256, B.AXE_FP8_E4M3, B.AXE_BF16, B.AXE_TILE_64x64x32
    elif kind in ("big_fp8", "big_fp8_mx"):
        M, N, K, dt, out, tile = 512, 768, 256, B.AXE_FP8_E4M3, B.AXE_BF16, B.AXE_TILE_256x256x64
    elif kind == "big_bf16_f32":
        M, N, K, dt, out, tile = 512, 768, 256, B.AXE_BF16, B.AXE_F32, B.AXE_TILE_256x256x64
    elif kind == "big_bf16_n224":
        # (problems this small go to the 64 x 64 tiles by themselves; the large tiles are asked for)
        M, N, K, dt, out, tile = 512, 672, 256, B.AXE_BF16, B.AXE_BF16, B.AXE_TILE_256x224x64
    else:
        M, N, K, dt, out, tile = 512, 768, 256, B.AXE_BF16, B.AXE_BF16, B.AXE_TILE_256x256x64
    scales = {}
    if kind == "big_fp8":
        # fp32 block scales: the 8-wave kernel that folds on the vector ALU.  describe never touches the
        # arrays; a non-NULL address stands for them.
        class _Fake:
            def data_ptr(self):
                return 0x1000
        scales = dict(scale_a=_Fake(), scale_b=_Fake())
    d = B.GemmDesc(M, N, K, dt, out, B.Layout(W.row_major_spec(M, K)), B.Layout(W.col_major_spec(K, N)),
                   B.Layout(W.row_major_spec(M, N)), M * K, N * K, M * N, tile_hint=tile, **scales)
    return d, (M, N, K)


def get(desc, which):
    spec, shape = B.axe_gemm_describe(desc, which)
    return Layout.from_spec(spec), shape


def table(L, shape):
    """All points: int array [E_D, E_R, 6] over AXES."""
    return R.evaluate_np(L, np.arange(prod(shape)), AXES)


# T x TN x BK: rows of A, rows of B (columns of C) and K elements per workgroup tile
GEO = {"small_bf16": dict(T=64, TN=64, BK=32, EB=2, waves=4, wn=2), "small_fp8": dict(T=64, TN=64, BK=128, EB=1, waves=4, wn=2),
       "big_bf16": dict(T=256, TN=256, BK=64, EB=2, waves=4, wn=2), "big_fp8": dict(T=256, TN=256, BK=128, EB=1, waves=8, wn=4),
       "big_bf16_n224": dict(T=256, TN=224, BK=64, EB=2, waves=4, wn=2),
       "big_bf16_f32": dict(T=256, TN=256, BK=64, EB=2, waves=4, wn=2),
       "big_fp8_mx": dict(T=256, TN=256, BK=128, EB=1, waves=4, wn=2)}
KINDS = ["small_bf16", "small_fp8", "big_bf16", "big_fp8", "big_bf16_n224", "big_fp8_mx", "big_bf16_f32"]
BIG = ("big_bf16", "big_fp8", "big_bf16_n224", "big_fp8_mx", "big_bf16_f32")
A_VIA_REGISTERS = ()                                                # (no kernel stages A through VGPRs and ds_write any more)
PAIRED_STORES = ("big_bf16", "big_fp8_mx")
TILE = {"small_bf16": B.AXE_TILE_64x64x32, "small_fp8": B.AXE_TILE_64x64x32, "big_bf16": B.AXE_TILE_256x256x64,
        "big_fp8": B.AXE_TILE_256x256x64, "big_bf16_n224": B.AXE_TILE_256x224x64, "big_fp8_mx": B.AXE_TILE_256x256x64,
        "big_bf16_f32": B.AXE_TILE_256x256x64}


@pytest.mark.parametrize("kind", KINDS)
def test_tile_shapes_and_kernel_choice(kind):
    desc, _ = desc_for(kind)
    geo = GEO[kind]
    assert B.axe_gemm_tile(desc) == TILE[kind]
    for which, want in ((B.AXE_DESC_A_G2L_THREADS, (geo["T"], geo["BK"])), (B.AXE_DESC_B_G2L_THREADS, (geo["BK"], geo["TN"])),
                        (B.AXE_DESC_A_LDS, (geo["T"], geo["BK"])), (B.AXE_DESC_B_LDS, (geo["BK"], geo["TN"])),
                        (B.AXE_DESC_A_OPERAND, (geo["T"], geo["BK"])), (B.AXE_DESC_B_OPERAND, (geo["BK"], geo["TN"])),
                        (B.AXE_DESC_C_STORE, (geo["T"], geo["TN"]))):
        L, shape = get(desc, which)
        assert shape == want and ax.admits(L, shape)


@pytest.mark.parametrize("kind", KINDS)
def test_accumulator_layout_is_a_bijection_and_a_tile_product(kind):
    desc, (M, N, K) = desc_for(kind)
    geo = GEO[kind]
    T, TN = geo["T"], geo["TN"]
    L, shape = get(desc, B.AXE_DESC_ACC)
    gm, gn = -(-M // T), -(-N // TN)
    assert shape == (gm * T, gn * TN)
    pts = table(L, shape)[:, 0, :]
    NW, WN = geo["waves"], geo["wn"]
    WM = NW // WN
    regs = T * TN // (64 * NW)
    box = np.stack(np.meshgrid(np.arange(gm * gn), np.arange(NW), np.arange(64), np.arange(regs), indexing="ij"), -1).reshape(-1, 4)
    got = pts[:, [2, 3, 4, 5]]
    assert np.all(pts[:, [0, 1]] == 0)
    assert len(got) == len(box) and np.array_equal(np.unique(got, axis=0), box)      # every accumulator exactly once
    # composition: grid (x) WM x WN waves (x) fragments-in-registers (x) MFMA accumulator fragment
    F = 16
    NFM, NFN = T // WM // F, TN // WN // F
    per = F * F // 64
    # 16x16 fragment with swapped operands: row -> lane, column 4b + c' -> lane + 16 b, reg c'
    frag = Layout.make((16, 4, 4), ("1@lane", "16@lane", "1@reg"))
    regs_t = Layout.make((NFM, NFN), (f"{NFN}@reg", "1@reg"))
    waves = Layout.make((WM, WN), (f"{WN}@wave", "1@wave"))
    grid = Layout.make((gm, gn), (f"{gn}@wg", "1@wg"))
    t1, s1 = ax.tile(regs_t, (NFM, NFN), frag, (F, F))
    t2, s2 = ax.tile(waves, (WM, WN), t1, (NFM * F, NFN * F))
    t3, s3 = ax.tile(grid, (gm, gn), t2, (T, TN))
    assert ax.span(frag)["reg"] == per
    want = R.evaluate_np(t3, np.arange(prod(shape)), AXES)[:, 0, :]
    assert np.array_equal(want, pts)


@pytest.mark.parametrize("kind", KINDS)
def test_global_to_lds_thread_map(kind):
    desc, _ = desc_for(kind)
    geo = GEO[kind]
    T, TN, BK, EB = geo["T"], geo["TN"], geo["BK"], geo["EB"]
    CE = 16 // EB
    for which_t, which_l, shape in ((B.AXE_DESC_A_G2L_THREADS, B.AXE_DESC_A_LDS, (T, BK)),
                                    (B.AXE_DESC_B_G2L_THREADS, B.AXE_DESC_B_LDS, (BK, TN))):
        R_ = shape[0] if which_l == B.AXE_DESC_A_LDS else shape[1]      # rows of this operand in the tile
        Lt, st = get(desc, which_t)
        Ll, sl = get(desc, which_l)
        assert st == sl == shape
        th = table(Lt, shape)[:, 0, :]
        NW = geo["waves"]
        regs = R_ * BK // (64 * NW)
        key = (th[:, 3] * 64 + th[:, 4]) * regs + th[:, 5]
        assert np.array_equal(np.sort(key), np.arange(R_ * BK))          # every thread register exactly once
        lds = table(Ll, shape)[:, 0, 1]
        # B block: right after A in the small kernels; the 256x256 bf16 kernel keeps two A blocks first
        base = 0 if which_l == B.AXE_DESC_A_LDS else T * BK * (2 if kind in BIG else 1)
        assert np.array_equal(np.sort(lds), np.arange(base, base + R_ * BK))  # LDS stage filled exactly once
        # each lane moves whole 16-byte chunks: CE consecutive registers <-> CE consecutive k <-> CE consecutive LDS elements
        order = np.argsort(key)
        lds_by_thread = lds[order].reshape(NW, 64, regs // CE, CE)
        assert np.all(np.diff(lds_by_thread, axis=-1) == 1) and np.all(lds_by_thread[..., 0] % CE == 0)
        if kind in BIG:
            # one wave instruction moves 8 rows x 128 bytes into a 1 KiB aligned piece of LDS
            first = lds_by_thread[..., 0] * EB                            # byte address of each lane's chunk
            for w, i in itertools.product(range(NW), range(regs // CE)):
                b0 = first[w, :, i].min()
                assert b0 % 1024 == 0
                if which_l == B.AXE_DESC_B_LDS or kind not in A_VIA_REGISTERS:
                    # direct-to-LDS load: lane l writes byte 16 l of the piece
                    assert np.array_equal(first[w, :, i], b0 + 16 * np.arange(64))
                else:
                    # through registers: the 8 lanes of a row write that row's 8 chunk positions, permuted
                    rows_ = (first[w, :, i] - b0) // 128
                    assert np.array_equal(rows_, np.arange(64) // 8)
                    for r in range(8):
                        assert sorted(((first[w, 8 * r:8 * r + 8, i] - b0) % 128 // 16).tolist()) == list(range(8))


# Lanes served together by one 16-byte-per-lane LDS read, as measured on gfx950 (a layout that is
# conflict-free for 16 consecutive lanes but not for these groups costs 8 instead of 4 LDS cycles per
# instruction, SQ_LDS_BANK_CONFLICT = 4 per instruction): per half-wave, lanes 0-3, 12-15, 20-23, 24-27
# and lanes 4-7, 8-11, 16-19, 28-31.
B128_GROUPS = [[h + l for q in qs for l in range(q, q + 4)] for h in (0, 32) for qs in ((0, 12, 20, 24), (4, 8, 16, 28))]


def bank_conflicts(byte_addrs):
    """64 banks of 4 bytes; a 16-byte read per lane is served 16 lanes at a time: conflict-free iff the
    16 lanes of a group touch 16 distinct 16-byte bank groups.  Returns the worst multiplicity."""
    worst = 1
    for lanes in B128_GROUPS:
        slots = (byte_addrs[lanes] // 16) % 16
        worst = max(worst, int(np.bincount(slots, minlength=16).max()))
    return worst


@pytest.mark.parametrize("kind", KINDS)
def test_operand_reads_cover_the_tile_and_are_bank_conflict_free(kind):
    desc, _ = desc_for(kind)
    geo = GEO[kind]
    T, TN, BK, EB = geo["T"], geo["TN"], geo["BK"], geo["EB"]
    CE = 16 // EB
    for which_o, which_l, shape in ((B.AXE_DESC_A_OPERAND, B.AXE_DESC_A_LDS, (T, BK)),
                                    (B.AXE_DESC_B_OPERAND, B.AXE_DESC_B_LDS, (BK, TN))):
        Lo, _ = get(desc, which_o)
        Ll, _ = get(desc, which_l)
        NW, WN = geo["waves"], geo["wn"]
        WM = NW // WN
        is_b = which_o == B.AXE_DESC_B_OPERAND
        repl = WM if is_b else WN                              # waves that hold the same operand rows
        op = table(Lo, shape)                                  # [E, replicas, 6]
        assert op.shape[1] == repl
        regs = ((TN // WN) if is_b else (T // WM)) * BK // 64
        key = ((op[:, :, 3] * 64 + op[:, :, 4]) * regs + op[:, :, 5]).reshape(-1)
        assert np.array_equal(np.sort(key), np.arange(NW * 64 * regs))     # each wave holds its share, once
        for swz, expect_clean in ((True, True), (False, False)):
            L = Ll if swz else Ll.with_(swizzle=None)
            lds = np.repeat(table(L, shape)[:, 0, 1], repl)
            addr = np.empty(NW * 64 * regs, dtype=np.int64)
            addr[key] = lds * EB
            addr = addr.reshape(NW, 64, regs // CE, CE)[..., 0]            # byte address of each 16-byte read
            worst = max(bank_conflicts(addr[w, :, i]) for w in range(NW) for i in range(addr.shape[2]))
            assert (worst == 1) == expect_clean, (kind, which_o, swz, worst)


@pytest.mark.parametrize("kind", ["small_bf16", "big_bf16", "big_fp8", "big_bf16_n224", "big_fp8_mx", "big_bf16_f32"])
def test_c_store_map(kind):
    desc, _ = desc_for(kind)
    T, TN, NW, WN = GEO[kind]["T"], GEO[kind]["TN"], GEO[kind]["waves"], GEO[kind]["wn"]
    L, shape = get(desc, B.AXE_DESC_C_STORE)
    pts = table(L, shape)[:, 0, :]
    regs = T * TN // (64 * NW)
    key = (pts[:, 3] * 64 + pts[:, 4]) * regs + pts[:, 5]
    assert np.array_equal(np.sort(key), np.arange(T * TN))
    if kind in BIG:
        # per = registers of one store instruction.  The fp8 and the 224-wide bf16 kernels store a fragment
        # at a time (4 registers = 4 columns per lane: 16 rows x 32 contiguous bytes); the 256-wide bf16
        # kernel stores fragment pairs (8 registers = 8 columns per lane: 16 rows x 64 contiguous bytes).
        # Either way the stores of a fragment row follow one another and complete TN / WN * 2 bytes per row.
        per = 8 if kind in PAIRED_STORES else 4
        lanes_per_row = 64 // 16
        per_row = TN // WN // (per * lanes_per_row)                   # store instructions per fragment row
        col = np.empty(T * TN, dtype=np.int64); row = np.empty(T * TN, dtype=np.int64)
        idx = np.arange(T * TN)
        row[key], col[key] = idx // TN, idx % TN
        row, col = row.reshape(NW, 64, regs // per, per), col.reshape(NW, 64, regs // per, per)
        assert np.all(np.diff(col, axis=-1) == 1) and np.all(row[..., 0:1] == row)
        assert np.all(col[..., 0] % per == 0)                         # aligned 8- or 16-byte stores
        for w, t in itertools.product(range(NW), range(regs // per)):
            r, c = row[w, :, t, 0], col[w, :, t, 0]
            assert len(set(r.tolist())) == 16
            for rr in set(r.tolist()):
                cs = np.sort(c[r == rr])
                assert np.array_equal(cs, cs[0] + per * np.arange(4)) and cs[0] % (4 * per) == 0
        for w, i in itertools.product(range(NW), range(8)):           # fragment row i
            c0 = np.sort(np.unique(col[w, :, per_row * i:per_row * i + per_row, :]))
            assert np.array_equal(c0, c0[0] + np.arange(TN // WN))
    if kind in PAIRED_STORES:
        # the exchange: lane group q = lane // 16 of the accumulator layout holds columns 4 q .. 4 q + 3 of
        # each fragment; the storing lane group of column c (inside its 32-column fragment pair) is
        # 2 * ((c % 16) // 8) + (c // 16): even groups store the first fragment, odd groups the second
        acc, _ = get(desc, B.AXE_DESC_ACC)
        for r, c in ((0, 0), (3, 5), (17, 12), (100, 16), (130, 27), (255, 255), (77, 200)):
            (p,) = ax.evaluate_at(L, shape, (r, c), AXES)
            cc = c % 32
            assert p[4] == r % 16 + 16 * (2 * ((cc % 16) // 8) + cc // 16)
            assert p[5] % 8 == 4 * ((cc % 8) // 4) + c % 4 and p[3] == 2 * (r // 128) + c // 128


@pytest.mark.parametrize("kind", KINDS)
def test_described_layouts_are_the_index_functions_the_kernels_compute_with(kind):
    """csrc/tile_maps.h states, as plain integer functions, where the kernels put things: the LDS chunk position of a
    row's chunk, the row a wave instruction's lane fetches, the chunk a lane group reads for its MFMA operand, the
    columns a lane stores.  The kernels call these functions; here every described layout, evaluated at every point of
    its tile by the host layer, must give the same coordinates as the functions (a test-only routine of the host
    library does the comparison in C++ against the header itself)."""
    import ctypes as C
    import os
    hc = C.CDLL(os.environ.get("AXE_TEST_HOST_LIB") or os.path.join(os.path.dirname(B.LIB_PATH), "libaxe_hostcheck.so"))
    fn = hc.axe_hostcheck_describe_vs_tile_maps
    fn.restype = C.c_int
    fn.argtypes = [C.POINTER(B.axe_gemm_desc_t)] + [C.c_int32] * 7 + [C.c_int64, C.c_int32]
    hc.axe_last_error.restype = C.c_char_p
    desc, _ = desc_for(kind)
    geo = GEO[kind]
    b_off = geo["T"] * geo["BK"] * (2 if kind in BIG else 1)
    for which in range(8):
        rc = fn(C.byref(desc.c), which, geo["T"], geo["TN"], geo["BK"], geo["EB"], geo["waves"], geo["wn"], b_off,
                int(kind in PAIRED_STORES))
        assert rc == 0, (kind, which, rc, hc.axe_last_error().decode())


def test_mfma_operand_layout_matches_its_statement():
    """MFMA 16x16x32 bf16: lane = row + 16 * (k // 8), 8 consecutive k per lane."""
    desc, _ = desc_for("big_bf16")
    L, shape = get(desc, B.AXE_DESC_A_OPERAND)
    for r, k in ((0, 0), (5, 7), (37, 8), (130, 17), (255, 63)):
        pts = ax.evaluate_at(L, shape, (r, k), AXES)
        wm, f, fr = r // 128, (r % 128) // 16, r % 16
        ks, fq, e = k // 32, (k % 32) // 8, k % 8
        assert sorted(p[3] for p in pts) == [2 * wm, 2 * wm + 1]
        assert {p[4] for p in pts} == {fr + 16 * fq} and {p[5] for p in pts} == {(ks * 8 + f) * 8 + e}
    desc, _ = desc_for("small_bf16")
    L, shape = get(desc, B.AXE_DESC_B_OPERAND)
    for k, n in ((0, 0), (9, 17), (31, 63)):
        pts = ax.evaluate_at(L, shape, (k, n), AXES)
        wn, f, fr = n // 32, (n % 32) // 16, n % 16
        assert sorted(p[3] for p in pts) == [wn, wn + 2]
        assert {p[4] for p in pts} == {fr + 16 * (k // 8)} and {p[5] for p in pts} == {f * 8 + k % 8}


def test_describe_errors():
    desc, _ = desc_for("small_bf16")
    with pytest.raises(B.AxeError) as e:
        B.axe_gemm_describe(desc, 99)
    assert e.value.code == B.AXE_EINVAL


def test_fp8_mfma_operand_layout_matches_its_statement():
    """MFMA 16x16x128 fp8 as the kernels feed it: lane = row + 16 * ((k % 64) // 16); the lane's 32 bytes
    are k = 16 q .. 16 q + 15 (registers 0..15) and k = 64 + 16 q .. (registers 16..31): the same two runs
    for A and for B, so every product pairs equal k."""
    for kind in ("small_fp8", "big_fp8", "big_fp8_mx"):
        desc, _ = desc_for(kind)
        T = GEO[kind]["T"]
        for which, shape_of in ((B.AXE_DESC_A_OPERAND, lambda r, k: (r, k)), (B.AXE_DESC_B_OPERAND, lambda r, k: (k, r))):
            L, shape = get(desc, which)
            for r, k in ((0, 0), (5, 15), (9, 16), (12, 63), (3, 64), (15, 127), (T // 4 + 17, 81)):
                pts = ax.evaluate_at(L, shape, shape_of(r, k), AXES)
                for p in pts:
                    assert p[4] == r % 16 + 16 * ((k % 64) // 16)
                    assert p[5] % 32 == 16 * (k // 64) + k % 16


# ----------------------------------------------------------------------------- grouped tile kernels
def _grouped_desc(M, kernel=B.AXE_GROUPED_AUTO, epilogue=B.AXE_EPI_NONE, dt=B.AXE_BF16):
    G, N, K = 4, 512, 256
    NC = N // 2 if epilogue == B.AXE_EPI_SWIGLU else N
    Bs = W.gated_b_spec(K, N, G) if epilogue == B.AXE_EPI_SWIGLU else W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")])
    return B.GroupedGemmDesc(M, N, K, G, B.Layout(W.row_major_spec(M, K)), B.Layout(Bs), B.Layout(W.row_major_spec(M, NC)),
                             M * K, G * N * K, M * NC, in_dtype=dt, out_dtype=dt, epilogue=epilogue, kernel_hint=kernel)


@pytest.mark.parametrize("T,hint", [(256, B.AXE_GROUPED_TILES_256), (128, B.AXE_GROUPED_TILES_128), (128, B.AXE_GROUPED_AUTO)])
def test_grouped_tile_kernels_report_the_dense_maps_at_their_tile_height(T, hint):
    desc = _grouped_desc(1000, hint)                       # 250 rows per group on average: tiles of 128 rows when left alone
    assert B.axe_gemm_grouped_kernel(desc) == (B.AXE_GROUPED_TILES_256 if T == 256 else B.AXE_GROUPED_TILES_128)
    def gget(which):
        spec, shape = B.axe_gemm_grouped_describe(desc, which)
        return Layout.from_spec(spec), shape
    dense, _ = desc_for("big_bf16")
    BK, TN, NW = 64, 256, 4
    for which, want in ((B.AXE_DESC_A_G2L_THREADS, (T, BK)), (B.AXE_DESC_B_G2L_THREADS, (BK, TN)), (B.AXE_DESC_A_LDS, (T, BK)),
                        (B.AXE_DESC_B_LDS, (BK, TN)), (B.AXE_DESC_A_OPERAND, (T, BK)), (B.AXE_DESC_B_OPERAND, (BK, TN)),
                        (B.AXE_DESC_ACC, (T, TN)), (B.AXE_DESC_C_STORE, (T, TN))):
        L, shape = gget(which)
        assert shape == want and ax.admits(L, shape)
        if T == 256 and which != B.AXE_DESC_ACC:           # the very layouts of the dense kernel
            Ld, sd = get(dense, which)
            assert sd == shape and np.array_equal(table(L, shape), table(Ld, sd))
    # thread maps: every register of every thread exactly once; LDS: A in its block's first T rows, B behind both A blocks
    for which_t, which_l, rows, base in ((B.AXE_DESC_A_G2L_THREADS, B.AXE_DESC_A_LDS, T, 0),
                                        (B.AXE_DESC_B_G2L_THREADS, B.AXE_DESC_B_LDS, TN, 2 * 256 * BK)):
        Lt, st = gget(which_t)
        th = table(Lt, st)[:, 0, :]
        regs = rows * BK // (64 * NW)
        key = (th[:, 3] * 64 + th[:, 4]) * regs + th[:, 5]
        assert np.array_equal(np.sort(key), np.arange(rows * BK))
        Ll, sl = gget(which_l)
        lds = table(Ll, sl)[:, 0, 1]
        assert np.array_equal(np.sort(lds), np.arange(base, base + rows * BK))
        first = (lds[np.argsort(key)].reshape(NW, 64, regs // 8, 8)[..., 0]) * 2       # byte address of each lane's chunk
        for w, i in itertools.product(range(NW), range(regs // 8)):                     # direct-to-LDS: lane l writes byte 16 l of its piece
            assert first[w, 0, i] % 1024 == 0 and np.array_equal(first[w, :, i], first[w, 0, i] + 16 * np.arange(64))
    # operands: A rows split over the wave rows and replicated over the wave columns, conflict-free reads
    La, sa = gget(B.AXE_DESC_A_OPERAND)
    ta = table(La, sa)
    assert ta.shape[1] == 2                                                             # two replicas: the waves wn = 0, 1
    Ll, sl = gget(B.AXE_DESC_A_LDS)
    lds_of = dict(zip(map(tuple, np.stack(np.unravel_index(np.arange(prod(sl)), sl), -1).tolist()), table(Ll, sl)[:, 0, 1].tolist()))
    rows_a, ks = np.unravel_index(np.arange(prod(sa)), sa)
    for frag in range(T // 2 // 16):
        for sub in range(2):
            addr = np.full(64, -1, dtype=np.int64)
            sel = (ta[:, 0, 3] == 0) & (ta[:, 0, 5] // 8 == sub * (T // 2 // 16) + frag) & (ta[:, 0, 5] % 8 == 0)
            for idx in np.nonzero(sel)[0]:
                addr[ta[idx, 0, 4]] = lds_of[(int(rows_a[idx]), int(ks[idx]))] * 2
            assert (addr >= 0).all() and bank_conflicts(addr) == 1
    # accumulators and the store map of one tile: every element once
    for which in (B.AXE_DESC_ACC, B.AXE_DESC_C_STORE):
        L, shape = gget(which)
        pts = table(L, shape)[:, 0, :]
        regs = T * TN // (64 * NW)
        key = (pts[:, 3] * 64 + pts[:, 4]) * regs + pts[:, 5]
        assert np.array_equal(np.sort(key), np.arange(T * TN)) and np.all(pts[:, [0, 1, 2]] == 0)


def test_grouped_describe_refusals():
    with pytest.raises(B.AxeError) as e:
        B.axe_gemm_grouped_describe(_grouped_desc(1000, B.AXE_GROUPED_STREAM), B.AXE_DESC_A_LDS)
    assert e.value.code == B.AXE_EUNSUPPORTED
    assert B.axe_gemm_grouped_kernel(_grouped_desc(16)) == B.AXE_GROUPED_STREAM        # 4 rows per group: streamed
    gated = _grouped_desc(1000, B.AXE_GROUPED_TILES_128, B.AXE_EPI_SWIGLU)
    B.axe_gemm_grouped_describe(gated, B.AXE_DESC_ACC)
    with pytest.raises(B.AxeError) as e:
        B.axe_gemm_grouped_describe(gated, B.AXE_DESC_C_STORE)
    assert e.value.code == B.AXE_EUNSUPPORTED
    with pytest.raises(B.AxeError) as e:
        B.axe_gemm_grouped_describe(_grouped_desc(1000), 99)
    assert e.value.code == B.AXE_EINVAL


def test_grouped_kernel_choice_follows_rows_per_group_and_k():
    """Left alone the library streams the weights while groups average few rows and takes the tile kernels beyond; the
    crossover lies higher when K is short (host logic only: the choice is made from M, G and K)."""
    def choice(M, K, G=4, fp8=False):
        N = 512
        if fp8:
            d = B.GroupedGemmDesc(M, N, K, G, B.Layout(W.row_major_spec(M, K)), B.Layout(W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")])),
                                  B.Layout(W.row_major_spec(M, N)), M * K, G * N * K, M * N, in_dtype=B.AXE_FP8_E4M3, out_dtype=B.AXE_BF16)
        else:
            d = B.GroupedGemmDesc(M, N, K, G, B.Layout(W.row_major_spec(M, K)), B.Layout(W.spec([(G, N * K, "m"), (K, 1, "m"), (N, K, "m")])),
                                  B.Layout(W.row_major_spec(M, N)), M * K, G * N * K, M * N)
        return B.axe_gemm_grouped_kernel(d)
    S, T = B.AXE_GROUPED_STREAM, B.AXE_GROUPED_TILES_128
    assert choice(13 * 4, 2048) == S and choice(13 * 4 + 1, 2048) == T
    assert choice(19 * 4, 768) == S and choice(19 * 4 + 1, 768) == T
    assert choice(8 * 4, 2048, fp8=True) == S and choice(8 * 4 + 1, 2048, fp8=True) == T
    assert choice(15 * 4, 768, fp8=True) == S and choice(15 * 4 + 1, 768, fp8=True) == T
    assert choice(384 * 4, 768, fp8=True) == T and choice(384 * 4 + 1, 768, fp8=True) == B.AXE_GROUPED_TILES_256
