"""The layout operators behind the C ABI (host code of the HIP library) against the oracle.

Equality is decided on MAPS, by brute force with the oracle's evaluator over the whole domain, so
that an operator may return a differently refined D as long as it denotes the same function; the
paper's printed examples (tests/golden/paper_examples.json) and its soundness theorems are the
yardstick.  Where an operator's conditions are only sufficient (grouping, tile-of, slice) the library
may fail (AXE_ENOFORM) where the oracle succeeds and vice versa; whatever it returns must be right.
CPU only."""
import itertools
import json
import os
import random
from math import prod

import pytest

from oracle import axe_layout as ax
from oracle.axe_layout import Iter, Layout, LayoutError
from paper_2601_19092_amd import binding as B

AXES = ["m", "lane", "reg"]
GOLDEN = json.load(open(os.path.join(os.path.dirname(__file__), "golden", "paper_examples.json")))


def spec_of(L: Layout) -> dict:
    z = L.swizzle
    return {"D": [(i.extent, i.stride, i.axis) for i in L.D], "R": [(i.extent, i.stride, i.axis) for i in L.R],
            "O": dict(L.O), "swizzle": (z.axis, z.bits, z.base, z.shift) if z else None}


def lib(L: Layout) -> B.Layout:
    return B.Layout(spec_of(L), AXES)


def orc(spec: dict) -> Layout:
    return Layout.from_spec(spec)


def mk(d, R=None, O=None):
    """{"extents": [...], "strides": [...]} as the golden file writes layouts."""
    return Layout.make(tuple(d["extents"]), tuple(d["strides"]), R=R, O=O)


def fmap(L: Layout):
    return [frozenset(ax.evaluate(L, x, AXES)) for x in range(L.E_D)]


def rand_iters(rng, n, max_e=4, neg=True, axes=AXES):
    out = []
    for _ in range(n):
        s = rng.choice([1, 2, 3, 4, 6, 8, 16])
        if neg and rng.random() < 0.2:
            s = -s
        out.append(Iter(rng.randint(1, max_e), s, rng.choice(axes)))
    return tuple(out)


def rand_layout(rng, nd=(1, 4), nr=(0, 2), max_e=4, neg=True):
    D = rand_iters(rng, rng.randint(*nd), max_e, neg)
    R = rand_iters(rng, rng.randint(*nr), 3, neg)
    O = {a: rng.randint(-5, 5) for a in AXES if rng.random() < 0.4}
    return Layout(D, R, ax._norm_offset(O))


def rand_shape_of(rng, E, rank=None):
    """A random factorisation of E into `rank` factors (1..3 when not given)."""
    shape = []
    for _ in range(rng.randint(0, 2) if rank is None else rank - 1):
        divs = [d for d in range(1, E + 1) if E % d == 0]
        d = rng.choice(divs)
        shape.append(d)
        E //= d
    shape.append(E)
    rng.shuffle(shape)
    return tuple(shape)


# ----------------------------------------------------------------------------- span, canonical forms
def test_span_is_the_closed_form_and_the_bruteforce_extent():
    rng = random.Random(11)
    for _ in range(150):
        L = rand_layout(rng)
        got = B.layout_span(lib(L))
        assert got == {a: ax.span_bruteforce(L, AXES)[a] for a in AXES}          # max - min + 1 over the whole image


def test_canonicalize_keeps_the_map_and_reaches_a_normal_form():
    rng = random.Random(12)
    for _ in range(300):
        L = rand_layout(rng, nd=(1, 5), nr=(0, 3))
        C = orc(B.layout_canonicalize(lib(L)))
        assert fmap(C) == fmap(L)                                                # same set-valued map
        assert all(i.extent > 1 for i in C.R) and all(i.stride > 0 for i in C.R)
        assert all(i.extent > 1 for i in C.D) or len(C.D) == 1
        for a, b in zip(C.D, C.D[1:]):                                           # no D1 chain left
            assert not (a.axis == b.axis and a.stride == b.extent * b.stride)
        again = orc(B.layout_canonicalize(lib(C)))
        assert again == C                                                        # idempotent
        want = ax.canonicalize(L)                                                # the oracle's normal form; R is a multiset
        assert (C.D, sorted(C.R, key=repr), C.O) == (want.D, sorted(want.R, key=repr), want.O)


def rewrite(rng, L: Layout) -> Layout:
    """Another way of writing the same set-valued map: unit iters inserted (D0, C0), a sharded iter
    split in two (the inverse of D1), replica iters flipped with their reach moved into O (C1), R shuffled."""
    D = []
    for it in L.D:
        divs = [d for d in range(2, it.extent) if it.extent % d == 0]
        if divs and rng.random() < 0.5:
            d = rng.choice(divs)
            D += [Iter(it.extent // d, d * it.stride, it.axis), Iter(d, it.stride, it.axis)]
        else:
            D.append(it)
        if rng.random() < 0.3:
            D.append(Iter(1, rng.choice([1, 5, -3]), rng.choice(AXES)))
    R, off = [], dict(L.offset)
    for it in L.R:
        if rng.random() < 0.5:
            off[it.axis] = off.get(it.axis, 0) + (it.extent - 1) * it.stride
            it = Iter(it.extent, -it.stride, it.axis)
        R.append(it)
    if rng.random() < 0.3:
        R.append(Iter(1, 9, rng.choice(AXES)))
    rng.shuffle(R)
    return Layout(tuple(D), tuple(R), ax._norm_offset(off))


def test_gap_condition_and_equality():
    rng = random.Random(13)
    differ = 0
    for _ in range(300):
        L1 = rand_layout(rng, nd=(1, 3), nr=(0, 2), max_e=4)
        gc = B.layout_gap_condition(lib(L1))
        r1, _ = ax.canon_OR(L1.R, L1.O)
        assert gc == ax.gap_condition(r1)
        if gc:                                                                   # then distinct replica digits give distinct points
            assert all(len(pts) == prod(i.extent for i in r1) for pts in fmap(L1))
        L2 = rewrite(rng, L1)
        assert fmap(L2) == fmap(L1)
        assert B.layout_equal(lib(L1), lib(L2)) and B.layout_equal(lib(L2), lib(L1))   # the normal form undoes the rewrite
        L3 = rand_layout(rng, nd=(1, 3), nr=(0, 2), max_e=4)
        same = L1.E_D == L3.E_D and fmap(L1) == fmap(L3)
        if B.layout_equal(lib(L1), lib(L3)):
            assert same                                                          # never a false positive
        differ += not same
    assert differ > 250
    # a swizzle stage is part of the identity of a layout
    Z = Layout.make((16, 64), (64, 1), swizzle=ax.Swizzle("m", 3, 3, 6))
    assert B.layout_equal(lib(Z), lib(Z)) and not B.layout_equal(lib(Z), lib(Z.with_(swizzle=None)))


# ----------------------------------------------------------------------------- group, tile, direct sum
def test_group_by_shape_refines_without_changing_the_map():
    rng = random.Random(14)
    ok = failed = 0
    for _ in range(400):
        L = rand_layout(rng, nd=(1, 4), nr=(0, 1), max_e=6)
        shape = rand_shape_of(rng, L.E_D)
        try:
            spec, ends = B.layout_group(lib(L), shape)
        except B.AxeError as e:
            assert e.code == B.AXE_ENOFORM
            with pytest.raises(LayoutError):                                     # the gcd step fails for both or for none
                ax.group(L.D, shape)
            failed += 1
            continue
        G = orc(spec)
        assert fmap(G) == fmap(L)
        lo = 0
        for T, hi in zip(shape, ends):
            assert prod(i.extent for i in G.D[lo:hi]) == T
            lo = hi
        assert lo == len(G.D) or all(i.extent == 1 for i in G.D[lo:])
        ok += 1
    assert ok > 150 and failed > 20


def test_tile_is_sound_and_matches_the_paper_example():
    g = GOLDEN["tile_example"]
    spec, ST = B.layout_tile(lib(mk(g["A"])), g["SA"], lib(mk(g["B"])), g["SB"])
    assert orc(spec) == mk(g["T"]) and ST == (2, 8, 3, 8)
    rng = random.Random(15)
    n = 0
    while n < 150:
        A, Bt = rand_layout(rng, nd=(1, 3), nr=(0, 1), max_e=3), rand_layout(rng, nd=(1, 3), nr=(0, 1), max_e=3)
        rank = rng.randint(1, 2)
        SA, SB = rand_shape_of(rng, A.E_D, rank), rand_shape_of(rng, Bt.E_D, rank)
        try:
            spec, ST = B.layout_tile(lib(A), SA, lib(Bt), SB)
        except B.AxeError as e:
            assert e.code == B.AXE_ENOFORM
            continue
        T = orc(spec)
        assert ST == tuple(v for p in zip(SA, SB) for v in p) and prod(ST) == T.E_D
        sig = ax.span_bruteforce(Bt, AXES)
        # f_T(x || y) = f_A(x) (.) span(B) + f_B(y)   (theorem of App. C), as sets of points
        for x in itertools.product(*[range(s) for s in SA]):
            fa = ax.evaluate_at(A, SA, x, AXES)
            for y in itertools.product(*[range(s) for s in SB]):
                u = tuple(v for p in zip(x, y) for v in p)
                want = {tuple(pa[k] * sig[AXES[k]] + pb[k] for k in range(3)) for pa in fa
                        for pb in ax.evaluate_at(Bt, SB, y, AXES)}
                assert set(ax.evaluate_at(T, ST, u, AXES)) == want
        n += 1


def test_direct_sum_example_and_scaled_direct_sum_is_tile():
    g = GOLDEN["direct_sum_example"]
    spec, ST = B.layout_direct_sum(lib(mk(g["A"])), (2, 2), lib(mk(g["B"])), (2, 2))
    S = orc(spec)
    assert ST == (2, 2, 2, 2)
    for p, i, q, j in itertools.product(range(2), repeat=4):
        assert ax.evaluate_at(S, ST, (p, i, q, j), ["m"]) == [(8 * p + 2 * q + 4 * i + j,)]
    rng = random.Random(16)
    n = 0
    while n < 100:
        A, Bt = rand_layout(rng, nd=(1, 3), nr=(0, 0), max_e=3), rand_layout(rng, nd=(1, 3), nr=(0, 1), max_e=3)
        A = A.with_(O={})
        SA, SB = (A.E_D,), (Bt.E_D,)
        W = B.layout_span(lib(Bt))
        scaled = A.with_(D=[Iter(i.extent, i.stride * W[i.axis], i.axis) for i in A.D])
        s1, _ = B.layout_direct_sum(lib(scaled), SA, lib(Bt), SB)
        s2, _ = B.layout_tile(lib(A), SA, lib(Bt), SB)
        assert fmap(orc(s1)) == fmap(orc(s2))                                    # (A . W) + B = A (x) B
        n += 1


def test_tile_keeps_a_swizzled_atom_when_the_tiler_steps_over_whole_periods():
    """The blocked, swizzled destination of the relayout workload as a product: a grid of tiles times a
    swizzled 128 x 64 atom (Sec. 3.4: the swizzle is a separate innermost layout)."""
    atom = Layout.make((128, 64), (64, 1), swizzle=ax.Swizzle("m", 3, 3, 6))
    grid = Layout.make((4, 2), (2, 1))
    spec, ST = B.layout_tile(B.Layout(spec_of(grid), ["m"]), (4, 2), B.Layout(spec_of(atom), ["m"]), (128, 64))
    T = orc(spec)
    assert T.swizzle == atom.swizzle and ST == (4, 128, 2, 64)
    for u in ((0, 0, 0, 0), (3, 77, 1, 13), (2, 127, 0, 63), (1, 5, 1, 40)):
        (base,), = ax.evaluate_at(grid, (4, 2), (u[0], u[2]), ["m"])
        (inner,), = ax.evaluate_at(atom, (128, 64), (u[1], u[3]), ["m"])
        assert ax.evaluate_at(T, ST, u, ["m"]) == [(base * 8192 + inner,)]
    # a tiler that lands inside a swizzle period is refused: 512-element period, atom span 192
    small = Layout.make((3, 64), (64, 1), swizzle=ax.Swizzle("m", 3, 3, 6))
    with pytest.raises(B.AxeError) as e:
        B.layout_tile(B.Layout(spec_of(grid), ["m"]), (4, 2), B.Layout(spec_of(small), ["m"]), (3, 64))
    assert e.value.code == B.AXE_EUNSUPPORTED


# ----------------------------------------------------------------------------- tile-of, slice
def test_tile_of_recovers_the_outer_layout():
    rng = random.Random(17)
    hit = 0
    for _ in range(400):
        Cl = rand_layout(rng, nd=(1, 3), nr=(0, 1), max_e=3, neg=False)
        Bt = rand_layout(rng, nd=(1, 3), nr=(0, 1), max_e=3, neg=False)
        rank = rng.randint(1, 2)
        SC, SB = rand_shape_of(rng, Cl.E_D, rank), rand_shape_of(rng, Bt.E_D, rank)
        try:
            A, SA = ax.tile(Cl, SC, Bt, SB)
        except LayoutError:
            continue
        SA2 = tuple(a * b for a, b in zip(SC, SB))
        if len(A.D) > 16 or len(A.R) > 8:
            continue
        try:
            spec, got_shape = B.layout_tile_of(lib(A), SA2, lib(Bt), SB)
        except B.AxeError as e:
            assert e.code == B.AXE_ENOFORM                                       # sufficient conditions only
            continue
        assert got_shape == SC
        back, _ = ax.tile(orc(spec), SC, Bt, SB)                                 # C recovered => C (x) B == A as maps
        assert fmap(back) == fmap(A)
        hit += 1
    assert hit > 120
    # the appendix's counter-example: (16):(1) is no tile of the strided atom
    g = GOLDEN["direct_sum_example"]
    with pytest.raises(B.AxeError) as e:
        B.layout_tile_of(lib(Layout.make((16,), (1,))), (4, 4), lib(mk(g["B"])), (2, 2))
    assert e.value.code == B.AXE_ENOFORM
    # and an aligned one: 16 x 24 row-major tiles of 8 x 8 inside a (2, 3) grid
    t = GOLDEN["tile_example"]
    spec, sc = B.layout_tile_of(lib(mk(t["T"])), (16, 24), lib(mk(t["B"])), t["SB"])
    assert sc == (2, 3) and fmap(orc(spec)) == fmap(mk(t["A"]))


def test_slice_matches_the_shifted_map_on_every_region_it_accepts():
    g = GOLDEN["slice_example"]
    S = orc(B.layout_slice(lib(mk(g["L"])), g["S"], g["begin"], g["size"]))
    assert fmap(S) == fmap(mk(g["result"], O={"m": g["result_offset"]}))
    rng = random.Random(18)
    accepted = refused = wraps = 0
    for _ in range(250):
        L = rand_layout(rng, nd=(1, 4), nr=(0, 1), max_e=5)
        shape = rand_shape_of(rng, L.E_D)
        try:
            ax.group(L.D, shape)
        except LayoutError:
            continue
        for _ in range(6):
            begin = tuple(rng.randrange(s) for s in shape)
            size = tuple(rng.randint(1, s - b) for s, b in zip(shape, begin))
            try:
                S = orc(B.layout_slice(lib(L), shape, begin, size))
            except B.AxeError as e:
                assert e.code == B.AXE_ENOFORM
                refused += 1
                continue
            assert ax.admits(S, size)
            for u in itertools.product(*[range(t) for t in size]):
                shifted = tuple(a + b for a, b in zip(u, begin))
                assert set(ax.evaluate_at(S, size, u, AXES)) == set(ax.evaluate_at(L, shape, shifted, AXES))
            accepted += 1
            wraps += any(i.extent == 2 and j.axis == i.axis for i, j in zip(S.D, S.D[1:])) and len(S.D) > len(shape)
    assert accepted > 300 and refused > 30
    # the symmetric one-wrap form: rows of 6 inside (4, 6):(6, 1), region [4, 8) of the flattened block
    L = Layout.make((4, 6), (10, 1))
    S = orc(B.layout_slice(lib(L), (24,), (4,), (4,)))
    assert [ax.evaluate(S, x, ["m"])[0][0] for x in range(4)] == [4, 5, 10, 11]
    # a slice of a swizzled layout keeps the stage (it acts on the sum D + R + O)
    Z = Layout.make((16, 64), (64, 1), swizzle=ax.Swizzle("m", 3, 3, 6))
    S = orc(B.layout_slice(B.Layout(spec_of(Z), ["m"]), (16, 64), (4, 16), (8, 32)))
    for u in ((0, 0), (7, 31), (3, 9)):
        assert ax.evaluate_at(S, (8, 32), u, ["m"]) == ax.evaluate_at(Z, (16, 64), (u[0] + 4, u[1] + 16), ["m"])


def test_errors_are_codes_not_crashes():
    L = lib(Layout.make((4, 6), (6, 1)))
    with pytest.raises(B.AxeError) as e:
        B.layout_group(L, (5, 5))
    assert e.value.code == B.AXE_ESHAPE
    with pytest.raises(B.AxeError) as e:
        B.layout_slice(L, (4, 6), (2, 0), (3, 6))
    assert e.value.code == B.AXE_ESHAPE
    with pytest.raises(B.AxeError) as e:
        B.layout_tile(L, (4, 6), lib(Layout.make((4,), (1,))), (3, 2))
    assert e.value.code == B.AXE_ESHAPE
    big = Layout(tuple(Iter(2, 3 ** k, "m") for k in range(12)))
    with pytest.raises(B.AxeError) as e:                                         # 24 iters do not fit a layout
        B.layout_tile(lib(big), (2 ** 12,), lib(big), (2 ** 12,))
    assert e.value.code == B.AXE_ERANGE


# ----------------------------------------------------------------------------- flatten (a thread-distributed layout as a memory image)
def test_flatten_is_the_weighted_sum_of_the_coordinates():
    """Oracle pinned to the definition by brute force: every replica of every point of flatten_axes(L) is
    sum_a pitch[a] * (coordinate of L on axis a); then the library against the oracle, as maps."""
    rng = random.Random(41)
    for _ in range(200):
        L = rand_layout(rng)
        pitch = {a: rng.choice([1, 2, 7, 64, 1000, -3]) for a in AXES}
        to = rng.choice(AXES)
        F = ax.flatten_axes(L, pitch, to)
        k = AXES.index(to)
        for x in range(L.E_D):
            want = sorted(sum(pitch[a] * c[i] for i, a in enumerate(AXES)) for c in ax.evaluate(L, x, AXES))
            got = sorted(c[k] for c in ax.evaluate(F, x, AXES))
            assert got == want
            assert all(c[i] == 0 for c in ax.evaluate(F, x, AXES) for i in range(len(AXES)) if i != k)
        got = orc(B.layout_flatten(lib(L), pitch, to))
        assert fmap(got) == fmap(F)


def test_flatten_the_tensor_core_tile_of_the_paper_into_warp_lane_reg_memory():
    """Sec. 2.2's 8 x 16 tensor-core tile on (lane, warp, reg) with its replication and offset, written to memory as
    [warp][lane][reg] (32 lanes, 2 registers): the two replicas of the 128 elements fill exactly the 64-element
    images of the four warps the paper lists, each address once."""
    g = GOLDEN["tensor_core_tile"]
    axes = ["m", "lane", "warp", "reg"]
    L = Layout.make(tuple(g["D"]["extents"]), tuple(g["D"]["strides"]), R=(tuple(g["R"]["extents"]), tuple(g["R"]["strides"])), O=g["O"])
    per_warp = g["lanes"] * g["regs"]
    pitch = {"warp": per_warp, "lane": g["regs"], "reg": 1, "m": 1}
    F = ax.flatten_axes(L, pitch, "m")
    n = prod(g["shape"])
    addrs = sorted(c[0] for x in range(n) for c in ax.evaluate(F, x, axes))
    assert addrs == sorted(per_warp * w + t for w in g["warps_with_offset"] for t in range(per_warp))
    for x in range(n):                                            # and point by point, the definition
        for c, f in zip(sorted(ax.evaluate(L, x, axes)), sorted(ax.evaluate(F, x, axes))):
            assert f == (per_warp * c[2] + g["regs"] * c[1] + c[3], 0, 0, 0)
    got = Layout.from_spec(B.layout_flatten(B.Layout(spec_of(L), axes), pitch, "m"))
    assert all(sorted(ax.evaluate(got, x, axes)) == sorted(ax.evaluate(F, x, axes)) for x in range(n))


def test_flatten_refusals():
    L = Layout.make((4, 8), ("1@lane", "1@reg"))
    with pytest.raises(B.AxeError) as e:
        B.layout_flatten(lib(L), {"lane": 8}, "m")                 # axis reg carries an iter and has no pitch
    assert e.value.code == B.AXE_EINVAL
    with pytest.raises(LayoutError):
        ax.flatten_axes(L, {"lane": 8}, "m")
    sw = Layout.make((4, 8), ("8@m", "1@m")).with_(swizzle=ax.Swizzle("m", 2, 0, 3))
    with pytest.raises(B.AxeError) as e:
        B.layout_flatten(lib(sw), {"m": 1}, "m")
    assert e.value.code == B.AXE_EUNSUPPORTED
    with pytest.raises(LayoutError):
        ax.flatten_axes(sw, {"m": 1}, "m")
