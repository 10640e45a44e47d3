"""Pins for the layout oracle: the worked examples the paper prints (tests/golden/paper_examples.json)
and the lemmas / theorems of its appendices as brute-force property tests on small layouts.
CPU only."""
import itertools
import random
from math import prod

import numpy as np
import pytest

from oracle import axe_layout as ax
from oracle.axe_layout import Iter, Layout, LayoutError, Swizzle
from oracle.axe_ref import evaluate_np


def mk(d, R=None, O=None):
    r = (R["extents"], R["strides"]) if R else None
    return Layout.make(d["extents"], d["strides"], R=r, O=O)


# ----------------------------------------------------------------------------- worked examples
def test_tensor_core_tile(golden):
    g = golden["tensor_core_tile"]
    axes = ["warp", "lane", "reg"]
    no_off = mk(g["D"], g["R"])
    with_off = mk(g["D"], g["R"], g["O"])
    shape = g["shape"]
    for L, warps in ((no_off, g["warps_without_offset"]), (with_off, g["warps_with_offset"])):
        seen = set()
        hits = {}
        for i in range(shape[0]):
            for j in range(shape[1]):
                pts = ax.evaluate_at(L, shape, (i, j), axes)
                assert len(pts) == g["replicas"] == len(set(pts))
                for p in pts:
                    seen.add(p[0])
                    hits[p] = hits.get(p, 0) + 1
        assert sorted(seen) == warps
        assert all(v == 1 for v in hits.values())
        assert len(hits) == len(warps) * g["lanes"] * g["regs"]
    # D alone covers warp{0,1} x lane[32] x reg[2] exactly once; row -> 4@lane, column -> warp, lane, reg
    d_only = mk(g["D"])
    cnt = ax.image_counts(d_only, axes)
    assert set(cnt) == set(itertools.product(range(2), range(32), range(2))) and set(cnt.values()) == {1}
    for i in range(8):
        for j in range(16):
            (w, l, r), = ax.evaluate_at(d_only, shape, (i, j), axes)
            assert (w, l, r) == (j // 8, 4 * i + (j // 2) % 4, j % 2)


def test_mesh_fully_sharded(golden):
    g = golden["mesh_fully_sharded"]
    L = mk(g["D"])
    dev = g["device_matrix_rows_cols"]
    per = {}
    for i in range(64):
        for j in range(128):
            (gpu, m), = ax.evaluate_at(L, g["shape"], (i, j), ["gpuid", "m"])
            assert gpu == dev[i // 32][j // 64]
            assert m == 128 * (i % 32) + (j % 64)
            per[gpu] = per.get(gpu, 0) + 1
    assert per == {k: g["per_gpu_elements"] for k in range(4)}


def test_mesh_shard_replica(golden):
    g = golden["mesh_shard_replica"]
    L = mk(g["D"], g["R"])
    for i in range(64):
        for j in (0, 1, 77, 127):
            pts = ax.evaluate_at(L, g["shape"], (i, j), ["gpuid", "m"])
            assert sorted(p[0] for p in pts) == g["gpus_of_row_half"][i // 32]
            assert {p[1] for p in pts} == {128 * (i % 32) + j}


@pytest.mark.parametrize("name", ["scratchpad", "tensor_memory"])
def test_native_memory_spans(golden, name):
    g = golden[name]
    L = mk(g["D"])
    assert ax.span(L) == g["span"]
    assert ax.span_bruteforce(L) == g["span"]


def test_cute_partition(golden):
    g = golden["cute_partition"]
    L = mk(g["D"], O=g["O"])
    C = ax.row_major(g["tensor_shape"])
    assert g["O"]["m"] == 16 * 128 + 64
    # bind the first two iters to tx//8, tx%8: each thread keeps (2,4):(4,1) + offset
    for tx in range(g["threads"]):
        off = (tx // 8) * 128 + (tx % 8) * 8 + 2112
        per = mk(g["per_thread"], O={"m": off})
        row0, col0 = 16 + tx // 8, 64 + 8 * (tx % 8)
        got = [ax.evaluate(per, x, ["m"])[0][0] for x in range(8)]
        want = [ax.evaluate_at(C, g["tensor_shape"], (row0, col0 + c), ["m"])[0][0] for c in range(8)]
        assert got == want
        # the same addresses through the full partition layout with the thread digits fixed
        full = [ax.evaluate_at(L, (16, 8, 2, 4), (tx // 8, tx % 8, a, b), ["m"])[0][0]
                for a in range(2) for b in range(4)]
        assert full == want
    # the partition is the slice of the row-major tensor on that region
    S = ax.slice_layout(C, g["tensor_shape"], g["region_begin"], g["region_size"])
    for u in itertools.product(range(16), range(64)):
        assert ax.evaluate_at(S, (16, 64), u, ["m"]) == ax.evaluate_at(L, (16, 64), u, ["m"])


def test_triton_local(golden):
    g = golden["triton_local"]
    L = mk(g["D"])
    cnt = ax.image_counts(L, ["tx", "reg"])
    assert set(cnt) == set(itertools.product(range(g["tx"]), range(g["reg"])))
    assert set(cnt.values()) == {1}
    # element (r, c) of the 16x64 region sits in thread 8r + c//8, register c%8
    for r in range(16):
        for c in range(64):
            assert ax.evaluate_at(L, (16, 64), (r, c), ["tx", "reg"]) == [(8 * r + c // 8, c % 8)]


def test_tile_example(golden):
    g = golden["tile_example"]
    A, B = mk(g["A"]), mk(g["B"])
    T, ST = ax.tile(A, g["SA"], B, g["SB"])
    assert T == mk(g["T"])
    assert ST == (2, 8, 3, 8)
    assert ax.span(B)["m"] == g["span_B"] == ax.span_bruteforce(B)["m"]
    # 16x24 matrix stored as a 2x3 grid of contiguous 8x8 tiles
    for i in range(16):
        for j in range(24):
            (m,), = ax.evaluate_at(T, (16, 24), (i, j), ["m"])
            assert m == ((i // 8) * 3 + j // 8) * 64 + (i % 8) * 8 + j % 8


def test_slice_example(golden):
    g = golden["slice_example"]
    L = mk(g["L"])
    S = ax.slice_layout(L, g["S"], g["begin"], g["size"])
    assert S == mk(g["result"], O={"m": g["result_offset"]})
    for u in itertools.product(range(8), range(16)):
        assert (ax.evaluate_at(S, g["size"], u, ["m"])
                == ax.evaluate_at(L, g["S"], (u[0] + g["begin"][0], u[1] + g["begin"][1]), ["m"]))


def test_direct_sum_example(golden):
    g = golden["direct_sum_example"]
    A, B = mk(g["A"]), mk(g["B"])
    assert sorted(ax.evaluate(A, x, ["m"])[0][0] for x in range(4)) == g["image_A"]
    assert sorted(ax.evaluate(B, x, ["m"])[0][0] for x in range(4)) == g["image_B"]
    S, ST = ax.direct_sum(A, (2, 2), B, (2, 2))
    # grouped by the interleaved shape (2,2,2,2) = (p, i, q, j):  8p + 4i + 2q + j
    assert ST == (2, 2, 2, 2)
    for p, i, q, j in itertools.product(range(2), repeat=4):
        assert ax.evaluate_at(S, ST, (p, i, q, j), ["m"]) == [(8 * p + 2 * q + 4 * i + j,)]
    assert sorted(ax.evaluate(S, x, ["m"])[0][0] for x in range(16)) == list(range(16))
    # the paper lists the blocks as A then B (domain order p,q,i,j): same image
    listed = mk(g["sum_D"])
    assert sorted(ax.evaluate(listed, x, ["m"])[0][0] for x in range(16)) == list(range(16))
    # the D1 chain printed in the appendix
    chain = [mk(c) for c in g["chain"]]
    for a, b in zip(chain, chain[1:]):
        assert [ax.evaluate(a, x, ["m"]) for x in range(16)] == [ax.evaluate(b, x, ["m"]) for x in range(16)]
    assert ax.canon_D(chain[0].D) == chain[-1].D
    # tiling cannot reach (16):(1): every value of C (x) B is congruent to {0,1,4,5} mod 6
    assert ax.span(B)["m"] == g["span_B"]
    for C in (Layout.make((4,), (1,)), Layout.make((2, 2), (2, 1)), Layout.make((2, 2), (1, 2))):
        T, ST = ax.tile(C, (2, 2) if len(C.D) == 2 else (4, 1), B, (2, 2))
        res = {ax.evaluate(T, x, ["m"])[0][0] % 6 for x in range(16)}
        assert res <= set(g["residues_mod_span"])
    with pytest.raises(LayoutError):
        ax.tile_of(Layout.make((16,), (1,)), (4, 4), B, (2, 2))


def test_non_bit_linear(golden):
    g = golden["non_bit_linear"]
    L = Layout.make((24, 24), (1, 24))       # column-major 24x24: f(i) = i//24 + 24*(i%24)
    f = lambda x: ax.evaluate(L, x, ["m"])[0][0]
    assert (f(1), f(2), f(3)) == (g["f1"], g["f2"], g["f3"])
    assert f(1) ^ f(2) == g["f1_xor_f2"] != f(1 ^ 2)


def test_reduce_scatter_signature(golden):
    g = golden["reduce_scatter_signature"]
    n = g["devices"]
    src = Layout.make((n, 64, 64), ("1@gpuid", 64, 1))               # (4,64,64) sharded on dim 0
    dst = Layout.make((n, 64 // n, 64), ("1@gpuid", 64, 1))          # (64,64) sharded on dim 0
    assert ax.admits(src, g["in_shape"]) and ax.admits(dst, g["out_shape"])
    owners = {ax.evaluate_at(dst, g["out_shape"], (r, 0), ["gpuid", "m"])[0][0] for r in range(64)}
    assert owners == set(range(n))


# ----------------------------------------------------------------------------- random layouts
AXES = ["m", "lane", "reg"]


def rand_iters(rng, n, max_e=4, axes=AXES, neg=True):
    out = []
    for _ in range(n):
        s = rng.choice([1, 2, 3, 4, 6, 8, 16])
        if neg and rng.random() < 0.2:
            s = -s
        out.append(Iter(rng.randint(1, max_e), s, rng.choice(axes)))
    return tuple(out)


def rand_layout(rng, nd=(1, 4), nr=(0, 2), max_e=4, axes=AXES):
    D = rand_iters(rng, rng.randint(*nd), max_e, axes)
    R = rand_iters(rng, rng.randint(*nr), 3, axes)
    O = {a: rng.randint(-5, 5) for a in axes if rng.random() < 0.4}
    return Layout(D, R, ax._norm_offset(O))


def fmap(L, axes=AXES):
    return [frozenset(ax.evaluate(L, x, axes)) for x in range(L.E_D)]


def test_unflatten_is_lexicographic_and_digit_identity():
    rng = random.Random(1)
    for _ in range(200):
        ext = [rng.randint(1, 5) for _ in range(rng.randint(1, 5))]
        E = prod(ext)
        all_digits = [ax.unflatten(x, ext) for x in range(E)]
        assert all_digits == list(itertools.product(*[range(e) for e in ext]))   # textbook odometer
        assert all_digits == [tuple(int(v) for v in np.unravel_index(x, ext)) for x in range(E)]
        # App. A exact digit identity: d_i = phi_i - e_i * phi_{i-1}
        for x in range(E):
            phi_prev = 0
            for i, e in enumerate(ext):
                phi = x // prod(ext[i + 1:])
                assert all_digits[x][i] == phi - e * phi_prev
                phi_prev = phi


def test_row_major_matches_numpy_strides():
    rng = random.Random(2)
    for _ in range(50):
        shape = tuple(rng.randint(1, 5) for _ in range(rng.randint(1, 4)))
        arr = np.arange(prod(shape)).reshape(shape)
        L = ax.row_major(shape)
        for u in itertools.product(*[range(s) for s in shape]):
            assert ax.evaluate_at(L, shape, u, ["m"]) == [(int(arr[u]),)]
        # a transposed (column-major) view: strides from numpy
        t = np.asfortranarray(arr)
        Lt = Layout.make(shape, [s // t.itemsize for s in t.strides])
        flat = t.ravel(order="K")
        for u in itertools.product(*[range(s) for s in shape]):
            (addr,), = ax.evaluate_at(Lt, shape, u, ["m"])
            assert flat[addr] == arr[u]


def test_replica_count_and_set_semantics():
    rng = random.Random(3)
    for _ in range(200):
        L = rand_layout(rng)
        for x in range(L.E_D):
            pts = ax.evaluate(L, x, AXES)
            assert len(pts) == L.E_R                       # |f_L(x)| = E_R as a multiset
            d = ax.f_D(L, x)
            want = set()
            for r in itertools.product(*[range(i.extent) for i in L.R]):
                c = dict(d)
                for a, v in ax.f_R(L, r).items():
                    c[a] = c.get(a, 0) + v
                for a, v in L.O:
                    c[a] = c.get(a, 0) + v
                want.add(tuple(c.get(a, 0) for a in AXES))
            assert set(pts) == want


def test_span_closed_form_equals_bruteforce():
    rng = random.Random(4)
    for _ in range(300):
        L = rand_layout(rng)
        assert ax.span(L, AXES) == ax.span_bruteforce(L, AXES)


def test_canon_D_preserves_map_and_is_normal():
    rng = random.Random(5)
    merged = 0
    for _ in range(400):
        D = list(rand_iters(rng, rng.randint(1, 5), 4))
        # plant mergeable chains now and then
        if rng.random() < 0.6 and len(D) >= 2:
            i = rng.randrange(len(D) - 1)
            D[i] = Iter(D[i].extent, D[i + 1].extent * D[i + 1].stride, D[i + 1].axis)
        L = Layout(tuple(D))
        C = Layout(ax.canon_D(L.D))
        assert fmap(L) == fmap(C)
        merged += len(C.D) < len([i for i in D if i.extent > 1])
        for a, b in zip(C.D, C.D[1:]):
            assert not (a.axis == b.axis and a.stride == b.extent * b.stride)
        assert all(i.extent > 1 for i in C.D) or (len(C.D) == 1 and L.E_D == 1)
        assert ax.canon_D(C.D) == C.D
    assert merged > 20


def test_split_and_fuse_rules():
    rng = random.Random(6)
    for _ in range(200):
        D = list(rand_iters(rng, rng.randint(1, 3), 3))
        e1, e2 = rng.randint(1, 4), rng.randint(1, 4)
        s, a = rng.choice([1, 2, -3, 5]), rng.choice(AXES)
        pos = rng.randint(0, len(D))
        whole = Layout(tuple(D[:pos] + [Iter(e1 * e2, s, a)] + D[pos:]))
        split = Layout(tuple(D[:pos] + [Iter(e1, e2 * s, a), Iter(e2, s, a)] + D[pos:]))
        assert fmap(whole) == fmap(split)


def test_canon_OR_preserves_set_map():
    rng = random.Random(7)
    absorbed = 0
    for _ in range(400):
        L = rand_layout(rng, nr=(0, 3))
        if rng.random() < 0.5 and L.R:
            # plant an absorbable multiple, including the boundary q = extent
            base = L.R[0]
            if base.extent > 1:
                q = rng.choice([1, base.extent, max(1, base.extent - 1)])
                L = L.with_(R=L.R + (Iter(rng.randint(2, 3), q * abs(base.stride) * (1 if base.stride > 0 else -1), base.axis),))
        R2, O2 = ax.canon_OR(L.R, L.O)
        C = Layout(L.D, R2, O2)
        assert fmap(L) == fmap(C)
        assert all(i.stride > 0 and i.extent > 1 for i in R2)
        absorbed += len(R2) < len([i for i in L.R if i.extent > 1])
    assert absorbed > 20


def test_c2_boundary_cases_bruteforce():
    # q = e_i is still exact (union of runs is contiguous); q = e_i + 1 leaves a hole
    for e1 in range(2, 5):
        for e2 in range(2, 4):
            for q in range(1, e1 + 2):
                vals = {r1 + q * r2 for r1 in range(e1) for r2 in range(e2)}
                contiguous = vals == set(range(e1 + q * (e2 - 1)))
                assert contiguous == (q <= e1)
                R2, _ = ax.canon_OR((Iter(e1, 1, "m"), Iter(e2, q, "m")), ())
                if q <= e1:
                    assert R2 == (Iter(e1 + q * (e2 - 1), 1, "m"),)
                else:
                    assert len(R2) == 2


def test_gap_condition_means_distinct_replicas():
    rng = random.Random(8)
    seen_true = seen_false = 0
    for _ in range(300):
        R = tuple(Iter(rng.randint(2, 3), rng.choice([1, 2, 3, 4, 6, 8, 12]), "m") for _ in range(rng.randint(1, 3)))
        R2, _ = ax.canon_OR(R, ())
        L = Layout((Iter(1, 1, "m"),), R2)
        pts = ax.evaluate(L, 0, ["m"])
        if ax.gap_condition(R2):
            seen_true += 1
            assert len(set(pts)) == len(pts)
        else:
            seen_false += 1
    assert seen_true > 20 and seen_false > 5


def test_canonical_form_decides_equality_under_gc():
    rng = random.Random(9)
    for _ in range(200):
        L = rand_layout(rng, nr=(0, 1))
        # a structurally different writing of the same map: split an iter, add unit iters, flip an R sign
        D = []
        for it in L.D:
            if it.extent % 2 == 0 and rng.random() < 0.5:
                D += [Iter(2, (it.extent // 2) * it.stride, it.axis), Iter(it.extent // 2, it.stride, it.axis)]
            else:
                D.append(it)
            if rng.random() < 0.3:
                D.append(Iter(1, 7, "reg"))
        R, O = [], dict(L.O)
        for it in L.R:
            O[it.axis] = O.get(it.axis, 0) + (it.extent - 1) * it.stride
            R.append(Iter(it.extent, -it.stride, it.axis))
        L2 = Layout(tuple(D), tuple(R), ax._norm_offset(O))
        assert fmap(L) == fmap(L2)
        assert ax.equivalent_by_canon(L, L2)


def test_group_by_shape():
    rng = random.Random(10)
    ok = fail = 0
    for _ in range(500):
        D = rand_iters(rng, rng.randint(1, 4), 6, neg=False)
        E = prod(i.extent for i in D)
        # random factorisation of E into 1..3 factors
        shape, rest = [], E
        for _ in range(rng.randint(0, 2)):
            divs = [d for d in range(1, rest + 1) if rest % d == 0]
            f = rng.choice(divs)
            shape.append(f)
            rest //= f
        shape.append(rest)
        L = Layout(D)
        try:
            G, bounds = ax.grouped(L, shape)
        except LayoutError:
            fail += 1
            continue
        ok += 1
        assert fmap(G) == fmap(L)
        lo = 0
        for hi, s in zip(bounds, shape):
            assert prod(i.extent for i in G.D[lo:hi]) == s
            lo = hi
    assert ok > 100 and fail > 20
    # a case the gcd step must reject: (6):(1) by (4, ...) style splits
    with pytest.raises(LayoutError):
        ax.group((Iter(3, 1, "m"), Iter(4, 3, "m")), (2, 6))
    with pytest.raises(LayoutError):
        ax.group((Iter(4, 1, "m"),), (2, 3))


def test_tile_soundness():
    rng = random.Random(11)
    done = 0
    while done < 150:
        A, B = rand_layout(rng, nd=(1, 3), max_e=3), rand_layout(rng, nd=(1, 3), max_e=3)
        r = rng.randint(1, 2)
        def shape_for(L):
            E = L.E_D
            if r == 1:
                return (E,)
            divs = [d for d in range(1, E + 1) if E % d == 0]
            f = rng.choice(divs)
            return (f, E // f)
        SA, SB = shape_for(A), shape_for(B)
        try:
            T, ST = ax.tile(A, SA, B, SB)
            GA, _ = ax.grouped(A, SA)
            GB, _ = ax.grouped(B, SB)
        except LayoutError:
            continue
        done += 1
        sig = ax.span_bruteforce(B, AXES)
        assert ax.admits(T, ST)
        for x in itertools.product(*[range(s) for s in SA]):
            fa = ax.evaluate_at(GA, SA, x, AXES)
            for y in itertools.product(*[range(s) for s in SB]):
                fb = ax.evaluate_at(GB, SB, y, AXES)
                u = tuple(v for pair in zip(x, y) for v in pair)
                got = frozenset(ax.evaluate_at(T, ST, u, AXES))
                want = frozenset(tuple(pa[i] * sig[a] + pb[i] for i, a in enumerate(AXES))
                                 for pa in fa for pb in fb)
                assert got == want


def test_scaled_direct_sum_is_tile():
    rng = random.Random(12)
    done = 0
    while done < 100:
        A = Layout(rand_iters(rng, rng.randint(1, 3), 3))            # R^A empty, O^A = 0
        B = rand_layout(rng, nd=(1, 3), max_e=3)
        SA, SB = (A.E_D,), (B.E_D,)
        T, ST = ax.tile(A, SA, B, SB)
        S, ST2 = ax.direct_sum(ax.scale_D(A, ax.span(B, AXES)), SA, B, SB)
        assert ST == ST2 and fmap(T) == fmap(S)
        done += 1


def test_tile_of_recovers_outer_layout():
    rng = random.Random(13)
    ok = 0
    for _ in range(400):
        C = Layout(rand_iters(rng, rng.randint(1, 2), 3, neg=False), (), ax._norm_offset({"m": rng.randint(0, 2)}))
        B = Layout(rand_iters(rng, rng.randint(1, 2), 3, neg=False), (), ax._norm_offset({"m": rng.randint(0, 2)}))
        SC, SB = (C.E_D,), (B.E_D,)
        T, ST = ax.tile(C, SC, B, SB)
        SA = (SC[0] * SB[0],)
        try:
            C2, SC2 = ax.tile_of(T, SA, B, SB)
        except LayoutError:
            continue
        ok += 1
        assert SC2 == SC
        T2, _ = ax.tile(C2, SC2, B, SB)
        assert fmap(T2) == fmap(T)                       # recovered C satisfies C (x) B == A
    assert ok > 150
    # the printed example: recover (2,3):(3,1) from the blocked 16x24 layout
    A = Layout.make((2, 8, 3, 8), (192, 8, 64, 1))
    C, SC = ax.tile_of(A, (16, 24), Layout.make((8, 8), (8, 1)), (8, 8))
    assert SC == (2, 3) and C.D == Layout.make((2, 3), (3, 1)).D


def test_slice_equality_on_every_sliceable_region():
    rng = random.Random(14)
    ok = fail = wraps = 0
    for _ in range(250):
        L = rand_layout(rng, nd=(1, 4), max_e=4)
        E = L.E_D
        divs = [d for d in range(1, E + 1) if E % d == 0]
        f = rng.choice(divs)
        shape = (f, E // f)
        try:
            ax.group(L.D, shape)
        except LayoutError:
            continue
        for b0 in range(shape[0]):
            for t0 in range(1, shape[0] - b0 + 1):
                b1 = rng.randrange(shape[1])
                t1 = rng.randint(1, shape[1] - b1)
                try:
                    S = ax.slice_layout(L, shape, (b0, b1), (t0, t1))
                except LayoutError:
                    fail += 1
                    continue
                ok += 1
                assert ax.admits(S, (t0, t1))
                for u in itertools.product(range(t0), range(t1)):
                    assert (frozenset(ax.evaluate_at(S, (t0, t1), u, AXES))
                            == frozenset(ax.evaluate_at(L, shape, (u[0] + b0, u[1] + b1), AXES)))
    assert ok > 300 and fail > 50


def test_slice_one_wrap_form():
    # block (4,6):(100,1) on one axis, region [4, 8) of the flattened 24: digits (0,4) .. (1,1):
    # pivot digit wraps once, T=4 even, d0 + T/2 = 6 = E_k
    L = Layout.make((4, 6), (100, 1))
    S = ax.slice_layout(L, (24,), (4,), (4,))
    assert S.D == (Iter(2, 100 - 4 * 1, "m"), Iter(2, 1, "m"))
    assert [ax.evaluate(S, x, ["m"])[0][0] for x in range(4)] == [4, 5, 100, 101]
    # the carry must not wrap digit k-1 (last row): region [22, 24+2) does not exist; [16,20) would
    # need digit 0 to go 2 -> 3 (fine), [22,24) is no-wrap
    S2 = ax.slice_layout(L, (24,), (16,), (4,))
    assert [ax.evaluate(S2, x, ["m"])[0][0] for x in range(4)] == [204, 205, 300, 301]
    # three-level block where the carry out of digit k-1 would propagate: must be refused
    L3 = Layout.make((2, 2, 6), (1000, 100, 1))
    with pytest.raises(LayoutError):
        ax.slice_layout(L3, (24,), (10,), (4,))          # digits (0,1,4): carry 1 -> 0 and into digit 0
    # and without the refusal the single-iter form would indeed be wrong there
    want = [ax.evaluate(L3, x, ["m"])[0][0] for x in range(10, 14)]
    assert want == [104, 105, 1000, 1001]


def test_swizzle_is_an_involution_on_aligned_blocks():
    for bits, base, shift in ((3, 3, 6), (3, 0, 3), (2, 4, 7), (0, 0, 0), (1, 0, 5)):
        z = Swizzle("m", bits, base, shift)
        block = 1 << (shift + bits)
        for start in (0, block, 5 * block):
            img = [z.apply(x) for x in range(start, start + block)]
            assert sorted(img) == list(range(start, start + block))
            assert [z.apply(y) for y in img] == list(range(start, start + block))
    with pytest.raises(ValueError):
        Swizzle("m", 3, 4, 6)
    # 16-byte chunk index ^= row mod 8 for 64-element rows of 2-byte elements
    z = Swizzle("m", 3, 3, 6)
    for row in range(16):
        for chunk in range(8):
            for e in range(8):
                x = row * 64 + chunk * 8 + e
                assert z.apply(x) == row * 64 + ((chunk ^ (row & 7)) * 8) + e


def test_evaluate_np_matches_scalar_evaluator():
    rng = random.Random(15)
    for _ in range(150):
        L = rand_layout(rng)
        if rng.random() < 0.4:
            # swizzle needs non-negative coordinates on its axis
            lo = min(p[0] for x in range(L.E_D) for p in ax.evaluate(L, x, AXES))
            if lo < 0:
                L = L.with_(O={**L.offset, "m": L.offset.get("m", 0) - lo})
            L = L.with_(swizzle=Swizzle("m", 2, 0, 2))
        xs = np.arange(L.E_D, dtype=np.int64)
        got = evaluate_np(L, xs, AXES)
        want = np.array([ax.evaluate(L, int(x), AXES) for x in xs], dtype=np.int64)
        assert got.shape == (L.E_D, L.E_R, len(AXES))
        assert np.array_equal(got, want)


def test_invalid_iters_rejected():
    with pytest.raises(ValueError):
        Iter(0, 1, "m")
    with pytest.raises(ValueError):
        Iter(-2, 1, "m")
    with pytest.raises(ValueError):
        Iter(2, 0, "m")
    with pytest.raises(ValueError):
        Layout(())
    L = Layout.make((4, 4), (4, 1))
    with pytest.raises(ValueError):
        ax.evaluate_at(L, (4, 5), (0, 0))
    with pytest.raises(IndexError):
        ax.evaluate(L, 16)
