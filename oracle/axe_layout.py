"""CPU oracle for Axe layouts -- TEST INFRASTRUCTURE, not part of the product path.

Plain, slow, exact (Python integers) implementation of what the paper defines:

  * iter / layout / induced set-valued map            (Sec. 2.3, Defs. 2.1-2.3)
  * shape admission and the row-major flattener        (Sec. 2.3, "Shape admission")
  * axis-wise span                                     (Sec. 2.3; closed form: App. C, Lemma "Axis-wise span")
  * canonicalisation D0/D1 and C0/C1/C2, gap condition (App. A)
  * Group-By-Shape                                     (App. B, Alg. 1)
  * tile / Kronecker product                           (Sec. 3.3, App. C, Alg. 2)
  * tile-of check and recovery of C in A = C (x) B     (App. D, Alg. 3)
  * slice                                              (Sec. 3.3, App. E, Alg. 4)
  * direct sum on the tiling domain                    (App. F)
  * the swizzle stage                                  (Sec. 3.4 step (2) names it; see below)

Nothing here is imported by the HIP library or its Python binding; only tests, the smoke check
and the CPU-baseline leg of the benchmark may use it.

Readings taken where the paper is silent or garbled:

  * span: span_a = max Vals_a - min Vals_a + 1, per axis; an axis no iter touches has span 1.
  * tile: in A (x) B the left factor A is the outer grid and B the inner tile (the formula,
    Alg. 2 and the printed numbers agree on this; one prose sentence says the reverse).
  * swizzle: the paper only says the hardware swizzle is "a separate innermost" layout.  Here
    it is one optional stage applied to a single axis after D + R + O:
        y = x ^ (((x >> shift) & (2**bits - 1)) << base),   base + bits <= shift,
    an involution that permutes every aligned block of 2**(shift+bits) coordinates.
  * replica order: the map is a set; `evaluate` lists replicas in lexicographic order of R as
    written (last R iter fastest) so that arrays can be compared position by position.
  * C2 side condition: the rule text says 1 <= q < e_i, the exactness paragraph 1 <= q <= E_1;
    the union of runs is contiguous for q <= e_i, which is what is implemented.
  * slice: "rem = 0" in Alg. 4 is read as "every digit was peeled".  A one-wrap pivot whose
    carry crosses to another axis would need an iter with a two-axis stride, which Def. 2.1
    does not allow; that case reports failure (the conditions are only sufficient anyway).
"""
from __future__ import annotations

from dataclasses import dataclass, field
from itertools import product
from math import gcd, prod
from typing import Dict, Iterable, List, Optional, Sequence, Tuple, Union

DEFAULT_AXIS = "m"  # Fig. 7 caption: a stride with no axis is on the memory axis m


# --------------------------------------------------------------------------------------
# Data structures (Defs. 2.1, 2.2)
# --------------------------------------------------------------------------------------
@dataclass(frozen=True)
class Iter:
    """Def. 2.1: extent e > 0, stride s != 0, axis a;  f_I(x) = (x*s)@a."""
    extent: int
    stride: int
    axis: str = DEFAULT_AXIS

    def __post_init__(self):
        if not (isinstance(self.extent, int) and self.extent > 0):
            raise ValueError(f"iter extent must be a positive integer, got {self.extent!r}")
        if not (isinstance(self.stride, int) and self.stride != 0):
            raise ValueError(f"iter stride must be a non-zero integer, got {self.stride!r}")

    def __repr__(self):
        return f"({self.extent}:{self.stride}@{self.axis})"


@dataclass(frozen=True)
class Swizzle:
    """XOR stage on one axis: y = x ^ (((x >> shift) & (2**bits-1)) << base)."""
    axis: str
    bits: int
    base: int
    shift: int

    def __post_init__(self):
        if self.bits < 0 or self.base < 0 or self.shift < 0:
            raise ValueError("swizzle fields must be non-negative")
        if self.base + self.bits > self.shift:
            raise ValueError("swizzle needs base + bits <= shift (source and target bits disjoint)")

    def apply(self, x: int) -> int:
        if x < 0:
            raise ValueError("swizzle is defined on non-negative coordinates")
        return x ^ (((x >> self.shift) & ((1 << self.bits) - 1)) << self.base)


def _parse_stride(s: Union[int, str, Tuple[int, str]]) -> Tuple[int, str]:
    if isinstance(s, tuple):
        return int(s[0]), s[1]
    if isinstance(s, str):
        if "@" in s:
            v, a = s.split("@")
            return int(v), a
        return int(s), DEFAULT_AXIS
    return int(s), DEFAULT_AXIS


def iters(extents: Sequence[int], strides: Sequence[Union[int, str, Tuple[int, str]]]) -> Tuple[Iter, ...]:
    if len(extents) != len(strides):
        raise ValueError("extents and strides differ in length")
    out = []
    for e, s in zip(extents, strides):
        v, a = _parse_stride(s)
        out.append(Iter(int(e), v, a))
    return tuple(out)


@dataclass(frozen=True)
class Layout:
    """Def. 2.2: L = (D, R, O); plus the optional swizzle stage."""
    D: Tuple[Iter, ...]
    R: Tuple[Iter, ...] = ()
    O: Tuple[Tuple[str, int], ...] = ()          # sorted (axis, value) pairs, zeros dropped
    swizzle: Optional[Swizzle] = None

    def __post_init__(self):
        if len(self.D) < 1:
            raise ValueError("a layout needs at least one sharded iter (n_D >= 1)")

    # -- construction helpers ---------------------------------------------------------
    @staticmethod
    def make(extents, strides, R=None, O=None, swizzle=None) -> "Layout":
        """Layout.make((8,2,4,2), ("4@lane","1@warp","1@lane","1@reg"),
                       R=((2,), ("4@warp",)), O={"warp": 5})"""
        d = iters(extents, strides)
        r = iters(*R) if R else ()
        return Layout(d, r, _norm_offset(O), swizzle)

    @staticmethod
    def from_spec(spec: dict) -> "Layout":
        """From the plain-data description {"D": [(e, s, axis)...], "R": [...], "O": {...},
        "swizzle": None | (axis, bits, base, shift)}."""
        D = tuple(Iter(int(e), int(s), a) for e, s, a in spec["D"])
        R = tuple(Iter(int(e), int(s), a) for e, s, a in spec.get("R", ()))
        z = spec.get("swizzle")
        return Layout(D, R, _norm_offset(spec.get("O")), Swizzle(*z) if z else None)

    @property
    def offset(self) -> Dict[str, int]:
        return dict(self.O)

    @property
    def E_D(self) -> int:
        return prod(i.extent for i in self.D)

    @property
    def E_R(self) -> int:
        return prod(i.extent for i in self.R)  # empty product = 1

    def axes(self) -> List[str]:
        """Axes in order of first appearance (D, then R, then O)."""
        seen: List[str] = []
        for it in self.D + self.R:
            if it.axis not in seen:
                seen.append(it.axis)
        for a, _ in self.O:
            if a not in seen:
                seen.append(a)
        if self.swizzle and self.swizzle.axis not in seen:
            seen.append(self.swizzle.axis)
        return seen

    def with_(self, D=None, R=None, O=None, swizzle="keep") -> "Layout":
        return Layout(tuple(D) if D is not None else self.D,
                      tuple(R) if R is not None else self.R,
                      _norm_offset(O) if O is not None else self.O,
                      self.swizzle if swizzle == "keep" else swizzle)

    def __repr__(self):
        s = "(" + ",".join(repr(i) for i in self.D) + ")"
        if self.R:
            s += "+[" + ",".join(repr(i) for i in self.R) + "]"
        if self.O:
            s += "+" + "+".join(f"{v}@{a}" for a, v in self.O)
        if self.swizzle:
            z = self.swizzle
            s += f" swz({z.axis};bits={z.bits},base={z.base},shift={z.shift})"
        return s


def _norm_offset(O) -> Tuple[Tuple[str, int], ...]:
    if O is None:
        return ()
    if isinstance(O, dict):
        items = O.items()
    else:
        items = O
    acc: Dict[str, int] = {}
    for a, v in items:
        acc[a] = acc.get(a, 0) + int(v)
    return tuple(sorted((a, v) for a, v in acc.items() if v != 0))


Coord = Dict[str, int]


def _add(c: Coord, axis: str, v: int) -> None:
    c[axis] = c.get(axis, 0) + v


# --------------------------------------------------------------------------------------
# Evaluation (Def. 2.3, shape admission)
# --------------------------------------------------------------------------------------
def unflatten(x: int, extents: Sequence[int]) -> Tuple[int, ...]:
    """Lexicographic unflattening iota: first extent is the slowest digit.

    Uses the digit formula of App. A: d_i = floor(x / p_i) mod e_i with p_i the product of
    the extents to the right of i."""
    E = prod(extents)
    if not 0 <= x < E:
        raise IndexError(f"index {x} outside [0, {E})")
    digits = []
    for i, e in enumerate(extents):
        p_i = prod(extents[i + 1:])
        digits.append((x // p_i) % e)
    return tuple(digits)


def flatten(u: Sequence[int], shape: Sequence[int]) -> int:
    """Row-major flattener flat_S (last coordinate fastest)."""
    if len(u) != len(shape):
        raise ValueError("rank mismatch")
    x = 0
    for ui, si in zip(u, shape):
        if not 0 <= ui < si:
            raise IndexError(f"coordinate {ui} outside [0, {si})")
        x = x * si + ui
    return x


def f_D(L: Layout, x: int) -> Coord:
    """f_D(x) = sum_k (iota(x)_k * s_k) @ a_k."""
    c: Coord = {}
    for d, it in zip(unflatten(x, [i.extent for i in L.D]), L.D):
        _add(c, it.axis, d * it.stride)
    return c


def f_R(L: Layout, r: Sequence[int]) -> Coord:
    """f_R(r) = sum_t (r_t * s_t) @ a_t."""
    c: Coord = {}
    for rt, it in zip(r, L.R):
        if not 0 <= rt < it.extent:
            raise IndexError("replica digit out of range")
        _add(c, it.axis, rt * it.stride)
    return c


def evaluate(L: Layout, x: int, axes: Optional[Sequence[str]] = None) -> List[Tuple[int, ...]]:
    """f_L(x) as a list of E_R coordinate tuples over `axes` (default L.axes()), replicas in
    lexicographic order of R; the swizzle stage, if any, is applied last."""
    axes = list(axes) if axes is not None else L.axes()
    base = f_D(L, x)
    for a, v in L.O:
        _add(base, a, v)
    out = []
    for r in product(*[range(it.extent) for it in L.R]):   # one empty tuple when R is empty
        c = dict(base)
        for a, v in f_R(L, r).items():
            _add(c, a, v)
        if L.swizzle is not None:
            c[L.swizzle.axis] = L.swizzle.apply(c.get(L.swizzle.axis, 0))
        for a in c:
            if c[a] != 0 and a not in axes:
                raise ValueError(f"axis {a!r} carries a coordinate but was not requested")
        out.append(tuple(c.get(a, 0) for a in axes))
    return out


def evaluate_set(L: Layout, x: int, axes: Optional[Sequence[str]] = None) -> frozenset:
    return frozenset(evaluate(L, x, axes))


def admits(L: Layout, shape: Sequence[int]) -> bool:
    return prod(shape) == L.E_D


def evaluate_at(L: Layout, shape: Sequence[int], u: Sequence[int], axes=None):
    """f_{L<S>}(u) = f_L(flat_S(u)); S must be admitted."""
    if not admits(L, shape):
        raise ValueError(f"shape {tuple(shape)} is not admitted (E_D = {L.E_D})")
    return evaluate(L, flatten(u, shape), axes)


def evaluate_all(L: Layout, axes=None) -> List[List[Tuple[int, ...]]]:
    return [evaluate(L, x, axes) for x in range(L.E_D)]


# --------------------------------------------------------------------------------------
# Span (Sec. 2.3; App. C closed form)
# --------------------------------------------------------------------------------------
def span(L: Layout, axes: Optional[Sequence[str]] = None) -> Dict[str, int]:
    """Closed form: span_a = 1 + sum |s|(e-1) over the D and R iters on a.  O does not enter."""
    axes = list(axes) if axes is not None else L.axes()
    out = {a: 1 for a in axes}
    for it in L.D + L.R:
        out[it.axis] = out.get(it.axis, 1) + abs(it.stride) * (it.extent - 1)
    return out


def span_bruteforce(L: Layout, axes: Optional[Sequence[str]] = None) -> Dict[str, int]:
    """max Vals - min Vals + 1 per axis by enumerating the whole image (no swizzle)."""
    axes = list(axes) if axes is not None else L.axes()
    plain = L.with_(swizzle=None)
    lo = {a: None for a in axes}
    hi = {a: None for a in axes}
    for x in range(L.E_D):
        for pt in evaluate(plain, x, axes):
            for a, v in zip(axes, pt):
                lo[a] = v if lo[a] is None else min(lo[a], v)
                hi[a] = v if hi[a] is None else max(hi[a], v)
    return {a: (hi[a] - lo[a] + 1) for a in axes}


# --------------------------------------------------------------------------------------
# Canonicalisation (App. A)
# --------------------------------------------------------------------------------------
def canon_D(D: Sequence[Iter], keep_one: bool = True) -> Tuple[Iter, ...]:
    """Apply D0 (drop extent 1) and D1 (merge (e_i, e_{i+1}s_{i+1}, a)(e_{i+1}, s_{i+1}, a))
    until neither applies.  If everything is dropped and keep_one is set, a single (1:1@m)
    iter is kept because Def. 2.2 requires n_D >= 1."""
    cur = [it for it in D if it.extent != 1]               # D0
    changed = True
    while changed:
        changed = False
        for i in range(len(cur) - 1):
            a, b = cur[i], cur[i + 1]
            if a.axis == b.axis and a.stride == b.extent * b.stride:   # D1
                cur[i:i + 2] = [Iter(a.extent * b.extent, b.stride, a.axis)]
                changed = True
                break
    if not cur and keep_one:
        axis = D[0].axis if len(D) else DEFAULT_AXIS
        cur = [Iter(1, 1, axis)]
    return tuple(cur)


def canon_OR(R: Sequence[Iter], O) -> Tuple[Tuple[Iter, ...], Tuple[Tuple[str, int], ...]]:
    """C0 (drop extent 1), C1 (make strides positive, move (e-1)*s into O), C2 (absorb an
    iter whose stride is q times another's, 1 <= q <= extent of that other) to a fixpoint.
    The result is sorted by (axis, stride) since R is a multiset."""
    off = dict(_norm_offset(O))
    cur: List[Iter] = []
    for it in R:
        if it.extent == 1:                                  # C0
            continue
        if it.stride < 0:                                   # C1
            off[it.axis] = off.get(it.axis, 0) + (it.extent - 1) * it.stride
            it = Iter(it.extent, -it.stride, it.axis)
        cur.append(it)
    changed = True
    while changed:                                          # C2
        changed = False
        cur.sort(key=lambda t: (t.axis, t.stride, t.extent))
        for i in range(len(cur)):
            for j in range(len(cur)):
                if i == j or cur[i].axis != cur[j].axis:
                    continue
                si, sj = cur[i].stride, cur[j].stride
                if sj % si != 0:
                    continue
                q = sj // si
                if 1 <= q <= cur[i].extent:
                    merged = Iter(cur[i].extent + q * (cur[j].extent - 1), si, cur[i].axis)
                    cur = [t for k, t in enumerate(cur) if k not in (i, j)] + [merged]
                    changed = True
                    break
            if changed:
                break
    cur.sort(key=lambda t: (t.axis, t.stride, t.extent))
    return tuple(cur), _norm_offset(off)


def gap_condition(R: Sequence[Iter]) -> bool:
    """GC: per axis, with strides sorted increasingly, sigma_{k+1} > E_k * sigma_k.
    Expects sign-normalised R (all strides positive)."""
    by_axis: Dict[str, List[Iter]] = {}
    for it in R:
        if it.stride <= 0:
            raise ValueError("gap condition is stated for sign-normalised R")
        by_axis.setdefault(it.axis, []).append(it)
    for its in by_axis.values():
        its.sort(key=lambda t: t.stride)
        for k in range(len(its) - 1):
            if not its[k + 1].stride > its[k].extent * its[k].stride:
                return False
    return True


def canonicalize(L: Layout) -> Layout:
    r, o = canon_OR(L.R, L.O)
    return Layout(canon_D(L.D), r, o, L.swizzle)


def equivalent_by_canon(L1: Layout, L2: Layout) -> bool:
    """Equality test through canonical forms (exact under the gap condition)."""
    return canonicalize(L1) == canonicalize(L2)


# --------------------------------------------------------------------------------------
# Group-By-Shape (App. B, Alg. 1)
# --------------------------------------------------------------------------------------
class LayoutError(Exception):
    """An operator's sufficient conditions do not hold (the paper's FAILURE / FAIL)."""


def group(D: Sequence[Iter], shape: Sequence[int]) -> List[List[Iter]]:
    """Grouping by a shape (App. B, Alg. 1 defines the result): refine D, without changing f_D, so that it
    falls into len(shape) consecutive blocks with extent products shape[i].

    Stated through prefix products: read left to right, the iters of D place their extents at the mixed-radix
    positions 1, e_0, e_0 e_1, ...; block i has to end at position shape[0] ... shape[i].  An iter that ends
    before or at the end of the open block goes into it whole; an iter inside which the block ends is cut
    there -- (e, s, a) with e = q t becomes (q, t s, a), (t, s, a), the split lemma of App. B -- which needs
    the block's remaining extent q to divide e.  When neither divides the other no refinement exists and a
    LayoutError is raised (the algorithm's gcd step would reach 1).  Unit iters carry no digit; each stays in
    the block of the piece before it (block 0 if there is none)."""
    if prod(it.extent for it in D) != prod(shape):
        raise LayoutError("shape is not admitted")
    ends = []                                   # position at which block i is complete
    for T in shape:
        ends.append((ends[-1] if ends else 1) * T)
    blocks: List[List[Iter]] = [[] for _ in shape]
    b, pos = 0, 1                               # block being filled, product of the extents placed so far
    for it in D:
        left = it.extent                        # extent of the part of this iter not placed yet
        if left == 1:
            blocks[b].append(it)
            continue
        while left > 1:
            while pos == ends[b]:               # complete blocks (also the empty ones of unit shape entries)
                b += 1
            need = ends[b] // pos
            if need % left == 0:
                q = left
            elif left % need == 0:
                q = need
            else:
                raise LayoutError(f"iter {it}: a block of {shape[b]} ends inside it at a position that does not divide it")
            left //= q
            blocks[b].append(Iter(q, left * it.stride, it.axis))
            pos *= q
    return blocks


def grouped(L: Layout, shape: Sequence[int]) -> Tuple[Layout, List[int]]:
    """L_{||S}: same map, refined D; returns the layout and the block boundaries."""
    blocks = group(L.D, shape)
    flat = [it for b in blocks for it in b]
    bounds, n = [], 0
    for b in blocks:
        n += len(b)
        bounds.append(n)
    if not flat:
        flat = [Iter(1, 1, L.D[0].axis)]
    return L.with_(D=flat), bounds


# --------------------------------------------------------------------------------------
# Tile (Alg. 2), direct sum (App. F), tile-of (Alg. 3)
# --------------------------------------------------------------------------------------
def _need_no_swizzle(*Ls: Layout):
    for L in Ls:
        if L.swizzle is not None:
            raise LayoutError("layout operators act on (D, R, O); strip the swizzle stage first")


def tile(A: Layout, SA: Sequence[int], B: Layout, SB: Sequence[int]) -> Tuple[Layout, Tuple[int, ...]]:
    """T = A_{||SA} (x) B_{||SB}: A is the outer grid, B the inner tile.
    f_T(x || y) = f_A(x) (.) span(f_B) + f_B(y).  Returns (T, interleaved shape S_T)."""
    _need_no_swizzle(A, B)
    if len(SA) != len(SB):
        raise LayoutError("tile needs shapes of equal rank")
    ba = group(A.D, SA)
    bb = group(B.D, SB)
    sigma = span(B)                         # closed form, D and R of B; O does not enter
    sc = lambda it: Iter(it.extent, sigma.get(it.axis, 1) * it.stride, it.axis)
    D: List[Iter] = []
    for i in range(len(SA)):
        D += [sc(it) for it in ba[i]]
        D += list(bb[i])
    R = tuple(sc(it) for it in A.R) + tuple(B.R)
    O: Dict[str, int] = {}
    for a, v in A.O:
        _add(O, a, v * sigma.get(a, 1))
    for a, v in B.O:
        _add(O, a, v)
    ST = tuple(v for pair in zip(SA, SB) for v in pair)
    if not D:
        D = [Iter(1, 1, DEFAULT_AXIS)]
    return Layout(tuple(D), R, _norm_offset(O)), ST


def direct_sum(A: Layout, SA: Sequence[int], B: Layout, SB: Sequence[int]) -> Tuple[Layout, Tuple[int, ...]]:
    """A + B on the tiling domain: blocks interleaved, no span scaling;
    f(x || y) = f_A(x) + f_B(y)."""
    _need_no_swizzle(A, B)
    if len(SA) != len(SB):
        raise LayoutError("direct sum needs shapes of equal rank")
    ba = group(A.D, SA)
    bb = group(B.D, SB)
    D: List[Iter] = []
    for i in range(len(SA)):
        D += list(ba[i]) + list(bb[i])
    O: Dict[str, int] = {}
    for a, v in A.O + B.O:
        _add(O, a, v)
    ST = tuple(v for pair in zip(SA, SB) for v in pair)
    return Layout(tuple(D), tuple(A.R) + tuple(B.R), _norm_offset(O)), ST


def scale_D(A: Layout, W: Dict[str, int]) -> Layout:
    """A . W of App. F: multiply every D stride on axis a by W[a]; R and O are kept."""
    return A.with_(D=[Iter(it.extent, it.stride * W.get(it.axis, 1), it.axis) for it in A.D])


def flatten_axes(L: Layout, pitch: Dict[str, int], to_axis: str) -> Layout:
    """The layout on the single axis `to_axis` that L becomes when a coordinate c on axis a is stored at
    sum_a c[a] * pitch[a] -- how a thread-distributed layout (axes wave, lane, reg: Sec. 2.2) is laid out in a
    linear memory, [wave][lane][reg] say.  By Def. 2.1 an iter contributes x * stride on its axis, so every iter
    (e, s @ a) of D and R becomes (e, s * pitch[a] @ to_axis) and the offsets add up: f_flat(x) = sum_a pitch[a] f_L(x)[a]
    for every replica.  Not defined for a swizzled L (the stage acts on one axis' coordinate, not on the sum)."""
    if L.swizzle is not None:
        raise LayoutError("flatten_axes is defined on (D, R, O)")
    def conv(it: Iter) -> Iter:
        if it.axis not in pitch or (pitch[it.axis] == 0 and it.extent > 1):
            raise LayoutError(f"no pitch for axis {it.axis}")
        return Iter(it.extent, it.stride * pitch[it.axis] if pitch[it.axis] else it.stride, to_axis)
    off = 0
    for a, v in L.O:
        if a not in pitch:
            raise LayoutError(f"no pitch for axis {a}")
        off += v * pitch[a]
    return Layout(tuple(conv(i) for i in L.D), tuple(conv(i) for i in L.R), _norm_offset({to_axis: off}))


def tile_of(A: Layout, SA: Sequence[int], B: Layout, SB: Sequence[int]) -> Tuple[Layout, Tuple[int, ...]]:
    """Decide A = C (x) B and return (C, S_C) with S_C = SA / SB; LayoutError otherwise.
    R of A must be empty or equal to R of B (the general Minkowski decomposition of a
    replicated A is not attempted); offsets must satisfy O_A = O_C (.) W + O_B."""
    _need_no_swizzle(A, B)
    if len(SA) != len(SB):
        raise LayoutError("rank mismatch")
    if any(a % b for a, b in zip(SA, SB)):
        raise LayoutError("S_B does not divide S_A coordinatewise")
    SC = tuple(a // b for a, b in zip(SA, SB))
    # group A by the interleaved shape so every block of A splits at the C/B boundary sizes
    blocksA = [canon_D(b, keep_one=False) for b in group(A.D, SA)]
    blocksB = [canon_D(b, keep_one=False) for b in group(B.D, SB)]
    W = span(B)
    DC: List[Iter] = []
    for j in range(len(SA)):
        # refine A's block so that B's iters can appear verbatim: regroup by (SC[j], SB[j]) is not
        # enough in general (interleaving), so scan with on-demand splitting of A's iters.
        blkA = list(blocksA[j])
        blkB = list(blocksB[j])
        p = q = 0
        C: List[Iter] = []
        while p < len(blkA):
            ia = blkA[p]
            if q < len(blkB):
                ib = blkB[q]
                if ia == ib:
                    p += 1
                    q += 1
                    continue
                # A's iter may be a fusion "outer part . B's iter" on the same axis: split it
                if (ia.axis == ib.axis and ia.stride == ib.stride and ia.extent % ib.extent == 0
                        and ia.extent > ib.extent):
                    head = Iter(ia.extent // ib.extent, ib.extent * ib.stride, ia.axis)
                    blkA[p:p + 1] = [head, ib]
                    ia = head
            w = W.get(ia.axis, 1)
            if ia.stride % w != 0:
                raise LayoutError(f"iter {ia} is neither the next iter of B nor span-scaled")
            C.append(Iter(ia.extent, ia.stride // w, ia.axis))
            p += 1
        if q != len(blkB):
            raise LayoutError("B's block was not matched as a subsequence")
        if prod(it.extent for it in C) != SC[j]:
            raise LayoutError("extent product of the recovered block differs from S_C")
        DC += C
    # offsets and replicas
    if tuple(sorted(A.R, key=repr)) != tuple(sorted(B.R, key=repr)):
        raise LayoutError("replication of A is not that of B")
    OC: Dict[str, int] = {}
    oa, ob = A.offset, B.offset
    for a in set(oa) | set(ob):
        diff = oa.get(a, 0) - ob.get(a, 0)
        w = W.get(a, 1)
        if diff % w:
            raise LayoutError("offsets are not consistent with a span-scaled outer offset")
        OC[a] = diff // w
    if not DC:
        DC = [Iter(1, 1, DEFAULT_AXIS)]
    return Layout(tuple(DC), (), _norm_offset(OC)), SC


# --------------------------------------------------------------------------------------
# Slice (Alg. 4)
# --------------------------------------------------------------------------------------
def _slice_block(block: Sequence[Iter], b: int, T: int) -> List[Iter]:
    """One grouped block, region [b, b+T) of its flattened index.  Returns the iters that
    enumerate the region (slow -> fast); the constant part lives in the caller's O*."""
    blk = list(canon_D(block, keep_one=False))
    E = [it.extent for it in blk]
    m = len(blk)
    if m == 0:
        if (b, T) != (0, 1):
            raise LayoutError("region outside a unit block")
        return []
    d0 = unflatten(b, E)
    rem = T
    peeled: List[Iter] = []
    k = None
    for j in range(m - 1, -1, -1):
        if d0[j] == 0 and rem % E[j] == 0:
            peeled.insert(0, blk[j])
            rem //= E[j]
        else:
            k = j
            break
    if k is None:                           # every digit peeled: the region is the whole block
        if rem != 1:
            raise LayoutError("region larger than the block")
        return peeled
    if d0[k] + rem <= E[k]:                 # no-wrap form
        return [Iter(rem, blk[k].stride, blk[k].axis)] + peeled
    c = rem // 2
    if rem % 2 == 0 and d0[k] + c == E[k]:  # symmetric one-wrap form
        if k == 0:
            raise LayoutError("one-wrap at the slowest digit leaves the block")
        # The carry adds 1 to digit k-1.  The appendix states the capacity test as
        # d_{k-1} + 1 <= E_{k-1}, which always holds; what its proof needs ("no further
        # carry") is that digit k-1 itself does not wrap, i.e. d_{k-1} + 1 <= E_{k-1} - 1.
        if not d0[k - 1] + 1 <= E[k - 1] - 1:
            raise LayoutError("carry into digit k-1 would wrap")
        if blk[k - 1].axis != blk[k].axis:
            raise LayoutError("one-wrap carry crosses axes: not expressible as a single iter")
        delta = blk[k - 1].stride - (E[k] - c) * blk[k].stride
        if delta == 0:
            raise LayoutError("one-wrap increment is zero")
        return [Iter(2, delta, blk[k].axis), Iter(c, blk[k].stride, blk[k].axis)] + peeled
    raise LayoutError("region is not covered by the sufficient slicing forms")


def slice_layout(L: Layout, shape: Sequence[int], begin: Sequence[int], size: Sequence[int]) -> Layout:
    """L[R:S] for R = prod_i [begin_i, begin_i + size_i): a layout admitting `size` with
    f_{L[R:S]<T>}(u) = f_{L<S>}(u + b).  Per grouped block; O* = f_{L<S>}(b) (with O, no R)."""
    _need_no_swizzle(L)
    if not admits(L, shape):
        raise LayoutError("shape is not admitted")
    for bi, ti, si in zip(begin, size, shape):
        if not (0 <= bi and ti >= 1 and bi + ti <= si):
            raise LayoutError("region outside the shape")
    blocks = group(L.D, shape)
    D: List[Iter] = []
    for blk, bi, ti in zip(blocks, begin, size):
        part = _slice_block(blk, bi, ti)
        if not part:
            part = [Iter(1, (blk[-1].stride if blk else 1), (blk[-1].axis if blk else DEFAULT_AXIS))]
        # keep exactly the block's region size as extent product
        D += part
    ostar = f_D(L, flatten(begin, shape))
    for a, v in L.O:
        _add(ostar, a, v)
    return Layout(tuple(D), L.R, _norm_offset(ostar))


# --------------------------------------------------------------------------------------
# Helpers used by tests of kernels' layouts
# --------------------------------------------------------------------------------------
def image_counts(L: Layout, axes: Optional[Sequence[str]] = None) -> Dict[Tuple[int, ...], int]:
    """How many (x, r) pairs land on each coordinate: a bijection onto a box has every count 1."""
    axes = list(axes) if axes is not None else L.axes()
    cnt: Dict[Tuple[int, ...], int] = {}
    for x in range(L.E_D):
        for pt in evaluate(L, x, axes):
            cnt[pt] = cnt.get(pt, 0) + 1
    return cnt


def is_injective(L: Layout, axes: Optional[Sequence[str]] = None) -> bool:
    return all(v == 1 for v in image_counts(L, axes).values())


def row_major(shape: Sequence[int], axis: str = DEFAULT_AXIS) -> Layout:
    strides, acc = [], 1
    for s in reversed(shape):
        strides.append(acc)
        acc *= s
    strides.reverse()
    return Layout(tuple(Iter(int(e), int(s), axis) for e, s in zip(shape, strides)))
