"""CPU oracle, array side -- TEST INFRASTRUCTURE, not part of the product path.

  * evaluate_np   : the induced map of Def. 2.3 for many indices at once (NumPy int64),
                    the same digit formula as the scalar evaluator, used where 2**26 points
                    would be too slow one by one;
  * relayout_ref  : dst[f_dst(x)] = src[f_src(x)] for every logical x -- the `copy` operator
                    between two layouts of one logical tensor (Sec. 3.2, operators) on raw words;
  * bf16 / e4m3   : exact decoders written from the formats' definitions;
  * gemm_ref      : C[i,j] = sum_k a[i,k] b[k,j] in fp64, natural k order (Sec. 4.1 workloads),
                    optionally with one fp32 scale per (128-row, 128-k) block of A and per
                    (128-col, 128-k) block of B (the block-scaled fp8 GEMM of Sec. 4.1; the
                    scale type is this build's, the paper's being e8m0).

Only tests, the smoke check and the benchmark's cpu_baseline leg may import this module.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from math import prod
from typing import Optional, Sequence

import numpy as np

from .axe_layout import Layout, admits

_HERE = os.path.dirname(os.path.abspath(__file__))


# --------------------------------------------------------------------------------------
# Vectorised layout evaluation (Def. 2.3)
# --------------------------------------------------------------------------------------
def evaluate_np(L: Layout, xs: np.ndarray, axes: Sequence[str]) -> np.ndarray:
    """Returns int64 array [len(xs), E_R, len(axes)]: replica t (lexicographic over R as
    written, last iter fastest) of f_L(xs[n]) on each requested axis.  Swizzle applied last."""
    xs = np.asarray(xs, dtype=np.int64)
    if xs.size and (xs.min() < 0 or xs.max() >= L.E_D):
        raise IndexError("logical index outside [0, E_D)")
    axes = list(axes)
    col = {a: i for i, a in enumerate(axes)}
    for it in L.D + L.R:
        if it.axis not in col:
            raise ValueError(f"axis {it.axis!r} not requested")
    for a, v in L.O:
        if a not in col and v != 0:
            raise ValueError(f"axis {a!r} not requested")
    n = xs.shape[0]
    base = np.zeros((n, len(axes)), dtype=np.int64)
    ext = [it.extent for it in L.D]
    for k, it in enumerate(L.D):
        p_k = prod(ext[k + 1:])
        digit = (xs // p_k) % it.extent
        base[:, col[it.axis]] += digit * it.stride
    for a, v in L.O:
        base[:, col[a]] += v
    ER = L.E_R
    out = np.empty((n, ER, len(axes)), dtype=np.int64)
    rext = [it.extent for it in L.R]
    for t in range(ER):
        rep = np.zeros(len(axes), dtype=np.int64)
        for k, it in enumerate(L.R):
            p_k = prod(rext[k + 1:])
            rep[col[it.axis]] += ((t // p_k) % it.extent) * it.stride
        out[:, t, :] = base + rep
    if L.swizzle is not None:
        z = L.swizzle
        c = col[z.axis]
        v = out[:, :, c]
        if v.size and v.min() < 0:
            raise ValueError("swizzle is defined on non-negative coordinates")
        out[:, :, c] = v ^ (((v >> z.shift) & ((1 << z.bits) - 1)) << z.base)
    return out


def flat_indices(shape: Sequence[int]) -> np.ndarray:
    return np.arange(prod(shape), dtype=np.int64)


# --------------------------------------------------------------------------------------
# Relayout
# --------------------------------------------------------------------------------------
def relayout_ref(src_L: Layout, dst_L: Layout, shape: Sequence[int], src: np.ndarray,
                 dst: np.ndarray, mem_axis: str = "m", chunk: int = 1 << 22) -> np.ndarray:
    """For every logical index x of `shape`: every replica address of dst_L receives the word
    found at the first replica address of src_L.  `src`, `dst` are 1-D arrays of raw words
    (uint8/16/32/64 or a void dtype for 16-byte elements); dst is modified in place and
    returned; words no x maps to keep their previous contents.  Coordinates on axes other
    than mem_axis are ignored (one device holds the whole tensor)."""
    if not (admits(src_L, shape) and admits(dst_L, shape)):
        raise ValueError("shape not admitted by both layouts")
    if src.ndim != 1 or dst.ndim != 1 or src.dtype != dst.dtype:
        raise ValueError("src and dst must be 1-D arrays of one word type")
    E = prod(shape)
    sa, da = src_L.axes(), dst_L.axes()
    if mem_axis not in sa or mem_axis not in da:
        raise ValueError("layouts have no memory axis")
    for lo in range(0, E, chunk):
        xs = np.arange(lo, min(E, lo + chunk), dtype=np.int64)
        s_addr = evaluate_np(src_L, xs, sa)[:, 0, sa.index(mem_axis)]
        d_addr = evaluate_np(dst_L, xs, da)[:, :, da.index(mem_axis)]
        if s_addr.min() < 0 or s_addr.max() >= src.shape[0]:
            raise IndexError("source address outside the source buffer")
        if d_addr.min() < 0 or d_addr.max() >= dst.shape[0]:
            raise IndexError("destination address outside the destination buffer")
        vals = src[s_addr]
        for t in range(d_addr.shape[1]):
            dst[d_addr[:, t]] = vals
    return dst


# --------------------------------------------------------------------------------------
# Number formats
# --------------------------------------------------------------------------------------
def bf16_to_f64(bits: np.ndarray) -> np.ndarray:
    """bfloat16 = the upper 16 bits of an IEEE binary32."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.uint32) << np.uint32(16)
    return b.view(np.float32).astype(np.float64)


def f16_to_f64(bits: np.ndarray) -> np.ndarray:
    """IEEE binary16 from its definition: 1 sign bit, 5 exponent bits (bias 15), 10 fraction bits;
    exponent 0 holds the subnormals m / 1024 * 2^-14, exponent 31 infinities (m = 0) and NaNs."""
    b = np.asarray(bits, dtype=np.uint16).astype(np.int64)
    s, e, m = b >> 15, (b >> 10) & 31, (b & 1023).astype(np.float64)
    v = np.where(e == 0, m / 1024.0 * 2.0 ** -14, (1.0 + m / 1024.0) * np.exp2((e - 15).astype(np.float64)))
    v = np.where(e == 31, np.where(m == 0, np.inf, np.nan), v)
    return np.where(s == 1, -v, v)


def e4m3_table() -> np.ndarray:
    """All 256 values of OCP FP8 E4M3 (the 'fn' flavour: bias 7, no infinities, the two
    codes S.1111.111 are NaN, largest finite 448)."""
    t = np.empty(256, dtype=np.float64)
    for code in range(256):
        s = -1.0 if code & 0x80 else 1.0
        e = (code >> 3) & 0xF
        m = code & 0x7
        if e == 0xF and m == 0x7:
            v = float("nan")
        elif e == 0:
            v = s * (m / 8.0) * 2.0 ** (1 - 7)
        else:
            v = s * (1.0 + m / 8.0) * 2.0 ** (e - 7)
        t[code] = v
    return t


def e4m3_to_f64(bits: np.ndarray) -> np.ndarray:
    return e4m3_table()[np.asarray(bits, dtype=np.uint8)]


# --------------------------------------------------------------------------------------
# GEMM
# --------------------------------------------------------------------------------------
AXE_BF16 = 1
AXE_FP8_E4M3 = 2
AXE_F16 = 4


def decode(bits: np.ndarray, dtype: int) -> np.ndarray:
    if dtype == AXE_BF16:
        return bf16_to_f64(bits)
    if dtype == AXE_FP8_E4M3:
        return e4m3_to_f64(bits)
    if dtype == AXE_F16:
        return f16_to_f64(bits)
    raise ValueError("unknown input dtype")


def e8m0_decode(codes: np.ndarray) -> np.ndarray:
    """E8M0 scale codes (OCP microscaling formats: 8 exponent bits, no sign, no mantissa) -> fp64:
    2^(code - 127) for codes 0..254, NaN for 255.  Every value is a power of two, so the fp32 the
    GEMM oracle takes holds it exactly for codes 1..254."""
    c = np.asarray(codes, dtype=np.uint8).astype(np.int64)
    out = np.ldexp(1.0, c - 127)
    return np.where(c == 255, np.nan, out)


def gemm_ref_numpy(a_bits: np.ndarray, b_bits: np.ndarray, dtype: int,
                   scale_a: Optional[np.ndarray] = None, scale_b: Optional[np.ndarray] = None,
                   block: int = 128, block_m_a: Optional[int] = None) -> np.ndarray:
    """a_bits: logical (M, K); b_bits: logical (K, N) (any strides).  fp64 result (M, N).
    With scales: C = sum_kb sA[i//block_m_a, kb] sB[j//block, kb] (A_kb @ B_kb); block_m_a defaults to block."""
    A = decode(a_bits, dtype)
    B = decode(b_bits, dtype)
    M, K = A.shape
    N = B.shape[1]
    if scale_a is None and scale_b is None:
        return A @ B
    C = np.zeros((M, N), dtype=np.float64)
    ri = np.arange(M) // (block if block_m_a is None else block_m_a)
    cj = np.arange(N) // block
    for kb in range((K + block - 1) // block):
        ks = slice(kb * block, min(K, (kb + 1) * block))
        part = A[:, ks] @ B[ks, :]
        sa = scale_a[ri, kb].astype(np.float64) if scale_a is not None else np.ones(M)
        sb = scale_b[cj, kb].astype(np.float64) if scale_b is not None else np.ones(N)
        C += sa[:, None] * sb[None, :] * part
    return C


def build_c_oracle(force: bool = False) -> str:
    """Compile oracle/gemm_ref.c with gcc into oracle/libaxe_oracle.so (plain C, OpenMP)."""
    src = os.path.join(_HERE, "gemm_ref.c")
    out = os.path.join(_HERE, "libaxe_oracle.so")
    if force or not os.path.exists(out) or os.path.getmtime(out) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", out, src, "-lm"])
    return out


_clib = None


def _c():
    global _clib
    if _clib is None:
        lib = ctypes.CDLL(build_c_oracle())
        i64, vp = ctypes.c_int64, ctypes.c_void_p
        lib.axe_oracle_gemm.restype = ctypes.c_int
        lib.axe_oracle_gemm.argtypes = [ctypes.c_int, i64, i64, i64,
                                        vp, i64, i64, vp, i64, i64,
                                        vp, vp, i64, i64,
                                        vp, i64, vp, i64, vp]
        lib.axe_oracle_threads.restype = ctypes.c_int
        _clib = lib
    return _clib


def oracle_threads() -> int:
    return int(_c().axe_oracle_threads())


def gemm_ref(a_bits: np.ndarray, b_bits: np.ndarray, dtype: int,
             scale_a: Optional[np.ndarray] = None, scale_b: Optional[np.ndarray] = None,
             block: int = 128, rows: Optional[np.ndarray] = None,
             cols: Optional[np.ndarray] = None, block_m_a: Optional[int] = None) -> np.ndarray:
    """The plain C triple loop.  a_bits logical (M, K), b_bits logical (K, N), any (element)
    strides; result fp64 [len(rows), len(cols)] (all rows / cols when None)."""
    M, K = a_bits.shape
    K2, N = b_bits.shape
    if K != K2:
        raise ValueError("inner dimensions differ")
    isz = a_bits.dtype.itemsize
    want = 1 if dtype == AXE_FP8_E4M3 else 2
    if isz != want or b_bits.dtype.itemsize != want:
        raise ValueError("bit arrays have the wrong word size")
    rows = np.arange(M, dtype=np.int64) if rows is None else np.ascontiguousarray(rows, dtype=np.int64)
    cols = np.arange(N, dtype=np.int64) if cols is None else np.ascontiguousarray(cols, dtype=np.int64)
    if rows.size and (rows.min() < 0 or rows.max() >= M):
        raise IndexError("row index")
    if cols.size and (cols.min() < 0 or cols.max() >= N):
        raise IndexError("col index")
    out = np.empty((rows.size, cols.size), dtype=np.float64)
    sa = sb = None
    if scale_a is not None or scale_b is not None:
        nkb = (K + block - 1) // block
        sa = np.ascontiguousarray(scale_a, dtype=np.float32)
        sb = np.ascontiguousarray(scale_b, dtype=np.float32)
        bma = block if block_m_a is None else block_m_a          # rows of A that share a scale (1: one scale per row and k block)
        if sa.shape != ((M + bma - 1) // bma, nkb) or sb.shape != ((N + block - 1) // block, nkb):
            raise ValueError("scale arrays have the wrong shape")
    rc = _c().axe_oracle_gemm(
        dtype, M, N, K,
        a_bits.ctypes.data, a_bits.strides[0] // isz, a_bits.strides[1] // isz,
        b_bits.ctypes.data, b_bits.strides[0] // isz, b_bits.strides[1] // isz,
        sa.ctypes.data if sa is not None else None,
        sb.ctypes.data if sb is not None else None, block, (block if block_m_a is None else block_m_a),
        rows.ctypes.data, rows.size, cols.ctypes.data, cols.size, out.ctypes.data)
    if rc != 0:
        raise RuntimeError(f"axe_oracle_gemm failed ({rc})")
    return out


def gemm_grouped_ref(a_bits: np.ndarray, b_bits: np.ndarray, group_rows: Sequence[int], dtype: int,
                     rows: Optional[np.ndarray] = None, cols: Optional[np.ndarray] = None,
                     scale_a: Optional[np.ndarray] = None, scale_b: Optional[np.ndarray] = None, block: int = 128) -> np.ndarray:
    """Grouped GEMM, the building block of the fused MoE layer of Sec. 4.1 (its two "group GEMMs"):
    the rows of A are sorted by group (expert), group g owns rows group_rows[g] .. group_rows[g+1]-1
    and has its own right-hand side:  C[r, :] = A[r, :] @ B[g]  for r in that range.

    a_bits logical (M, K); b_bits logical (G, K, N) (any strides); group_rows G+1 non-decreasing
    integers, 0 <= group_rows[0], group_rows[G] <= M.  fp64 result [len(rows), len(cols)]; a row that
    belongs to no group is NaN (the operation does not define, and must not write, it).
    Each group is one call of the plain triple loop (gemm_ref): nothing is blocked or fused.
    Block-scaled form (both scale arrays or neither): scale_a fp32 (M, ceil(K/block)), one scale per row of A and
    k block (activations); scale_b fp32 (G, ceil(N/block), ceil(K/block)), one per block x block tile of each B[g]:
        C[r, j] = sum_kb scale_a[r, kb] * scale_b[g, j // block, kb] * sum_{k in block kb} A[r, k] B[g, k, j]."""
    M, K = a_bits.shape
    G, K2, N = b_bits.shape
    off = [int(x) for x in group_rows]
    if len(off) != G + 1 or K2 != K:
        raise ValueError("group_rows needs G + 1 entries; inner dimensions must agree")
    if off[0] < 0 or off[-1] > M or any(off[g] > off[g + 1] for g in range(G)):
        raise ValueError("group_rows must be non-decreasing within [0, M]")
    rows = np.arange(M, dtype=np.int64) if rows is None else np.asarray(rows, dtype=np.int64)
    cols = np.arange(N, dtype=np.int64) if cols is None else np.asarray(cols, dtype=np.int64)
    out = np.full((rows.size, cols.size), np.nan, dtype=np.float64)
    for g in range(G):
        sel = np.nonzero((rows >= off[g]) & (rows < off[g + 1]))[0]
        if sel.size:
            if scale_a is None and scale_b is None:
                out[sel, :] = gemm_ref(a_bits, b_bits[g], dtype, rows=rows[sel], cols=cols)
            else:
                out[sel, :] = gemm_ref(a_bits, b_bits[g], dtype, scale_a, scale_b[g], block, rows=rows[sel], cols=cols, block_m_a=1)
    return out


def swiglu_ref(p: np.ndarray) -> np.ndarray:
    """The gated activation between the two group GEMMs of the MoE layer (Sec. 4.1 names the layer of
    Qwen3-30B-A3B, whose experts are gated SiLU units): for P = [gate | up] of shape (M, 2 I),
        H[r, c] = silu(P[r, c]) * P[r, c + I],      silu(x) = x / (1 + exp(-x)),
    in fp64.  NaN rows (rows no group owns) stay NaN."""
    if p.shape[1] % 2:
        raise ValueError("the gate and up halves must have equal widths")
    half = p.shape[1] // 2
    gate, up = p[:, :half], p[:, half:]
    with np.errstate(over="ignore"):
        return gate / (1.0 + np.exp(-gate)) * up


def rel_frobenius(c: np.ndarray, ref: np.ndarray) -> float:
    """|| c - ref ||_F / || ref ||_F in fp64."""
    c = np.asarray(c, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    den = np.linalg.norm(ref)
    return float(np.linalg.norm(c - ref) / den) if den > 0 else float(np.linalg.norm(c - ref))
