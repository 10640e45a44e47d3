"""Seeded synthetic inputs for the five benchmark configurations.

This module only draws random numbers and casts them to the storage formats; it holds none of
the arithmetic of layout evaluation, relayout or GEMM, so that the HIP path and the CPU oracle
can both be fed the very same bits.  Everything is generated on the host with
numpy.random.Philox; the casts are PyTorch's CPU round-to-nearest-even conversions.

The paper's own GEMM workload (batch 8192 against LLM weight shapes, Sec. 4.1) is only given
in a figure; these synthetic shapes stand in for it.
"""
from __future__ import annotations

from dataclasses import dataclass
from typing import Optional, Tuple

import numpy as np
import torch

SEED_BASE = 19092


def _rng(seed: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(seed))


def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> bf16 (round to nearest even) -> raw uint16 words."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.bfloat16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def to_f16_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> IEEE binary16 (round to nearest even) -> raw uint16 words."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).to(torch.float16)
    return t.view(torch.int16).numpy().view(np.uint16).copy()


def to_e4m3_bits(x: np.ndarray) -> np.ndarray:
    """fp32 -> clip to the finite range [-448, 448] -> OCP e4m3 (round to nearest even) -> raw bytes."""
    t = torch.from_numpy(np.ascontiguousarray(x, dtype=np.float32)).clamp_(-448.0, 448.0)
    return t.to(torch.float8_e4m3fn).view(torch.uint8).numpy().copy()


def normal(seed: int, shape, std: float = 1.0) -> np.ndarray:
    return (_rng(seed).standard_normal(shape, dtype=np.float32) * np.float32(std)).astype(np.float32)


def uniform(seed: int, shape, lo: float, hi: float) -> np.ndarray:
    return _rng(seed).uniform(lo, hi, size=shape).astype(np.float32)


@dataclass
class GemmInputs:
    """A is logical (M, K) stored row-major; B is logical (K, N) stored column-major, i.e. the
    array `b_nk` below is its memory image, a row-major (N, K) matrix."""
    M: int
    N: int
    K: int
    dtype: str                      # "bf16" | "f16" | "fp8"
    a_mk: np.ndarray                # raw words, shape (M, K)
    b_nk: np.ndarray                # raw words, shape (N, K)
    scale_a: Optional[np.ndarray] = None   # fp32, or uint8 E8M0 codes, (ceil(M/128), ceil(K/128))
    scale_b: Optional[np.ndarray] = None   # same, (ceil(N/128), ceil(K/128))
    out_dtype: str = "bf16"         # "f32" | "bf16"
    scale_dtype: str = "f32"        # "f32" | "e8m0" (one byte per block, the power of two 2^(code - 127))


def gemm_bf16(M: int, N: int, K: int, seed: int, std_a: float = 1.0, std_b: float = 1.0,
              out_dtype: str = "bf16") -> GemmInputs:
    a = to_bf16_bits(normal(seed, (M, K), std_a))
    b = to_bf16_bits(normal(seed + 1000, (N, K), std_b))
    return GemmInputs(M, N, K, "bf16", a, b, out_dtype=out_dtype)


def gemm_f16(M: int, N: int, K: int, seed: int, std_a: float = 1.0, std_b: float = 1.0,
             out_dtype: str = "f16") -> GemmInputs:
    """The same draws as gemm_bf16, cast to IEEE binary16 (the fused MoE layer of the paper is an FP16 layer)."""
    a = to_f16_bits(normal(seed, (M, K), std_a))
    b = to_f16_bits(normal(seed + 1000, (N, K), std_b))
    return GemmInputs(M, N, K, "f16", a, b, out_dtype=out_dtype)


def gemm_fp8(M: int, N: int, K: int, seed: int, block: int = 128, scaled=True) -> GemmInputs:
    """scaled: False, True (fp32 scales uniform in [0.5, 2]) or "e8m0" (codes 124..130: powers of two 1/8 .. 8)."""
    a = to_e4m3_bits(normal(seed, (M, K)))
    b = to_e4m3_bits(normal(seed + 1000, (N, K)))
    sa = sb = None
    kb = -(-K // block)
    if scaled == "e8m0":
        sa = (124 + np.floor(uniform(seed + 2000, (-(-M // block), kb), 0.0, 7.0))).astype(np.uint8)
        sb = (124 + np.floor(uniform(seed + 3000, (-(-N // block), kb), 0.0, 7.0))).astype(np.uint8)
        return GemmInputs(M, N, K, "fp8", a, b, sa, sb, out_dtype="bf16", scale_dtype="e8m0")
    if scaled:
        sa = uniform(seed + 2000, (-(-M // block), kb), 0.5, 2.0)
        sb = uniform(seed + 3000, (-(-N // block), kb), 0.5, 2.0)
    return GemmInputs(M, N, K, "fp8", a, b, sa, sb, out_dtype="bf16")


@dataclass
class GroupedGemmInputs:
    """Grouped GEMM over experts: A (M, K) row-major, rows sorted by group; B logical (G, K, N) whose memory
    image `b_gnk` is (G, N, K) (each group's matrix column-major, as in GemmInputs); group_rows = G + 1 row
    offsets (int32, non-decreasing, group_rows[G] <= M)."""
    M: int
    N: int
    K: int
    G: int
    a_mk: np.ndarray
    b_gnk: np.ndarray
    group_rows: np.ndarray
    dtype: str = "bf16"             # "bf16" | "f16" (inputs and output) | "fp8" (e4m3 inputs, bf16 output)
    scale_a: Optional[np.ndarray] = None   # fp8: (M, ceil(K/128)), one per row and k block; fp32 or uint8 E8M0 codes
    scale_b: Optional[np.ndarray] = None   # fp8: (G, N/128, ceil(K/128)), one per 128 x 128 block of each group's matrix
    scale_dtype: str = "f32"


def moe_group_rows(tokens: int, experts: int, topk: int, seed: int, skew: float = 0.5) -> np.ndarray:
    """Rows per expert of a synthetic top-k routing: every token picks `topk` distinct experts by
    Gumbel-top-k on expert popularities drawn from N(0, skew^2) (mildly unbalanced, like a trained
    router; skew 0 = uniform).  Returns the experts + 1 offsets of the rows sorted by expert."""
    rng = _rng(seed)
    pop = rng.standard_normal(experts) * skew
    keys = pop[None, :] + rng.gumbel(size=(tokens, experts))
    pick = np.argpartition(-keys, topk - 1, axis=1)[:, :topk]
    counts = np.bincount(pick.ravel(), minlength=experts)
    return np.concatenate([[0], np.cumsum(counts)]).astype(np.int32)


def gemm_grouped_bf16(group_rows, N: int, K: int, seed: int, M: Optional[int] = None, std_a: float = 1.0,
                      std_b: Optional[float] = None, dtype: str = "bf16") -> GroupedGemmInputs:
    group_rows = np.ascontiguousarray(group_rows, dtype=np.int32)
    G = group_rows.size - 1
    M = int(group_rows[-1]) if M is None else M
    std_b = K ** -0.5 if std_b is None else std_b
    cast = to_f16_bits if dtype == "f16" else to_bf16_bits
    return GroupedGemmInputs(M, N, K, G, cast(normal(seed, (M, K), std_a)), cast(normal(seed + 7919, (G, N, K), std_b)),
                             group_rows, dtype)


def gemm_grouped_fp8(group_rows, N: int, K: int, seed: int, M: Optional[int] = None, scale_dtype: str = "f32") -> GroupedGemmInputs:
    """e4m3 operands with the usual block scaling of an fp8 MoE layer: activations one scale per row and 128-wide
    k block, weights one per 128 x 128 block; fp32 scales U[0.5, 2] or E8M0 codes 124..130."""
    group_rows = np.ascontiguousarray(group_rows, dtype=np.int32)
    G = group_rows.size - 1
    M = int(group_rows[-1]) if M is None else M
    nkb = (K + 127) // 128
    a = to_e4m3_bits(normal(seed, (M, K)))
    b = to_e4m3_bits(normal(seed + 7919, (G, N, K)))
    rng = _rng(seed + 31)
    if scale_dtype == "e8m0":
        sa = rng.integers(124, 131, (M, nkb)).astype(np.uint8)
        sb = rng.integers(124, 131, (G, N // 128, nkb)).astype(np.uint8)
    else:
        sa = rng.uniform(0.5, 2.0, (M, nkb)).astype(np.float32)
        sb = rng.uniform(0.5, 2.0, (G, N // 128, nkb)).astype(np.float32)
    return GroupedGemmInputs(M, N, K, G, a, b, group_rows, "fp8", sa, sb, scale_dtype)


# the MoE layer of Qwen3-30B-A3B (the configuration the paper's fused-MoE figure is measured on):
# hidden size, expert intermediate size, experts, experts per token
MOE_HIDDEN, MOE_INTER, MOE_EXPERTS, MOE_TOPK = 2048, 768, 128, 8


def moe_gemm1(tokens: int, seed: int = SEED_BASE + 11, dtype: str = "bf16") -> GroupedGemmInputs:
    """First grouped GEMM of the layer: routed tokens (tokens * topk rows of the hidden size) against each
    expert's gate and up projections side by side (N = 2 * intermediate)."""
    return gemm_grouped_bf16(moe_group_rows(tokens, MOE_EXPERTS, MOE_TOPK, seed), 2 * MOE_INTER, MOE_HIDDEN, seed + 1, dtype=dtype)


def moe_gemm2(tokens: int, seed: int = SEED_BASE + 11, dtype: str = "bf16") -> GroupedGemmInputs:
    """Second grouped GEMM: the activations (intermediate size) against each expert's down projection."""
    return gemm_grouped_bf16(moe_group_rows(tokens, MOE_EXPERTS, MOE_TOPK, seed), MOE_HIDDEN, MOE_INTER, seed + 2, dtype=dtype)


def relayout_words(rows: int, cols: int, seed: int, kind: str = "uniform") -> np.ndarray:
    """Raw bf16 words of a (rows, cols) tensor.  kind="uniform": i.i.d. uniform[-1, 1] cast to
    bf16; kind="index": word = (flat index * 40503) mod 65536, so that a misplaced chunk cannot
    hide behind equal values."""
    if kind == "uniform":
        return to_bf16_bits(uniform(seed, (rows, cols), -1.0, 1.0))
    if kind == "index":
        idx = np.arange(rows * cols, dtype=np.uint64).reshape(rows, cols)
        return ((idx * np.uint64(40503)) % np.uint64(65536)).astype(np.uint16)
    raise ValueError(kind)


# The five configurations --------------------------------------------------------------
def config1() -> GemmInputs:
    """bf16 GEMM M=N=K=256, entries N(0,1), fp32 output."""
    return gemm_bf16(256, 256, 256, SEED_BASE + 1, out_dtype="f32")


def config2(kind: str = "uniform", rows: int = 8192, cols: int = 8192) -> np.ndarray:
    """bf16 tensor to be re-laid out from row-major to swizzled 128x64 tiles."""
    return relayout_words(rows, cols, SEED_BASE + 2, kind)


def config3(M: int = 8192, N: int = 8192, K: int = 8192) -> GemmInputs:
    """bf16 GEMM 8192^3, entries N(0, sigma) with sigma = K^-1/2, bf16 output."""
    s = float(K) ** -0.5
    return gemm_bf16(M, N, K, SEED_BASE + 3, s, s)


def config4(M: int = 4096, N: int = 3584, K: int = 8192) -> GemmInputs:
    """One shard (of 8) of a tensor-parallel linear layer: activations N(0,1), weights N(0, 0.02)."""
    return gemm_bf16(M, N, K, SEED_BASE + 4, 1.0, 0.02)


def config5(M: int = 8192, N: int = 8192, K: int = 8192) -> GemmInputs:
    """fp8 e4m3 GEMM with fp32 scales per 128x128 block, uniform[0.5, 2]."""
    return gemm_fp8(M, N, K, SEED_BASE + 5)


# Layout descriptions of the configurations (plain data; no layout arithmetic here) ------
# A spec is {"D": [(extent, stride, axis), ...], "R": [...], "O": {axis: value},
#            "swizzle": None | (axis, bits, base, shift)}.
def spec(D, R=(), O=None, swizzle=None) -> dict:
    return {"D": [tuple(i) for i in D], "R": [tuple(i) for i in R], "O": dict(O or {}), "swizzle": swizzle}


def row_major_spec(rows: int, cols: int) -> dict:
    return spec([(rows, cols, "m"), (cols, 1, "m")])


def col_major_spec(rows: int, cols: int) -> dict:
    """Logical (rows, cols) whose element (r, c) sits at c*rows + r."""
    return spec([(rows, 1, "m"), (cols, rows, "m")])


def blocked_swizzled_spec(rows: int, cols: int, tr: int = 128, tc: int = 64, swizzle: bool = True) -> dict:
    """Logical (rows, cols) stored as a row-major grid of contiguous tr x tc row-major tiles,
    the 16-byte chunk index inside each tile row XOR-ed with (row mod 8) -- 2-byte elements."""
    if rows % tr or cols % tc:
        raise ValueError("shape is not a multiple of the tile")
    D = [(rows // tr, (cols // tc) * tr * tc, "m"), (tr, tc, "m"), (cols // tc, tr * tc, "m"), (tc, 1, "m")]
    swz = None
    if swizzle:
        if tc != 64:
            raise ValueError("the swizzle is stated for 64-element (128-byte) tile rows")
        swz = ("m", 3, 3, 6)
    return spec(D, swizzle=swz)


def gemm_specs(g: "GemmInputs", device_axis: bool = False, shard: int = 0) -> Tuple[dict, dict, dict]:
    """A (M,K) row-major, B (K,N) column-major, C (M,N) row-major.  With device_axis the weight
    carries an extent-1 iter on a `gpuid` axis plus the shard number as its offset (one GPU's
    shard of a column-parallel linear layer)."""
    A = row_major_spec(g.M, g.K)
    C = row_major_spec(g.M, g.N)
    if device_axis:
        B = spec([(g.K, 1, "m"), (1, 1, "gpuid"), (g.N, g.K, "m")], O={"gpuid": shard})
    else:
        B = col_major_spec(g.K, g.N)
    return A, B, C


def grouped_gemm_specs(g: "GroupedGemmInputs", lda: Optional[int] = None, ldb: Optional[int] = None,
                       ldg: Optional[int] = None, ldc: Optional[int] = None) -> Tuple[dict, dict, dict]:
    """Layout specs of a grouped GEMM's operands: A (M, K) and C (M, N) row-major, B (G, K, N) with each
    group's matrix column-major; optional pitches in elements."""
    lda = g.K if lda is None else lda
    ldb = g.K if ldb is None else ldb
    ldg = g.N * ldb if ldg is None else ldg
    ldc = g.N if ldc is None else ldc
    return (spec([(g.M, lda, "m"), (g.K, 1, "m")]),
            spec([(g.G, ldg, "m"), (g.K, 1, "m"), (g.N, ldb, "m")]),
            spec([(g.M, ldc, "m"), (g.N, 1, "m")]))


# ---- operands stored in 256 x 64 blocks (rows x k), each block contiguous, blocks of one row block side by side
def blocked_iters(Rn: int, K: int, rb: int = 256, kb: int = 64):
    """(row iters, k iters), as Axe iters on "m", of a (R, K) matrix stored as contiguous rb x kb blocks: block
    (r / rb, k / kb) at ((r / rb) * (K / kb) + k / kb) * rb * kb, row-major inside the block."""
    return [(Rn // rb, rb * K, "m"), (rb, kb, "m")], [(K // kb, rb * kb, "m"), (kb, 1, "m")]


def blocked_a_spec(M: int, K: int) -> dict:
    r, k = blocked_iters(M, K)
    return spec(r + k)


def blocked_b_spec(K: int, N: int, G: Optional[int] = None) -> dict:
    """B logical (K, N), or (G, K, N) with the groups' images one after the other."""
    r, k = blocked_iters(N, K)
    return spec(([(G, N * K, "m")] if G is not None else []) + k + r)


# ---- gate and up projections of an expert interleaved in runs of 16 rows (what the gated epilogue reads)
def gated_b_spec(K: int, N: int, G: int, blocked: bool = False) -> dict:
    """Layout of the logical (G, K, N) right-hand sides with gate and up rows interleaved: memory row 32 f + 16 h + i holds
    (h ? up : gate)[16 f + i]; blocked: that image stored in contiguous 256 x 64 blocks."""
    if not blocked:
        return spec([(G, N * K, "m"), (K, 1, "m"), (2, 16 * K, "m"), (N // 32, 32 * K, "m"), (16, K, "m")])
    return spec([(G, N * K, "m"), (K // 64, 256 * 64, "m"), (64, 1, "m"),
                 (2, 16 * 64, "m"), (N // 256, 256 * K, "m"), (8, 32 * 64, "m"), (16, 64, "m")])
