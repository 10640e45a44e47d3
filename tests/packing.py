"""Memory images of packed GEMM operands built with NumPy reshape / transpose -- checker code for the tests: what
axe_relayout must produce, and inputs for kernels that read packed operands.  Independent of the layout evaluator."""
import numpy as np


def pack_blocked(rows_k: np.ndarray, rb: int = 256, kb: int = 64) -> np.ndarray:
    """Memory image of a (R, K) matrix (unit stride along k in the plain form) stored as contiguous rb x kb
    blocks: block (r / rb, k / kb) at ((r / rb) * (K / kb) + k / kb) * rb * kb, row-major inside the block.
    Leading dimensions are kept: (..., R, K) -> (..., R * K)."""
    *lead, Rn, K = rows_k.shape
    v = rows_k.reshape(*lead, Rn // rb, rb, K // kb, kb)
    n = len(lead)
    return np.ascontiguousarray(v.transpose(*range(n), n, n + 2, n + 1, n + 3)).reshape(*lead, Rn * K)



def pack_gate_up(b_gnk: np.ndarray) -> np.ndarray:
    """(G, N, K) with rows [gate 0 .. I-1 | up 0 .. I-1] -> rows 32 f + 16 h + i = (h ? up : gate)[16 f + i]."""
    G, N, K = b_gnk.shape
    return np.ascontiguousarray(b_gnk.reshape(G, 2, N // 32, 16, K).transpose(0, 2, 1, 3, 4)).reshape(G, N, K)
