"""The matrix instructions' operand and accumulator maps, pinned on the device: one MFMA of one wave is run on operand
registers filled according to the layouts axe_gemm_describe reports (evaluated by the oracle), and its accumulator
registers, read back through the reported accumulator layout, must hold A B exactly.  The maps are not in the paper
(its register-tile example, Sec. 2.2, is for another vendor's tensor cores); this is what ties the described layouts
to what the hardware does, independently of any GEMM kernel."""
import ctypes as C
import os

import numpy as np
import pytest
import torch

from oracle import axe_layout as ax
from oracle import axe_ref as R
from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W
from test_describe import AXES, desc_for, get

pytestmark = pytest.mark.gpu


def probe():
    P = C.CDLL(os.path.join(os.path.dirname(B.LIB_PATH), "libaxe_probe.so"))
    P.axe_probe_mfma_fragment.restype = C.c_int
    P.axe_probe_mfma_fragment.argtypes = [C.c_int32, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p, C.c_void_p]
    return P


def e4m3_codes_of_small_integers(v):
    """OCP e4m3 codes of integers -8 .. 8 (all exactly representable), by search in the oracle's decoding table."""
    table = R.e4m3_table()
    codes = {int(x): int(np.nonzero(table == float(x))[0][0]) for x in range(-8, 9)}
    return np.vectorize(codes.__getitem__)(v).astype(np.uint8)


@pytest.mark.parametrize("kind", ["bf16", "f16", "fp8", "fp8_scaled"])
def test_one_mfma_lands_where_the_described_layouts_say(kind):
    fp8 = kind.startswith("fp8")
    desc, _ = desc_for("big_fp8_mx" if fp8 else "big_bf16")
    K = 128 if fp8 else 32                                # k of one instruction
    bytes_per_lane = 32 if fp8 else 16
    rng = np.random.default_rng(len(kind))
    A = rng.integers(-8, 9, (16, K))                      # small integers: every product and sum is exact
    Bm = rng.integers(-8, 9, (K, 16))
    if fp8:
        a_bits, b_bits = e4m3_codes_of_small_integers(A), e4m3_codes_of_small_integers(Bm)
    elif kind == "bf16":
        a_bits, b_bits = W.to_bf16_bits(A.astype(np.float32)), W.to_bf16_bits(Bm.astype(np.float32))
    else:
        a_bits, b_bits = A.astype(np.float16).view(np.uint16), Bm.astype(np.float16).view(np.uint16)
    # operand registers, lane by lane, from the described operand layouts (rows 0..15 of wave 0: its first fragment;
    # the k of the instruction: the first K elements of the K-tile -> the fragment's first registers)
    La, sa_ = get(desc, B.AXE_DESC_A_OPERAND)
    Lb, sb_ = get(desc, B.AXE_DESC_B_OPERAND)
    per_lane = bytes_per_lane // a_bits.dtype.itemsize
    a_regs = np.zeros((64, per_lane), dtype=a_bits.dtype)
    b_regs = np.zeros((64, per_lane), dtype=a_bits.dtype)
    seen_a, seen_b = set(), set()
    for r in range(16):
        for k in range(K):
            pa = [p for p in ax.evaluate_at(La, sa_, (r, k), AXES) if p[3] == 0][0]      # the replica held by wave 0
            pb = [p for p in ax.evaluate_at(Lb, sb_, (k, r), AXES) if p[3] == 0][0]
            assert pa[5] < per_lane and pb[5] < per_lane
            a_regs[pa[4], pa[5]] = a_bits[r, k]
            b_regs[pb[4], pb[5]] = b_bits[k, r]
            seen_a.add((pa[4], pa[5])); seen_b.add((pb[4], pb[5]))
    assert len(seen_a) == len(seen_b) == 64 * per_lane    # every register of every lane is filled exactly once
    dA = torch.from_numpy(a_regs.view(np.uint8).reshape(-1).copy()).cuda()
    dB = torch.from_numpy(b_regs.view(np.uint8).reshape(-1).copy()).cuda()
    dAcc = torch.zeros(64 * 4, dtype=torch.float32, device="cuda")
    want = (A @ Bm).astype(np.float64)
    code = {"bf16": 0, "f16": 1, "fp8": 2, "fp8_scaled": 3}[kind]
    dSa = dSb = None
    if kind == "fp8_scaled":
        # one E8M0 code per row of A and per column of B: a lane supplies the code of the row (column) it holds
        ca, cb = rng.integers(120, 135, 16), rng.integers(120, 135, 16)
        lane_row = np.arange(64) % 16
        dSa = torch.from_numpy(ca[lane_row].astype(np.int32)).cuda()
        dSb = torch.from_numpy(cb[lane_row].astype(np.int32)).cuda()
        want = want * np.exp2(ca.astype(np.float64) - 127)[:, None] * np.exp2(cb.astype(np.float64) - 127)[None, :]
    rc = probe().axe_probe_mfma_fragment(code, dA.data_ptr(), dB.data_ptr(), dSa.data_ptr() if dSa is not None else None,
                                         dSb.data_ptr() if dSb is not None else None, dAcc.data_ptr(),
                                         torch.cuda.current_stream().cuda_stream)
    assert rc == 0
    torch.cuda.synchronize()
    acc = dAcc.cpu().numpy().reshape(64, 4).astype(np.float64)
    Lc, sc_ = get(desc, B.AXE_DESC_ACC)
    got = np.empty((16, 16))
    for i in range(16):
        for j in range(16):
            (p,) = ax.evaluate_at(Lc, sc_, (i, j), AXES)
            assert p[2] == 0 and p[3] == 0 and p[5] < 4
            got[i, j] = acc[p[4], p[5]]
    assert np.array_equal(got, want)
