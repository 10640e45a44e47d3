"""axe_gemm_grouped_pair_static -- the fused pair of grouped GEMMs on the library's own workspace (a __device__ array;
nothing is allocated) -- against axe_gemm_grouped_pair with a caller's workspace: same H and C, bit for bit, on two
calls in a row, the second on a smaller input (the array keeps the first call's counts: what the second call uses it
must have cleared)."""
import numpy as np
import pytest
import torch

from packing import pack_blocked, pack_gate_up
from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W

pytestmark = pytest.mark.gpu


def dev(words):
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int16)).cuda()


def layer(off, hidden, inter, out, seed):
    g = W.gemm_grouped_bf16(off, 2 * inter, hidden, seed, std_b=2.0 * hidden ** -0.5)
    w2 = W.to_bf16_bits(W.normal(seed + 1, (g.G, out, inter), inter ** -0.5))
    M, G = g.M, g.G
    d1 = B.GroupedGemmDesc(M, 2 * inter, hidden, G, B.Layout(W.row_major_spec(M, hidden)), B.Layout(W.gated_b_spec(hidden, 2 * inter, G, True)),
                           B.Layout(W.row_major_spec(M, inter)), M * hidden, G * 2 * inter * hidden, M * inter, epilogue=B.AXE_EPI_SWIGLU)
    d2 = B.GroupedGemmDesc(M, out, inter, G, B.Layout(W.row_major_spec(M, inter)), B.Layout(W.blocked_b_spec(inter, out, G=G)),
                           B.Layout(W.row_major_spec(M, out)), M * inter, G * out * inter, M * out)
    bufs = (dev(g.a_mk.reshape(-1)), dev(pack_blocked(pack_gate_up(g.b_gnk)).reshape(-1)), dev(pack_blocked(w2).reshape(-1)),
            torch.from_numpy(g.group_rows).cuda())
    return M, inter, out, d1, d2, bufs


def test_static_workspace_entry_point_equals_the_workspace_one_on_two_calls_in_a_row():
    cases = [layer([0, 300, 520, 1300, 1301, 2900], 512, 384, 512, 700),       # 2900 rows
             layer([0, 40, 41, 600, 900], 256, 256, 256, 710)]                # then a smaller one: 900 rows, other shapes
    for M, inter, out, d1, d2, (dA, dW1, dW2, dR) in cases:
        assert B.axe_gemm_grouped_pair_fused(d1, d2)
        want_h = torch.full((M * inter,), 0x7FC1, dtype=torch.int16, device="cuda")
        want_c = torch.full((M * out,), 0x7FC1, dtype=torch.int16, device="cuda")
        sync = torch.zeros(M + 1, dtype=torch.int32, device="cuda")
        B.axe_gemm_grouped_pair(d1, d2, dA, dW1, want_h, dW2, want_c, dR, sync)
        B.axe_gemm_grouped_pair_status(sync, M)
        got_h, got_c = torch.full_like(want_h, 0x7FC1), torch.full_like(want_c, 0x7FC1)
        B.axe_gemm_grouped_pair_static(d1, d2, dA, dW1, got_h, dW2, got_c, dR)
        B.axe_gemm_grouped_pair_status(None, M)
        assert torch.equal(got_h, want_h) and torch.equal(got_c, want_c), M
