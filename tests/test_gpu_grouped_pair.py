"""The two grouped GEMMs of an MoE layer's expert computation as one launch (axe_gemm_grouped_pair; Sec. 4.1, fused MoE
layer): gemm1 with the gated activation writes H, gemm2 reads H, and a row block of gemm2 starts once gemm1's column
tiles for those rows are stored.  Checked against the oracle's composition of the two grouped GEMMs (H rounded to the
16-bit type in between, as the layer stores it) on every 128 x 128 block of every group, and bit for bit against two
separate axe_gemm_grouped launches: a row block read before it was complete would change bits."""
import os

import numpy as np
import pytest

torch = pytest.importorskip("torch")
if not torch.cuda.is_available():
    pytest.skip("needs a GPU", allow_module_level=True)

from oracle import axe_ref as R
from packing import pack_blocked, pack_gate_up
from paper_2601_19092_amd import binding as B
from paper_2601_19092_amd import workloads as W

pytestmark = pytest.mark.gpu
SENTINEL = 0x7FC1
TOL = {"bf16": 5e-3, "f16": 2e-3}
ODT = {"bf16": R.AXE_BF16, "f16": R.AXE_F16}
BDT = {"bf16": B.AXE_BF16, "f16": B.AXE_F16}


def dev(words):
    return torch.from_numpy(np.ascontiguousarray(words).view(np.int16 if words.dtype == np.uint16 else words.dtype)).cuda()


class Layer:
    """Seeded inputs of one layer: routed rows sorted by expert, gate/up weights (G, 2 I, K1), down weights (G, N2, I)."""

    def __init__(self, off, hidden, inter, out, seed, dtype="bf16", M=None):
        self.dtype = dtype
        self.g1 = W.gemm_grouped_bf16(off, 2 * inter, hidden, seed, M=M, std_b=2.0 * hidden ** -0.5, dtype=dtype)
        cast = W.to_f16_bits if dtype == "f16" else W.to_bf16_bits
        self.w2 = cast(W.normal(seed + 1, (self.g1.G, out, inter), inter ** -0.5))
        self.M, self.G, self.K1, self.I, self.N2 = self.g1.M, self.g1.G, hidden, inter, out
        self.off = self.g1.group_rows

    def descs(self, hint):
        M, G, K1, I, N2 = self.M, self.G, self.K1, self.I, self.N2
        dt = BDT[self.dtype]
        d1 = B.GroupedGemmDesc(M, 2 * I, K1, G, B.Layout(W.row_major_spec(M, K1)), B.Layout(W.gated_b_spec(K1, 2 * I, G, True)),
                               B.Layout(W.row_major_spec(M, I)), M * K1, G * 2 * I * K1, M * I, in_dtype=dt, out_dtype=dt,
                               epilogue=B.AXE_EPI_SWIGLU, kernel_hint=hint)
        d2 = B.GroupedGemmDesc(M, N2, I, G, B.Layout(W.row_major_spec(M, I)), B.Layout(W.blocked_b_spec(I, N2, G=G)),
                               B.Layout(W.row_major_spec(M, N2)), M * I, G * N2 * I, M * N2, in_dtype=dt, out_dtype=dt, kernel_hint=hint)
        return d1, d2

    def device(self):
        w1 = pack_blocked(pack_gate_up(self.g1.b_gnk))
        w2 = pack_blocked(self.w2)
        return dev(self.g1.a_mk.reshape(-1)), dev(w1.reshape(-1)), dev(w2.reshape(-1)), torch.from_numpy(self.off).cuda()

    def oracle(self):
        """(H, C) in fp64, NaN rows where no group owns the row; H is rounded to the layer's 16-bit type before gemm2."""
        h = R.swiglu_ref(R.gemm_grouped_ref(self.g1.a_mk, self.g1.b_gnk.transpose(0, 2, 1), self.off, ODT[self.dtype]))
        cast = W.to_f16_bits if self.dtype == "f16" else W.to_bf16_bits
        h_bits = cast(np.nan_to_num(h, nan=0.0).astype(np.float32))
        c = R.gemm_grouped_ref(h_bits, self.w2.transpose(0, 2, 1), self.off, ODT[self.dtype])
        return h, c


def decode(raw, dtype):
    return R.bf16_to_f64(raw) if dtype == "bf16" else R.f16_to_f64(raw)


def check_blocks(off, got, raw, ref, tol, what):
    owned = ~np.isnan(ref[:, 0])
    assert (raw[~owned] == SENTINEL).all(), f"{what}: a row outside every group was written"
    assert np.isfinite(got[owned]).all(), what
    assert R.rel_frobenius(got[owned], ref[owned]) <= tol, what
    for e in range(len(off) - 1):
        for i in range(off[e], off[e + 1], 128):
            for j in range(0, ref.shape[1], 128):
                blk = (slice(i, min(i + 128, off[e + 1])), slice(j, j + 128))
                err = R.rel_frobenius(got[blk], ref[blk])
                assert err <= tol, f"{what}: group {e} rows {i} columns {j}: {err:.3e}"


def run_pair(L: Layer, hint, fused=True):
    d1, d2 = L.descs(hint)
    dA, dW1, dW2, dR = L.device()
    dH = torch.full((L.M * L.I,), SENTINEL, dtype=torch.int16, device="cuda")
    dC = torch.full((L.M * L.N2,), SENTINEL, dtype=torch.int16, device="cuda")
    sync = torch.full((L.M + 1,), 12345, dtype=torch.int32, device="cuda") if fused else None      # (the library clears it)
    B.axe_gemm_grouped_pair(d1, d2, dA, dW1, dH, dW2, dC, dR, sync)
    if fused:
        B.axe_gemm_grouped_pair_status(sync, L.M)
        assert int(sync[L.M].item()) == 0
    torch.cuda.synchronize()
    return (dH.cpu().numpy().view(np.uint16).reshape(L.M, L.I), dC.cpu().numpy().view(np.uint16).reshape(L.M, L.N2), sync)


CASES = [
    # (row offsets, hidden, intermediate, out, M)
    ([0, 300, 520, 1300, 1301, 2000], 512, 384, 512, 2003),       # ragged groups, a single-row group, rows no group owns
    ([0, 0, 700, 701, 1500, 1800, 1800], 256, 256, 768, None),    # empty groups first and last; the smallest K on both sides
    ([5, 6, 6, 270, 1100], 1024, 128 * 3, 256, 1100),             # rows before the first group
]


@pytest.mark.parametrize("hint", [B.AXE_GROUPED_TILES_256, B.AXE_GROUPED_TILES_128])
@pytest.mark.parametrize("case", range(len(CASES)))
@pytest.mark.parametrize("dtype", ["bf16", "f16"])
def test_pair_against_the_oracle_and_two_launches(case, hint, dtype):
    off, hidden, inter, out, M = CASES[case]
    L = Layer(off, hidden, inter, out, 500 + case, dtype, M=M)
    d1, d2 = L.descs(hint)
    assert B.axe_gemm_grouped_pair_fused(d1, d2)
    h_raw, c_raw, _ = run_pair(L, hint)
    h_ref, c_ref = L.oracle()
    check_blocks(L.off, decode(h_raw, dtype), h_raw, h_ref, TOL[dtype], "H")
    check_blocks(L.off, decode(c_raw, dtype), c_raw, c_ref, TOL[dtype], "C")
    h2, c2, _ = run_pair(L, hint, fused=False)                     # no workspace: one launch after the other
    assert np.array_equal(h_raw, h2) and np.array_equal(c_raw, c2)


def test_pair_moe_layer_shapes_512_tokens():
    """The benchmark's layer (hidden 2048, intermediate 768, 128 experts, 8 per token) in fp16, whole-layer oracle."""
    off = W.moe_group_rows(512, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
    L = Layer(off, W.MOE_HIDDEN, W.MOE_INTER, W.MOE_HIDDEN, 510, "f16")
    d1, d2 = L.descs(B.AXE_GROUPED_AUTO)
    assert B.axe_gemm_grouped_pair_fused(d1, d2)
    h_raw, c_raw, _ = run_pair(L, B.AXE_GROUPED_AUTO)
    h_ref, c_ref = L.oracle()
    check_blocks(L.off, decode(h_raw, "f16"), h_raw, h_ref, TOL["f16"], "H")
    check_blocks(L.off, decode(c_raw, "f16"), c_raw, c_ref, TOL["f16"], "C")
    h2, c2, _ = run_pair(L, B.AXE_GROUPED_AUTO, fused=False)
    assert np.array_equal(h_raw, h2) and np.array_equal(c_raw, c2)


def test_pair_second_gemm_follows_the_first_onto_the_tile_kernels():
    """256 tokens: 16 rows per expert on average.  Alone, the second GEMM (K = 768) would still go to the streaming
    kernel; in a pair it follows the first (K = 2048: tiles), so the pair is fused, and runs the same kernels -- same
    bits -- with and without a workspace."""
    off = W.moe_group_rows(256, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
    L = Layer(off, W.MOE_HIDDEN, W.MOE_INTER, W.MOE_HIDDEN, 511, "f16")
    d1, d2 = L.descs(B.AXE_GROUPED_AUTO)
    assert B.axe_gemm_grouped_kernel(d1) == B.AXE_GROUPED_TILES_128 and B.axe_gemm_grouped_kernel(d2) == B.AXE_GROUPED_STREAM
    assert B.axe_gemm_grouped_pair_fused(d1, d2)
    h_raw, c_raw, _ = run_pair(L, B.AXE_GROUPED_AUTO)
    h_ref, c_ref = L.oracle()
    check_blocks(L.off, decode(h_raw, "f16"), h_raw, h_ref, TOL["f16"], "H")
    check_blocks(L.off, decode(c_raw, "f16"), c_raw, c_ref, TOL["f16"], "C")
    h2, c2, _ = run_pair(L, B.AXE_GROUPED_AUTO, fused=False)
    assert np.array_equal(h_raw, h2) and np.array_equal(c_raw, c2)


_FULL = {}


def full_size_layer():
    """The layer at 4096 tokens (32768 routed rows), bf16: inputs, the fused launch's H and C, the two-launch H and C."""
    if not _FULL:
        off = W.moe_group_rows(4096, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
        L = Layer(off, W.MOE_HIDDEN, W.MOE_INTER, W.MOE_HIDDEN, 511, "bf16")
        d1, d2 = L.descs(B.AXE_GROUPED_AUTO)
        assert B.axe_gemm_grouped_pair_fused(d1, d2)
        h_raw, c_raw, _ = run_pair(L, B.AXE_GROUPED_AUTO)
        h2, c2, _ = run_pair(L, B.AXE_GROUPED_AUTO, fused=False)
        _FULL.update(L=L, h=h_raw, c=c_raw, h2=h2, c2=c2)
    return _FULL


def test_pair_moe_layer_full_size_equals_two_launches():
    f = full_size_layer()
    assert np.array_equal(f["h"], f["h2"]) and np.array_equal(f["c"], f["c2"])


def test_pair_moe_layer_full_size_first_gemm_against_the_oracle():
    f = full_size_layer()
    L = f["L"]
    h_ref = R.swiglu_ref(R.gemm_grouped_ref(L.g1.a_mk, L.g1.b_gnk.transpose(0, 2, 1), L.off, R.AXE_BF16))
    f["h_ref"] = h_ref
    check_blocks(L.off, decode(f["h"], "bf16"), f["h"], h_ref, TOL["bf16"], "H")


def test_pair_moe_layer_full_size_second_gemm_against_the_oracle():
    f = full_size_layer()
    L = f["L"]
    h_ref = f.get("h_ref")
    if h_ref is None:                                               # (run alone: the first GEMM's oracle result is needed as input)
        h_ref = R.swiglu_ref(R.gemm_grouped_ref(L.g1.a_mk, L.g1.b_gnk.transpose(0, 2, 1), L.off, R.AXE_BF16))
    h_bits = W.to_bf16_bits(np.nan_to_num(h_ref, nan=0.0).astype(np.float32))
    c_ref = R.gemm_grouped_ref(h_bits, L.w2.transpose(0, 2, 1), L.off, R.AXE_BF16)
    check_blocks(L.off, decode(f["c"], "bf16"), f["c"], c_ref, TOL["bf16"], "C")


def test_pair_is_bitwise_repeatable_and_reuses_its_workspace():
    """40 launches on one workspace, inputs alternating between two sets of group sizes: every result equals the
    two-launch result of its inputs (a stale count in the workspace, or rows read early, would show)."""
    hidden, inter, out = 512, 256, 512
    offs = [[0, 300, 520, 1300, 1301, 2000], [0, 64, 900, 901, 1200, 2000]]
    Ls = [Layer(o, hidden, inter, out, 520, "bf16") for o in offs]
    want = [run_pair(L, B.AXE_GROUPED_TILES_128, fused=False)[:2] for L in Ls]
    d1, d2 = Ls[0].descs(B.AXE_GROUPED_TILES_128)
    bufs = [L.device() for L in Ls]
    M = Ls[0].M
    dH = torch.empty(M * inter, dtype=torch.int16, device="cuda")
    dC = torch.empty(M * out, dtype=torch.int16, device="cuda")
    sync = torch.zeros(M + 1, dtype=torch.int32, device="cuda")
    for it in range(40):
        k = it & 1
        dA, dW1, dW2, dR = bufs[k]
        dH.fill_(SENTINEL)
        dC.fill_(SENTINEL)
        B.axe_gemm_grouped_pair(d1, d2, dA, dW1, dH, dW2, dC, dR, sync)
        B.axe_gemm_grouped_pair_status(sync, M)
        assert np.array_equal(dH.cpu().numpy().view(np.uint16).reshape(M, inter), want[k][0]), it
        assert np.array_equal(dC.cpu().numpy().view(np.uint16).reshape(M, out), want[k][1]), it


def test_pair_wait_that_cannot_end_gives_up_and_is_reported(monkeypatch):
    """The host asks every wait for one column tile more than the first GEMM has, with a limit of a few polls: every
    wave still leaves the kernel, the waits are counted, and the status call reports them."""
    L = Layer([0, 300, 520, 1300], 256, 256, 256, 530, "bf16")
    monkeypatch.setenv("AXE_GROUPED_PAIR_TEST_NEVER", "1")
    monkeypatch.setenv("AXE_GROUPED_PAIR_POLLS", "3")
    d1, d2 = L.descs(B.AXE_GROUPED_TILES_128)
    dA, dW1, dW2, dR = L.device()
    dH = torch.zeros(L.M * L.I, dtype=torch.int16, device="cuda")
    dC = torch.zeros(L.M * L.N2, dtype=torch.int16, device="cuda")
    sync = torch.zeros(L.M + 1, dtype=torch.int32, device="cuda")
    B.axe_gemm_grouped_pair(d1, d2, dA, dW1, dH, dW2, dC, dR, sync)
    with pytest.raises(B.AxeError) as ei:
        B.axe_gemm_grouped_pair_status(sync, L.M)
    assert ei.value.code == B.AXE_ETIMEOUT
    torch.cuda.synchronize()
    assert int(sync[L.M].item()) > 0
    monkeypatch.delenv("AXE_GROUPED_PAIR_TEST_NEVER")
    monkeypatch.delenv("AXE_GROUPED_PAIR_POLLS")
    B.axe_gemm_grouped_pair(d1, d2, dA, dW1, dH, dW2, dC, dR, sync)          # and the next call is unaffected
    B.axe_gemm_grouped_pair_status(sync, L.M)


def test_pair_falls_back_to_two_launches():
    """Problems that cannot share a launch (here: only two K-steps in the second) run one after the other."""
    L = Layer([0, 300, 520, 1300], 256, 128, 256, 540, "bf16")
    d1, d2 = L.descs(B.AXE_GROUPED_TILES_256)
    assert not B.axe_gemm_grouped_pair_fused(d1, d2)
    h_raw, c_raw, _ = run_pair(L, B.AXE_GROUPED_TILES_256)
    h_ref, c_ref = L.oracle()
    check_blocks(L.off, decode(h_raw, "bf16"), h_raw, h_ref, TOL["bf16"], "H")
    check_blocks(L.off, decode(c_raw, "bf16"), c_raw, c_ref, TOL["bf16"], "C")


def test_pair_can_be_captured_in_a_hip_graph():
    """A serving loop records the layer once and replays it: the fused pair (on a caller's workspace and on the
    library's own) clears its counters with a kernel, allocates nothing and never synchronises.  Every replay, with
    eager work and synchronisations in between and other group sizes in the same buffers, must equal the eager result."""
    hidden, inter, out = 512, 256, 512
    offs = [[0, 300, 520, 1300, 1301, 2000], [0, 64, 900, 901, 1200, 2000]]
    Ls = [Layer(o, hidden, inter, out, 550, "bf16") for o in offs]
    want = [run_pair(L, B.AXE_GROUPED_TILES_128, fused=False)[:2] for L in Ls]
    d1, d2 = Ls[0].descs(B.AXE_GROUPED_TILES_128)
    M = Ls[0].M
    dA, dW1, dW2, dR = Ls[0].device()
    rows = [torch.from_numpy(L.off).cuda() for L in Ls]
    dH = torch.zeros(M * inter, dtype=torch.int16, device="cuda")
    dC = torch.zeros(M * out, dtype=torch.int16, device="cuda")
    dH2, dC2 = torch.zeros_like(dH), torch.zeros_like(dC)
    sync = torch.zeros(M + 1, dtype=torch.int32, device="cuda")

    def layer_twice():
        B.axe_gemm_grouped_pair(d1, d2, dA, dW1, dH, dW2, dC, dR, sync)
        B.axe_gemm_grouped_pair_static(d1, d2, dA, dW1, dH2, dW2, dC2, dR)

    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):                                   # warm-up on the capture stream (also takes the array's address)
        layer_twice()
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph, stream=side):
        layer_twice()
    for rep in range(3):
        for k in (0, 1):
            dR.copy_(rows[k])
            for t in (dH, dC, dH2, dC2):
                t.fill_(SENTINEL)
            torch.randn(1 << 20, device="cuda").sum().item()        # eager work and a synchronisation between replays
            graph.replay()
            torch.cuda.synchronize()
            B.axe_gemm_grouped_pair_status(sync, M)
            B.axe_gemm_grouped_pair_status(None, M)
            for h, c in ((dH, dC), (dH2, dC2)):
                assert np.array_equal(h.cpu().numpy().view(np.uint16).reshape(M, inter), want[k][0]), (rep, k)
                assert np.array_equal(c.cpu().numpy().view(np.uint16).reshape(M, out), want[k][1]), (rep, k)


def test_pair_beside_a_dense_gemm_of_another_stream():
    """The fused pair launched while a dense GEMM of another stream holds compute units: its workgroups then do not
    all start together, the waits for rows last longer -- and still end (the status stays clean), and H, C and the
    dense result are the bits of the quiet launches."""
    g = W.gemm_bf16(4352, 4096, 2048, 91)
    As, Bs, Cs = W.gemm_specs(g)
    d = B.GemmDesc(g.M, g.N, g.K, B.AXE_BF16, B.AXE_BF16, B.Layout(As), B.Layout(Bs), B.Layout(Cs), g.M * g.K, g.N * g.K, g.M * g.N)
    gA, gB = dev(g.a_mk.reshape(-1)), dev(g.b_nk.reshape(-1))
    gC = torch.zeros(g.M * g.N, dtype=torch.int16, device="cuda")
    off = W.moe_group_rows(2048, W.MOE_EXPERTS, W.MOE_TOPK, W.SEED_BASE + 11)
    L = Layer(off, W.MOE_HIDDEN, W.MOE_INTER, W.MOE_HIDDEN, 560, "f16")
    d1, d2 = L.descs(B.AXE_GROUPED_AUTO)
    assert B.axe_gemm_grouped_pair_fused(d1, d2)
    dA, dW1, dW2, dR = L.device()
    dH = torch.zeros(L.M * L.I, dtype=torch.int16, device="cuda")
    dC = torch.zeros(L.M * L.N2, dtype=torch.int16, device="cuda")
    sync = torch.zeros(L.M + 1, dtype=torch.int32, device="cuda")
    B.axe_gemm(d, gA, gB, gC)
    B.axe_gemm_grouped_pair(d1, d2, dA, dW1, dH, dW2, dC, dR, sync)
    torch.cuda.synchronize()
    quiet = (gC.clone(), dH.clone(), dC.clone())
    s1, s2 = torch.cuda.Stream(), torch.cuda.Stream()
    for it in range(30):
        for t in (gC, dH, dC):
            t.zero_()
        torch.cuda.synchronize()
        with torch.cuda.stream(s1):
            B.axe_gemm(d, gA, gB, gC)
            B.axe_gemm(d, gA, gB, gC)
        with torch.cuda.stream(s2):
            B.axe_gemm_grouped_pair(d1, d2, dA, dW1, dH, dW2, dC, dR, sync)
        torch.cuda.synchronize()
        B.axe_gemm_grouped_pair_status(sync, L.M)
        assert torch.equal(gC, quiet[0]) and torch.equal(dH, quiet[1]) and torch.equal(dC, quiet[2]), it
