"""What the hand-scheduled GEMM kernels rely on, checked on the ISA hipcc actually emits (CPU only:
the kernels are cross-compiled to assembly, nothing runs).

The kernels count their own memory waits (s_waitcnt vmcnt(N)) and issue some loads and stores as
asm statements the compiler cannot see; that is only sound while the compiler adds nothing of its
own inside the K loops.  These tests fail when a change of source or compiler breaks one of the
assumptions silently:
  * no scratch (spill) traffic and no compiler-inserted vmcnt wait inside a K loop -- a spilled
    register that an asm-issued load is still filling would be saved before the data arrives;
  * the waits inside the K loops are exactly the counted ones;
  * every asm-issued buffer instruction is preceded by its s_nop padding (an SGPR written by the
    vector ALU must not be read by a vector-memory instruction less than 5 wait states later);
  * the bf16 and E8M0 kernels keep their accumulators in AGPRs: no v_accvgpr moves inside a K loop.
"""
import os
import re
import subprocess

import pytest

from paper_2601_19092_amd import build as BLD

HIPCC = os.environ.get("HIPCC", "/opt/rocm/bin/hipcc")


def kernel_asm(source: str, tmp_path_factory) -> dict:
    out = tmp_path_factory.mktemp("isa") / (source + ".s")
    subprocess.check_call([HIPCC, *BLD.FLAGS, "-I", BLD.CSRC, "-S", "--cuda-device-only", os.path.join(BLD.CSRC, source),
                           "-o", str(out)], stderr=subprocess.DEVNULL)
    text = open(out).read()
    kernels = {}
    for m in re.finditer(r"^(_ZN3axe\w+):[^\n]*\n(.*?)\n\ts_endpgm", text, re.S | re.M):
        kernels[m.group(1)] = m.group(2).split("\n")
    return kernels


@pytest.fixture(scope="module")
def isa(tmp_path_factory):
    return {src: kernel_asm(src, tmp_path_factory)
            for src in ("kernels_gemm_bf16.hip", "kernels_gemm_fp8.hip", "kernels_gemm_fp8_e8m0.hip")}


def k_loops(lines):
    """Line ranges [first MFMA of a loop body .. its backward branch] of the loops that contain MFMAs."""
    labels = {l[:-1].split(":")[0]: i for i, l in enumerate(lines) if re.match(r"^\.LBB\d+_\d+:", l)}
    loops = []
    for i, l in enumerate(lines):
        m = re.match(r"\ts_cbranch_\w+ (\.LBB\d+_\d+)", l)
        if m and m.group(1) in labels and labels[m.group(1)] < i:
            body = lines[labels[m.group(1)]:i]
            if sum("v_mfma" in x for x in body) >= 32:
                loops.append((labels[m.group(1)], i))
    # keep innermost ones only
    inner = [a for a in loops if not any(b != a and a[0] <= b[0] and b[1] <= a[1] for b in loops)]
    return inner


# (source, kernel, counted waits, accumulators in AGPRs, asm-issued global loads allowed in a loop)
CASES = [("kernels_gemm_bf16.hip", "gemm_bf16_256_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_bf16_256x224_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_bf16_256_grouped_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_bf16_256_blocked_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_bf16_256_grouped_gated_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_bf16_256_f32out_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_bf16_256_ragged_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_f16_256_ragged_f32out_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_f16_256_ragged_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_bf16_128_grouped_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_f16_128_grouped_gated_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_f16_256_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_f16_256_grouped_kernel", {8}, True, 0),
         ("kernels_gemm_bf16.hip", "gemm_f16_256_grouped_gated_kernel", {8}, True, 0),
         ("kernels_gemm_fp8_e8m0.hip", "gemm_fp8_e8m0_256_kernel", {8}, True, 0),
         # the fp32-scale kernel prefetches the next tile's two scale words with asm-issued loads of its own
         ("kernels_gemm_fp8.hip", "gemm_fp8_256_kernel", {4}, False, 2)]


@pytest.mark.parametrize("source,kernel,waits,agpr_acc,asm_loads", CASES)
def test_k_loops_hold_only_the_counted_waits(isa, source, kernel, waits, agpr_acc, asm_loads):
    (name, lines), = [(k, v) for k, v in isa[source].items() if kernel + "E" in k]
    if asm_loads:
        # registers that asm-issued loads are still filling must never be saved to scratch: no spills at all
        assert not [l for l in lines if "scratch_" in l], f"{kernel}: spills in a kernel with asm-issued global loads"
        src = open(os.path.join(BLD.CSRC, source)).read()
        assert len(re.findall(r'asm volatile\("global_load_dword', src)) == asm_loads
    loops = k_loops(lines)
    assert len(loops) >= 2, "steady loop and next-tile loop expected"
    for a, b in loops:
        body = lines[a:b]
        assert not [l for l in body if "scratch_" in l], f"{kernel}: spill traffic inside a K loop"
        seen = {int(n) for l in body for n in re.findall(r"vmcnt\((\d+)\)", l)}
        assert seen == waits, f"{kernel}: waits {sorted(seen)} inside a K loop, expected {sorted(waits)}"
        if agpr_acc:
            assert not [l for l in body if "v_accvgpr" in l], f"{kernel}: accumulator moves inside a K loop"
        loads = [l for l in body if re.search(r"\bflat_load|\bglobal_load", l)]
        assert len(loads) <= asm_loads, f"{kernel}: a compiler-visible global load inside a K loop: {loads}"
        mfma = sum("v_mfma" in l for l in body)
        assert mfma % 32 == 0 or mfma % 56 == 0, "whole K-steps of one wave"


@pytest.mark.parametrize("source", ["kernels_gemm_bf16.hip", "kernels_gemm_fp8.hip", "kernels_gemm_fp8_e8m0.hip"])
def test_asm_issued_buffer_instructions_are_padded(isa, source):
    src = open(os.path.join(BLD.CSRC, source)).read()
    asm_buffer = re.findall(r'asm volatile\("([^"]*buffer_(?:load|store)[^"]*)"', src)
    assert asm_buffer, "the kernel issues buffer instructions as asm statements"
    assert all(a.startswith("s_nop 4\\n\\t") for a in asm_buffer)
    # and in the emitted ISA: each such instruction (register destination or store) directly follows the padding
    for name, lines in isa[source].items():
        for i, l in enumerate(lines):
            if re.match(r"\tbuffer_store_dwordx[24] ", l) or re.match(r"\tbuffer_load_dwordx4 v\[\d+:\d+\], v\d+, s\[\d+:\d+\], s\d+ offen$", l):
                assert lines[i - 1].strip() == "s_nop 4", (name, i, lines[i - 1], l)
            # ... and every store is followed by wait states of its own: the compiler does not know the asm statement
            # reads its data registers for a while after issue, and would let the next vector-ALU instruction overwrite them
            if re.match(r"\tbuffer_store_dwordx[24] ", l):
                assert re.match(r"s_nop [3-9]$", lines[i + 1].strip()), (name, i, l, lines[i + 1])


@pytest.mark.parametrize("kernel", ["gemm_bf16_128_grouped_pair_kernel", "gemm_f16_128_grouped_pair_kernel",
                                    "gemm_bf16_256_grouped_pair_kernel", "gemm_f16_256_grouped_pair_kernel"])
def test_fused_pair_publishes_with_write_through_stores_and_acquires_before_it_reads(isa, kernel):
    """The hand-over between the two grouped GEMMs of a fused pair, on the emitted ISA: the first GEMM's tiles are
    stored at device scope (sc1: written through to memory) and the kernel holds no write-back of the whole L2 (the
    language's device-scope release, measured slower than two launches); the polls of the row block's word are
    device-scope loads; a device-scope invalidate stands between the polls and the second GEMM's loads; and both
    bodies' K loops keep the invariants of the single kernels."""
    (name, lines), = [(k, v) for k, v in isa["kernels_gemm_bf16.hip"].items() if kernel + "E" in k]
    stores = [l for l in lines if re.match(r"\tbuffer_store_dwordx4 ", l)]
    sc1 = [l for l in stores if l.rstrip().endswith("sc1")]
    assert sc1 and len(sc1) < len(stores), "the first GEMM stores at device scope, the second does not"
    assert not [l for l in lines if "buffer_wbl2" in l]
    assert [l for l in lines if re.match(r"\tglobal_load_dword v\d+, v\d+, s\[\d+:\d+\] sc1", l)], "device-scope polls"
    inv = [i for i, l in enumerate(lines) if "buffer_inv sc1" in l]
    assert inv, "device-scope acquire"
    # every poll loop (s_sleep) is followed by an invalidate before the next direct-to-LDS load
    for i, l in enumerate(lines):
        if "s_sleep" in l:
            nxt_inv = min(j for j in inv if j > i)
            nxt_lds_load = min((j for j, x in enumerate(lines) if j > i and re.search(r"buffer_load_dwordx4 .* lds$", x)), default=len(lines))
            assert nxt_inv < nxt_lds_load, (kernel, i)
    loops = k_loops(lines)
    assert len(loops) >= 4, "steady and next-tile loops of both bodies"
    for a, b in loops:
        body = lines[a:b]
        assert not [l for l in body if "scratch_" in l]
        assert {int(n) for l in body for n in re.findall(r"vmcnt\((\d+)\)", l)} == {8}
        assert not [l for l in body if "v_accvgpr" in l or "buffer_inv" in l or "s_sleep" in l]
