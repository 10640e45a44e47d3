/* Measurement aids of the Axe-layout hot path: measured ceilings of the matrix pipe and of plain HBM streams.
 *
 * Not part of the hot path and not part of libaxe_hip.so: these live in libaxe_probe.so, which only
 * the benchmark's --ceilings mode loads.  They answer the question the roofline fraction alone
 * cannot: what does the matrix pipe sustain on this data when nothing but MFMAs is issued?
 */
#ifndef AXE_PROBE_H
#define AXE_PROBE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define AXE_PROBE_SAMPLE_BF16 (16 * 256 * 16) /* bytes of operand sample the bf16 loop reads */
#define AXE_PROBE_SAMPLE_FP8 (12 * 256 * 32)  /* bytes of operand sample the fp8 loop reads  */

/* Launches, on `stream` (a hipStream_t, NULL = default stream), a register-only loop of the MFMA
 * instruction, wave count and accumulator order of the 256 x 256 GEMM kernel of that input type
 * (fp8 = 0: bf16, v_mfma_f32_16x16x32_bf16, one wave per SIMD, 8 x 8 fragments; fp8 = 1: e4m3,
 * v_mfma_f32_16x16x128_f8f6f4, two waves per SIMD, 8 x 4 fragments), one workgroup per compute unit,
 * `iters` passes over the wave's fragments.
 *   sample       device pointer, 32-byte aligned, at least AXE_PROBE_SAMPLE_* bytes of operand codes
 *                (a piece of the real input, so that the loop toggles the datapath as the GEMM does);
 *                read only
 *   sink         device pointer to sink_floats floats, at least one per launched thread
 *                (512 x compute units covers both); written, content meaningless
 *   flops        host pointer; receives the flops the launch performs
 * The call is asynchronous; the caller times it with events on `stream`.  Returns 0, 1 for a bad
 * argument, 2 if the launch failed.  Nothing is allocated. */
int axe_probe_mfma(int32_t fp8, const void* sample, size_t sample_bytes, int32_t iters, float* sink, size_t sink_floats,
                   double* flops, void* stream);

/* The bf16 loop of axe_probe_mfma with its 64 MFMAs per pass issued in another order (same instructions, operands and
 * accumulators): what the order alone does to the power the matrix pipe draws, hence to the clock, hence to the rate.
 * walk 0: the GEMM kernel's (fragment rows in pairs, every other pair from the last column back; = axe_probe_mfma),
 * 1: row by row, 2: rows in pairs all in one direction, 3: diagonal (both operands change at every MFMA), 4: rows in
 * blocks of four.  Arguments and return value as axe_probe_mfma (sample: AXE_PROBE_SAMPLE_BF16 bytes; sink: 256 floats
 * per compute unit). */
int axe_probe_mfma_walk(int32_t walk, const void* sample, size_t sample_bytes, int32_t iters, float* sink, size_t sink_floats,
                        double* flops, void* stream);

/* Launches, on `stream`, ONE matrix instruction of one wave on operand registers the caller supplies, and returns the
 * accumulator registers: the experiment that shows which (lane, register) holds which element of the operands and of
 * the result.  The instruction is issued as the GEMM kernels issue it (B fragment first, A fragment second, zero
 * accumulator).  kind 0: v_mfma_f32_16x16x32_bf16, 1: v_mfma_f32_16x16x32_f16 (16 bytes per lane and operand);
 * 2: v_mfma_f32_16x16x128_f8f6f4 with e4m3 operands (32 bytes per lane and operand), 3: the same through the scale
 * path, with the E8M0 code of lane l's operand in byte 0 of a_scale[l] / b_scale[l].
 *   a_regs, b_regs  device pointers, 32-byte aligned: lane l's operand registers at byte offset l * 16 (l * 32)
 *   a_scale, b_scale  device pointers to 64 words (kind 3 only, else ignored)
 *   acc_regs        device pointer, 32-byte aligned, to 64 x 4 floats: lane l's accumulator registers 0..3
 * Asynchronous; returns 0, 1 for a bad argument, 2 if the launch failed.  Nothing is allocated. */
int axe_probe_mfma_fragment(int32_t kind, const void* a_regs, const void* b_regs, const uint32_t* a_scale, const uint32_t* b_scale,
                            float* acc_regs, void* stream);

/* Launches, on `stream`, one pass of a plain HBM stream over `bytes` bytes (a multiple of 16; buffers 16-byte
 * aligned): 128-bit non-temporal accesses, four per thread, the access shape of the relayout kernels without
 * any address arithmetic.  kind 0: copy src -> dst; 1: read src only (dst may be NULL); 2: write dst only
 * (src ignored).  The figure the relayout can be held against on the box it runs on.  Asynchronous; returns 0,
 * 1 for a bad argument, 2 if the launch failed.  Nothing is allocated. */
int axe_probe_stream(int32_t kind, const void* src, void* dst, size_t bytes, void* stream);

#ifdef __cplusplus
}
#endif
#endif
