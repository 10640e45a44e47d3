// Measured ceilings of the matrix pipe (measurement aids, not part of the hot path; a library of
// their own, libaxe_probe.so, loaded only by bench.py --ceilings).
//
// A register-only loop of the very MFMA instruction, wave shape and accumulator walk of the GEMM
// kernel it stands for: operands are loaded once from a caller-supplied sample of the real input,
// then the loop issues nothing but MFMAs.  What it sustains on that data is what the kernel could
// reach if LDS, L2 and HBM cost neither time nor power; on random data this is well below the
// nominal peak because the chip runs into its power limit.
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "../../include/axe_probe.h"
#include "gemm_common.h"
#include "kernels.h"

namespace {
using axe::bf16x8;
using axe::f32x4;
using axe::i32x8;

// bf16: one wave per SIMD (4 per workgroup), 8 x 8 fragments of v_mfma_f32_16x16x32_bf16, fragment rows in pairs with j
// innermost, every other pair backwards, as the kernel walks them (asm statements: the order issued is the order written).
// WALK: 0 = the kernel's (rows in pairs, every other pair backwards), 1 = row by row, 2 = rows in pairs all in one
// direction, 3 = diagonal (both operands change at every MFMA), 4 = rows in blocks of four.
template <int WALK>
__device__ __forceinline__ void probe_bf16_body(const bf16x8* __restrict__ in, float* out, int iters) {
  bf16x8 a[8], b[8];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = in[i * 256 + threadIdx.x];
#pragma unroll
  for (int j = 0; j < 8; ++j) b[j] = in[(8 + j) * 256 + threadIdx.x];
  f32x4 acc[8][8];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int t = 0; t < 64; ++t) {
      int i, j;
      if (WALK == 0) i = 2 * (t >> 4) + (t & 1), j = ((t >> 4) & 1) ? 7 - ((t >> 1) & 7) : (t >> 1) & 7;
      else if (WALK == 1) i = t >> 3, j = t & 7;
      else if (WALK == 2) i = 2 * (t >> 4) + (t & 1), j = (t >> 1) & 7;
      else if (WALK == 3) i = t & 7, j = ((t >> 3) + t) & 7;
      else i = 4 * (t >> 5) + (t & 3), j = (t >> 2) & 7;
      asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc[i][j]) : "v"(b[j]), "v"(a[i]));
    }
  }
  asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");              // the MFMAs retire before their results are read
  __builtin_amdgcn_sched_barrier(0);
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  out[blockIdx.x * 256 + threadIdx.x] = s;
}
__global__ __launch_bounds__(256, 1) void probe_bf16_kernel(const bf16x8* __restrict__ in, float* out, int iters) { probe_bf16_body<0>(in, out, iters); }
__global__ __launch_bounds__(256, 1) void probe_bf16_rows_kernel(const bf16x8* __restrict__ in, float* out, int iters) { probe_bf16_body<1>(in, out, iters); }
__global__ __launch_bounds__(256, 1) void probe_bf16_pairs_kernel(const bf16x8* __restrict__ in, float* out, int iters) { probe_bf16_body<2>(in, out, iters); }
__global__ __launch_bounds__(256, 1) void probe_bf16_diagonal_kernel(const bf16x8* __restrict__ in, float* out, int iters) { probe_bf16_body<3>(in, out, iters); }
__global__ __launch_bounds__(256, 1) void probe_bf16_fours_kernel(const bf16x8* __restrict__ in, float* out, int iters) { probe_bf16_body<4>(in, out, iters); }

// fp8: two waves per SIMD (8 per workgroup), 8 x 4 fragments of v_mfma_f32_16x16x128_f8f6f4, j innermost.
__global__ __launch_bounds__(512, 1) void probe_fp8_kernel(const i32x8* __restrict__ in, float* out, int iters) {
  const int t = threadIdx.x & 255;
  i32x8 a[8], b[4];
#pragma unroll
  for (int i = 0; i < 8; ++i) a[i] = in[i * 256 + t];
#pragma unroll
  for (int j = 0; j < 4; ++j) b[j] = in[(8 + j) * 256 + t];
  f32x4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int it = 0; it < iters; ++it) {
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(b[j], a[i], acc[i][j], 0, 0, 0, 0, 0, 0);
  }
  float s = 0.f;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) s += acc[i][j][0] + acc[i][j][1] + acc[i][j][2] + acc[i][j][3];
  out[blockIdx.x * 512 + threadIdx.x] = s;
}
// One MFMA on operand registers the caller supplies, lane by lane: where do the products land?  The instruction is
// issued the way the GEMM kernels issue it -- the B fragment as the first operand, the A fragment as the second, so
// that a lane's accumulator registers hold consecutive columns of one row -- with a zero accumulator.  KIND 0:
// v_mfma_f32_16x16x32_bf16, 1: v_mfma_f32_16x16x32_f16, 2: v_mfma_f32_16x16x128_f8f6f4 (e4m3, unscaled), 3: the
// same on the scale path, each lane supplying the E8M0 code of its operand in byte 0 of a register.
template <int KIND>
__global__ __launch_bounds__(64) void probe_fragment_kernel(const uint8_t* __restrict__ a, const uint8_t* __restrict__ b,
                                                            const uint32_t* __restrict__ sa, const uint32_t* __restrict__ sb,
                                                            float* __restrict__ acc_out) {
  const int lane = threadIdx.x;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  if constexpr (KIND <= 1) {
    const bf16x8 fa = *(const bf16x8*)(a + lane * 16), fb = *(const bf16x8*)(b + lane * 16);
    if constexpr (KIND == 0) acc = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb, fa, acc, 0, 0, 0);
    else {
      typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
      acc = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, fb), __builtin_bit_cast(f16x8, fa), acc, 0, 0, 0);
    }
  } else {
    const i32x8 fa = *(const i32x8*)(a + lane * 32), fb = *(const i32x8*)(b + lane * 32);
    if constexpr (KIND == 2) acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb, fa, acc, 0, 0, 0, 0, 0, 0);
    else acc = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb, fa, acc, 0, 0, 0, (int)sb[lane], 0, (int)sa[lane]);
  }
#pragma unroll
  for (int e = 0; e < 4; ++e) acc_out[lane * 4 + e] = acc[e];
}

// HBM streams: what this machine's memory system gives a plain kernel -- 16 bytes per lane and access, four accesses per
// thread issued together, non-temporal, one pass over the buffers.  KIND 0: copy, 1: read only (the words are
// folded into a sum nobody needs, written only if it has an impossible value so that the loads stay), 2: write only.
typedef __attribute__((ext_vector_type(4))) unsigned int probe_u32x4;
template <int KIND>
__global__ __launch_bounds__(256) void probe_stream_kernel(const probe_u32x4* __restrict__ src, probe_u32x4* __restrict__ dst, size_t n) {
  const size_t i = (size_t)blockIdx.x * 1024 + threadIdx.x;
  probe_u32x4 v[4];
#pragma unroll
  for (int u = 0; u < 4; ++u) {
    if (KIND == 2) v[u] = probe_u32x4{(unsigned)i, 1u, 2u, 3u};
    else if (i + u * 256 < n) v[u] = __builtin_nontemporal_load(&src[i + u * 256]);
    else v[u] = probe_u32x4{0u, 0u, 0u, 0u};
  }
  if (KIND == 1) {
    unsigned x = 0;
#pragma unroll
    for (int u = 0; u < 4; ++u) x ^= v[u][0] ^ v[u][1] ^ v[u][2] ^ v[u][3];
    if (x == 0x9e3779b9u && n == 1) dst[0] = v[0];                 // (never with the buffers the benchmark passes)
    return;
  }
#pragma unroll
  for (int u = 0; u < 4; ++u)
    if (i + u * 256 < n) __builtin_nontemporal_store(v[u], &dst[i + u * 256]);
}
}  // namespace

extern "C" int axe_probe_mfma_fragment(int32_t kind, const void* a_regs, const void* b_regs, const uint32_t* a_scale,
                                       const uint32_t* b_scale, float* acc_regs, void* stream) {
  if (kind < 0 || kind > 3 || !a_regs || !b_regs || !acc_regs || (kind == 3 && (!a_scale || !b_scale)) ||
      (((uintptr_t)a_regs | (uintptr_t)b_regs | (uintptr_t)acc_regs) & 31))
    return 1;
  hipStream_t st = (hipStream_t)stream;
  const uint8_t *a = (const uint8_t*)a_regs, *b = (const uint8_t*)b_regs;
  switch (kind) {
    case 0: hipLaunchKernelGGL(probe_fragment_kernel<0>, dim3(1), dim3(64), 0, st, a, b, a_scale, b_scale, acc_regs); break;
    case 1: hipLaunchKernelGGL(probe_fragment_kernel<1>, dim3(1), dim3(64), 0, st, a, b, a_scale, b_scale, acc_regs); break;
    case 2: hipLaunchKernelGGL(probe_fragment_kernel<2>, dim3(1), dim3(64), 0, st, a, b, a_scale, b_scale, acc_regs); break;
    default: hipLaunchKernelGGL(probe_fragment_kernel<3>, dim3(1), dim3(64), 0, st, a, b, a_scale, b_scale, acc_regs); break;
  }
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

extern "C" int axe_probe_stream(int32_t kind, const void* src, void* dst, size_t bytes, void* stream) {
  if (kind < 0 || kind > 2 || bytes == 0 || bytes % 16 || (kind != 2 && !src) || (kind != 1 && !dst) ||
      (((uintptr_t)src | (uintptr_t)dst) & 15))
    return 1;
  const size_t n = bytes / 16, nwg = (n + 1023) / 1024;
  if (nwg > 0x7fffffffu || (kind == 1 && n < 2)) return 1;       // (n >= 2: the read-only kernel's guarded store can never happen)
  const dim3 grid((unsigned)nwg), block(256);
  hipStream_t st = (hipStream_t)stream;
  if (kind == 0) hipLaunchKernelGGL(probe_stream_kernel<0>, grid, block, 0, st, (const probe_u32x4*)src, (probe_u32x4*)dst, n);
  else if (kind == 1) hipLaunchKernelGGL(probe_stream_kernel<1>, grid, block, 0, st, (const probe_u32x4*)src, (probe_u32x4*)(dst ? dst : (void*)src), n);
  else hipLaunchKernelGGL(probe_stream_kernel<2>, grid, block, 0, st, (const probe_u32x4*)dst, (probe_u32x4*)dst, n);
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

extern "C" int axe_probe_mfma_walk(int32_t walk, const void* sample, size_t sample_bytes, int32_t iters, float* sink, size_t sink_floats,
                                   double* flops, void* stream) {
  const int cus = axe::cu_count();
  if (walk < 0 || walk > 4 || !sample || !sink || !flops || iters <= 0 || sample_bytes < AXE_PROBE_SAMPLE_BF16 ||
      sink_floats < (size_t)cus * 256 || ((uintptr_t)sample & 31))
    return 1;
  const dim3 grid(cus), block(256);
  hipStream_t st = (hipStream_t)stream;
  const bf16x8* in = (const bf16x8*)sample;
  switch (walk) {
    case 0: hipLaunchKernelGGL(probe_bf16_kernel, grid, block, 0, st, in, sink, iters); break;
    case 1: hipLaunchKernelGGL(probe_bf16_rows_kernel, grid, block, 0, st, in, sink, iters); break;
    case 2: hipLaunchKernelGGL(probe_bf16_pairs_kernel, grid, block, 0, st, in, sink, iters); break;
    case 3: hipLaunchKernelGGL(probe_bf16_diagonal_kernel, grid, block, 0, st, in, sink, iters); break;
    default: hipLaunchKernelGGL(probe_bf16_fours_kernel, grid, block, 0, st, in, sink, iters); break;
  }
  *flops = 2.0 * 16 * 16 * 32 * 64 * (double)iters * 4 * cus;
  return hipGetLastError() == hipSuccess ? 0 : 2;
}

extern "C" int axe_probe_mfma(int32_t fp8, const void* sample, size_t sample_bytes, int32_t iters, float* sink,
                              size_t sink_floats, double* flops, void* stream) {
  const int cus = axe::cu_count();
  const size_t need = fp8 ? AXE_PROBE_SAMPLE_FP8 : AXE_PROBE_SAMPLE_BF16;
  const size_t threads = (size_t)cus * (fp8 ? 512 : 256);
  if (!sample || !sink || !flops || iters <= 0 || sample_bytes < need || sink_floats < threads || ((uintptr_t)sample & 31)) return 1;
  if (fp8) {
    hipLaunchKernelGGL(probe_fp8_kernel, dim3(cus), dim3(512), 0, (hipStream_t)stream, (const i32x8*)sample, sink, iters);
    *flops = 2.0 * 16 * 16 * 128 * 32 * (double)iters * 8 * cus;
  } else {
    hipLaunchKernelGGL(probe_bf16_kernel, dim3(cus), dim3(256), 0, (hipStream_t)stream, (const bf16x8*)sample, sink, iters);
    *flops = 2.0 * 16 * 16 * 32 * 64 * (double)iters * 4 * cus;
  }
  return hipGetLastError() == hipSuccess ? 0 : 2;
}
