// Small-tile GEMM for gfx950: workgroup tile 64 x 64, K step of one LDS row (bf16: 32 elements
// = 64 B, fp8: 128 elements = 128 B), 4 waves in a 2 x 2 grid, each wave a 32 x 32 sub-tile made
// of 2 x 2 MFMA 16x16 fragments.  Ragged M / N are handled by zero-filled loads and guarded
// stores, so this kernel serves every shape the library accepts; the large-tile kernel takes
// over for big aligned problems.
//
// Tile movements (all K-contiguous, A row-major and B column-major):
//   HBM -> VGPR : thread t fetches 16-byte chunk (row = t / CH, chunk = t % CH) of the tile
//   VGPR -> LDS : row-major rows of ROWB bytes, 16-byte chunk index XOR-ed with row bits
//   LDS -> VGPR : lane l reads row (l % 16) of a fragment and K chunk l / 16 (bf16: the MFMA operand
//                 layout) or K chunks l / 16 and l / 16 + 4 (fp8: the 32 k of a lane are two runs of
//                 16, the same two for A and for B, so the products pair up as they should).  An LDS
//                 unit serves a 16-byte-per-lane read 16 lanes at a time, and not 16 consecutive ones:
//                 lanes 0-3, 12-15, 20-23, 24-27 go together, then 4-7, 8-11, 16-19, 28-31 (measured
//                 with the bank-conflict counter); key and chunk choice make each such group hit 16
//                 distinct 16-byte bank groups.
//   MFMA        : operands swapped (B rows as the first operand) so that the accumulator
//                 fragment holds 4 consecutive columns of one C row per lane -> vector stores
#include <hip/hip_runtime.h>
#include <stdlib.h>

#include "device_types.h"
#include "kernels.h"
#include "tile_maps.h"

namespace axe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;

__device__ __forceinline__ uint16_t f32_to_bf16_rne(float f) {
  __bf16 h = (__bf16)f;                       // v_cvt_pk_bf16_f32: round to nearest even
  return __builtin_bit_cast(uint16_t, h);
}

__device__ __forceinline__ uint16_t f32_to_f16_rne(float f) {
  _Float16 h = (_Float16)f;
  return __builtin_bit_cast(uint16_t, h);
}

// F16 (with FP8 = false): 16-bit inputs and a 16-bit output are IEEE binary16 instead of bf16
template <bool FP8, bool F16 = false>
__global__ __launch_bounds__(256) void gemm_small_kernel(GemmArgs g) {
  constexpr int EB = FP8 ? 1 : 2;             // element bytes
  constexpr int ROWB = FP8 ? 128 : 64;        // bytes of K per LDS row
  constexpr int CH = ROWB / 16;               // 16-byte chunks per row
  constexpr int BK = ROWB / EB;               // elements per K step
  constexpr int PER = (64 * CH) / 256;        // chunks per thread per operand

  __shared__ __attribute__((aligned(16))) uint8_t lds[2][2][64 * ROWB];   // [stage][A|B]

  const int tid = threadIdx.x;
  const int lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
  const uint8_t* Ab = (const uint8_t*)g.A;
  const uint8_t* Bb = (const uint8_t*)g.B;
  const int64_t nk = (g.K + BK - 1) / BK;

  uint4 ra[PER], rb[PER];
  auto fetch = [&](int64_t kt) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int c = tid + p * 256;
      int row = c / CH, ch = c % CH;
      int64_t k = kt * BK + (int64_t)ch * (16 / EB);
      uint4 z = {0, 0, 0, 0};
      ra[p] = (m0 + row < g.M && k < g.K) ? *(const uint4*)(Ab + ((m0 + row) * g.lda + k) * EB) : z;
      rb[p] = (n0 + row < g.N && k < g.K) ? *(const uint4*)(Bb + ((n0 + row) * g.ldb + k) * EB) : z;
    }
  };
  auto stash = [&](int st) {
#pragma unroll
    for (int p = 0; p < PER; ++p) {
      int c = tid + p * 256;
      int row = c / CH, ch = c % CH;
      int pc = maps::lds_chunk_pos(row, ch, CH);
      *(uint4*)(&lds[st][0][row * ROWB + pc * 16]) = ra[p];
      *(uint4*)(&lds[st][1][row * ROWB + pc * 16]) = rb[p];
    }
  };

  f32x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int frow = lane & 15, fgrp = lane >> 4;
  const int sa_row = (int)(m0 / 128), sb_row = (int)(n0 / 128);

  fetch(0);
  stash(0);
  __syncthreads();
  for (int64_t kt = 0; kt < nk; ++kt) {
    const int st = (int)(kt & 1);
    if (kt + 1 < nk) fetch(kt + 1);
    if constexpr (!FP8) {
      bf16x8 fa[2], fb[2];
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        int r = wm * 32 + f * 16 + frow;
        fa[f] = *(const bf16x8*)(&lds[st][0][r * ROWB + maps::lds_chunk_pos(r, maps::operand_chunk_16bit(0, fgrp), CH) * 16]);
        r = wn * 32 + f * 16 + frow;
        fb[f] = *(const bf16x8*)(&lds[st][1][r * ROWB + maps::lds_chunk_pos(r, maps::operand_chunk_16bit(0, fgrp), CH) * 16]);
      }
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          if constexpr (F16) {
            typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, fb[j]), __builtin_bit_cast(f16x8, fa[i]),
                                                               acc[i][j], 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j], fa[i], acc[i][j], 0, 0, 0);
          }
    } else {
      i32x8 fa[2], fb[2];
#pragma unroll
      for (int f = 0; f < 2; ++f) {
        int r = wm * 32 + f * 16 + frow;
        i32x4 lo = *(const i32x4*)(&lds[st][0][r * ROWB + maps::lds_chunk_pos(r, maps::operand_chunk_fp8(0, fgrp), CH) * 16]);
        i32x4 hi = *(const i32x4*)(&lds[st][0][r * ROWB + maps::lds_chunk_pos(r, maps::operand_chunk_fp8(1, fgrp), CH) * 16]);
        fa[f] = i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
        r = wn * 32 + f * 16 + frow;
        lo = *(const i32x4*)(&lds[st][1][r * ROWB + maps::lds_chunk_pos(r, maps::operand_chunk_fp8(0, fgrp), CH) * 16]);
        hi = *(const i32x4*)(&lds[st][1][r * ROWB + maps::lds_chunk_pos(r, maps::operand_chunk_fp8(1, fgrp), CH) * 16]);
        fb[f] = i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
      }
      if (g.scale_a) {
        // one K step is one 128-deep scale block: accumulate it alone, then scale and add.  A's scale is
        // that of the tile's 128-row block, or (scale_a_rows == 1) of the lane's own row of each fragment.
        float sc[2];
#pragma unroll
        for (int i = 0; i < 2; ++i) {
          int64_t ar = sa_row;
          if (g.scale_a_rows == 1) {
            ar = m0 + wm * 32 + i * 16 + frow;
            ar = ar < g.M ? ar : g.M - 1;        // rows past the end are never stored
          }
          if (g.scale_e8m0) {        // 2^(ca - 127) * 2^(cb - 127), built as the bits of two floats (codes 1..254 are normal numbers)
            const uint32_t ca = ((const uint8_t*)g.scale_a)[ar * g.nkb + kt], cb = ((const uint8_t*)g.scale_b)[(int64_t)sb_row * g.nkb + kt];
            sc[i] = __builtin_bit_cast(float, ca << 23) * __builtin_bit_cast(float, cb << 23);
          } else {
            sc[i] = g.scale_a[ar * g.nkb + kt] * g.scale_b[(int64_t)sb_row * g.nkb + kt];
          }
        }
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j) {
            f32x4 part = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb[j], fa[i], f32x4{0.f, 0.f, 0.f, 0.f},
                                                                        0, 0, 0, 0, 0, 0);
#pragma unroll
            for (int e = 0; e < 4; ++e) acc[i][j][e] = __builtin_fmaf(sc[i], part[e], acc[i][j][e]);
          }
      } else {
#pragma unroll
        for (int i = 0; i < 2; ++i)
#pragma unroll
          for (int j = 0; j < 2; ++j)
            acc[i][j] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb[j], fa[i], acc[i][j], 0, 0, 0, 0, 0, 0);
      }
    }
    if (kt + 1 < nk) stash(st ^ 1);
    __syncthreads();
  }

  // accumulator fragment (operands swapped): lane holds C[m][n .. n+3], m = frag row base + lane % 16,
  // n = frag col base + 4 * (lane / 16)
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      int64_t m = m0 + wm * 32 + i * 16 + frow;
      int64_t n = n0 + wn * 32 + j * 16 + 4 * fgrp;
      if (m >= g.M) continue;
      if (g.out_bf16) {
        uint16_t* C = (uint16_t*)g.C + m * g.ldc + n;
        uint16_t h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = F16 ? f32_to_f16_rne(acc[i][j][e]) : f32_to_bf16_rne(acc[i][j][e]);
        if (n + 3 < g.N && ((g.ldc & 3) == 0)) {
          *(uint2*)C = uint2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < g.N) C[e] = h[e];
        }
      } else {
        float* C = (float*)g.C + m * g.ldc + n;
        if (n + 3 < g.N && ((g.ldc & 3) == 0)) {
          *(float4*)C = float4{acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
        } else {
#pragma unroll
          for (int e = 0; e < 4; ++e)
            if (n + e < g.N) C[e] = acc[i][j][e];
        }
      }
    }
}

// Short K, few tiles: the time of such a launch is latency -- of the launch itself and of K-step after K-step each
// waiting for its own loads.  This variant asks for everything at once: all K-tiles (64 elements = one 128-byte row
// each) of the workgroup's 64 rows of A and 64 rows of B go straight from HBM into LDS in one burst of direct-to-LDS
// loads, every K-tile into an 8 KiB block of its own (up to 8 of them per operand: 128 KiB), in K order; the K loop then
// waits only for the K-tile it is about to multiply (a counted wait: 4 loads per wave and K-tile) and never for a
// load it has yet to issue.  LDS image, swizzle, operand reads and the MFMA order inside a K-tile are those of the
// 256-row kernels (tile_maps.h).  16-bit inputs, whole tiles (M and N multiples of 64, K a multiple of 64).
template <bool F16>
__global__ __launch_bounds__(256) void gemm_small_preload_kernel(GemmArgs g) {
  constexpr int kRow = maps::kLargeRowBytes;
  constexpr int kBlk = 64 * kRow;                  // 64 rows of one operand, one K-tile
  constexpr int kMaxTiles = 8;
  typedef __attribute__((address_space(3))) void* lds_ptr;
  typedef __attribute__((address_space(3))) uint8_t* lds_u8;
  __shared__ __attribute__((aligned(1024))) uint8_t lds_mem[2 * kMaxTiles * kBlk];   // A's K-tiles, then B's
  const lds_u8 lds3 = (lds_u8)lds_mem;
  const int tid = threadIdx.x, lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = w >> 1, wn = w & 1;
  const int nkt = (int)(g.K / 64);
  const int64_t m0 = (int64_t)blockIdx.y * 64, n0 = (int64_t)blockIdx.x * 64;
  const int a_pitch = (int)(g.lda * 2), b_pitch = (int)(g.ldb * 2);
  // the tile's 64 rows of either operand (reads past the end return zero; the host admits whole tiles only)
  const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.A + m0 * g.lda * 2), 0,
                                                                      63 * a_pitch + (int)g.K * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.B + n0 * g.ldb * 2), 0,
                                                                      63 * b_pitch + (int)g.K * 2, 0x00020000);
  // one wave instruction = 8 rows x 128 bytes; wave w takes the row groups w and w + 4
  const int lr = lane / maps::kLargeChunks, lp = lane % maps::kLargeChunks;
  int a_voff[2], b_voff[2];
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int row = maps::piece_row(w, i, lr, 4);
    a_voff[i] = row * a_pitch + maps::lds_chunk_pos(row, lp, maps::kLargeChunks) * maps::kChunkBytes;
    b_voff[i] = row * b_pitch + maps::lds_chunk_pos(row, lp, maps::kLargeChunks) * maps::kChunkBytes;
  }
  for (int t = 0; t < nkt; ++t) {
#pragma unroll
    for (int i = 0; i < 2; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(ra, (lds_ptr)(lds3 + t * kBlk + maps::piece_row(w, i, 0, 4) * kRow), 16, a_voff[i], t * kRow, 0, 0);
#pragma unroll
    for (int i = 0; i < 2; ++i)
      __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_ptr)(lds3 + (kMaxTiles + t) * kBlk + maps::piece_row(w, i, 0, 4) * kRow), 16, b_voff[i],
                                               t * kRow, 0, 0);
  }

  const int fr = lane % maps::kFrag, fq = lane / maps::kFrag;
  int pos[2];
#pragma unroll
  for (int s = 0; s < 2; ++s) pos[s] = maps::lds_chunk_pos(fr, maps::operand_chunk_16bit(s, fq), maps::kLargeChunks) * maps::kChunkBytes;
  const lds_u8 pa = lds3 + (wm * 32 + fr) * kRow, pb = lds3 + kMaxTiles * kBlk + (wn * 32 + fr) * kRow;

  f32x4 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  for (int t = 0; t < nkt; ++t) {
    // the 4 (nkt - 1 - t) loads of the later K-tiles may still be in flight
    switch (nkt - 1 - t) {
      case 0: asm volatile("s_waitcnt vmcnt(0)" ::: "memory"); break;
      case 1: asm volatile("s_waitcnt vmcnt(4)" ::: "memory"); break;
      case 2: asm volatile("s_waitcnt vmcnt(8)" ::: "memory"); break;
      case 3: asm volatile("s_waitcnt vmcnt(12)" ::: "memory"); break;
      case 4: asm volatile("s_waitcnt vmcnt(16)" ::: "memory"); break;
      case 5: asm volatile("s_waitcnt vmcnt(20)" ::: "memory"); break;
      case 6: asm volatile("s_waitcnt vmcnt(24)" ::: "memory"); break;
      default: asm volatile("s_waitcnt vmcnt(28)" ::: "memory"); break;
    }
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    bf16x8 fa[2][2], fb[2][2];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int s = 0; s < 2; ++s) {
        fa[f][s] = *(__attribute__((address_space(3))) const bf16x8*)(pa + t * kBlk + f * 16 * kRow + pos[s]);
        fb[f][s] = *(__attribute__((address_space(3))) const bf16x8*)(pb + t * kBlk + f * 16 * kRow + pos[s]);
      }
#pragma unroll
    for (int s = 0; s < 2; ++s)
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j)
          if constexpr (F16) {
            typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, fb[j][s]), __builtin_bit_cast(f16x8, fa[i][s]),
                                                               acc[i][j], 0, 0, 0);
          } else {
            acc[i][j] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(fb[j][s], fa[i][s], acc[i][j], 0, 0, 0);
          }
  }

  // accumulator fragment (operands swapped): lane holds C[m][n .. n + 3]
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j) {
      const int64_t m = m0 + wm * 32 + i * 16 + fr;
      const int64_t n = n0 + wn * 32 + j * 16 + maps::kAccCols * fq;
      if (g.out_bf16) {
        uint16_t h[4];
#pragma unroll
        for (int e = 0; e < 4; ++e) h[e] = F16 ? f32_to_f16_rne(acc[i][j][e]) : f32_to_bf16_rne(acc[i][j][e]);
        *(uint2*)((uint16_t*)g.C + m * g.ldc + n) = uint2{(uint32_t)h[0] | ((uint32_t)h[1] << 16), (uint32_t)h[2] | ((uint32_t)h[3] << 16)};
      } else {
        *(float4*)((float*)g.C + m * g.ldc + n) = float4{acc[i][j][0], acc[i][j][1], acc[i][j][2], acc[i][j][3]};
      }
    }
}

// The burst variant serves 16-bit problems made of whole 64 x 64 tiles with at most 8 K-tiles of 64 (K <= 512), C
// rows aligned for the vector stores, and few enough tiles that they are all on the chip at once (a workgroup holds
// 16 KiB of LDS per K-tile, so at most one or two fit a compute unit: with many tiles the regular kernel's higher
// occupancy wins).
bool small_preload_fits(const GemmArgs& g, bool fp8) {
  static const bool enabled = [] { const char* v = getenv("AXE_SMALL_BURST"); return !v || atoi(v) != 0; }();
  if (!enabled || fp8 || g.M % 64 || g.N % 64 || g.K % 64 || g.K > 512 || g.K <= 0) return false;
  if (g.ldc % 4 || 64 * g.lda * 2 >= (int64_t(1) << 31) || 64 * g.ldb * 2 >= (int64_t(1) << 31)) return false;
  return (g.M / 64) * (g.N / 64) <= cu_count();
}

hipError_t launch_gemm_small(const GemmArgs& g, bool fp8, hipStream_t s) {
  dim3 grid((unsigned)((g.N + 63) / 64), (unsigned)((g.M + 63) / 64));
  if (small_preload_fits(g, fp8)) {
    if (g.f16) hipLaunchKernelGGL(gemm_small_preload_kernel<true>, grid, dim3(256), 0, s, g);
    else hipLaunchKernelGGL(gemm_small_preload_kernel<false>, grid, dim3(256), 0, s, g);
    return hipGetLastError();
  }
  if (fp8)
    hipLaunchKernelGGL(gemm_small_kernel<true>, grid, dim3(256), 0, s, g);
  else if (g.f16)
    hipLaunchKernelGGL((gemm_small_kernel<false, true>), grid, dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_small_kernel<false>, grid, dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace axe
