// fp8 (OCP e4m3) GEMM for gfx950 (MI355X) with optional fp32 scales per 128 x 128 block:
// workgroup tile 256 x 256 x 128, 4 waves (one per SIMD), each a 128 x 128 sub-tile = 4 x 4 MFMA
// 32x32x64 fragments.  A row-major, B column-major (both K contiguous).
//
// Tile movements, each an Axe layout (reported by axe_gemm_describe):
//   HBM -> LDS  : global_load_lds_dwordx4; one wave instruction fills 8 LDS rows of 128 bytes; the
//                 XOR swizzle is applied on the global side: lane (r = lane / 8, p = lane % 8)
//                 fetches chunk p ^ key(r) of row r, key(r) = (r >> 1) & 7 (64 LDS banks: conflict-free).
//   LDS layout  : two stages of 64 KiB, A tile then B tile, rows of 128 bytes (128 fp8).
//   LDS -> VGPR : lane l reads row l % 32 of a fragment and the two adjacent 16-byte chunks
//                 4 * ks + 2 * (l / 32) + {0, 1}: 32 consecutive k per lane, the operand layout
//                 of MFMA 32x32x64 (A and B are loaded the same way, so the pairing of k is kept).
//   scales      : one K step is one 128-deep scale block; it is accumulated on its own (MFMA with a
//                 zero accumulator), then acc += (sA * sB) * block on the vector ALU.
//   VGPR -> HBM : accumulators -> bf16 -> LDS -> 16-byte coalesced stores.
#include <hip/hip_runtime.h>

#include "device_types.h"
#include "gemm_common.h"
#include "kernels.h"

namespace axe {

namespace {
constexpr int kRowB = 128;                        // bytes of K per LDS row
constexpr int kOperandB = kTile * kRowB;          // 32 KiB per operand per stage
constexpr int kStageB = 2 * kOperandB;            // 64 KiB
static_assert(2 * kStageB <= kEpiB, "the epilogue staging area covers both stages");
}  // namespace

__global__ __launch_bounds__(256, 1) void gemm_fp8_256_kernel(GemmArgs g) {
  constexpr int EB = 1;
  constexpr int BK = kRowB / EB;                  // 128 fp8 per K step
  __shared__ __attribute__((aligned(1024))) uint8_t lds[kEpiB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave id, kept scalar
  const int wm = w >> 1, wn = w & 1;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, g.grid_m, g.grid_n, tm, tn);
  const int64_t m0 = (int64_t)tm * kTile, n0 = (int64_t)tn * kTile;
  const int nk = (int)(g.K / BK);

  // ---- HBM -> LDS: per wave and K step, 8 instructions for A and 8 for B; instruction i of wave w
  //      covers LDS rows (4 i + w) * 8 .. + 7
  const int lr = lane >> 3;                                   // row inside the 8-row group
  const int lc = (lane & 7) ^ ((4 * (w & 1) + (lr >> 1)) & 7);  // global chunk this lane fetches: p ^ key(row)
  const uint8_t* ga = (const uint8_t*)g.A + ((m0 + w * 8 + lr) * g.lda) * EB + lc * 16;
  const uint8_t* gb = (const uint8_t*)g.B + ((n0 + w * 8 + lr) * g.ldb) * EB + lc * 16;
  const int64_t a_step = 32 * g.lda * EB, b_step = 32 * g.ldb * EB;   // bytes between instructions

  auto issue_loads = [&](int kt, int stage) {
    const uint8_t* pa = ga + (int64_t)kt * kRowB;
    const uint8_t* pb = gb + (int64_t)kt * kRowB;
    uint8_t* la = lds + stage * kStageB + w * 8 * kRowB;
    uint8_t* lb = la + kOperandB;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_global_load_lds(pa + i * a_step, (__attribute__((address_space(3))) void*)(la + i * 32 * kRowB), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(pb + i * b_step, (__attribute__((address_space(3))) void*)(lb + i * 32 * kRowB), 16, 0, 0);
    }
  };

  // ---- LDS -> VGPR: fragment f of this wave's A (B) rows: row = base + f * 32 + lane % 32
  const int fr = lane & 31, fh = lane >> 5;
  const int fkey = (fr >> 1) & 7;
  const uint8_t* fa_base = lds + (wm * 128 + fr) * kRowB;
  const uint8_t* fb_base = lds + kOperandB + (wn * 128 + fr) * kRowB;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  // fp8: one K step = one 128-deep scale block = two MFMA 32x32x64 (ks = 0, 1); a lane's operand
  // fragment is 32 bytes = two adjacent 16-byte chunks.  B fragments of the step stay resident,
  // A fragments are streamed one fragment row ahead of the MFMAs that use them.
  i32x8 fb[2][4], fa[2][2];
  auto read_frag = [&](const uint8_t* base, int stage, int ks, int f) -> i32x8 {
    const int o0 = stage * kStageB + (((4 * ks + 2 * fh) ^ fkey) << 4);
    const int o1 = stage * kStageB + (((4 * ks + 2 * fh + 1) ^ fkey) << 4);
    i32x4 lo = *(const i32x4*)(base + o0 + f * 32 * kRowB);
    i32x4 hi = *(const i32x4*)(base + o1 + f * 32 * kRowB);
    return i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
  };
  const bool scaled = g.scale_a != nullptr;
  const float* sa = scaled ? g.scale_a + (int64_t)((m0 + wm * 128) / 128) * g.nkb : nullptr;
  const float* sb = scaled ? g.scale_b + (int64_t)((n0 + wn * 128) / 128) * g.nkb : nullptr;

  issue_loads(0, 0);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  wg_barrier();
  if (nk > 1) issue_loads(1, 1);
  for (int kt = 0; kt < nk; ++kt) {
    const int st = kt & 1;
    const float sc = scaled ? sa[kt] * sb[kt] : 1.0f;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks)
#pragma unroll
      for (int j = 0; j < 4; ++j) fb[ks][j] = read_frag(fb_base, st, ks, j);
    fa[0][0] = read_frag(fa_base, st, 0, 0);
    fa[0][1] = read_frag(fa_base, st, 1, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      if (i + 1 < 4) {
        fa[(i + 1) & 1][0] = read_frag(fa_base, st, 0, i + 1);
        fa[(i + 1) & 1][1] = read_frag(fa_base, st, 1, i + 1);
      } else {
        // every LDS read of this step has been issued: once they land, stage st can be refilled
        asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
        wg_barrier();
        if (kt + 2 < nk) issue_loads(kt + 2, st);
      }
      if (scaled) {
        // the 128-deep block is accumulated on its own, then scaled into the running sum
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          f32x16 part;
#pragma unroll
          for (int e = 0; e < 16; ++e) part[e] = 0.f;
          part = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[0][j], fa[i & 1][0], part, 0, 0, 0, 0, 0, 0);
          part = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[1][j], fa[i & 1][1], part, 0, 0, 0, 0, 0, 0);
#pragma unroll
          for (int e = 0; e < 16; ++e) acc[i][j][e] = __builtin_fmaf(sc, part[e], acc[i][j][e]);
        }
      } else {
#pragma unroll
        for (int j = 0; j < 4; ++j) {
          acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[0][j], fa[i & 1][0], acc[i][j], 0, 0, 0, 0, 0, 0);
          acc[i][j] = __builtin_amdgcn_mfma_scale_f32_32x32x64_f8f6f4(fb[1][j], fa[i & 1][1], acc[i][j], 0, 0, 0, 0, 0, 0);
        }
      }
    }
  }

  // ---- epilogue: one more barrier so that no wave overwrites fragments another wave is still to read
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  wg_barrier();
  store_tile_bf16(acc, lds, w, lane, (uint16_t*)g.C + (m0 + wm * 128) * g.ldc + n0 + wn * 128, g.ldc);
}

hipError_t launch_gemm_fp8_256(const GemmArgs& g, hipStream_t s) {
  unsigned nwg = (unsigned)(g.grid_m * g.grid_n);
  hipLaunchKernelGGL(gemm_fp8_256_kernel, dim3(nwg), dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace axe
