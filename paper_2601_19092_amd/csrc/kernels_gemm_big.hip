// Large-tile GEMM for gfx950 (MI355X): workgroup tile 256 x 256, one workgroup of 4 waves per CU
// (one wave per SIMD), each wave a 128 x 128 sub-tile = 4 x 4 MFMA 32x32 fragments held in 256
// accumulator registers.  A is row-major (K contiguous), B column-major (K contiguous).
//
// Tile movements, each an Axe layout (reported by axe_gemm_describe):
//   HBM -> LDS  : global_load_lds_dwordx4, 16 bytes per lane straight into LDS.  One wave
//                 instruction fills 8 consecutive LDS rows of 128 bytes; because the LDS side of
//                 such a load is linear in the lane id, the XOR swizzle is applied on the global
//                 side: lane (r = lane / 8, p = lane % 8) fetches chunk p ^ key(r) of row r.
//   LDS layout  : per stage, A tile then B tile, rows of 128 bytes (64 bf16 / 128 fp8), 16-byte
//                 chunk c of row r stored at chunk position c ^ key(r), key(r) = (r & 7) ^ ((r >> 3) & 1):
//                 any 8 or 16 consecutive rows reading the same logical chunk hit distinct banks
//                 for both a 32-bank and a 64-bank LDS.
//   LDS -> VGPR : ds_read_b128, lane l reads row l % 32 of a fragment and K chunk 2 * ks + l / 32
//                 -- exactly the MFMA 32x32x16 operand layout (8 consecutive k per lane).
//   MFMA        : operands swapped (B fragment first) so the accumulator fragment of a lane holds
//                 groups of 4 consecutive columns of one C row.
//   VGPR -> HBM : accumulators -> bf16 -> LDS (row pitch 272 bytes) -> 16-byte coalesced stores,
//                 256 contiguous bytes per row per wave.
//
// Pipeline: two LDS stages of 64 KiB.  The loads of K-tile kt+1 are issued one whole K step
// (64 MFMAs per wave) before they are needed; the only workgroup barrier of a step sits before
// the last quarter of its MFMAs, which hide the barrier skew and the first fragment reads of the
// next tile.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_types.h"
#include "kernels.h"

namespace axe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kTile = 256;            // workgroup tile edge (M and N)
constexpr int kRowB = 128;            // bytes of K per LDS row
constexpr int kOperandB = kTile * kRowB;          // 32 KiB per operand per stage
constexpr int kStageB = 2 * kOperandB;            // 64 KiB
constexpr int kEpiPitch = 272;                    // bytes per accumulator row in the epilogue staging
constexpr int kLdsB = 4 * 128 * kEpiPitch;        // 139264 >= 2 * kStageB

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 v = {(__bf16)lo, (__bf16)hi};            // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}

// Workgroup id -> (tile row, tile col).  Consecutive workgroup ids go to different XCDs (8 of
// them, each with its own L2), so ids are first regrouped per XCD, then walked in column-major
// groups of 8 tile rows so that the tiles resident on one XCD share A and B panels.
__device__ __forceinline__ void tile_of_block(int bid, int nwg, int grid_m, int grid_n, int& tm, int& tn) {
  int lin = bid;
  if ((nwg & 7) == 0) lin = (bid & 7) * (nwg >> 3) + (bid >> 3);
  const int GM = 8;
  int per_group = GM * grid_n;
  int group = lin / per_group;
  int first_m = group * GM;
  int gsz = grid_m - first_m < GM ? grid_m - first_m : GM;
  int in_group = lin - group * per_group;
  tm = first_m + in_group % gsz;
  tn = in_group / gsz;
}

template <bool FP8>
__global__ __launch_bounds__(256, 1) void gemm_256_kernel(GemmArgs g) {
  constexpr int EB = FP8 ? 1 : 2;
  constexpr int BK = kRowB / EB;                  // 64 bf16 or 128 fp8 per K step
  __shared__ __attribute__((aligned(1024))) uint8_t lds[kLdsB];

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
  const int lc = (lane & 7) ^ lr ^ (w & 1);                   // global chunk this lane fetches
  // address = wave-uniform base (scalar registers) + 32-bit per-lane offset that never changes
  const uint8_t* sa_base = (const uint8_t*)g.A + (m0 + w * 8) * g.lda * EB;
  const uint8_t* sb_base = (const uint8_t*)g.B + (n0 + w * 8) * g.ldb * EB;
  const uint32_t va_off = (uint32_t)(lr * g.lda * EB + lc * 16);
  const uint32_t vb_off = (uint32_t)(lr * g.ldb * EB + lc * 16);
  const int64_t a_step = 32 * g.lda * EB, b_step = 32 * g.ldb * EB;   // bytes between instructions

  auto issue_loads = [&](int kt, int stage) {
    const uint8_t* pa = sa_base + (int64_t)kt * kRowB;
    const uint8_t* pb = sb_base + (int64_t)kt * kRowB;
    uint8_t* la = lds + stage * kStageB + w * 8 * kRowB;
    uint8_t* lb = la + kOperandB;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      __builtin_amdgcn_global_load_lds(pa + i * a_step + va_off, (__attribute__((address_space(3))) void*)(la + i * 32 * kRowB), 16, 0, 0);
      __builtin_amdgcn_global_load_lds(pb + i * b_step + vb_off, (__attribute__((address_space(3))) void*)(lb + i * 32 * kRowB), 16, 0, 0);
    }
  };

  // ---- LDS -> VGPR: fragment f of this wave's A (B) rows: row = base + f * 32 + lane % 32
  const int fr = lane & 31, fh = lane >> 5;
  const int fkey = (fr & 7) ^ ((fr >> 3) & 1);
  const uint8_t* fa_base = lds + (wm * 128 + fr) * kRowB;
  const uint8_t* fb_base = lds + kOperandB + (wn * 128 + fr) * kRowB;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  if constexpr (!FP8) {
    bf16x8 fa[2][4], fb[2][4];
    auto read_frags = [&](int buf, int stage, int ks) {
      const int off = stage * kStageB + (((2 * ks + fh) ^ fkey) << 4);
#pragma unroll
      for (int f = 0; f < 4; ++f) {
        fa[buf][f] = *(const bf16x8*)(fa_base + off + f * 32 * kRowB);
        fb[buf][f] = *(const bf16x8*)(fb_base + off + f * 32 * kRowB);
      }
    };
    auto mfma_all = [&](int buf) {
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
    };

    // One K step.  Instruction order is pinned with sched_group_barrier (0x008 = MFMA,
    // 0x100 = LDS read, 0x020 = VMEM read): the 8 fragment reads of the next sub-step are
    // interleaved one-to-one with the first MFMAs of the current one, and in the last sub-step
    // the 16 loads of K-tile kt+2 are interleaved with its 16 MFMAs.
    auto step = [&](int kt, auto loads_c, auto next_c) {
      constexpr bool LOADS = decltype(loads_c)::value, NEXT = decltype(next_c)::value;
      const int st = kt & 1;
#pragma unroll
      for (int ks = 0; ks < 3; ++ks) {
        read_frags((ks + 1) & 1, st, ks + 1);
        mfma_all(ks & 1);
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 8, 0);
      }
      // fragments of sub-step 3 are in registers: this wave is done with stage st
      asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
      __syncthreads();
      if constexpr (LOADS) issue_loads(kt + 2, st);
      if constexpr (NEXT) read_frags(0, st ^ 1, 0);
      mfma_all(1);
      if constexpr (NEXT) {
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
          if constexpr (LOADS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
#pragma unroll
        for (int q = 0; q < 8; ++q) {
          __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
          if constexpr (LOADS) __builtin_amdgcn_sched_group_barrier(0x020, 1, 0);
        }
      }
    };
    using T = std::true_type;
    using F = std::false_type;

    issue_loads(0, 0);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
    if (nk > 1) issue_loads(1, 1);
    read_frags(0, 0, 0);
    int kt = 0;
    for (; kt + 2 < nk; ++kt) step(kt, T{}, T{});
    if (kt + 1 < nk) step(kt++, F{}, T{});
    step(kt, F{}, F{});
  } else {
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
    __syncthreads();
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
          __syncthreads();
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
  }

  // ---- epilogue: every wave has passed the last barrier after its final LDS reads were issued and
  //      waited for, but other waves may still be reading fragments: one more barrier, then each
  //      wave stages its own 128 x 128 sub-tile
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __syncthreads();
  uint8_t* ew = lds + w * 128 * kEpiPitch;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 v = {pack_bf16(acc[i][j][4 * a + 0], acc[i][j][4 * a + 1]),
                   pack_bf16(acc[i][j][4 * a + 2], acc[i][j][4 * a + 3])};
        *(uint2*)(ew + (i * 32 + fr) * kEpiPitch + (j * 32 + 8 * a + 4 * fh) * 2) = v;
      }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  uint16_t* C = (uint16_t*)g.C + (m0 + wm * 128) * g.ldc + n0 + wn * 128;
  const int er = lane >> 4, ec = lane & 15;
#pragma unroll 4
  for (int t = 0; t < 32; ++t) {
    int row = t * 4 + er;
    uint4 v = *(const uint4*)(ew + row * kEpiPitch + ec * 16);
    *(uint4*)(C + (int64_t)row * g.ldc + ec * 8) = v;
  }
}

static hipError_t launch_256(const GemmArgs& g, bool fp8, hipStream_t s) {
  unsigned nwg = (unsigned)(g.grid_m * g.grid_n);
  if (fp8)
    hipLaunchKernelGGL(gemm_256_kernel<true>, dim3(nwg), dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_256_kernel<false>, dim3(nwg), dim3(256), 0, s, g);
  return hipGetLastError();
}

hipError_t launch_gemm_bf16_256(const GemmArgs& g, hipStream_t s) { return launch_256(g, false, s); }
hipError_t launch_gemm_fp8_256(const GemmArgs& g, hipStream_t s) { return launch_256(g, true, s); }

}  // namespace axe
