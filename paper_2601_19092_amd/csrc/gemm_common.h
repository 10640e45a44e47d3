// Pieces shared by the large-tile GEMM kernels (device code only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "device_types.h"

namespace axe {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(8))) int i32x8;
typedef __attribute__((ext_vector_type(4))) int i32x4;

constexpr int kTile = 256;                        // workgroup tile edge (M and N)
constexpr int kEpiPitch = 272;                    // bytes per accumulator row in the epilogue staging
constexpr int kEpiB = 4 * 128 * kEpiPitch;        // 139264 bytes: 4 waves x 128 rows
constexpr int kEpiPitch8 = 144;                   // same for the 8-wave kernels (128 x 64 per wave)
constexpr int kEpiB8 = 8 * 128 * kEpiPitch8;      // 147456 bytes: 8 waves x 128 rows

// Workgroup barrier without the memory fence of __syncthreads().  That fence waits for every
// outstanding global load (vmcnt(0)), which would drain the load pipeline at each K step; the
// kernels wait explicitly, with s_waitcnt, for exactly the loads and LDS reads a barrier publishes.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

__device__ __forceinline__ uint32_t pack_bf16(float lo, float hi) {
  typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
  bf16x2 v = {(__bf16)lo, (__bf16)hi};            // v_cvt_pk_bf16_f32, round to nearest even
  return __builtin_bit_cast(uint32_t, v);
}

// Workgroup id -> (tile row, tile col).  Consecutive workgroup ids go to different XCDs (8 of
// them, each with its own L2, 32 CUs each), so the id is split into (XCD, position on that XCD).
// When the tile grid is made of 16 x 16 blocks, one round of 256 concurrent workgroups covers one
// block (32 panels, 128 MiB for K = 8192: half the last-level cache), XCD x owning an 8 x 4
// sub-block of it (12 panels through its L2), and the blocks are visited in snake order so that
// consecutive rounds share 16 panels.  Other grids: regroup per XCD, then column-major groups of 8
// tile rows.
__device__ __forceinline__ void tile_of_block(int bid, int nwg, int grid_m, int grid_n, int& tm, int& tn) {
  if (((grid_m | grid_n) & 15) == 0) {
    const int xcd = bid & 7, idx = bid >> 3;
    const int round = idx >> 5, cu = idx & 31;
    const int bpr = grid_n >> 4;
    const int br = round / bpr;
    int bc = round - br * bpr;
    if (br & 1) bc = bpr - 1 - bc;
    tm = br * 16 + (xcd >> 2) * 8 + (cu & 7);
    tn = bc * 16 + (xcd & 3) * 4 + (cu >> 3);
    return;
  }
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

// Epilogue of a 256 x 256 tile held as 4 x 4 MFMA 32x32 accumulator fragments per wave (operands
// swapped: lane l holds, for fragment (i, j) and a = 0..3, the 4 consecutive columns
// j*32 + 8a + 4*(l/32) .. +3 of row i*32 + l%32).  Each wave converts to bf16, stages its 128 x 128
// sub-tile in its own LDS region (row pitch 272 bytes) and writes it out with 16-byte stores, 256
// contiguous bytes per row.  The caller guarantees that no wave still reads the pipeline stages.
__device__ __forceinline__ void store_tile_bf16(const f32x16 (&acc)[4][4], uint8_t* lds, int w, int lane, uint16_t* C,
                                                int64_t ldc) {
  const int fr = lane & 31, fh = lane >> 5;
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
  const int er = lane >> 4, ec = lane & 15;
#pragma unroll 4
  for (int t = 0; t < 32; ++t) {
    int row = t * 4 + er;
    uint4 v = *(const uint4*)(ew + row * kEpiPitch + ec * 16);
    *(uint4*)(C + (int64_t)row * ldc + ec * 8) = v;
  }
}

// Epilogue of a 256 x 256 tile held by 4 waves as 8 x 8 MFMA 16x16 accumulator fragments each
// (operands swapped: lane l holds, for fragment (i, j), the 4 consecutive columns
// j*16 + 4*(l/16) .. +3 of row i*16 + l%16 of the wave's 128 x 128 sub-tile).  Each wave converts to
// bf16, stages its sub-tile in its own LDS region (row pitch 272 bytes: the 8-byte writes of a
// wave instruction fall on 64 distinct banks) and writes it out with 16-byte stores, 256
// contiguous bytes per row.  The caller guarantees that no wave still reads the pipeline stages.
__device__ __forceinline__ void store_tile_bf16_16(const f32x4 (&acc)[8][8], uint8_t* lds, int w, int lane,
                                                   uint16_t* C, int64_t ldc) {
  const int fr = lane & 15, fq = lane >> 4;
  uint8_t* ew = lds + w * 128 * kEpiPitch;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j) {
      uint2 v = {pack_bf16(acc[i][j][0], acc[i][j][1]), pack_bf16(acc[i][j][2], acc[i][j][3])};
      *(uint2*)(ew + (i * 16 + fr) * kEpiPitch + (j * 16 + 4 * fq) * 2) = v;
    }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  const int er = lane >> 4, ec = lane & 15;
#pragma unroll 4
  for (int t = 0; t < 32; ++t) {
    int row = t * 4 + er;
    uint4 v = *(const uint4*)(ew + row * kEpiPitch + ec * 16);
    *(uint4*)(C + (int64_t)row * ldc + ec * 8) = v;
  }
}

// Epilogue of a 256 x 256 tile held by 8 waves as 8 x 4 MFMA 16x16 accumulator fragments each (lane l
// holds, for fragment (i, j), the 4 consecutive columns j*16 + 4*(l/16) .. +3 of row i*16 + l%16 of the
// wave's 128 x 64 sub-tile).  Staging and stores as in store_tile_bf16_w8.
__device__ __forceinline__ void store_tile_bf16_w8_16(const f32x4 (&acc)[8][4], uint8_t* lds, int w, int lane,
                                                      uint16_t* C, int64_t ldc) {
  const int fr = lane & 15, fq = lane >> 4;
  uint8_t* ew = lds + w * 128 * kEpiPitch8;
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      uint2 v = {pack_bf16(acc[i][j][0], acc[i][j][1]), pack_bf16(acc[i][j][2], acc[i][j][3])};
      *(uint2*)(ew + (i * 16 + fr) * kEpiPitch8 + (j * 16 + 4 * fq) * 2) = v;
    }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  const int er = lane >> 3, ec = lane & 7;
#pragma unroll 4
  for (int t = 0; t < 16; ++t) {
    int row = t * 8 + er;
    uint4 v = *(const uint4*)(ew + row * kEpiPitch8 + ec * 16);
    *(uint4*)(C + (int64_t)row * ldc + ec * 8) = v;
  }
}

// Epilogue of a 256 x 256 tile held by 8 waves as 4 x 2 MFMA 32x32 accumulator fragments each
// (operands swapped: lane l holds, for fragment (i, j) and a = 0..3, the 4 consecutive columns
// j*32 + 8a + 4*(l/32) .. +3 of row i*32 + l%32 of the wave's 128 x 64 sub-tile).  Each wave converts
// to bf16, stages its sub-tile in its own LDS region (row pitch 144 bytes) and writes it out with
// 16-byte stores, 128 contiguous bytes per row.  The caller guarantees that no wave still reads
// the pipeline stages.
__device__ __forceinline__ void store_tile_bf16_w8(const f32x16 (&acc)[4][2], uint8_t* lds, int w, int lane,
                                                   uint16_t* C, int64_t ldc) {
  const int fr = lane & 31, fh = lane >> 5;
  uint8_t* ew = lds + w * 128 * kEpiPitch8;
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int a = 0; a < 4; ++a) {
        uint2 v = {pack_bf16(acc[i][j][4 * a + 0], acc[i][j][4 * a + 1]),
                   pack_bf16(acc[i][j][4 * a + 2], acc[i][j][4 * a + 3])};
        *(uint2*)(ew + (i * 32 + fr) * kEpiPitch8 + (j * 32 + 8 * a + 4 * fh) * 2) = v;
      }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_wave_barrier();
  const int er = lane >> 3, ec = lane & 7;
#pragma unroll 4
  for (int t = 0; t < 16; ++t) {
    int row = t * 8 + er;
    uint4 v = *(const uint4*)(ew + row * kEpiPitch8 + ec * 16);
    *(uint4*)(C + (int64_t)row * ldc + ec * 8) = v;
  }
}

}  // namespace axe
