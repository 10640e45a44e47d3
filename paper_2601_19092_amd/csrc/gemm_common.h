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

// Workgroup barrier without the memory fence of __syncthreads().  That fence waits for every
// outstanding global load (vmcnt(0)), which would drain the load pipeline at each K step; the
// kernels wait explicitly, with s_waitcnt, for exactly the loads and LDS reads a barrier publishes.
__device__ __forceinline__ void wg_barrier() {
  asm volatile("" ::: "memory");
  __builtin_amdgcn_s_barrier();
  asm volatile("" ::: "memory");
}

// Checking build (-DAXE_PARANOID, a library of its own that only a GPU test loads): the large-tile kernels rely on
// counted waits, on loads and stores issued as asm statements that the compiler's own bookkeeping does not see, and on
// one barrier per K-step.  In the checking build every load into LDS and every store is followed by a full wait, and
// every row of MFMAs by a full wait and a workgroup barrier: nothing is in flight when anything is read.  The
// arithmetic and its order are untouched, so both builds must produce the same bits; if they do not, the fast build
// reads something before it has arrived.
#ifdef AXE_PARANOID
#define AXE_PARANOID_WAIT() asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory")
#define AXE_PARANOID_SYNC()                                         \
  do {                                                              \
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");     \
    __builtin_amdgcn_s_barrier();                                   \
    asm volatile("" ::: "memory");                                  \
  } while (0)
#else
#define AXE_PARANOID_WAIT() \
  do {                      \
  } while (0)
#define AXE_PARANOID_SYNC() \
  do {                      \
  } while (0)
#endif

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

// A buffer instruction written as an asm statement is opaque to the compiler's hazard recogniser.
// One hazard of this chip can then go unpadded: a vector-memory instruction that reads an SGPR
// (descriptor word or scalar offset) needs 5 wait states after a vector-ALU instruction wrote that
// SGPR -- and the register allocator does write SGPRs that way (v_readfirstlane / v_readlane from a
// uniform value it parked in a VGPR).  Unpadded, the instruction now and then used the stale offset:
// a fragment stored over its neighbour.  Every such asm statement therefore starts with s_nop 4; the
// MFMAs issued before keep the matrix pipe busy meanwhile.
//
// The other hazard of such a store is on its data: the instruction reads its data registers a little after it has
// issued, and the compiler -- which does not know that the asm statement is a store -- lets the very next vector-ALU
// instruction overwrite them (the gated epilogue computed the next fragment into the registers of the 16-byte store
// just issued).  In a quiet machine the store won the race; with a copy kernel of another stream saturating the
// memory pipeline one group of four lanes of one store in a launch of a few million did not: 32 wrong elements in a
// quarter of the launches.  Every asm-issued store is therefore followed by wait states of its own.
#ifndef AXE_AFTER_STORE
#define AXE_AFTER_STORE "\n\ts_nop 3"
#endif
//
// Descriptor words for a buffer store issued as an asm statement: base address, byte range, raw
// 32-bit data format.  The words are wave-uniform by construction; readfirstlane tells the compiler so
// (they must sit in SGPRs).
__device__ __forceinline__ i32x4 raw_rsrc(const void* p, uint32_t bytes) {
  const uint64_t a = (uint64_t)p;
  return i32x4{__builtin_amdgcn_readfirstlane((int)(uint32_t)a), __builtin_amdgcn_readfirstlane((int)((a >> 32) & 0xffffu)),
               __builtin_amdgcn_readfirstlane((int)bytes), 0x00020000};
}

}  // namespace axe
