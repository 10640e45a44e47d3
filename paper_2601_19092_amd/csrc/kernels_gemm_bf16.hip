// bf16 GEMM for gfx950 (MI355X), workgroup tile 256 x 256 x 64, one workgroup of 8 waves per CU
// (two waves per SIMD); each wave owns a 128 x 64 sub-tile = 4 x 2 MFMA 32x32x16 fragments in 128
// accumulator registers.  A is row-major (K contiguous), B column-major (K contiguous).
//
// What bounds this kernel besides the matrix pipe is the L2 -> CU path: a 256 x 256 tile pulls
// 64 KiB per 64 K-elements, about three quarters of what the L2s can deliver to all CUs at once, and
// only when every request is a whole 128-byte line (half-line requests of a 32-wide K-tile reach
// 60 % of that rate).  Hence 64-wide K-tiles: every load instruction fetches 8 rows x 128 bytes.
// A memory system that busy answers late (a wave's eight loads of one K-tile complete 1500 - 2300
// cycles after issue), so every load is given at least two K-steps (4096 cycles) before it is
// needed.  160 KiB of LDS hold five 32 KiB operand blocks, not the six that two-step prefetch of
// both operands through LDS would take, so the operands travel differently:
//   B: global_load ... lds (direct to LDS) into a ring of three blocks, issued two to three steps ahead;
//   A: global load into 8 x 4 staging registers per lane, issued two steps ahead, ds_write_b128 into
//      a double-buffered block one step ahead of use.
//
// Tile movements, each an Axe layout (reported by axe_gemm_describe):
//   HBM -> LDS/VGPR : one wave instruction covers 8 rows x 128 bytes (lane = 8 * row + chunk).
//   LDS layout  : rows of 128 bytes (64 bf16); 16-byte chunk c of row r sits at chunk position
//                 c ^ key(r), key(r) = (r >> 1) & 7.  With 64 banks of 4 bytes, 16 consecutive rows
//                 reading the same logical chunk touch 16 distinct 16-byte bank groups.  A direct-to-LDS
//                 load writes LDS linearly in the lane id, so for B the XOR is applied on the global
//                 side (lane (r, p) fetches chunk p ^ key(r)); for A on the ds_write address.
//   LDS -> VGPR : ds_read_b128; lane l reads row l % 32 of a fragment, K chunk 2 * ks + l / 32:
//                 the MFMA 32x32x16 operand layout (8 consecutive k per lane).
//   MFMA        : operands swapped (B fragment first) so that a lane's accumulator fragment holds
//                 groups of 4 consecutive columns of one C row.
//   VGPR -> HBM : accumulators -> bf16 -> LDS -> 16-byte coalesced stores.
//
// Schedule.  A K-step is four sub-steps of 8 MFMAs per wave; sub-step (kt, ks) also reads the six
// fragments of the next sub-step, writes one staged A piece to LDS, reloads that staging slot and
// issues one B load.  One workgroup barrier per K-step, after sub-step 2: by then every LDS read of
// tile kt has completed, and the barrier publishes tile kt+1.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_types.h"
#include "gemm_common.h"
#include "kernels.h"

namespace axe {

namespace {
constexpr int kRow = 128;                         // bytes of K per LDS row (64 bf16)
constexpr int kBlk = kTile * kRow;                // 32 KiB: one operand, one K-tile
constexpr int kBoff = 2 * kBlk;                   // A: blocks 0, 1 (double buffer); B: blocks 2, 3, 4 (ring)
constexpr int kLds = 5 * kBlk;                    // 160 KiB
constexpr int kRot = 8;                           // K-rotation window, in K-tiles
static_assert(kEpiB8 <= kLds, "the epilogue staging area fits");
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(3))) uint8_t* lds_u8;
__device__ __forceinline__ bf16x8 lds_read(lds_u8 p) { return *(__attribute__((address_space(3))) const bf16x8*)p; }
}  // namespace

__global__ __launch_bounds__(512, 1) void gemm_bf16_256_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds_mem[kLds];
  uint8_t* const lds = lds_mem;                                    // generic view, for the epilogue
  const lds_u8 lds3 = (lds_u8)lds_mem;                             // 32-bit LDS addresses for the main loop

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave id 0..7, kept scalar
  const int wm = w >> 2, wn = w & 3;                               // wave grid 2 x 4
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, g.grid_m, g.grid_n, tm, tn);
  const int64_t m0 = (int64_t)tm * kTile, n0 = (int64_t)tn * kTile;
  const int nk = (int)(g.K / 64);
  // K rotation.  The workgroups that share an A or B panel run side by side on one XCD and would ask
  // for the same 128-byte line of every row at the same time, then for the next line one K-step
  // later: HBM sees isolated 128-byte reads scattered over rows 16 KiB apart.  Instead each
  // workgroup walks every aligned window of kRot K-tiles in its own rotated order (the sum over k
  // does not care), so that neighbours fetch the kRot adjacent lines of a row at once -- one 1 KiB
  // burst per row -- and find the other lines in L2 during the rest of the window (measured on the
  // bare load stream: 16 -> 21.5 TB/s).
  const int rot = (tm + tn) & (kRot - 1);
  const int nk_rot = nk & ~(kRot - 1);                            // tiles beyond the last full window keep their order
  auto kcol = [&](int T) -> int {                                  // K-tile visited at position T -> byte column
    const int t = T < nk_rot ? ((T & ~(kRot - 1)) | ((T + rot) & (kRot - 1))) : T;
    return t * kRow;
  };

  // ---- global side.  Per K-tile and operand 32 wave instructions of 8 rows; wave w issues pieces
  //      i = 0..3 = row groups w, w + 8, w + 16, w + 24.  Buffer addressing: the descriptor covers the
  //      256 rows of the tile, the per-lane offset is fixed, K-tile and piece go into the scalar offset.
  const int lr = lane >> 3, lp = lane & 7;
  const int lkey = (4 * w + (lr >> 1)) & 7;                        // key(row) of row (w + 8 i) * 8 + lr
  const int a_pitch = (int)(g.lda * 2), b_pitch = (int)(g.ldb * 2);
  const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc(
      (void*)((const uint8_t*)g.A + m0 * g.lda * 2), 0, 255 * a_pitch + (int)g.K * 2, 0x00020000);
  const __amdgpu_buffer_rsrc_t rb = __builtin_amdgcn_make_buffer_rsrc(
      (void*)((const uint8_t*)g.B + n0 * g.ldb * 2), 0, 255 * b_pitch + (int)g.K * 2, 0x00020000);
  const int a_voff = (w * 8 + lr) * a_pitch + lp * 16;
  const int b_voff = (w * 8 + lr) * b_pitch + ((lp ^ lkey) << 4);
  const int a_piece = 64 * a_pitch, b_piece = 64 * b_pitch;        // bytes between pieces
  const lds_u8 a_wr = lds3 + (w * 8 + lr) * kRow + ((lp ^ lkey) << 4);    // + stage * kBlk + i * 8192

  u32x4 stg[8];                                                    // A staging: slot (T & 1) * 4 + i
  auto a_load = [&](int T, int i) -> u32x4 {
    return __builtin_amdgcn_raw_buffer_load_b128(ra, a_voff, i * a_piece + kcol(T), 0);
  };
  auto a_write = [&](int stage, int i, u32x4 v) {
    *(__attribute__((address_space(3))) u32x4*)(a_wr + stage * kBlk + i * 8192) = v;
  };
  // B ring: byte offsets of the blocks that hold tiles kt, kt+1, kt+2 (tile kt+3 reuses the first)
  int bo0 = kBoff, bo1 = kBoff + kBlk, bo2 = kBoff + 2 * kBlk;
  auto b_load = [&](int T, int i, int slot_off) {
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rb, (lds_ptr)(lds3 + slot_off + (w + 8 * i) * 1024), 16, b_voff,
                                             i * b_piece + kcol(T), 0, 0);
  };

  // ---- LDS -> VGPR: fragment f of this wave's A (B) rows: row = base + f * 32 + lane % 32
  const int fr = lane & 31, fh = lane >> 5;
  const int fkey = (fr >> 1) & 7;
  lds_u8 fax[4], fbx[4];                                           // row base + swizzled chunk, per sub-step
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    fax[ks] = lds3 + (wm * 128 + fr) * kRow + (((2 * ks + fh) ^ fkey) << 4);
    fbx[ks] = lds3 + (wn * 64 + fr) * kRow + (((2 * ks + fh) ^ fkey) << 4);
  }

  f32x16 acc[4][2];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  bf16x8 fa[2][4], fb[2][2];

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;
  using I2 = std::integral_constant<int, 2>;
  using I3 = std::integral_constant<int, 3>;

  // Sub-step KS of K-step kt (PAR = kt & 1), in exact program order (sched_barrier(0) forbids any
  // reordering across it).  Nothing is guarded against the end of K: loads of tiles past the end stay
  // inside the buffer descriptors (which return zero beyond the tile's last row), land in staging
  // slots and LDS blocks that are free by then, and are never multiplied.
  auto substep = [&](auto par_c, auto ks_c, int kt) {
    constexpr int PAR = decltype(par_c)::value, KS = decltype(ks_c)::value;
    constexpr int CUR = KS & 1, NXT = CUR ^ 1;
    // fragments read now: sub-step KS + 1 of this tile, or sub-step 0 of the next one
    constexpr int RKS = KS < 3 ? KS + 1 : 0;
    constexpr int RST = KS < 3 ? PAR : PAR ^ 1;                    // A stage of that tile
    const lds_u8 pa = fax[RKS] + RST * kBlk;
    const lds_u8 pb = fbx[RKS] + (KS < 3 ? bo0 : bo1);
    // staged A piece written now and the load that refills its slot; B piece loaded now
    constexpr int PI = KS == 3 ? 0 : KS + 1;                       // piece index
    const int wT = KS == 3 ? kt + 2 : kt + 1;                      // tile whose piece goes to LDS
    constexpr int WST = KS == 3 ? PAR : PAR ^ 1;                   // its stage = wT & 1
    constexpr int SLOT = WST * 4 + PI;
    const int aT = wT + 2;                                         // tile loaded into the freed slot
    const int bT = KS == 3 ? kt + 3 : kt + 2;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      const int i = q >> 1, j = q & 1;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[CUR][j], fa[CUR][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (q == 0) fa[NXT][0] = lds_read(pa);
      if (q == 1) fb[NXT][0] = lds_read(pb);
      if (q == 2) fb[NXT][1] = lds_read(pb + 32 * kRow);
      if (q == 3) fa[NXT][1] = lds_read(pa + 32 * kRow);
      if (q == 4) fa[NXT][2] = lds_read(pa + 64 * kRow);
      if (q == 5) fa[NXT][3] = lds_read(pa + 96 * kRow);
      if (q == 3) b_load(bT, PI, KS == 3 ? bo0 : bo2);
      if (q == 6) {
        // the load that filled SLOT was issued 8 sub-steps ago; 15 loads have been issued since
        asm volatile("s_waitcnt vmcnt(15)" ::: "memory");
        a_write(WST, PI, stg[SLOT]);
        stg[SLOT] = a_load(aT, PI);
      }
      __builtin_amdgcn_sched_barrier(0);
    }
    if (KS == 2) {
      // Own reads of tile kt and own writes of tile kt+1 are complete, and so are own B loads of tile
      // kt+1 (the 9 younger loads may still be in flight).  After the barrier tile kt+1 is readable
      // by every wave and nobody reads tile kt any more.
      asm volatile("s_waitcnt vmcnt(9) lgkmcnt(0)" ::: "memory");
      wg_barrier();
    }
  };
  auto step = [&](auto par_c, int kt) {
    substep(par_c, I0{}, kt);
    substep(par_c, I1{}, kt);
    substep(par_c, I2{}, kt);
    substep(par_c, I3{}, kt);
    const int t = bo0;
    bo0 = bo1, bo1 = bo2, bo2 = t;
  };

  // ---- prologue: the loads the sub-steps before (0, 0) would have issued, oldest first in the order
  //      the loop consumes them, so that the counted waits of the first steps hold as well.  Tile 0 and
  //      piece 0 of tile 1 go to LDS from temporaries; the rest stays in the staging slots.
  {
    u32x4 t0[4], t1;
#pragma unroll
    for (int i = 0; i < 4; ++i) t0[i] = a_load(0, i);
    t1 = a_load(1, 0);
#pragma unroll
    for (int i = 1; i < 4; ++i) stg[4 + i] = a_load(1, i);
#pragma unroll
    for (int i = 0; i < 4; ++i) stg[i] = a_load(2, i);
    stg[4] = a_load(3, 0);
#pragma unroll
    for (int i = 0; i < 4; ++i) b_load(0, i, bo0);
#pragma unroll
    for (int i = 0; i < 4; ++i) b_load(1, i, bo1);
    b_load(2, 0, bo2);
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
#pragma unroll
    for (int i = 0; i < 4; ++i) a_write(0, i, t0[i]);
    a_write(1, 0, t1);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    wg_barrier();
  }
#pragma unroll
  for (int f = 0; f < 4; ++f) fa[0][f] = lds_read(fax[0] + f * 32 * kRow);
#pragma unroll
  for (int f = 0; f < 2; ++f) fb[0][f] = lds_read(fbx[0] + bo0 + f * 32 * kRow);

  int kt = 0;
  for (; kt + 1 < nk; kt += 2) {
    step(I0{}, kt);
    step(I1{}, kt + 1);
  }
  if (kt < nk) step(I0{}, kt);

  // ---- epilogue: all LDS reads of the last tile were waited for before the last barrier; one more
  //      barrier so that no wave overwrites fragments another wave is still to read
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  wg_barrier();
  store_tile_bf16_w8(acc, lds, w, lane, (uint16_t*)g.C + (m0 + wm * 128) * g.ldc + n0 + wn * 64, g.ldc);
}

hipError_t launch_gemm_bf16_256(const GemmArgs& g, hipStream_t s) {
  unsigned nwg = (unsigned)(g.grid_m * g.grid_n);
  hipLaunchKernelGGL(gemm_bf16_256_kernel, dim3(nwg), dim3(512), 0, s, g);
  return hipGetLastError();
}

}  // namespace axe
