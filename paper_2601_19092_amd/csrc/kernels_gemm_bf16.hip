// bf16 GEMM for gfx950 (MI355X), workgroup tile 256 x 256 x 32, one workgroup of 4 waves per CU
// (one wave per SIMD); each wave owns a 128 x 128 sub-tile = 4 x 4 MFMA 32x32x16 fragments in 256
// accumulator registers.  A is row-major (K contiguous), B column-major (K contiguous).
//
// Tile movements, each an Axe layout (reported by axe_gemm_describe):
//   HBM -> LDS  : global_load_lds_dwordx4, 16 bytes per lane straight into LDS.  One wave
//                 instruction fills 16 consecutive LDS rows of 64 bytes.  The LDS side of such a
//                 load is linear in the lane id, so the XOR swizzle is applied on the global side:
//                 lane (r = lane / 4, p = lane % 4) fetches chunk p ^ key(r) of row r.
//   LDS layout  : ring of 4 stages of 32 KiB; per stage the A tile then the B tile, rows of 64
//                 bytes (32 bf16); 16-byte chunk c of row r sits at chunk position c ^ key(r),
//                 key(r) = (r >> 2) & 3.  The LDS has 64 banks of 4 bytes (256 bytes = 4 rows per bank
//                 cycle): 16 consecutive rows reading the same logical chunk then touch 16 distinct
//                 16-byte bank groups (measured conflict-free; without the swizzle reads take 2.3x).
//   LDS -> VGPR : ds_read_b128; lane l reads row l % 32 of a fragment, K chunk 2 * ks + l / 32:
//                 the MFMA 32x32x16 operand layout (8 consecutive k per lane).
//   MFMA        : operands swapped (B fragment first) so that a lane's accumulator fragment holds
//                 groups of 4 consecutive columns of one C row.
//   VGPR -> HBM : accumulators -> bf16 -> LDS -> 16-byte coalesced stores.
//
// Pipeline.  The L1 (TCP) path moves 64 bytes per clock per CU, so the 64 KiB a 256 x 256 tile
// needs per 64 K-elements take half of the MFMA time of those elements; loads issued in a burst
// stall the issuing wave (and with one wave per SIMD, its MFMAs) until the burst has drained.
// The ring therefore lets loads be issued all the time, one per four MFMAs: while K-tile kt is
// multiplied, tiles kt+1 and kt+2 are resident or landing and the loads of tile kt+3 / kt+4 are
// being issued into the stage freed by the single workgroup barrier of the step.  Every load has
// two to three K steps (2048 - 3072 MFMA cycles) to land before it is waited for.
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_types.h"
#include "gemm_common.h"
#include "kernels.h"

namespace axe {

namespace {
constexpr int kRow = 64;                          // bytes of K per LDS row (32 bf16)
constexpr int kOpnd = kTile * kRow;               // 16 KiB per operand per stage
constexpr int kStage = 2 * kOpnd;                 // 32 KiB
constexpr int kStages = 4;
static_assert(kStages * kStage <= kEpiB, "the epilogue staging area covers the ring");
}  // namespace

__global__ __launch_bounds__(256, 1) void gemm_bf16_256_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds[kEpiB];

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave id, kept scalar
  const int wm = w >> 1, wn = w & 1;
  int tm, tn;
  tile_of_block(blockIdx.x, gridDim.x, g.grid_m, g.grid_n, tm, tn);
  const int64_t m0 = (int64_t)tm * kTile, n0 = (int64_t)tn * kTile;
  const int nk = (int)(g.K / 32);

  // ---- HBM -> LDS.  Per K-tile and operand 16 wave instructions of 16 rows; wave w issues those
  //      of row groups w, w+4, w+8, w+12.
  const int lr = lane >> 2;                                              // row inside the 16-row group
  const int lkey = (lr >> 2) & 3;
  const int lc = (lane & 3) ^ lkey;                                      // global chunk this lane fetches
  const uint8_t* ga = (const uint8_t*)g.A + ((m0 + w * 16 + lr) * g.lda) * 2 + lc * 16;
  const uint8_t* gb = (const uint8_t*)g.B + ((n0 + w * 16 + lr) * g.ldb) * 2 + lc * 16;
  const int64_t a_step = 64 * g.lda * 2, b_step = 64 * g.ldb * 2;        // bytes between row groups w, w+4, ...

  // one load instruction: 16 rows (row group w + 4 i) of K-tile kt of A (op 0) or B (op 1)
  auto load_one = [&](int op, int kt, int i) {
    const uint8_t* p = (op ? gb + i * b_step : ga + i * a_step) + (int64_t)kt * kRow;
    uint8_t* l = lds + (kt & 3) * kStage + op * kOpnd + (w * 16 + i * 64) * kRow;
    __builtin_amdgcn_global_load_lds(p, (__attribute__((address_space(3))) void*)l, 16, 0, 0);
  };
  auto load_a = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) load_one(0, kt, i);
  };
  auto load_b = [&](int kt) {
#pragma unroll
    for (int i = 0; i < 4; ++i) load_one(1, kt, i);
  };

  // ---- LDS -> VGPR: fragment f of this wave's A (B) rows: row = base + f * 32 + lane % 32
  const int fr = lane & 31, fh = lane >> 5;
  const int fkey = (fr >> 2) & 3;
  const uint8_t* fa_base = lds + (wm * 128 + fr) * kRow;
  const uint8_t* fb_base = lds + kOpnd + (wn * 128 + fr) * kRow;

  f32x16 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 16; ++e) acc[i][j][e] = 0.f;

  bf16x8 fa[2][4], fb[2][4];
  auto read_frags = [&](int buf, int kt, int ks) {
    const int off = (kt & 3) * kStage + (((2 * ks + fh) ^ fkey) << 4);
#pragma unroll
    for (int f = 0; f < 4; ++f) {
      fa[buf][f] = *(const bf16x8*)(fa_base + off + f * 32 * kRow);
      fb[buf][f] = *(const bf16x8*)(fb_base + off + f * 32 * kRow);
    }
  };
  auto mfma_all = [&](int buf) {
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j)
        acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[buf][j], fa[buf][i], acc[i][j], 0, 0, 0);
  };
  // Half a K step in exact program order (sched_barrier(0) forbids any reordering across it):
  // 16 MFMAs on fragment buffer CUR; after MFMA q < 8 one fragment read into the other buffer
  // (fragments of K-tile rkt, sub-step rks); after MFMAs 1, 5, 9, 13 one load instruction of
  // operand OP of K-tile lkt.  Fragments are read in the order the next half step consumes them.
  auto half_step = [&](auto cur_c, auto op_c, int rkt, int rks, int lkt) {
    constexpr int CUR = decltype(cur_c)::value, OP = decltype(op_c)::value, NXT = CUR ^ 1;
    const int off = (rkt & 3) * kStage + (((2 * rks + fh) ^ fkey) << 4);
#pragma unroll
    for (int q = 0; q < 16; ++q) {
      const int i = q >> 2, j = q & 3;
      acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fb[CUR][j], fa[CUR][i], acc[i][j], 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (q < 8) {
        if (q & 1) fb[NXT][q >> 1] = *(const bf16x8*)(fb_base + off + (q >> 1) * 32 * kRow);
        else fa[NXT][q >> 1] = *(const bf16x8*)(fa_base + off + (q >> 1) * 32 * kRow);
      }
      if ((q & 3) == 1) load_one(OP, lkt, q >> 2);
      __builtin_amdgcn_sched_barrier(0);
    }
  };
  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;

  // Steady-state step kt.  Entering it, the loads of every K-tile up to kt+2 and the A half of tile
  // kt+3 have been issued, and fragments (tile kt, ks 0) are in buffer 0.
  auto step_full = [&](int kt) {
    half_step(I0{}, I1{}, kt, 1, kt + 3);          // MFMA buf 0; read (kt, ks 1) -> buf 1; load B of kt+3
    // Own reads of tile kt are complete and so are own loads of tile kt+1 (the 16 younger loads,
    // tiles kt+2 and kt+3, may still be in flight).  After the barrier tile kt+1 is readable by
    // every wave and nobody reads the stage of tile kt any more: it takes tile kt+4.
    asm volatile("s_waitcnt vmcnt(16) lgkmcnt(0)" ::: "memory");
    wg_barrier();
    half_step(I1{}, I0{}, kt + 1, 0, kt + 4);      // MFMA buf 1; read (kt+1, ks 0) -> buf 0; load A of kt+4
  };
  // Same step with every load and read guarded, for the first and last steps of short or ending loops.
  auto step_tail = [&](int kt) {
    read_frags(1, kt, 1);
    if (kt + 3 < nk) load_b(kt + 3);
    mfma_all(0);
    asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
    wg_barrier();
    if (kt + 1 < nk) read_frags(0, kt + 1, 0);
    if (kt + 4 < nk) load_a(kt + 4);
    mfma_all(1);
  };

  // prologue: tiles 0..2 and the A half of tile 3
#pragma unroll
  for (int t = 0; t < 3; ++t)
    if (t < nk) {
      load_a(t);
      load_b(t);
    }
  if (3 < nk) load_a(3);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  wg_barrier();
  read_frags(0, 0, 0);
  int kt = 0;
  for (; kt + 4 < nk; ++kt) step_full(kt);
  for (; kt < nk; ++kt) step_tail(kt);

  // ---- epilogue: all LDS reads of the last tile were waited for before the last barrier; one more
  //      barrier so that no wave overwrites fragments another wave is still to read
  asm volatile("s_waitcnt vmcnt(0) lgkmcnt(0)" ::: "memory");
  wg_barrier();
  store_tile_bf16(acc, lds, w, lane, (uint16_t*)g.C + (m0 + wm * 128) * g.ldc + n0 + wn * 128, g.ldc);
}

hipError_t launch_gemm_bf16_256(const GemmArgs& g, hipStream_t s) {
  unsigned nwg = (unsigned)(g.grid_m * g.grid_n);
  hipLaunchKernelGGL(gemm_bf16_256_kernel, dim3(nwg), dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace axe
