// bf16 (and fp16) GEMM for gfx950 (MI355X), workgroup tile 256 x 256 x 64 (or 256 x 224 x 64), one workgroup of 4 waves per CU (one
// wave per SIMD); each wave owns a 128 x 128 sub-tile = 8 x 8 MFMA 16x16x32 fragments in 256
// accumulator registers.  A is row-major (K contiguous), B column-major (K contiguous).
// One body, instantiated as: the dense kernel (256 or 224 columns per tile), the dense kernel for operands
// stored in blocks, the fp16 twins, and the grouped kernels of an MoE layer (tiles of 256 or 128 rows, plain or
// gated epilogue) -- see the template parameters of gemm_bf16_256_body.
//
// Two measured facts shape the kernel:
//  * On real (random) data the chip runs into its power limit long before the matrix pipe is full,
//    and what a flop costs depends on the instruction stream: a register-only loop of 16x16x32 MFMAs
//    that walks the accumulators in register order, issued by a single wave per SIMD, sustains
//    1.9 - 2.0 PFLOP/s where 32x32x16 MFMAs, or two interleaved waves per SIMD, sustain 1.7 - 1.8.
//    Hence one wave per SIMD, 16x16x32; and the order of the walk matters too: fragment rows in pairs,
//    (r, j), (r + 1, j) with j innermost, every other pair backwards, draw less than row by row (2.08 against
//    2.0 - 2.05 PFLOP/s register-only).
//  * The L2 -> CU path is the second bound: a 256 x 256 tile pulls 64 KiB per 64 K-elements, about
//    three quarters of what the L2s deliver to all CUs at once, and only when every request is a
//    whole 128-byte line.  Hence 64-wide K-tiles: every load instruction fetches 8 rows x 128 bytes.
//  (An earlier version let every workgroup walk each aligned window of 8 K-tiles in an order of its own, so that
//   the workgroups sharing a panel fetch 8 adjacent lines of a row together; that helped a bare load stream, but the
//   finished kernel runs 2 % faster with all of them on the same K-tile: 8192^3 1549 -> 1580 TFLOP/s.)
//
// Tile movements, each an Axe layout (reported by axe_gemm_describe):
//   HBM -> LDS  : one wave instruction covers 8 rows x 128 bytes (lane = 8 * row + chunk), direct to LDS.
//   LDS layout  : five 32 KiB blocks (one operand, one K-tile each): A double-buffered in blocks 0, 1,
//                 B in a ring of blocks 2, 3, 4.  Rows of 128 bytes (64 bf16); 16-byte chunk c of row r
//                 sits at chunk position c ^ key(r), key(r) = (r >> 1) & 7.  With 64 banks of 4 bytes, 16
//                 consecutive rows reading the same logical chunk touch 16 distinct 16-byte bank groups.
//                 A direct-to-LDS load writes LDS linearly in the lane id, so the XOR is applied on the
//                 global side (lane (r, p) fetches chunk p ^ key(r)).
//   LDS -> VGPR : ds_read_b128; lane l reads row l % 16 of a fragment, K chunk 4 * s + l / 16: the MFMA
//                 16x16x32 operand layout (8 consecutive k per lane).
//   MFMA        : operands swapped (B fragment first) so that a lane's accumulator fragment holds 4
//                 consecutive columns of one C row.
//   VGPR -> HBM : accumulators -> bf16, stored directly: two neighbouring fragments exchange halves between
//                 lane groups (v_permlane16_swap) so that a lane stores 16 contiguous bytes, an instruction
//                 64 contiguous bytes of 16 rows (the four pairs of a fragment row complete 256 bytes per
//                 row; L2 merges them).  The 224-wide tile stores fragment by fragment, 8 bytes per lane.
//
// Schedule.  A K-step is two sub-steps of 64 MFMAs; a sub-step also reads the 16 fragments of the
// next sub-step.  One workgroup barrier per K-step, early in sub-step 1: every LDS read of step kt has
// completed by then, and the barrier publishes step kt+1.  With one wave per SIMD nothing hides a late
// load, and a memory system that busy answers late (a wave's loads of one K-tile complete 1500 - 2300
// cycles after issue, a K-step takes about 2900).  160 KiB of LDS hold five 32 KiB blocks:
//   B: buffer_load ... lds (direct to LDS) into a ring of three blocks, 1 to 1.5 K-steps ahead;
//   A: buffer_load ... lds into the block of its step's parity, right after the barrier that frees it:
//      one K-step ahead.  (Staging A through registers and ds_write_b128 would give it two K-steps; measured,
//      the writes cost more than the distance is worth: 8192^3 runs 7 % faster without them.)
//
// Tile width.  The same kernel body exists with 224 instead of 256 columns of C per tile (7 instead
// of 8 fragments per wave along N): M = 4096, N = 3584 makes 16 x 16 such tiles, one per CU, where
// 256-wide tiles would leave 32 CUs idle (measured: 5 - 8 % faster; less than the 14 % of the tile
// count because the chip is power-limited and 224 busy CUs clock higher than 256).
//
// Tiles.  When there are more tiles than CUs (and the number of K-steps is even and at least 4) one
// workgroup per CU walks its tiles back to back: the load side simply runs on into the next tile's
// first K-steps, so only the first tile of a workgroup has a prologue, and a tile's stores overlap
// the arrival of the next tile's operands.
#include <hip/hip_runtime.h>

#include <stdlib.h>

#include <algorithm>
#include <mutex>
#include <type_traits>

#include "device_types.h"
#include "gemm_common.h"
#include "grouped_tiles.h"
#include "kernels.h"
#include "tile_maps.h"

namespace axe {

namespace {
constexpr int kRow = maps::kLargeRowBytes;         // bytes of K per LDS row (64 bf16)
constexpr int kBlk = kTile * kRow;                // 32 KiB: one operand, one K-tile
constexpr int kBoff = 2 * kBlk;                   // A: blocks 0, 1 (double buffer); B: blocks 2, 3, 4 (ring)
constexpr int kLds = 5 * kBlk;                    // 160 KiB
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(3))) uint8_t* lds_u8;
__device__ __forceinline__ bf16x8 lds_read(lds_u8 p) { return *(__attribute__((address_space(3))) const bf16x8*)p; }
// acc += a(16 x 32) * b(32 x 16).  Written as an asm statement with the accumulator constrained to
// the AGPR half of the register file: left to itself the register allocator spreads 256 accumulator
// registers over both halves and moves fragments between them around every MFMA.  No two MFMAs on
// the same accumulator are closer than 64 instructions, so the hardware's dependent-issue rules
// need no software padding here; the epilogue pads before it reads the accumulators.
// F16: the operands are IEEE binary16 instead of bf16 (same fragment layout, same rate); fragments are
// handled as 16 raw bytes either way.
template <bool F16>
__device__ __forceinline__ void mfma_16x16x32(f32x4& acc, bf16x8 a, bf16x8 b) {
  if constexpr (F16) asm volatile("v_mfma_f32_16x16x32_f16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
  else asm volatile("v_mfma_f32_16x16x32_bf16 %0, %1, %2, %0" : "+a"(acc) : "v"(a), "v"(b));
}
// two fp32 -> two 16-bit values of the output type, round to nearest even
template <bool F16>
__device__ __forceinline__ uint32_t pack16(float lo, float hi) {
  if constexpr (F16) {
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    const f16x2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
  } else {
    return pack_bf16(lo, hi);
  }
}
// The workgroup's 160 KiB of LDS.  One array whoever asks: a kernel that runs two bodies one after the other
// (the fused pair of grouped GEMMs) gives both the same blocks.
__device__ __forceinline__ lds_u8 tile_lds() {
  __shared__ __attribute__((aligned(1024))) uint8_t lds_mem[kLds];
  return (lds_u8)lds_mem;
}
}  // namespace

// NB = columns of C per tile (B rows per tile): 256, or 224 = 2 waves x 7 fragments for problems whose
// tile count then fills the compute units better (B pieces past row 223 are outside the tile's buffer
// descriptor: they cost no traffic and fill LDS rows nobody reads).
//
// GROUPED: the grouped GEMM of an MoE layer.  The rows of A and C are sorted by group, group e owns rows
// group_rows[e] .. group_rows[e + 1] - 1 (device memory: the host does not know them) and multiplies them with
// its own B.  A tile is (group, 256 or 128 rows of that group, 256 columns); the rows a group does not fill are
// outside the tile's buffer descriptors: they load as zero and their stores are dropped.  Each wave first
// works out which tiles its workgroup owns (group_tiles below) and keeps them one per lane; the pipeline
// then runs over them exactly as over the tiles of a dense problem.
//
// BLOCKED: the operands may be stored in blocks (see a_kstep below); without it the scalar offsets are
// the constants of a plain pitched matrix.
//
// GATED: the epilogue of the first group GEMM of an MoE layer.  B holds each expert's gate and up
// projections interleaved in runs of 16 rows (the host accepts only that layout), so that fragment pair
// (j, j + 1) of a wave is (gate, up) of the same 16 output columns in the same lanes; the tile stores
// silu(gate) * up, half as wide as the product.
//
// MR = fragment rows per wave: 8 (tile of 256 rows), or 4 for the grouped kernel when groups are small: a
// tile is then 128 rows x 256 columns, a wave owns 64 x 128 of it, a K-step is 2 x 32 MFMAs per wave instead of
// 2 x 64 and moves half as much of A (4 pieces per wave and K-step), so that the weights stream past twice as
// fast -- with few rows per group the time is that of reading B from HBM.  The A blocks in LDS keep their
// places (half of each is used); loads per K-step 12 instead of 16 (the wait count at the barrier is the same).
//
// RAGGED: a dense GEMM whose M is no multiple of the tile height and whose N is no multiple of 256 (but of 8:
// a lane stores 8 columns at once), run as a grouped one with a single group of all rows.  What M leaves over
// is handled like a group's last tile; what N leaves over: the B descriptor of a tile in the last column ends
// after the rows that exist (the others load as zero), and a lane whose 8 columns lie past N stores at an
// offset no buffer reaches, which drops the store.
//
// OUT32: C is fp32 -- the accumulators are stored as they are, a fragment at a time (a lane's 4 columns are 16
// bytes).  Dense kernels only (with ragged edges N is then a multiple of 4).
//
// PAIR: the body runs as one of the two grouped GEMMs of a fused pair (one launch; the first GEMM's C is the
// second's A).  1 = the first: a tile is stored at device scope (write-through) and then published (every wave
// waits for its stores, barrier, one count added to the row block's word).  2 = the second: before a tile's first
// load may be issued -- a tile ahead, because the load side of the pipeline crosses into the next tile -- wave 0
// polls the row block's word until all column tiles of the first GEMM are counted, acquires at device scope, and
// a barrier lets the other waves on.  A workgroup works through its tiles of the first GEMM before any of the
// second, all workgroups are resident at once (the host launches no more than there are compute units), and tiles
// of the first GEMM wait for nothing: every wait ends.  Should one not (the limit on polls is reached), the wait
// is counted in done[M] and the tile is computed from what is there: wrong rows, but every wave leaves the kernel.
template <int NB, bool GROUPED, bool BLOCKED, bool GATED = false, bool F16 = false, int MR = 8, bool RAGGED = false, bool OUT32 = false,
          int PAIR = 0>
__device__ __forceinline__ void gemm_bf16_256_body(const GemmArgs& g, const PairSync ps = PairSync{}) {
  static_assert(PAIR == 0 || (GROUPED && !RAGGED && !OUT32), "a fused pair is made of two grouped kernels");
  static_assert(!OUT32 || ((!GROUPED || RAGGED) && NB == 256), "the fp32 output exists for the dense 256-wide kernels");
  static_assert(!RAGGED || (GROUPED && !GATED && NB == 256), "ragged edges are handled by the grouped 256-wide kernel");
  static_assert(!GATED || (GROUPED && NB == 256), "the gated epilogue exists for the grouped 256-wide kernel");
  static_assert(MR == 8 || (MR == 4 && GROUPED), "128-row tiles exist for the grouped kernel");
  constexpr int TM = 32 * MR;                                      // rows of a tile
  constexpr int NA = MR;                                           // A pieces (8 rows x 128 bytes) per wave and K-step
  // loads issued after the last load of the next K-step's operands, at the barrier: the last A piece of step
  // kt + 1 is followed by 4 B loads of its sub-step and the 4 of the next sub-step
  constexpr int kWaitStep = 8;
  constexpr int NJ = NB / 32;                                      // fragments per wave along N
  const lds_u8 lds3 = tile_lds();                                  // 32-bit LDS addresses

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave id 0..3, kept scalar
  const int wm = w >> 1, wn = w & 1;                               // wave grid 2 x 2
  const int nk = (int)(g.K / 64);
  const int ntiles = g.grid_m * g.grid_n;

  // ---- the tiles of this workgroup: blockIdx.x, blockIdx.x + gridDim.x, ...  The load side of the
  //      pipeline runs two to four K-steps ahead of the MFMAs and crosses into the next tile before
  //      the current one is finished, so two tiles are described at any time: cur and nxt.
  const int a_pitch = (int)(g.lda * 2), b_pitch = (int)(g.ldb * 2);
  // Operands may be stored pre-tiled along K and blocked along their rows (Sec. 3.3: a blocked layout is a
  // tile product): element (row, k) sits at  (row / rb) * blk_stride + (row % rb) * pitch + (k / 64) * kstep
  // + k % 64  with rb a power-of-two multiple of the tile height.  The plain pitched matrix is kstep = 64,
  // blk_stride = rb * pitch.  All that changes here are scalar offsets: of a tile's first row, and between
  // K-tiles; with 256 x 64 blocks stored contiguously every K-step of a tile reads 32 contiguous KiB.
  const int a_kstep = BLOCKED ? g.a_kstep : kRow, b_kstep = BLOCKED ? g.b_kstep : kRow;   // bytes between K-tiles
  const int a_span = (nk - 1) * a_kstep + kRow, b_span = (nk - 1) * b_kstep + kRow;   // bytes a row of a tile reaches over
  auto a_tile_off = [&](int tm) -> int64_t {                       // elements
    if (!BLOCKED) return (int64_t)tm * kTile * g.lda;
    return (int64_t)(tm >> g.a_tpb_shift) * g.a_blk_stride + (int64_t)(tm & ((1 << g.a_tpb_shift) - 1)) * kTile * g.lda;
  };
  auto b_tile_off = [&](int tn) -> int64_t {
    if (!BLOCKED) return (int64_t)tn * NB * g.ldb;
    return (int64_t)(tn >> g.b_tpb_shift) * g.b_blk_stride + (int64_t)(tn & ((1 << g.b_tpb_shift) - 1)) * NB * g.ldb;
  };
  struct Tile {
    __amdgpu_buffer_rsrc_t ra, rb;
  };
  int tb_row0 = 0, tb_desc = 0;                                    // grouped: lane t = the workgroup's t-th tile
  if constexpr (GROUPED) group_tiles<TM, RAGGED>(g, lane, tb_row0, tb_desc);
  auto table_rows = [&](int t) __attribute__((always_inline)) -> int { return t < 64 ? desc_rows(__builtin_amdgcn_readlane(tb_desc, t)) : 0; };
  // dense: v = tile id; grouped: v = index into the workgroup's table
  auto describe = [&](int v) __attribute__((always_inline)) -> Tile {
    Tile t;
    if constexpr (GROUPED) {
      const int rows = table_rows(v);
      if (rows > 0) {
        const int row0 = __builtin_amdgcn_readlane(tb_row0, v), dsc = __builtin_amdgcn_readlane(tb_desc, v);
        const int grp = desc_group(dsc), tn = desc_tn(dsc);
        const uint8_t* pa = (const uint8_t*)g.A + (int64_t)row0 * g.lda * 2;
        t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)pa, 0, (rows - 1) * a_pitch + a_span, 0x00020000);
        int nb = NB;                                               // rows of B the tile has
        if constexpr (RAGGED) nb = (int)g.N - tn * NB < NB ? (int)g.N - tn * NB : NB;
        t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.B + ((int64_t)grp * g.ldg + b_tile_off(tn)) * 2), 0,
                                                 (nb - 1) * b_pitch + b_span, 0x00020000);
        return t;
      }
    }
    if (!GROUPED && v < ntiles) {
      int tm, tn;
      tile_of_block(v, ntiles, g.grid_m, g.grid_n, tm, tn);
      t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.A + a_tile_off(tm) * 2), 0, 255 * a_pitch + a_span, 0x00020000);
      t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.B + b_tile_off(tn) * 2), 0, (NB - 1) * b_pitch + b_span, 0x00020000);
    } else {                                                       // no such tile: every load returns zero
      t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)g.A, 0, 0, 0x00020000);
      t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)g.B, 0, 0, 0x00020000);
    }
    return t;
  };
  int v = GROUPED ? 0 : (int)blockIdx.x;
  const int vstep = GROUPED ? 1 : (int)gridDim.x;
  if (GROUPED && table_rows(0) <= 0) return;                       // more workgroups than tiles (the host sizes the launch for the worst case)
  // second GEMM of a pair: the rows of tile t of this workgroup have been produced (see PAIR above)
  auto wait_rows = [&](int t) __attribute__((always_inline)) {
    if constexpr (PAIR == 2) {
      if (table_rows(t) <= 0) return;                              // (uniform over the workgroup: every wave holds the same table)
      if (w == 0) {
        const int32_t* word = ps.done + __builtin_amdgcn_readlane(tb_row0, t);
        int polls = 0;
        while (__hip_atomic_load(word, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) < ps.need) {
          if (++polls > ps.spin_limit) {
            if (lane == 0) __hip_atomic_fetch_add(ps.done + ps.M, 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            break;
          }
          __builtin_amdgcn_s_sleep(8);
        }
        __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
      }
      wg_barrier();
    }
  };
  wait_rows(0);
  wait_rows(1);
  Tile cur = describe(v), nxt = describe(v + vstep);

  // ---- HBM -> LDS.  Per K-tile and operand 32 wave instructions of 8 rows; wave w issues pieces
  //      i = 0..7 = row groups w, w + 4, ..., w + 28.  Buffer addressing: the descriptor covers the 256
  //      rows of the tile (reads past its end return zero), the per-lane offset is fixed, K-tile and
  //      piece go into the scalar offset.
  const int lr = lane / maps::kLargeChunks, lp = lane % maps::kLargeChunks;
  const int lrow = maps::piece_row(w, 0, lr, 4);                   // row of piece 0; piece i lies 32 i rows further (same key)
  const int a_voff_x = lrow * a_pitch + maps::lds_chunk_pos(lrow, lp, maps::kLargeChunks) * maps::kChunkBytes;
  const int b_voff = lrow * b_pitch + maps::lds_chunk_pos(lrow, lp, maps::kLargeChunks) * maps::kChunkBytes;
  const int a_piece = maps::piece_row(0, 1, 0, 4) * a_pitch, b_piece = maps::piece_row(0, 1, 0, 4) * b_pitch;   // bytes between pieces
  // Both operands go from HBM straight into LDS (no staging registers, no ds_write: a ds_write_b128 keeps its
  // wave from issuing for about 20 cycles, and 8 of them per K-step cost 7 % of the whole kernel).  A direct
  // load fills 1 KiB of LDS linearly in the lane id, so the XOR of the LDS image is applied to the chunk a
  // lane fetches.  A has two blocks (the steps of either parity): the pieces of step kt + 2 are issued right
  // after the barrier of step kt has freed the block step kt occupied, and have to have landed at the barrier
  // of step kt + 1 -- a load distance of one K-step.  B has a ring of three blocks.
  // (the piece goes into the per-lane offset, one register per piece, so that the scalar offset is the K-tile's
  //  alone and shared by the 8 loads of a step: one scalar instruction less per load)
  int a_voff_p[NA], b_voff_p[8];
#pragma unroll
  for (int i = 0; i < NA; ++i) a_voff_p[i] = a_voff_x + i * a_piece;
#pragma unroll
  for (int i = 0; i < 8; ++i) b_voff_p[i] = b_voff + i * b_piece;
  auto a_dload = [&](int T, int i, bool cross) __attribute__((always_inline)) {   // piece i of step T into the A block of its parity
    const bool nx = cross && T >= nk;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(nx ? nxt.ra : cur.ra, (lds_ptr)(lds3 + (T & 1) * kBlk + maps::piece_row(w, i, 0, 4) * kRow), 16,
                                             a_voff_p[i], (nx ? T - nk : T) * a_kstep, 0, 0);   // (K-step T >= nk: step T - nk of the next tile)
    AXE_PARANOID_WAIT();
  };
  // B ring: byte offsets of the blocks that hold K-steps kt, kt+1, kt+2 (step kt+3 reuses the first)
  int bo0 = kBoff, bo1 = kBoff + kBlk, bo2 = kBoff + 2 * kBlk;
  auto b_load = [&](int T, int i, int slot_off, bool cross) __attribute__((always_inline)) {
    const bool nx = cross && T >= nk;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(nx ? nxt.rb : cur.rb, (lds_ptr)(lds3 + slot_off + maps::piece_row(w, i, 0, 4) * kRow), 16,
                                             b_voff_p[i], (nx ? T - nk : T) * b_kstep, 0, 0);
    AXE_PARANOID_WAIT();
  };

  // ---- LDS -> VGPR: fragment f of this wave's A (B) rows: row = base + f * 16 + lane % 16
  const int fr = lane % maps::kFrag, fq = lane / maps::kFrag;
  lds_u8 fax[2], fbx[2];                                           // row base + swizzled chunk, per sub-step
#pragma unroll
  for (int s = 0; s < 2; ++s) {
    // (the wave's first row is a multiple of 16 = one period of the key: the key is that of row fr)
    const int pos = maps::lds_chunk_pos(fr, maps::operand_chunk_16bit(s, fq), maps::kLargeChunks) * maps::kChunkBytes;
    fax[s] = lds3 + (wm * (16 * MR) + fr) * kRow + pos;
    fbx[s] = lds3 + (wn * (NB / 2) + fr) * kRow + pos;
  }

  f32x4 acc[MR][NJ];
#pragma unroll
  for (int i = 0; i < MR; ++i)
#pragma unroll
    for (int j = 0; j < NJ; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  bf16x8 fa[MR], fb[2][NJ];    // A fragment i serves the 8 MFMAs of its row and is re-read right after the last of them; B is double-buffered

  // ---- VGPR -> HBM.  Operands are swapped in the MFMA, so lane l holds, for fragment (i, j), the 4
  //      consecutive columns j*16 + 4*(l/16) .. +3 of row i*16 + l%16 of the wave's 128 x 128 sub-tile:
  //      8 bytes of bf16.  The eight stores of a fragment row fill 256 contiguous bytes of 16 rows one after
  //      the other; L2 merges them into whole lines.  The store is an asm statement so that the
  //      compiler's wait-count bookkeeping, which would otherwise turn every counted wait for a load
  //      into a wait for everything while a store is pending, does not see it: stores and loads share
  //      the hardware counter, but a counted wait for a load stays valid with stores in between,
  //      because loads complete in order among themselves.
  i32x4 rc;                                                        // descriptor of this wave's part of the C tile
  int c_rowblk;                                                    // bytes between fragment rows
  const int c_voff = (int)((fr * g.ldc + 4 * fq) * 2);
  int c_cw = 0;                                                    // ragged: columns of this wave's part of the tile that exist
  int c_nfr = MR;                                                  // grouped: fragment rows of this wave that hold rows of the tile
  auto set_output = [&](int vv) __attribute__((always_inline)) {
    if constexpr (GROUPED) {
      const int row0 = __builtin_amdgcn_readlane(tb_row0, vv), dsc = __builtin_amdgcn_readlane(tb_desc, vv);
      const int tn = desc_tn(dsc);
      int rows = desc_rows(dsc) - wm * (16 * MR);                    // rows of the tile that fall to this wave
      rows = rows < 0 ? 0 : (rows > 16 * MR ? 16 * MR : rows);
      constexpr int CW = GATED ? NB / 4 : NB / 2;                    // columns of C this wave writes
      int cw = CW;
      if constexpr (RAGGED) {
        cw = (int)g.N - tn * NB - wn * CW;                           // ... of which exist
        cw = cw < 0 ? 0 : (cw > CW ? CW : cw);
        if (cw == 0) rows = 0;
        c_cw = cw;
      }
      c_nfr = (rows + 15) >> 4;
      constexpr int OBG = OUT32 ? 4 : 2;                             // bytes per element of C
      rc = raw_rsrc((uint8_t*)g.C + (((int64_t)row0 + wm * (16 * MR)) * g.ldc + (int64_t)tn * (2 * CW) + wn * CW) * OBG,
                    rows ? (uint32_t)(((rows - 1) * g.ldc + cw) * OBG) : 0u);
      c_rowblk = (int)(16 * g.ldc * OBG);
      return;
    }
    int tm, tn;
    tile_of_block(vv, ntiles, g.grid_m, g.grid_n, tm, tn);
    constexpr int OB = OUT32 ? 4 : 2;                                // bytes per element of C
    rc = raw_rsrc((uint8_t*)g.C + (((int64_t)tm * kTile + wm * 128) * g.ldc + (int64_t)tn * NB + wn * (NB / 2)) * OB,
                  (uint32_t)((127 * g.ldc + NB / 2) * OB));
    c_rowblk = (int)(16 * g.ldc * OB);
  };
  // fp32 output: the fragment as it is, 16 bytes per lane (columns 4 q .. 4 q + 3 of row fr), 64 bytes per row
  const int c_voff32 = (int)((fr * g.ldc + 4 * fq) * 4);
  auto store_fragment32 = [&](int i, int j) __attribute__((always_inline)) {
    const f32x4 d = acc[i][j];                                     // (a copy in VGPRs: the accumulators live in AGPRs)
    const int soff = __builtin_amdgcn_readfirstlane(i * c_rowblk + j * 64);
    int voff = c_voff32;
    if constexpr (RAGGED) {                                          // the lane's 4 columns lie past N: an offset no descriptor reaches
      int l;
      asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
      if (j * 16 + 4 * (l >> 4) + 4 > c_cw) voff = (int)0x80000000u;
    }
    asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, %3 offen" AXE_AFTER_STORE ::"v"(d), "v"(voff), "s"(rc), "s"(soff) : "memory");
    AXE_PARANOID_WAIT();
    __builtin_amdgcn_sched_barrier(0);                             // one fragment at a time: copied out of the AGPRs and stored
  };
  auto store_fragment = [&](int i, int j) __attribute__((always_inline)) {
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
    const u32x2 d = {pack16<F16>(acc[i][j][0], acc[i][j][1]), pack16<F16>(acc[i][j][2], acc[i][j][3])};
    const int soff = __builtin_amdgcn_readfirstlane(i * c_rowblk + j * 32);
    asm volatile("s_nop 4\n\tbuffer_store_dwordx2 %0, %1, %2, %3 offen" AXE_AFTER_STORE ::"v"(d), "v"(c_voff), "s"(rc), "s"(soff) : "memory");
    AXE_PARANOID_WAIT();
  };
  // Two neighbouring fragments (i, j), (i, j + 1) in one 16-byte store per lane: lane groups q = l / 16
  // hold columns 4 q .. 4 q + 3 of each fragment; v_permlane16_swap exchanges the odd lane groups of
  // the first with the even lane groups of the second, after which an even group q owns columns
  // 4 q .. 4 q + 7 of fragment j and an odd group q columns 4 (q - 1) .. 4 q + 3 of fragment j + 1.
  // Half as many store instructions and write requests; 64 contiguous bytes per row and instruction.
  const int c_voff2 = (int)((fr * g.ldc + maps::pair_store_col(fq)) * 2);
  auto store_fragment_pair = [&](int i, int j) __attribute__((always_inline)) {
    const auto lo = __builtin_amdgcn_permlane16_swap(pack16<F16>(acc[i][j][0], acc[i][j][1]),
                                                     pack16<F16>(acc[i][j + 1][0], acc[i][j + 1][1]), false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(pack16<F16>(acc[i][j][2], acc[i][j][3]),
                                                     pack16<F16>(acc[i][j + 1][2], acc[i][j + 1][3]), false, false);
    const u32x4 d = {lo[0], hi[0], lo[1], hi[1]};
    const int soff = __builtin_amdgcn_readfirstlane(i * c_rowblk + j * 32);
    // (an offset of 2^31 is past the end of every descriptor -- their ranges stay below 2^31 bytes)
    int voff = c_voff2;
    if constexpr (RAGGED) {
      // the lane's first column, worked out here from the lane number (an asm statement, so that it is not
      // hoisted above the K loops, where it would occupy a register the pipeline needs)
      int l;
      asm volatile("v_mbcnt_lo_u32_b32 %0, -1, 0\n\tv_mbcnt_hi_u32_b32 %0, -1, %0" : "=v"(l));
      const int q = l >> 4;
      const int c0 = maps::pair_store_col(q);
      if (j * 16 + c0 + 8 > c_cw) voff = (int)0x80000000u;
    }
    asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, %3 offen" AXE_AFTER_STORE ::"v"(d), "v"(voff), "s"(rc), "s"(soff) : "memory");
    AXE_PARANOID_WAIT();
  };

  // Gated epilogue: h = silu(gate) * up for the fragment pairs (j, j + 1) and (j + 2, j + 3), stored like a
  // fragment pair (32 output columns, 64 contiguous bytes per row).  fp32 throughout; the exponential and
  // the reciprocal are the hardware's approximations (1 ulp), far inside the bf16 rounding of the result.
  auto store_gated_quad = [&](int i, int j) __attribute__((always_inline)) {
    float h[2][4];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float gate = acc[i][j + 2 * q][e], up = acc[i][j + 2 * q + 1][e];
        h[q][e] = gate * __builtin_amdgcn_rcpf(1.0f + __expf(-gate)) * up;
      }
    const auto lo = __builtin_amdgcn_permlane16_swap(pack16<F16>(h[0][0], h[0][1]), pack16<F16>(h[1][0], h[1][1]), false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(pack16<F16>(h[0][2], h[0][3]), pack16<F16>(h[1][2], h[1][3]), false, false);
    const u32x4 d = {lo[0], hi[0], lo[1], hi[1]};
    const int soff = __builtin_amdgcn_readfirstlane(i * c_rowblk + j * 16);
    // (first GEMM of a pair: the store is made at device scope -- it writes through this XCD's L2 to memory, where the
    //  other XCDs' workgroups will read it, so that publishing the tile needs no write-back of the whole L2)
    if constexpr (PAIR == 1)
      asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, %3 offen sc1" AXE_AFTER_STORE ::"v"(d), "v"(c_voff2), "s"(rc), "s"(soff) : "memory");
    else
      asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, %3 offen" AXE_AFTER_STORE ::"v"(d), "v"(c_voff2), "s"(rc), "s"(soff) : "memory");
    AXE_PARANOID_WAIT();
  };

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;

  // Sub-step S of K-step kt (PAR = kt & 1), in exact program order (sched_barrier(0) forbids any
  // reordering across it): 8 x NJ slots (i, j), j innermost, one MFMA each -- the fragments are walked in pairs of
  // rows (see the loop), the side work is placed by slot; in rows 0..3 the B fragments of the
  // next sub-step are read into the other buffer (after slots j = 1 and j = 5), and right after the last MFMA of
  // fragment row i the A fragment i of the next sub-step replaces the one just used; sub-step 0 issues four B loads (after
  // slot j = 2 of the even rows), sub-step 1 the 8 A pieces and four B loads.  Sub-step 1 of the 256-row tile has
  // its own placement (see LATE below).  Steps past the end of the tile are steps of the workgroup's next tile
  // (or of none: then their loads return zero).
  auto substep = [&](auto par_c, auto s_c, auto cross_c, int kt) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_c)::value, S = decltype(s_c)::value;
    constexpr bool CROSS = decltype(cross_c)::value != 0;          // the loads of this step may belong to the next tile
    constexpr int CUR = S, NXT = S ^ 1;
    // fragments read now: sub-step 1 of this step, or sub-step 0 of the next one
    constexpr int RST = S == 0 ? PAR : PAR ^ 1;                    // A stage of that step
    const lds_u8 pa = fax[NXT] + RST * kBlk;
    const lds_u8 pb = fbx[NXT] + (S == 0 ? bo0 : bo1);
    // B pieces loaded now: 4..7 of step kt+2 into its ring block (sub-step 0) or 0..3 of step kt+3 into the
    // block step kt has just left (sub-step 1); all A pieces of step kt+2 are loaded in sub-step 1, into the
    // block step kt has just left.
    const int bT = S == 0 ? kt + 2 : kt + 3;
    const int bslot = S == 0 ? bo2 : bo0;
    // With 256-row tiles the barrier of a K-step does not stand between the two sub-steps but two rows of MFMAs
    // (16 of them, 256 cycles) into sub-step 1: the wave reaches it with the last LDS read of sub-step 0 long
    // complete and a little more time for its loads to land, instead of draining the matrix pipe while it waits
    // for that read.  Everything that needs the barrier -- reads of step kt + 1, loads into what step kt
    // occupied -- is scheduled into rows 2..7 of sub-step 1; rows 0 and 1 only multiply what is in registers.
    constexpr bool LATE = MR == 8;
    auto step_barrier = [&]() __attribute__((always_inline)) {
      // Own reads of step kt are complete, and so are own loads of step kt+1 (the 8 younger loads may still
      // be in flight).  After the barrier step kt+1 is readable by every wave and nobody reads step kt any more.
      asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)" ::"n"(kWaitStep) : "memory");
      wg_barrier();
    };
#pragma unroll
    for (int i = 0; i < MR; ++i) {
#pragma unroll
      for (int j = 0; j < NJ; ++j) {
        // (i, j) is the slot of the schedule; the fragment multiplied in it is (mi, mj): the rows are walked in pairs,
        // (r, 0), (r + 1, 0), (r, 1), (r + 1, 1), ..., every other pair from the last column back to the first (so that
        // the B fragment stays when the pair changes) -- every accumulator sees the same sequence of K-steps as in a
        // row-by-row walk (same bits), but the matrix pipe draws less power, and power bounds these kernels: a
        // register-only loop of this MFMA on the same data sustains 2080 TFLOP/s in this order against 2015 row by
        // row (pairs all in the same direction 2068, four-row blocks 2020, a diagonal walk 1975), the 8192^3 GEMM
        // 1564 against 1539 with the pairs and another 0.4 % with the alternating direction.
        const int mr = (i & 1) * NJ + j;
        const int mi = 2 * (i >> 1) + (mr & 1), mj = ((i >> 1) & 1) ? NJ - 1 - (mr >> 1) : (mr >> 1);
        mfma_16x16x32<F16>(acc[mi][mj], fb[CUR][mj], fa[mi]);
        __builtin_amdgcn_sched_barrier(0);
        if constexpr (LATE && S == 1) {
          // side work of sub-step 1, rows 2..7 (NJ = 8, or 7 with the 224-wide tile: nothing sits at j = 7 but
          // the reload of the row's own A fragment, which goes with the row's last MFMA)
          if (i == 1 && j == NJ - 1) step_barrier();
          if (i >= 2 && i < 6 && (j == 1 || j == 5) && 2 * (i - 2) + (j == 5) < NJ)
            fb[NXT][2 * (i - 2) + (j == 5)] = lds_read(pb + (2 * (i - 2) + (j == 5)) * 16 * kRow);
          if (i == 2 && j == 4) fa[0] = lds_read(pa);
          if (i == 3 && j == 4) fa[1] = lds_read(pa + 16 * kRow);
          if (mi >= 2 && (mr >> 1) == NJ - 1) fa[mi] = lds_read(pa + mi * 16 * kRow);
          // the 8 A pieces of step kt + 2 first (they have one K-step to land), then four B loads
          if (i >= 2 && i < 6 && (j == 2 || j == 6)) a_dload(kt + 2, 2 * (i - 2) + (j == 6), CROSS);
          if (i >= 6 && (j == 2 || j == 6)) b_load(bT, 2 * (i - 6) + (j == 6), bslot, CROSS);
        } else {
          // (with 4 rows the reads sit earlier in the row: the last fragment is needed 9 MFMAs after row 3 ends)
          constexpr int jb0 = MR == 8 ? 1 : 0, jb1 = MR == 8 ? 5 : 3;
          if (i < 4 && (j == jb0 || j == jb1) && 2 * i + (j == jb1) < NJ)
            fb[NXT][2 * i + (j == jb1)] = lds_read(pb + (2 * i + (j == jb1)) * 16 * kRow);
          if ((mr >> 1) == NJ - 1) fa[mi] = lds_read(pa + mi * 16 * kRow);
          if constexpr (MR == 4 && S == 1) {
            // 128-row tiles, sub-step 1 (right after the barrier): the 4 A pieces of step kt + 2, then four B loads
            if (i < 2 && (j == 2 || j == 6)) a_dload(kt + 2, 2 * i + (j == 6), CROSS);
            if (i >= 2 && (j == 2 || j == 6)) b_load(bT, 2 * (i - 2) + (j == 6), bslot, CROSS);
          } else
          // four B loads per sub-step: after MFMA j = 2 of the even rows (8 rows), or of every row (4 rows)
          if (MR == 8 ? ((i & 1) == 0 && j == 2) : j == 2) b_load(bT, (S == 0 ? 4 : 0) + (MR == 8 ? i >> 1 : i), bslot, CROSS);
        }
        __builtin_amdgcn_sched_barrier(0);
      }
      AXE_PARANOID_SYNC();
    }
    if (S == 0 && !LATE) step_barrier();
  };
  auto step = [&](auto par_c, auto cross_c, int kt) __attribute__((always_inline)) {
    substep(par_c, I0{}, cross_c, kt);
    substep(par_c, I1{}, cross_c, kt);
    const int t = bo0;
    bo0 = bo1, bo1 = bo2, bo2 = t;
  };

  // ---- prologue (first tile only): what the sub-steps before (0, 0) would have done: steps 0 and 1 of A,
  //      steps 0, 1 and the first half of step 2 of B.  Step 0 of both operands first: the MFMAs start as soon as it
  //      has landed (the NA + 12 loads of step 1 and of step 2's first half may still be in flight; the barrier of
  //      step 0 waits for step 1 as the barrier of every step does, with step 2's eight B loads behind it).
#pragma unroll
  for (int i = 0; i < NA; ++i) a_dload(0, i, true);
#pragma unroll
  for (int i = 0; i < 8; ++i) b_load(0, i, bo0, true);
#pragma unroll
  for (int i = 0; i < NA; ++i) a_dload(1, i, true);                // (a single K-step per tile: step 1 is the next tile's step 0)
#pragma unroll
  for (int i = 0; i < 8; ++i) b_load(1, i, bo1, true);
#pragma unroll
  for (int i = 0; i < 4; ++i) b_load(2, i, bo2, true);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(NA + 12) : "memory");
  wg_barrier();
#pragma unroll
  for (int f = 0; f < NJ; ++f) fb[0][f] = lds_read(fbx[0] + bo0 + f * 16 * kRow);
#pragma unroll
  for (int f = 0; f < MR; ++f) fa[f] = lds_read(fax[0] + f * 16 * kRow);

  // ---- all K-steps of all tiles of this workgroup, one uninterrupted pipeline.  The host launches
  //      more than one tile per workgroup only when nk is even (the A block of a step is chosen by its
  //      parity, which must continue across the tile boundary) and at least 4 (the load side looks at most
  //      one tile ahead).
  for (;;) {
    set_output(v);
    int kt = 0;
    for (; kt + 5 < nk; kt += 2) {                                 // every load of these steps is of this tile (at most step kt + 5)
      step(I0{}, I0{}, kt);
      step(I1{}, I0{}, kt + 1);
    }
    for (; kt + 1 < nk; kt += 2) {                                 // the last steps load the next tile's first K-steps
      step(I0{}, I1{}, kt);
      step(I1{}, I1{}, kt + 1);
    }
    if (kt < nk) step(I0{}, I1{}, kt);                             // odd nk: only with one tile per workgroup
    // the tile is complete: store it while the loads of the next tile's first K-steps, issued by the
    // steps above, are on their way; the MFMAs have to retire before their results are read
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");
    __builtin_amdgcn_sched_barrier(0);                             // no accumulator read may move above the padding
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      // grouped: a fragment row without rows of the tile issues no stores (the buffer descriptor would drop them,
      // but each would still take its turn in the memory pipeline, ahead of the next tile's loads)
      if (!GROUPED || i < c_nfr) {
        if constexpr (OUT32) {
#pragma unroll
          for (int j = 0; j < NJ; ++j) store_fragment32(i, j);
        } else if constexpr (GATED) {
#pragma unroll
          for (int j = 0; j < NJ; j += 4) store_gated_quad(i, j);
        } else {
#pragma unroll
          for (int j = 0; j < NJ; j += 2) {
            if (NJ % 2 == 0) store_fragment_pair(i, j);            // (7 fragments per row do not pair up: stored one by one)
            else {
              store_fragment(i, j);
              if (j + 1 < NJ) store_fragment(i, j + 1);
            }
          }
        }
      }
#pragma unroll
      for (int j = 0; j < NJ; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;            // ready for the next tile
    }
    if constexpr (PAIR == 1) {
      // first GEMM of a pair: publish the tile.  Its stores were made at device scope (written through to memory,
      // see store_gated_quad); each wave waits until its own have been acknowledged -- they are asm statements the
      // compiler does not count, so the wait is written out (it also covers the next tile's first loads: a pause
      // of one load latency per tile) -- and after the barrier one lane counts the tile.  A device-scope release
      // fence in place of the write-through stores also works, and is what the language offers; it writes back
      // the XCD's whole L2 at every tile and made the pair slower than two launches (485 against 441 us on the
      // benchmark's layer at 4096 tokens; this way 425).
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      wg_barrier();
      if (w == 0 && lane == 0)
        __hip_atomic_fetch_add(ps.done + __builtin_amdgcn_readlane(tb_row0, v), 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    v += vstep;
    if (GROUPED ? table_rows(v) <= 0 : v >= ntiles) break;
    cur = nxt;
    wait_rows(v + vstep);
    nxt = describe(v + vstep);
  }
}

// (plain kernels around the template: a __global__ template would be instantiated by the host pass
//  too, which cannot parse the register constraints of the asm statements)
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_kernel(GemmArgs g) { gemm_bf16_256_body<256, false, false>(g); }
__global__ __launch_bounds__(256, 1) void gemm_bf16_256x224_kernel(GemmArgs g) { gemm_bf16_256_body<224, false, false>(g); }
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_blocked_kernel(GemmArgs g) { gemm_bf16_256_body<256, false, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_grouped_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_grouped_gated_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, true>(g); }
// IEEE binary16 inputs and output: the dense kernel (plain or blocked operands) and the grouped ones
__global__ __launch_bounds__(256, 1) void gemm_f16_256_kernel(GemmArgs g) { gemm_bf16_256_body<256, false, true, false, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_f16_256_grouped_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, false, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_f16_256_grouped_gated_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, true, true>(g); }
// grouped, tiles of 128 rows (small groups)
// fp32 output (plain or blocked operands)
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_f32out_kernel(GemmArgs g) { gemm_bf16_256_body<256, false, true, false, false, 8, false, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_f16_256_f32out_kernel(GemmArgs g) { gemm_bf16_256_body<256, false, true, false, true, 8, false, true>(g); }
// dense with ragged edges and an fp32 output (any M, N a multiple of 4)
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_ragged_f32out_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, false, false, 8, true, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_f16_256_ragged_f32out_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, false, true, 8, true, true>(g); }
// dense with ragged edges (any M, N a multiple of 8)
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_ragged_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, false, false, 8, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_f16_256_ragged_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, false, true, 8, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_bf16_128_grouped_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, false, false, 4>(g); }
__global__ __launch_bounds__(256, 1) void gemm_bf16_128_grouped_gated_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, true, false, 4>(g); }
__global__ __launch_bounds__(256, 1) void gemm_f16_128_grouped_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, false, true, 4>(g); }
__global__ __launch_bounds__(256, 1) void gemm_f16_128_grouped_gated_kernel(GemmArgs g) { gemm_bf16_256_body<256, true, true, true, true, 4>(g); }
// the fused pair: both GEMMs of an MoE layer's expert computation in one launch (gated first GEMM, plain second)
template <bool F16, int MR>
__device__ __forceinline__ void grouped_pair_body(const GemmArgs& g1, const GemmArgs& g2, const PairSync& ps) {
  gemm_bf16_256_body<256, true, true, true, F16, MR, false, false, 1>(g1, ps);
  gemm_bf16_256_body<256, true, true, false, F16, MR, false, false, 2>(g2, ps);
}
__global__ __launch_bounds__(256, 1) void gemm_bf16_256_grouped_pair_kernel(GemmArgs g1, GemmArgs g2, PairSync ps) { grouped_pair_body<false, 8>(g1, g2, ps); }
__global__ __launch_bounds__(256, 1) void gemm_f16_256_grouped_pair_kernel(GemmArgs g1, GemmArgs g2, PairSync ps) { grouped_pair_body<true, 8>(g1, g2, ps); }
__global__ __launch_bounds__(256, 1) void gemm_bf16_128_grouped_pair_kernel(GemmArgs g1, GemmArgs g2, PairSync ps) { grouped_pair_body<false, 4>(g1, g2, ps); }
__global__ __launch_bounds__(256, 1) void gemm_f16_128_grouped_pair_kernel(GemmArgs g1, GemmArgs g2, PairSync ps) { grouped_pair_body<true, 4>(g1, g2, ps); }

__global__ __launch_bounds__(256) void pair_sync_clear_kernel(int32_t* p, int64_t n) {
  const int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x;
  if (i < n) p[i] = 0;
}

hipError_t launch_gemm_bf16_256(const GemmArgs& g, hipStream_t s) {
  const int ntiles = g.grid_m * g.grid_n;
  const int nk = (int)(g.K / 64);
  const int cus = cu_count();
  // one resident workgroup per CU walks several tiles when the pipeline can continue across tiles
  const bool chain = (nk % 2 == 0) && nk >= 4 && ntiles > cus && (cus % 8 == 0);
  unsigned nwg = (unsigned)(chain ? cus : ntiles);
  const bool blocked = g.a_kstep != kRow || g.b_kstep != kRow || g.a_blk_stride != kTile * g.lda || g.b_blk_stride != g.tile_n * g.ldb;
  if (!g.out_bf16) {
    if (g.tile_n != 256) return hipErrorInvalidValue;
    if (g.f16) hipLaunchKernelGGL(gemm_f16_256_f32out_kernel, dim3(nwg), dim3(256), 0, s, g);
    else hipLaunchKernelGGL(gemm_bf16_256_f32out_kernel, dim3(nwg), dim3(256), 0, s, g);
  } else if (g.f16)
    hipLaunchKernelGGL(gemm_f16_256_kernel, dim3(nwg), dim3(256), 0, s, g);
  else if (g.tile_n == 224)
    hipLaunchKernelGGL(gemm_bf16_256x224_kernel, dim3(nwg), dim3(256), 0, s, g);
  else if (blocked)
    hipLaunchKernelGGL(gemm_bf16_256_blocked_kernel, dim3(nwg), dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_bf16_256_kernel, dim3(nwg), dim3(256), 0, s, g);
  return hipGetLastError();
}

// Grouped: the host does not know the group sizes, only that sum_e ceil(rows_e / 256) <= M / 256 + groups.
// One workgroup per CU walks its tiles when the pipeline can continue across tiles (a wave keeps at
// most 64 tiles, one per lane: beyond 64 x CUs tiles in the worst case more workgroups are launched);
// otherwise one workgroup per possible tile, those without a tile leave at once.
hipError_t launch_gemm_bf16_256_grouped(const GemmArgs& g, hipStream_t s) {
  const bool t128 = grouped_tile_rows(g.M, g.groups, g.tile_m) == 128;
  const int tm = t128 ? 128 : kTile;
  const int64_t worst = (g.M / tm + g.groups) * (int64_t)g.grid_n;
  const int nk = (int)(g.K / 64);
  const int cus = cu_count();
  const bool chain = (nk % 2 == 0) && nk >= 4;
  int64_t nwg = chain ? std::max<int64_t>(cus, (worst + 63) / 64) : worst;
  // more workgroups than compute units only in whole rounds (272 workgroups on 256 units take as long as 512)
  if (chain && nwg > cus) nwg = (nwg + cus - 1) / cus * cus;
  nwg = (nwg + 7) / 8 * 8;                                         // the tile sequence is cut into 8 parts, one per XCD
  if (nwg > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nwg), block(256);
  const int which = (t128 ? 4 : 0) + (g.f16 ? 2 : 0) + (g.gated ? 1 : 0);
  switch (which) {
    case 0: hipLaunchKernelGGL(gemm_bf16_256_grouped_kernel, grid, block, 0, s, g); break;
    case 1: hipLaunchKernelGGL(gemm_bf16_256_grouped_gated_kernel, grid, block, 0, s, g); break;
    case 2: hipLaunchKernelGGL(gemm_f16_256_grouped_kernel, grid, block, 0, s, g); break;
    case 3: hipLaunchKernelGGL(gemm_f16_256_grouped_gated_kernel, grid, block, 0, s, g); break;
    case 4: hipLaunchKernelGGL(gemm_bf16_128_grouped_kernel, grid, block, 0, s, g); break;
    case 5: hipLaunchKernelGGL(gemm_bf16_128_grouped_gated_kernel, grid, block, 0, s, g); break;
    case 6: hipLaunchKernelGGL(gemm_f16_128_grouped_kernel, grid, block, 0, s, g); break;
    default: hipLaunchKernelGGL(gemm_f16_128_grouped_gated_kernel, grid, block, 0, s, g); break;
  }
  return hipGetLastError();
}

hipError_t launch_pair_sync_clear(int32_t* p, int64_t n, hipStream_t s) {
  if (n <= 0) return hipSuccess;
  hipLaunchKernelGGL(pair_sync_clear_kernel, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, s, p, n);
  return hipGetLastError();
}

// The library's own workspace for callers that may not allocate (axe_gemm_grouped_pair_static): the counters of
// PairSync for up to kPairStaticRows rows, 4 MiB + 4 bytes of every device the library runs on, held until the
// process ends.  The array's name is only a handle on the host: its address on the current device is asked for
// once per device and kept.
static __device__ __align__(256) int32_t pair_scratch[kPairStaticRows + 1];

hipError_t pair_static_workspace(int32_t** out) {
  constexpr int kMaxDevices = 64;
  static std::mutex mu;
  static int32_t* ptr[kMaxDevices] = {};
  int dev = -1;
  if (hipError_t e = hipGetDevice(&dev); e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(mu);
  if (!ptr[dev]) {
    void* p = nullptr;
    if (hipError_t e = hipGetSymbolAddress(&p, HIP_SYMBOL(pair_scratch)); e != hipSuccess) return e;
    ptr[dev] = (int32_t*)p;
  }
  *out = ptr[dev];
  return hipSuccess;
}

// sync: M + 1 words of device memory (cleared here, on the stream, by a small kernel: a caller may be capturing a graph)
hipError_t launch_gemm_bf16_256_grouped_pair(const GemmArgs& g1, const GemmArgs& g2, int32_t* sync, int spin_limit, int need_extra,
                                             hipStream_t s) {
  if (!grouped_pair_fusable(g1, g2) || !sync) return hipErrorInvalidValue;
  const bool t128 = grouped_tile_rows(g1.M, g1.groups, g1.tile_m) == 128;
  if (hipError_t e = launch_pair_sync_clear(sync, g1.M + 1, s); e != hipSuccess) return e;
  PairSync ps;
  ps.done = sync;
  ps.need = g1.grid_n + need_extra;
  ps.spin_limit = spin_limit;
  ps.M = g1.M;
  const dim3 grid((unsigned)cu_count()), block(256);
  switch ((t128 ? 2 : 0) + (g1.f16 ? 1 : 0)) {
    case 0: hipLaunchKernelGGL(gemm_bf16_256_grouped_pair_kernel, grid, block, 0, s, g1, g2, ps); break;
    case 1: hipLaunchKernelGGL(gemm_f16_256_grouped_pair_kernel, grid, block, 0, s, g1, g2, ps); break;
    case 2: hipLaunchKernelGGL(gemm_bf16_128_grouped_pair_kernel, grid, block, 0, s, g1, g2, ps); break;
    default: hipLaunchKernelGGL(gemm_f16_128_grouped_pair_kernel, grid, block, 0, s, g1, g2, ps); break;
  }
  return hipGetLastError();
}

// Dense with ragged edges: the grouped kernel's machinery with one group of all M rows (g.groups = 1, no offsets
// array), tiles of 256 rows; the host knows the tile count exactly.
hipError_t launch_gemm_bf16_256_ragged(const GemmArgs& g, hipStream_t s) {
  const int64_t tiles = (g.M + kTile - 1) / kTile * (int64_t)g.grid_n;
  const int nk = (int)(g.K / 64);
  const int cus = cu_count();
  const bool chain = (nk % 2 == 0) && nk >= 4;
  int64_t nwg = chain ? std::min<int64_t>(tiles, std::max<int64_t>(cus, (tiles + 63) / 64)) : tiles;
  if (chain && nwg > cus) nwg = (nwg + cus - 1) / cus * cus;      // whole rounds of workgroups
  nwg = (nwg + 7) / 8 * 8;
  if (nwg > 0x7fffffff || g.groups != 1) return hipErrorInvalidValue;
  if (!g.out_bf16) {
    if (g.f16) hipLaunchKernelGGL(gemm_f16_256_ragged_f32out_kernel, dim3((unsigned)nwg), dim3(256), 0, s, g);
    else hipLaunchKernelGGL(gemm_bf16_256_ragged_f32out_kernel, dim3((unsigned)nwg), dim3(256), 0, s, g);
  } else if (g.f16)
    hipLaunchKernelGGL(gemm_f16_256_ragged_kernel, dim3((unsigned)nwg), dim3(256), 0, s, g);
  else
    hipLaunchKernelGGL(gemm_bf16_256_ragged_kernel, dim3((unsigned)nwg), dim3(256), 0, s, g);
  return hipGetLastError();
}

}  // namespace axe
