// fp8 (OCP e4m3) GEMM for gfx950 (MI355X) with power-of-two block scales (E8M0, one byte per
// 128 x 128 block: value 2^(e - 127)) or none, on the matrix cores' own scale path:
// v_mfma_scale_f32_16x16x128_f8f6f4 multiplies each operand by the scale its lane supplies and
// accumulates in place, so the running sums stay in AGPRs and no vector-ALU fold is needed (the
// kernel for arbitrary fp32 scales has to fold every product on the vector ALU).
//
// Structure and measured reasons are those of the bf16 kernel (kernels_gemm_bf16.hip): workgroup tile
// 256 x 256, one workgroup of 4 waves per CU, wave tile 128 x 128 = 8 x 8 fragments in 256 AGPRs, five
// 32 KiB LDS blocks (both operands direct to LDS: A into two blocks, one K-step ahead, B through a ring of
// three), tiles of a workgroup chained, direct paired stores.
// What differs:
//   K-step      : 128 elements = one LDS row = ONE MFMA per fragment (32 cycles); a K-step is 64 MFMAs,
//                 split in two halves by fragment rows (rows 0..3, rows 4..7), with the barrier
//                 between them.
//   Fragments   : 32 bytes per lane (two ds_read_b128: K chunks q and q + 4, q = lane / 16 -- exactly the
//                 order in which the instruction pairs the bytes of its operands: lane group q holds
//                 k = 16 q .. 16 q + 15 and k = 64 + 16 q .. 64 + 16 q + 15, and the scale of lane
//                 r + 16 b applies to the 32-wide block b of row r; found by experiment).  All 16
//                 fragments of step kt+1 are read in the second half of step kt; rows are processed
//                 in pairs so that a B fragment is re-read right after its last use (row 7) and is
//                 not needed again before 14 MFMAs later.
//   Scales      : two bytes per K-step and wave (its 128 rows and 128 columns lie in one scale block), kept one
//                 per lane for 64 K-steps and broadcast to the lanes.
//   Row scales  : (second instantiation) A carries one code per ROW and 128-wide k block -- the usual choice for
//                 activations -- instead of one per 128 x 128 block.  The instruction takes the scale of a row
//                 from the lanes that hold the row, so nothing changes in the matrix pipe: a lane keeps the codes
//                 of its row of each of the 8 fragment rows for a window of 8 K-steps (8 contiguous bytes of the
//                 row-major (M, K / 128) code array, 16 registers, plus 16 for the window being fetched) and hands
//                 the MFMAs of a K-step one byte of each.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <type_traits>

#include "device_types.h"
#include "gemm_common.h"
#include "grouped_tiles.h"
#include "kernels.h"
#include "tile_maps.h"

namespace axe {

namespace {
constexpr int kRow = maps::kLargeRowBytes;         // bytes of K per LDS row (128 fp8)
constexpr int kBlk = kTile * kRow;                // 32 KiB: one operand, one K-tile
constexpr int kBoff = 2 * kBlk;                   // A: blocks 0, 1 (double buffer); B: blocks 2, 3, 4 (ring)
constexpr int kLds = 5 * kBlk;                    // 160 KiB
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(3))) uint8_t* lds_u8;
__device__ __forceinline__ i32x8 lds_read32(lds_u8 p0, lds_u8 p1) {
  const i32x4 lo = *(__attribute__((address_space(3))) const i32x4*)p0;
  const i32x4 hi = *(__attribute__((address_space(3))) const i32x4*)p1;
  return i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}
// acc += (first * 2^(s_first - 127)) (16 x 128) * (second * 2^(s_second - 127)) (128 x 16), accumulator pinned to
// AGPRs (see the bf16 kernel).  The scale operands are VGPRs whose byte 0 is the E8M0 code.
__device__ __forceinline__ void mfma_scaled(f32x4& acc, i32x8 first, i32x8 second, uint32_t s_first, uint32_t s_second) {
  asm volatile("v_mfma_scale_f32_16x16x128_f8f6f4 %0, %1, %2, %0, %3, %4 op_sel_hi:[0,0,0]"
               : "+a"(acc)
               : "v"(first), "v"(second), "v"(s_first), "v"(s_second));
}
}  // namespace

// ROWS: one E8M0 code per row of A and k block (scale_a is (M, K / 128)) instead of one per 128 x 128 block; B's
// codes are per 128 x 128 block either way.
// GROUPED: the grouped GEMM of an MoE layer in fp8 (rows of A and C sorted by group, group e multiplies its rows with
// its own B; offsets on the device): the tile table, the clipped buffer descriptors and the chained walk of the
// 16-bit grouped kernel (kernels_gemm_bf16.hip), tiles of 256 or 128 rows (MR below), A scaled per row (ROWS), each group's B per
// 128 x 128 block, or no scales at all.
// GATED: B holds each group's gate and up rows interleaved in runs of 16, so that the wave's fragment pair (j, j + 1) is
// (gate, up) of the same 16 outputs; the tile stores silu(gate) * up, half as wide.  The gate and the up columns of a
// wave lie in different 128-wide blocks of the logical matrix: two B codes per K-step.
// MR = fragment rows per wave: 8 (tiles of 256 rows), or 4 for the grouped kernel when groups are small (tiles of 128
// rows, a wave owns 64 x 128: a K-step is 2 x 16 MFMAs per wave and moves half as much of A; as in the 16-bit kernel
// the A blocks in LDS keep their places, half of each is used).
template <bool ROWS, bool GROUPED = false, bool GATED = false, int MR = 8>
__device__ __forceinline__ void gemm_fp8_e8m0_256_body(const GemmArgs& g) {
  static_assert(!GROUPED || ROWS, "the grouped kernel scales A per row");
  static_assert(!GATED || GROUPED, "the gated epilogue exists for the grouped kernel");
  static_assert(MR == 8 || (MR == 4 && GROUPED), "128-row tiles exist for the grouped kernel");
  constexpr int TM = 32 * MR, WR = 16 * MR;                        // rows of a tile, of a wave's part of it
  __shared__ __attribute__((aligned(1024))) uint8_t lds_mem[kLds];
  const lds_u8 lds3 = (lds_u8)lds_mem;                             // 32-bit LDS addresses

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave id 0..3, kept scalar
  const int wm = w >> 1, wn = w & 1;                               // wave grid 2 x 2
  const int nk = (int)(g.K / 128);
  const int ntiles = g.grid_m * g.grid_n;
  const bool scaled = g.scale_a != nullptr;

  // ---- the tiles of this workgroup: blockIdx.x, blockIdx.x + gridDim.x, ... (cur and nxt, see the bf16 kernel);
  //      grouped: lane t of a wave holds the workgroup's t-th tile (grouped_tiles.h)
  const int a_pitch = (int)g.lda, b_pitch = (int)g.ldb;            // bytes
  struct Tile {
    __amdgpu_buffer_rsrc_t ra, rb;
    const uint8_t *sa, *sb, *sb2;                                  // E8M0 codes of this wave's row block (not ROWS) and column block(s), one per K-tile
    int sa_row;                                                    // ROWS: the lane's row of fragment row 0 (fragment row i: 16 i further)
  };
  int tb_row0 = 0, tb_desc = 0;
  if constexpr (GROUPED) group_tiles<TM, false>(g, lane, tb_row0, tb_desc);
  auto table_rows = [&](int t) __attribute__((always_inline)) -> int { return t < 64 ? desc_rows(__builtin_amdgcn_readlane(tb_desc, t)) : 0; };
  auto describe = [&](int v) __attribute__((always_inline)) -> Tile {
    Tile t;
    t.sa = (const uint8_t*)g.scale_a, t.sb = t.sb2 = (const uint8_t*)g.scale_b;   // (valid addresses where the codes are never used)
    t.sa_row = 0;
    if constexpr (GROUPED) {
      const int rows = table_rows(v);
      if (rows > 0) {
        const int row0 = __builtin_amdgcn_readlane(tb_row0, v), dsc = __builtin_amdgcn_readlane(tb_desc, v);
        const int grp = desc_group(dsc), tn = desc_tn(dsc);
        t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.A + (int64_t)row0 * g.lda), 0, (rows - 1) * a_pitch + (int)g.K, 0x00020000);
        t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.B + (int64_t)grp * g.ldg + (int64_t)tn * kTile * g.ldb), 0,
                                                 255 * b_pitch + (int)g.K, 0x00020000);
        t.sa_row = row0 + wm * WR + (lane & 15);
        const int64_t nb = g.N / 128;                              // 128-wide blocks of a group's logical columns
        if constexpr (GATED) {
          // memory rows 256 tn + 128 wn + 16 j + i of the group's image: j even = gate, j odd = up, of the logical columns
          // 128 tn + 64 wn + 16 (j / 2) + i (+ N / 2 for up): block tn of the gate half, block N / 256 + tn of the up half
          t.sb = (const uint8_t*)g.scale_b + ((int64_t)grp * nb + tn) * g.nkb;
          t.sb2 = (const uint8_t*)g.scale_b + ((int64_t)grp * nb + nb / 2 + tn) * g.nkb;
        } else {
          t.sb = t.sb2 = (const uint8_t*)g.scale_b + ((int64_t)grp * nb + 2 * tn + wn) * g.nkb;
        }
        return t;
      }
    }
    if (!GROUPED && v < ntiles) {
      int tm, tn;
      tile_of_block(v, ntiles, g.grid_m, g.grid_n, tm, tn);
      t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.B + (int64_t)tn * kTile * g.ldb), 0,
                                               255 * b_pitch + (int)g.K, 0x00020000);
      t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.A + (int64_t)tm * kTile * g.lda), 0,
                                               255 * a_pitch + (int)g.K, 0x00020000);
      if constexpr (ROWS) t.sa_row = tm * kTile + wm * 128 + (lane & 15);
      else t.sa = (const uint8_t*)g.scale_a + (int64_t)(2 * tm + wm) * g.nkb;
      t.sb = t.sb2 = (const uint8_t*)g.scale_b + (int64_t)(2 * tn + wn) * g.nkb;
    } else {                                                       // no such tile: every load returns zero
      t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)g.B, 0, 0, 0x00020000);
      t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)g.A, 0, 0, 0x00020000);
    }
    return t;
  };
  int v = GROUPED ? 0 : (int)blockIdx.x;
  const int vstep = GROUPED ? 1 : (int)gridDim.x;
  if (GROUPED && table_rows(0) <= 0) return;                       // more workgroups than tiles (the host sizes the launch for the worst case)
  Tile cur = describe(v), nxt = describe(v + vstep);

  // ---- block scales.  The wave's 128 rows and 128 columns lie in one scale block each, so a K-step
  //      needs two codes.  A register per operand holds the codes of 64 consecutive K-steps of the
  //      walk, one per lane; v_readlane hands out one per step.  The registers for the NEXT 64 steps
  //      (of this tile, or the first of the next tile) are fetched when a block of 64 steps begins and
  //      taken over when it ends.  These are ordinary loads: the compiler waits for them before the first
  //      use, once per 64 K-steps or per tile.
  uint32_t cva = 127u, cvb = 127u, nva = 127u, nvb = 127u;        // this block's and the next block's codes, lane = step % 64
  uint32_t cvb2 = 127u, nvb2 = 127u;                               // GATED: the codes of the up half
  auto fetch_codes = [&](const Tile& t, int base, uint32_t& oa, uint32_t& ob, uint32_t& ob2) __attribute__((always_inline)) {
    if (!scaled) return;
    const int T = base + lane;
    const int kt_ = T < nk ? T : nk - 1;
    if constexpr (!ROWS) oa = t.sa[kt_];
    ob = t.sb[kt_];
    if constexpr (GATED) ob2 = t.sb2[kt_];
  };
  // Row scales.  The codes of a row for a window of 8 K-steps are 8 contiguous bytes of the row-major (M, K / 128)
  // array (of the last, partial window fewer: the load then runs on into the next row, or, at the very end of the
  // array, starts earlier and is shifted down).  na: the window being fetched, as loaded; ca: the current window,
  // step t of the window uses byte t: the lowest byte now, moved down by one byte per step.  Without scales all
  // codes are 127 (2^0).
  uint32_t ca[MR][2], na[MR][2];
#pragma unroll
  for (int i = 0; i < MR; ++i) ca[i][0] = ca[i][1] = na[i][0] = na[i][1] = 0x7f7f7f7fu;
  bool more = false;                                               // the workgroup has another tile after the current one
  // where the 8 bytes of (row of fragment row i, window win) are read from, and by how many bytes that read starts
  // early (only at the very end of the array).  32-bit arithmetic: the host admits code arrays below 2^31 bytes.
  const int codes_total = (int)(g.M * (int64_t)g.nkb);             // bytes of the code array (at least 8)
  const int codes_last_row = codes_total - g.nkb;
  auto row_codes_at = [&](int sa_row, int i, int win, int& at, int& over) __attribute__((always_inline)) {
    int off = (sa_row + 16 * i) * g.nkb;
    off = off < codes_last_row ? off : codes_last_row;             // rows past the end belong to no group: their codes are never used
    off += 8 * win;
    at = off < codes_total - 8 ? off : codes_total - 8;
    over = off - at;
  };
  auto fetch_rows = [&](const Tile& t, int win) __attribute__((always_inline)) {
    if (!scaled) return;
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      int at, over;
      row_codes_at(t.sa_row, i, win, at, over);
      uint64_t c;
      __builtin_memcpy(&c, (const uint8_t*)g.scale_a + at, 8);
      na[i][0] = (uint32_t)c, na[i][1] = (uint32_t)(c >> 32);      // (used 8 K-steps later: nothing here may wait for the load)
    }
  };
  // na -> ca at the first step of window win of the current tile: shifted down if the read started early
  auto take_rows = [&](int win) __attribute__((always_inline)) {
    if (!scaled) {                                                 // a fresh window of codes 127 (the steps shift them out)
#pragma unroll
      for (int i = 0; i < MR; ++i) ca[i][0] = ca[i][1] = 0x7f7f7f7fu;
      return;
    }
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      int at, over;
      row_codes_at(cur.sa_row, i, win, at, over);
      const uint64_t c = (((uint64_t)na[i][1] << 32) | na[i][0]) >> (8 * over);
      ca[i][0] = (uint32_t)c, ca[i][1] = (uint32_t)(c >> 32);
    }
  };
  auto lane_value = [](uint32_t val, int l) -> uint32_t { return (uint32_t)__builtin_amdgcn_readlane((int)val, l); };

  // ---- HBM -> LDS, both operands directly (as in the bf16 kernel; pitches and columns in bytes = elements): a wave
  //      instruction fills 8 rows x 128 bytes linearly in the lane id, so the XOR of the LDS image is applied to
  //      the chunk a lane fetches.  A has two blocks (the steps of either parity), B a ring of three.
  const int lr = lane / maps::kLargeChunks, lp = lane % maps::kLargeChunks;
  const int lrow = maps::piece_row(w, 0, lr, 4);                   // row of piece 0; piece i lies 32 i rows further (same key)
  const int a_voff_x = lrow * a_pitch + maps::lds_chunk_pos(lrow, lp, maps::kLargeChunks) * maps::kChunkBytes;
  const int b_voff = lrow * b_pitch + maps::lds_chunk_pos(lrow, lp, maps::kLargeChunks) * maps::kChunkBytes;
  const int a_piece = maps::piece_row(0, 1, 0, 4) * a_pitch, b_piece = maps::piece_row(0, 1, 0, 4) * b_pitch;   // bytes between pieces
  // (the piece goes into the per-lane offset, one register per piece: the scalar offset is the K-tile's alone)
  int a_voff_p[MR], b_voff_p[8];                                   // (A: MR pieces of 8 rows per wave and K-step)
#pragma unroll
  for (int i = 0; i < MR; ++i) a_voff_p[i] = a_voff_x + i * a_piece;
#pragma unroll
  for (int i = 0; i < 8; ++i) b_voff_p[i] = b_voff + i * b_piece;
  auto a_dload = [&](int T, int i, bool cross) __attribute__((always_inline)) {   // piece i of step T into the A block of its parity
    const bool nx = cross && T >= nk;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(nx ? nxt.ra : cur.ra, (lds_ptr)(lds3 + (T & 1) * kBlk + maps::piece_row(w, i, 0, 4) * kRow), 16, a_voff_p[i],
                                             (nx ? T - nk : T) * kRow, 0, 0);   // (K-step T >= nk: step T - nk of the next tile)
    AXE_PARANOID_WAIT();
  };
  int bo0 = kBoff, bo1 = kBoff + kBlk, bo2 = kBoff + 2 * kBlk;     // B ring: blocks of K-steps kt, kt+1, kt+2
  auto b_load = [&](int T, int i, int slot_off, bool cross) __attribute__((always_inline)) {
    const bool nx = cross && T >= nk;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(nx ? nxt.rb : cur.rb, (lds_ptr)(lds3 + slot_off + maps::piece_row(w, i, 0, 4) * kRow), 16, b_voff_p[i],
                                             (nx ? T - nk : T) * kRow, 0, 0);
    AXE_PARANOID_WAIT();
  };

  // ---- LDS -> VGPR: fragment f of this wave's A (B) rows: row = base + f * 16 + lane % 16, chunks q and q + 4
  const int fr = lane % maps::kFrag, fq = lane / maps::kFrag;
  const int pos0 = maps::lds_chunk_pos(fr, maps::operand_chunk_fp8(0, fq), maps::kLargeChunks) * maps::kChunkBytes;
  const int pos1 = maps::lds_chunk_pos(fr, maps::operand_chunk_fp8(1, fq), maps::kLargeChunks) * maps::kChunkBytes;
  const lds_u8 fax0 = lds3 + (wm * WR + fr) * kRow + pos0;
  const lds_u8 fax1 = lds3 + (wm * WR + fr) * kRow + pos1;
  const lds_u8 fbx0 = lds3 + (wn * 128 + fr) * kRow + pos0;
  const lds_u8 fbx1 = lds3 + (wn * 128 + fr) * kRow + pos1;
  auto read_a = [&](int f, int off) __attribute__((always_inline)) -> i32x8 {
    return lds_read32(fax0 + off + f * 16 * kRow, fax1 + off + f * 16 * kRow);
  };
  auto read_b = [&](int f, int off) __attribute__((always_inline)) -> i32x8 {
    return lds_read32(fbx0 + off + f * 16 * kRow, fbx1 + off + f * 16 * kRow);
  };

  f32x4 acc[MR][8];
#pragma unroll
  for (int i = 0; i < MR; ++i)
#pragma unroll
    for (int j = 0; j < 8; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  i32x8 fa[MR], fb[8];      // all fragments of the current K-step; each is re-read for the next step right after its last use

  // ---- VGPR -> HBM (as in the bf16 kernel: fragment pairs exchange halves, 16 bytes per lane)
  i32x4 rc;
  int c_rowblk;
  int c_nfr = MR;                                                  // grouped: fragment rows of this wave that hold rows of the tile
  const int c_voff2 = (int)((fr * g.ldc + maps::pair_store_col(fq)) * 2);
  auto set_output = [&](int vv) __attribute__((always_inline)) {
    if constexpr (GROUPED) {
      const int row0 = __builtin_amdgcn_readlane(tb_row0, vv), dsc = __builtin_amdgcn_readlane(tb_desc, vv);
      const int tn = desc_tn(dsc);
      int rows = desc_rows(dsc) - wm * WR;                           // rows of the tile that fall to this wave
      rows = rows < 0 ? 0 : (rows > WR ? WR : rows);
      c_nfr = (rows + 15) >> 4;
      constexpr int CW = GATED ? 64 : 128;                           // columns of C this wave writes
      rc = raw_rsrc((uint16_t*)g.C + ((int64_t)row0 + wm * WR) * g.ldc + (int64_t)tn * (2 * CW) + wn * CW,
                    rows ? (uint32_t)(((rows - 1) * g.ldc + CW) * 2) : 0u);   // the stores of rows the group does not have are dropped
      c_rowblk = (int)(16 * g.ldc * 2);
      return;
    }
    int tm, tn;
    tile_of_block(vv, ntiles, g.grid_m, g.grid_n, tm, tn);
    rc = raw_rsrc((uint16_t*)g.C + ((int64_t)tm * kTile + wm * 128) * g.ldc + (int64_t)tn * kTile + wn * 128,
                  (uint32_t)((127 * g.ldc + 128) * 2));
    c_rowblk = (int)(16 * g.ldc * 2);
  };
  auto store_fragment_pair = [&](int i, int j) __attribute__((always_inline)) {
    const auto lo = __builtin_amdgcn_permlane16_swap(pack_bf16(acc[i][j][0], acc[i][j][1]),
                                                     pack_bf16(acc[i][j + 1][0], acc[i][j + 1][1]), false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(pack_bf16(acc[i][j][2], acc[i][j][3]),
                                                     pack_bf16(acc[i][j + 1][2], acc[i][j + 1][3]), false, false);
    const u32x4 d = {lo[0], hi[0], lo[1], hi[1]};
    const int soff = __builtin_amdgcn_readfirstlane(i * c_rowblk + j * 32);
    asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, %3 offen" AXE_AFTER_STORE ::"v"(d), "v"(c_voff2), "s"(rc), "s"(soff) : "memory");
    AXE_PARANOID_WAIT();
  };

  // Gated epilogue (see the 16-bit grouped kernel): h = silu(gate) * up for the fragment pairs (j, j + 1) and
  // (j + 2, j + 3), stored like a fragment pair (32 output columns, 64 contiguous bytes per row).
  auto store_gated_quad = [&](int i, int j) __attribute__((always_inline)) {
    float h[2][4];
#pragma unroll
    for (int q = 0; q < 2; ++q)
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        const float gate = acc[i][j + 2 * q][e], up = acc[i][j + 2 * q + 1][e];
        h[q][e] = gate * __builtin_amdgcn_rcpf(1.0f + __expf(-gate)) * up;
      }
    const auto lo = __builtin_amdgcn_permlane16_swap(pack_bf16(h[0][0], h[0][1]), pack_bf16(h[1][0], h[1][1]), false, false);
    const auto hi = __builtin_amdgcn_permlane16_swap(pack_bf16(h[0][2], h[0][3]), pack_bf16(h[1][2], h[1][3]), false, false);
    const u32x4 d = {lo[0], hi[0], lo[1], hi[1]};
    const int soff = __builtin_amdgcn_readfirstlane(i * c_rowblk + j * 16);
    asm volatile("s_nop 4\n\tbuffer_store_dwordx4 %0, %1, %2, %3 offen" AXE_AFTER_STORE ::"v"(d), "v"(c_voff2), "s"(rc), "s"(soff) : "memory");
    AXE_PARANOID_WAIT();
  };

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;

  // Half H of K-step kt (PAR = kt & 1), in exact program order: fragment rows 4 H .. 4 H + 3, two rows at a
  // time with j innermost: MFMAs (r, j), (r + 1, j) for even j and (r + 1, j), (r, j) for odd j -- 2 x 2 blocks walked
  // as a snake, the order in which this MFMA draws least power (register-only loop on e4m3 data: 4415 TFLOP/s against
  // 4325 with (r, j), (r + 1, j) throughout and 4400 row by row; the ranking differs from the 16-bit MFMA's).  Loads: in the first half pieces 4..7 of B of step kt + 2
  // (after MFMAs 2, 10, 18, 26); in the second half, after the barrier has freed what step kt occupied, the 8
  // pieces of A of step kt + 2 (after MFMAs 0, 2, .., 14: they have one K-step to land) and pieces 0..3 of B of
  // step kt + 3 (after MFMAs 18, 22, 26, 30).  The second half also reads the 16 fragments of step kt+1, each right after the
  // last MFMA that uses the register it goes to: A fragments 0..3 during rows 4, 5; A fragments 4, 5
  // and, after MFMA (7, j), B fragment j during rows 6, 7; A fragments 6, 7 at the end.
  // With 4 fragment rows per wave (MR = 4) a half is one pair of rows, 16 MFMAs: the first half loads pieces 4..7 of B
  // of step kt + 2 (after MFMAs 2, 6, 10, 14); the second the 4 pieces of A of step kt + 2 (after MFMAs 0, 2, 4, 6) and
  // pieces 0..3 of B of step kt + 3 (after MFMAs 8, 10, 12, 14), and reads step kt + 1: A fragments 0, 1 after MFMAs
  // 1, 3, B fragment j after MFMA (3, j), A fragments 2, 3 at the end.
  auto half = [&](auto par_c, auto h_c, auto cross_c, int kt, const uint32_t (&va)[MR], uint32_t vb, uint32_t vb2, bool pref) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_c)::value, H = decltype(h_c)::value;
    constexpr bool CROSS = decltype(cross_c)::value != 0;
    const int bT = H == 0 ? kt + 2 : kt + 3;
    const int bslot = H == 0 ? bo2 : bo0;
    constexpr int pa = (PAR ^ 1) * kBlk;                           // step kt+1: A stage, B ring block
    const int pb = bo1;
#pragma unroll
    for (int q = 0; q < 4 * MR; ++q) {
      const int i = (MR / 2) * H + 2 * (q >> 4) + ((q & 1) ^ ((q >> 1) & 1)), j = (q >> 1) & 7;
      mfma_scaled(acc[i][j], fb[j], fa[i], (GATED && (j & 1)) ? vb2 : vb, va[ROWS ? i : 0]);
      __builtin_amdgcn_sched_barrier(0);
      if constexpr (ROWS && H == 1) {
        // the row codes of the next window of the walk (of this tile, or the first of the next tile), once per 8
        // K-steps, before the A pieces: older than they are, so complete at the next barrier at the latest
        if (q == 0 && pref) {
          if (kt + 8 < nk) fetch_rows(cur, (kt >> 3) + 1);
          else if (more) fetch_rows(nxt, 0);
        }
      }
      if constexpr (MR == 8) {
        if (H == 1) {
          if (q < 16 && (q & 3) == 1) fa[q >> 2] = read_a(q >> 2, pa);
          if (q == 16) fa[4] = read_a(4, pa);
          if (q == 18) fa[5] = read_a(5, pa);
          if (q >= 16 && (q & 1) == 1) fb[j] = read_b(j, pb);
          if (q == 31) {
            fa[6] = read_a(6, pa);
            fa[7] = read_a(7, pa);
          }
        }
        if (H == 0) {
          if ((q & 7) == 2) b_load(bT, 4 + (q >> 3), bslot, CROSS);
        } else {
          if (q < 16 && (q & 1) == 0) a_dload(kt + 2, q >> 1, CROSS);
          if (q >= 16 && (q & 3) == 2) b_load(bT, (q - 16) >> 2, bslot, CROSS);
        }
      } else {
        if (H == 1) {
          if (q == 1) fa[0] = read_a(0, pa);
          if (q == 3) fa[1] = read_a(1, pa);
          if ((q & 1) == 1) fb[j] = read_b(j, pb);
          if (q == 15) {
            fa[2] = read_a(2, pa);
            fa[3] = read_a(3, pa);
          }
        }
        if (H == 0) {
          if ((q & 3) == 2) b_load(bT, 4 + (q >> 2), bslot, CROSS);
        } else {
          if (q < 8 && (q & 1) == 0) a_dload(kt + 2, q >> 1, CROSS);
          if (q >= 8 && (q & 1) == 0) b_load(bT, (q - 8) >> 1, bslot, CROSS);
        }
      }
      __builtin_amdgcn_sched_barrier(0);
      if ((q & 7) == 7) AXE_PARANOID_SYNC();
    }
    if (H == 0) {
      // Own loads of step kt+1 are complete (its last A piece was followed by 8 B loads, which may still be in
      // flight); nobody has read LDS since the last barrier's second half.  After the barrier step kt+1 is
      // readable by every wave and the blocks of step kt are free.
      asm volatile("s_waitcnt vmcnt(8) lgkmcnt(0)" ::: "memory");
      wg_barrier();
    }
  };
  auto step = [&](auto par_c, auto cross_c, int kt, bool pref = false) __attribute__((always_inline)) {
    uint32_t va[MR], vb = lane_value(cvb, kt & 63), vb2 = GATED ? lane_value(cvb2, kt & 63) : 0u;
    // the codes are now in VGPRs, written by the vector ALU; the MFMA is an asm statement, so the compiler's
    // hazard recogniser cannot pad between that write and the matrix core's read of its scale operands
    if constexpr (ROWS) {
      // step t of the window uses byte t of the codes: the lowest byte now, then the 64 bits move down by one
      // byte (no register is ever indexed by t: that would put the array into scratch memory)
#pragma unroll
      for (int i = 0; i < MR; ++i) {
        va[i] = ca[i][0] & 0xffu;
        ca[i][0] = __builtin_amdgcn_alignbit(ca[i][1], ca[i][0], 8);
        ca[i][1] >>= 8;
      }
      if constexpr (MR == 4)
        asm volatile("s_nop 3" : "+v"(va[0]), "+v"(va[1]), "+v"(va[2]), "+v"(va[3]), "+v"(vb), "+v"(vb2));
      else if constexpr (GATED)
        asm volatile("s_nop 3" : "+v"(va[0]), "+v"(va[1]), "+v"(va[2]), "+v"(va[3]), "+v"(va[4 % MR]), "+v"(va[5 % MR]), "+v"(va[6 % MR]), "+v"(va[7 % MR]), "+v"(vb), "+v"(vb2));
      else
        asm volatile("s_nop 3" : "+v"(va[0]), "+v"(va[1]), "+v"(va[2]), "+v"(va[3]), "+v"(va[4 % MR]), "+v"(va[5 % MR]), "+v"(va[6 % MR]), "+v"(va[7 % MR]), "+v"(vb));
    } else {
      va[0] = lane_value(cva, kt & 63);
      asm volatile("s_nop 3" : "+v"(va[0]), "+v"(vb));
    }
    half(par_c, I0{}, cross_c, kt, va, vb, vb2, pref);
    half(par_c, I1{}, cross_c, kt, va, vb, vb2, pref);
    const int t = bo0;
    bo0 = bo1, bo1 = bo2, bo2 = t;
  };
  // ROWS: at the first step of a window of 8 the codes fetched during the previous window are taken over and the
  // step fetches the next window's
  auto window = [&](int kt) __attribute__((always_inline)) -> bool {
    if constexpr (ROWS) {
      if ((kt & 7) == 0) {
        take_rows(kt >> 3);
        return true;
      }
    }
    return false;
  };

  // ---- prologue (first tile only): steps 0 and 1 of A, steps 0, 1 and half of 2 of B
  //      Step 0 of both operands and the scale codes first: the MFMAs start as soon as these have landed (the MR + 12 loads
  //      of step 1 and of step 2's first half may still be in flight, as at the barrier of every later step).
#pragma unroll
  for (int i = 0; i < MR; ++i) a_dload(0, i, true);
#pragma unroll
  for (int i = 0; i < 8; ++i) b_load(0, i, bo0, true);
  fetch_codes(cur, 0, cva, cvb, cvb2);
  if constexpr (ROWS) fetch_rows(cur, 0);
#pragma unroll
  for (int i = 0; i < MR; ++i) a_dload(1, i, true);                // (a single K-step per tile: step 1 is the next tile's step 0)
#pragma unroll
  for (int i = 0; i < 8; ++i) b_load(1, i, bo1, true);
#pragma unroll
  for (int i = 0; i < 4; ++i) b_load(2, i, bo2, true);
  asm volatile("s_waitcnt vmcnt(%0)" ::"n"(MR + 12) : "memory");
  wg_barrier();
#pragma unroll
  for (int f = 0; f < 8; ++f) fb[f] = read_b(f, bo0);
#pragma unroll
  for (int f = 0; f < MR; ++f) fa[f] = read_a(f, 0);

  // ---- all K-steps of all tiles of this workgroup, one uninterrupted pipeline (nk even and >= 4 when chained)
  for (;;) {
    set_output(v);
    more = GROUPED ? table_rows(v + 1) > 0 : v + vstep < ntiles;
    int kt = 0;
    for (int base = 0; base < nk; base += 64) {
      const int end = nk < base + 64 ? nk : base + 64;
      // the next 64 steps of the walk: of this tile, or the first of the next tile
      if (end < nk) fetch_codes(cur, end, nva, nvb, nvb2);
      else if (more) fetch_codes(nxt, 0, nva, nvb, nvb2);
      for (; kt + 1 < end && kt + 5 < nk; kt += 2) {               // every load of these steps is of this tile (at most step kt + 5)
        step(I0{}, I0{}, kt, window(kt));
        step(I1{}, I0{}, kt + 1);
      }
      for (; kt + 1 < end; kt += 2) {                              // the last steps load the next tile's first K-steps
        step(I0{}, I1{}, kt, window(kt));
        step(I1{}, I1{}, kt + 1);
      }
      if (kt < end) {                                              // odd nk: only with one tile per workgroup
        step(I0{}, I1{}, kt, window(kt));
        ++kt;
      }
      if (end < nk) cva = nva, cvb = nvb, cvb2 = nvb2;
    }
    asm volatile("s_nop 15\n\ts_nop 15" ::: "memory");             // the last MFMAs retire before their results are read
    __builtin_amdgcn_sched_barrier(0);
#pragma unroll
    for (int i = 0; i < MR; ++i) {
      // grouped: a fragment row without rows of the tile issues no stores (see the 16-bit kernel)
      if (!GROUPED || i < c_nfr) {
        if constexpr (GATED) {
#pragma unroll
          for (int j = 0; j < 8; j += 4) store_gated_quad(i, j);
        } else {
#pragma unroll
          for (int j = 0; j < 8; j += 2) store_fragment_pair(i, j);
        }
      }
#pragma unroll
      for (int j = 0; j < 8; ++j)
#pragma unroll
        for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;            // ready for the next tile
    }
    v += vstep;
    if (GROUPED ? table_rows(v) <= 0 : v >= ntiles) break;
    cva = nva, cvb = nvb, cvb2 = nvb2;
    cur = nxt;
    nxt = describe(v + vstep);
  }
}

__global__ __launch_bounds__(256, 1) void gemm_fp8_e8m0_256_kernel(GemmArgs g) { gemm_fp8_e8m0_256_body<false>(g); }
__global__ __launch_bounds__(256, 1) void gemm_fp8_e8m0_256_rows_kernel(GemmArgs g) { gemm_fp8_e8m0_256_body<true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_fp8_e8m0_256_grouped_kernel(GemmArgs g) { gemm_fp8_e8m0_256_body<true, true>(g); }
__global__ __launch_bounds__(256, 1) void gemm_fp8_e8m0_256_grouped_gated_kernel(GemmArgs g) { gemm_fp8_e8m0_256_body<true, true, true>(g); }
// grouped, tiles of 128 rows (small groups)
__global__ __launch_bounds__(256, 1) void gemm_fp8_e8m0_128_grouped_kernel(GemmArgs g) { gemm_fp8_e8m0_256_body<true, true, false, 4>(g); }
__global__ __launch_bounds__(256, 1) void gemm_fp8_e8m0_128_grouped_gated_kernel(GemmArgs g) { gemm_fp8_e8m0_256_body<true, true, true, 4>(g); }

hipError_t launch_gemm_fp8_e8m0_256(const GemmArgs& g, hipStream_t s) {
  const int ntiles = g.grid_m * g.grid_n;
  const int nk = (int)(g.K / 128);
  const int cus = cu_count();
  const bool chain = (nk % 2 == 0) && nk >= 4 && ntiles > cus && (cus % 8 == 0);
  unsigned nwg = (unsigned)(chain ? cus : ntiles);
  if (g.scale_a && g.scale_a_rows == 1) {
    if (!g.scale_e8m0 || g.M * (int64_t)g.nkb < 8 || g.M * (int64_t)g.nkb >= (int64_t(1) << 30)) return hipErrorInvalidValue;   // (a row's codes are fetched 8 bytes at a time, 32-bit offsets)
    hipLaunchKernelGGL(gemm_fp8_e8m0_256_rows_kernel, dim3(nwg), dim3(256), 0, s, g);
  } else
    hipLaunchKernelGGL(gemm_fp8_e8m0_256_kernel, dim3(nwg), dim3(256), 0, s, g);
  return hipGetLastError();
}

// Grouped (see launch_gemm_bf16_256_grouped): the host knows only that sum_e ceil(rows_e / TM) <= M / TM + groups.
hipError_t launch_gemm_fp8_e8m0_256_grouped(const GemmArgs& g, hipStream_t s) {
  if (g.scale_a && (!g.scale_e8m0 || g.M * (int64_t)g.nkb < 8 || g.M * (int64_t)g.nkb >= (int64_t(1) << 30))) return hipErrorInvalidValue;
  const bool t128 = grouped_fp8_tile_rows(g.M, g.groups, g.tile_m) == 128;
  const int64_t worst = (g.M / (t128 ? 128 : kTile) + g.groups) * (int64_t)g.grid_n;
  const int nk = (int)(g.K / 128);
  const int cus = cu_count();
  const bool chain = (nk % 2 == 0) && nk >= 4;
  int64_t nwg = chain ? std::max<int64_t>(cus, (worst + 63) / 64) : worst;
  if (chain && nwg > cus) nwg = (nwg + cus - 1) / cus * cus;      // more workgroups than compute units only in whole rounds
  nwg = (nwg + 7) / 8 * 8;                                         // the tile sequence is cut into 8 parts, one per XCD
  if (nwg > 0x7fffffff) return hipErrorInvalidValue;
  const dim3 grid((unsigned)nwg), block(256);
  switch ((t128 ? 2 : 0) + (g.gated ? 1 : 0)) {
    case 0: hipLaunchKernelGGL(gemm_fp8_e8m0_256_grouped_kernel, grid, block, 0, s, g); break;
    case 1: hipLaunchKernelGGL(gemm_fp8_e8m0_256_grouped_gated_kernel, grid, block, 0, s, g); break;
    case 2: hipLaunchKernelGGL(gemm_fp8_e8m0_128_grouped_kernel, grid, block, 0, s, g); break;
    default: hipLaunchKernelGGL(gemm_fp8_e8m0_128_grouped_gated_kernel, grid, block, 0, s, g); break;
  }
  return hipGetLastError();
}

}  // namespace axe
