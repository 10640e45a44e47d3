// fp8 (OCP e4m3) GEMM for gfx950 (MI355X) with optional fp32 scales per 128 x 128 block: workgroup
// tile 256 x 256 x 128, 8 waves (two per SIMD), each a 128 x 64 sub-tile = 8 x 4 MFMA 16x16x128
// fragments.  A row-major, B column-major (both K contiguous).
//
// One K-tile is one 128-deep scale block and one MFMA per fragment: every MFMA starts from a zero
// accumulator, and its result P is folded into the running sum on the vector ALU,
// acc += (sA * sB) * P, three MFMAs later.  The vector ALU cannot address the AGPR half of the
// register file, so the running sums live in ordinary VGPRs; that is what sets the wave tile: 128
// accumulator registers, four P buffers, four A and four B fragments of 8 registers each stay below
// the 256 registers a wave has when two waves share a SIMD.
//
// Tile movements, each an Axe layout (the LDS side as in the bf16 kernel, reported by axe_gemm_describe):
//   HBM -> LDS  : buffer_load ... lds, 16 bytes per lane straight into LDS; one wave instruction
//                 covers 8 rows x 128 bytes.  The LDS side of such a load is linear in the lane id,
//                 so the XOR swizzle is applied on the global side: lane (r = lane / 8, p = lane % 8)
//                 fetches chunk p ^ key(r) of row r.
//   LDS layout  : five 32 KiB blocks (one operand, one K-tile each): A double-buffered in blocks 0, 1,
//                 B in a ring of blocks 2, 3, 4.  Rows of 128 bytes (128 fp8); 16-byte chunk c of row r
//                 sits at chunk position c ^ key(r), key(r) = (r >> 1) & 7 (64 LDS banks: conflict-free).
//   LDS -> VGPR : lane l reads row l % 16 of a fragment and the 16-byte chunks l / 16 and l / 16 + 4.
//                 MFMA 16x16x128 multiplies the 32 bytes of a lane of A with the 32 bytes of the
//                 same lane group of B; which k they are is free as long as A and B agree, and
//                 this choice keeps the reads free of bank conflicts: an LDS unit serves a
//                 16-byte-per-lane read 16 lanes at a time, lanes 0-3, 12-15, 20-23, 24-27 together
//                 and then 4-7, 8-11, 16-19, 28-31 (measured: with adjacent chunks 2 q, 2 q + 1
//                 every read took 8 LDS cycles instead of 4), so neighbouring lane groups must
//                 differ in chunk bit 0 for the key below to separate them.
//   VGPR -> HBM : accumulators -> bf16, 8 bytes per lane and fragment, stored directly (the four
//                 fragments of a fragment row complete 128 contiguous bytes per row; L2 merges them).
//
// Schedule.  A K-step is 32 MFMAs per wave, fragment (i, j) with j innermost.  A fragments are read
// three rows ahead of their use, so every LDS read of A of tile kt has been issued when row 4 ends;
// the B fragments of a tile are read during the last row of the tile before.  One workgroup barrier
// per K-step, after row 4: it publishes tile kt+1 and frees the A block of tile kt and the B block of
// tile kt (read at the end of step kt-1).  Between two barriers a wave issues A of tile kt+2 (into
// the block just freed: one K-step to land, so it goes first) and then B of tile kt+3 (ring of
// three blocks: a little more than one K-step).
// The workgroup -> tile order and the chaining of a workgroup's tiles into one
// pipeline are those of the bf16 kernel.  (Measured: chaining gains nothing here.  With the MFMAs
// taken out, the loads, LDS reads and barriers of this kernel alone run at the equivalent of 4.9
// PFLOP/s -- 19 TB/s from the L2s, about what they deliver -- and a register-only loop of the MFMAs
// and folds alone runs at 4.9 PFLOP/s as well: two streams that each nearly fill the time overlap
// imperfectly.  The L2 -> CU path carries twice the bytes per flop of the bf16 kernel; a larger
// tile would need more accumulator registers than two waves per SIMD have.)
#include <hip/hip_runtime.h>

#include <type_traits>

#include "device_types.h"
#include "gemm_common.h"
#include "kernels.h"
#include "tile_maps.h"

namespace axe {

namespace {
constexpr int kRow = maps::kLargeRowBytes;         // bytes of K per LDS row (128 fp8)
constexpr int kBlk = kTile * kRow;                // 32 KiB: one operand, one K-tile
constexpr int kBoff = 2 * kBlk;                   // A: blocks 0, 1 (double buffer); B: blocks 2, 3, 4 (ring)
constexpr int kLds = 5 * kBlk;                    // 160 KiB
constexpr int kFD = 3;                            // an MFMA's result is folded into the running sum kFD MFMAs later
constexpr int kNP = 4;                            // product buffers (a power of two above kFD)
typedef __attribute__((address_space(3))) void* lds_ptr;
typedef __attribute__((address_space(3))) uint8_t* lds_u8;
__device__ __forceinline__ i32x8 lds_read32(lds_u8 p0, lds_u8 p1) {
  const i32x4 lo = *(__attribute__((address_space(3))) const i32x4*)p0;
  const i32x4 hi = *(__attribute__((address_space(3))) const i32x4*)p1;
  return i32x8{lo[0], lo[1], lo[2], lo[3], hi[0], hi[1], hi[2], hi[3]};
}
}  // namespace

__global__ __launch_bounds__(512, 1) void gemm_fp8_256_kernel(GemmArgs g) {
  __shared__ __attribute__((aligned(1024))) uint8_t lds_mem[kLds];
  const lds_u8 lds3 = (lds_u8)lds_mem;                             // 32-bit LDS addresses

  const int tid = threadIdx.x;
  const int lane = tid & 63;
  const int w = __builtin_amdgcn_readfirstlane(tid >> 6);          // wave id 0..7, kept scalar
  const int wm = w >> 2, wn = w & 3;                               // wave grid 2 x 4
  const int nk = (int)(g.K / 128);
  const int ntiles = g.grid_m * g.grid_n;
  const bool scaled = g.scale_a != nullptr;

  // ---- the tiles of this workgroup: blockIdx.x, blockIdx.x + gridDim.x, ...  The loads run two
  //      K-steps ahead of the MFMAs and cross into the next tile before the current one is finished,
  //      so two tiles are described at any time: cur and nxt.
  const int a_pitch = (int)g.lda, b_pitch = (int)g.ldb;            // bytes
  struct Tile {
    __amdgpu_buffer_rsrc_t ra, rb;
    const float *sa, *sb;                                          // block scales of this wave's rows (A) and columns (B)
  };
  auto describe = [&](int v) __attribute__((always_inline)) -> Tile {
    Tile t;
    if (v < ntiles) {
      int tm, tn;
      tile_of_block(v, ntiles, g.grid_m, g.grid_n, tm, tn);
      t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.A + (int64_t)tm * kTile * g.lda), 0,
                                               255 * a_pitch + (int)g.K, 0x00020000);
      t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.B + (int64_t)tn * kTile * g.ldb), 0,
                                               255 * b_pitch + (int)g.K, 0x00020000);
      t.sa = scaled ? g.scale_a + (int64_t)(2 * tm + wm) * g.nkb : nullptr;
      t.sb = scaled ? g.scale_b + (int64_t)(2 * tn + (wn >> 1)) * g.nkb : nullptr;
    } else {                                                       // no such tile: every load returns zero
      t.ra = __builtin_amdgcn_make_buffer_rsrc((void*)g.A, 0, 0, 0x00020000);
      t.rb = __builtin_amdgcn_make_buffer_rsrc((void*)g.B, 0, 0, 0x00020000);
      t.sa = t.sb = nullptr;
    }
    return t;
  };
  int v = blockIdx.x;
  Tile cur = describe(v), nxt = describe(v + (int)gridDim.x);

  // ---- HBM -> LDS.  Per K-tile and operand 32 wave instructions of 8 rows; wave w issues pieces
  //      i = 0..3 = row groups w, w + 8, w + 16, w + 24.  Step T >= nk of the current tile is step
  //      T - nk of the next one (cross = false: the caller knows T < nk).
  const int lr = lane / maps::kLargeChunks, lp = lane % maps::kLargeChunks;
  const int lrow = maps::piece_row(w, 0, lr, 8);                   // row of piece 0; piece i lies 64 i rows further (same key)
  const int a_voff = lrow * a_pitch + maps::lds_chunk_pos(lrow, lp, maps::kLargeChunks) * maps::kChunkBytes;
  const int b_voff = lrow * b_pitch + maps::lds_chunk_pos(lrow, lp, maps::kLargeChunks) * maps::kChunkBytes;
  const int a_piece = maps::piece_row(0, 1, 0, 8) * a_pitch, b_piece = maps::piece_row(0, 1, 0, 8) * b_pitch;   // bytes between pieces
  auto a_load = [&](int T, int i, int stage, bool cross) __attribute__((always_inline)) {
    const bool nx = cross && T >= nk;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(nx ? nxt.ra : cur.ra, (lds_ptr)(lds3 + stage * kBlk + maps::piece_row(w, i, 0, 8) * kRow), 16,
                                             a_voff, i * a_piece + (nx ? T - nk : T) * kRow, 0, 0);
    AXE_PARANOID_WAIT();
  };
  // B ring: byte offsets of the blocks that hold tiles kt, kt+1, kt+2 (tile kt+3 reuses the first)
  int bo0 = kBoff, bo1 = kBoff + kBlk, bo2 = kBoff + 2 * kBlk;
  auto b_load = [&](int T, int i, int slot_off, bool cross) __attribute__((always_inline)) {
    const bool nx = cross && T >= nk;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(nx ? nxt.rb : cur.rb, (lds_ptr)(lds3 + slot_off + maps::piece_row(w, i, 0, 8) * kRow), 16,
                                             b_voff, i * b_piece + (nx ? T - nk : T) * kRow, 0, 0);
    AXE_PARANOID_WAIT();
  };

  // ---- LDS -> VGPR: fragment f of this wave's A (B) rows: row = base + f * 16 + lane % 16; the lane's
  //      32 bytes are the chunks q and q + 4 (q = lane / 16), found at positions q ^ key, (q + 4) ^ key
  const int fr = lane % maps::kFrag, fq = lane / maps::kFrag;
  const int pos0 = maps::lds_chunk_pos(fr, maps::operand_chunk_fp8(0, fq), maps::kLargeChunks) * maps::kChunkBytes;
  const int pos1 = maps::lds_chunk_pos(fr, maps::operand_chunk_fp8(1, fq), maps::kLargeChunks) * maps::kChunkBytes;
  const lds_u8 fa0 = lds3 + (wm * 128 + fr) * kRow + pos0;
  const lds_u8 fa1 = lds3 + (wm * 128 + fr) * kRow + pos1;
  const lds_u8 fb0 = lds3 + (wn * 64 + fr) * kRow + pos0;
  const lds_u8 fb1 = lds3 + (wn * 64 + fr) * kRow + pos1;

  f32x4 acc[8][4];
#pragma unroll
  for (int i = 0; i < 8; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j)
#pragma unroll
      for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;

  // Block scales: one product sA * sB per K-step of this wave.  A register holds those of 64
  // consecutive K-steps, one per lane (no scalar or vector memory access in the steady loop); it is
  // refilled every 64 steps.
  auto scales_from = [&](int base) -> float {
    if (!scaled) return 1.0f;
    const int T = base + lane;
    const int t = T < nk ? T : nk - 1;
    return cur.sa[t] * cur.sb[t];
  };
  auto lane_value = [](float v, int l) -> float {
    return __builtin_bit_cast(float, __builtin_amdgcn_readlane(__builtin_bit_cast(int, v), l));
  };

  i32x8 fa[4], fb[4];      // A fragment i sits in slot i % 4 (read three rows ahead of its use); B fragments 0..3 of the tile
  f32x4 P[kNP];            // results of the last kNP MFMAs

  using I0 = std::integral_constant<int, 0>;
  using I1 = std::integral_constant<int, 1>;

  auto read_a = [&](int f, int stage) {
    fa[f & 3] = lds_read32(fa0 + stage * kBlk + f * 16 * kRow, fa1 + stage * kBlk + f * 16 * kRow);
  };
  auto read_b = [&](int f, int slot_off) {
    fb[f] = lds_read32(fb0 + slot_off + f * 16 * kRow, fb1 + slot_off + f * 16 * kRow);
  };
  auto fold = [&](int i, int j, int buf, float s) {
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[i][j][e] = __builtin_fmaf(s, P[buf][e], acc[i][j][e]);
  };

  // K-step kt (PAR = kt & 1) in exact program order (sched_barrier(0) forbids any reordering across
  // it).  Slot q = 4 i + j: MFMA (i, j) from a zero accumulator; then the result of MFMA q - 3 (long
  // complete, so the fold never waits) is folded into the running sum.  Row i also reads A fragment i + 3 (rows 5..7: fragments 0..2 of
  // the next tile) into the slot row i - 1 has just left; in row 7 B fragment j of the next tile
  // replaces fragment j right after its last use.  The barrier follows row 4, when the last A read of
  // the tile has been issued.  Slots 2, 6, 10, 14 load B of tile kt+2; slots 20, 22, 24, 26 load A of
  // tile kt+2.  Nothing is guarded against the end of K: loads of tiles past the end stay inside the
  // buffer descriptors, land in blocks that are free by then, and are never multiplied.
  auto step = [&](auto par_c, auto cross_c, int kt, float sc, float sc_prev) __attribute__((always_inline)) {
    constexpr int PAR = decltype(par_c)::value;
    constexpr bool CROSS = decltype(cross_c)::value != 0;          // the loads of this step may belong to the next tile
#pragma unroll
    for (int q = 0; q < 32; ++q) {
      const int i = q >> 2, j = q & 3;
      P[q % kNP] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(fb[j], fa[i & 3], f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
      __builtin_amdgcn_sched_barrier(0);
      if (q >= kFD) fold((q - kFD) >> 2, (q - kFD) & 3, (q - kFD) % kNP, sc);
      else if (kt > 0) fold(7, 4 + q - kFD, (32 + q - kFD) % kNP, sc_prev);
      if (j == 1) {
        if (i < 5) read_a(i + 3, PAR);
        else read_a(i - 5, PAR ^ 1);
      }
      if (i == 7) read_b(j, bo1);
      if (q < 16 && j == 2) b_load(kt + 2, i, bo2, CROSS);
      if (q >= 20 && q < 28 && (q & 1) == 0) a_load(kt + 2, (q - 20) >> 1, PAR, CROSS);
      if (q == 19) {
        // Own reads of tile kt are complete and so are own loads of tile kt+1 (the 4 B loads issued
        // since may still be in flight).  After the barrier tile kt+1 is readable by every wave and
        // nobody reads the blocks of tile kt any more.
        asm volatile("s_waitcnt vmcnt(4) lgkmcnt(0)" ::: "memory");
        wg_barrier();
      }
      __builtin_amdgcn_sched_barrier(0);
      if ((q & 3) == 3) AXE_PARANOID_SYNC();
    }
    const int t = bo0;
    bo0 = bo1, bo1 = bo2, bo2 = t;
  };

  // ---- VGPR -> HBM.  Operands are swapped in the MFMA, so lane l holds, for fragment (i, j), the 4
  //      consecutive columns j*16 + 4*(l/16) .. +3 of row i*16 + l%16 of the wave's 128 x 64 sub-tile:
  //      8 bytes of bf16, stored directly (the four fragments of a fragment row complete 128
  //      contiguous bytes per row; L2 merges them).  An asm statement, for the reason given in the
  //      bf16 kernel: the compiler's wait-count bookkeeping must not see the store.
  i32x4 rc;                                                        // descriptor of this wave's part of the C tile
  const int c_rowblk = (int)(16 * g.ldc * 2);                      // bytes between fragment rows
  const int c_voff = (int)((fr * g.ldc + 4 * fq) * 2);
  auto set_output = [&](int vv) __attribute__((always_inline)) {
    int tm, tn;
    tile_of_block(vv, ntiles, g.grid_m, g.grid_n, tm, tn);
    rc = raw_rsrc((uint16_t*)g.C + ((int64_t)tm * kTile + wm * 128) * g.ldc + (int64_t)tn * kTile + wn * 64,
                  (uint32_t)((127 * g.ldc + 64) * 2));
  };
  auto store_fragment = [&](int i, int j) __attribute__((always_inline)) {
    typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;
    const u32x2 d = {pack_bf16(acc[i][j][0], acc[i][j][1]), pack_bf16(acc[i][j][2], acc[i][j][3])};
    const int soff = __builtin_amdgcn_readfirstlane(i * c_rowblk + j * 32);
    asm volatile("s_nop 4\n\tbuffer_store_dwordx2 %0, %1, %2, %3 offen" AXE_AFTER_STORE ::"v"(d), "v"(c_voff), "s"(rc), "s"(soff) : "memory");
    AXE_PARANOID_WAIT();
#pragma unroll
    for (int e = 0; e < 4; ++e) acc[i][j][e] = 0.f;                // ready for the next tile
  };

  // ---- prologue (first tile only): tiles 0 and 1 of both operands
#pragma unroll
  for (int i = 0; i < 4; ++i) a_load(0, i, 0, true);
#pragma unroll
  for (int i = 0; i < 4; ++i) b_load(0, i, bo0, true);
#pragma unroll
  for (int i = 0; i < 4; ++i) a_load(1, i, 1, true);
#pragma unroll
  for (int i = 0; i < 4; ++i) b_load(1, i, bo1, true);
  asm volatile("s_waitcnt vmcnt(8)" ::: "memory");                  // tile 0 has landed; the 8 loads of tile 1 may still be in flight
  wg_barrier();
#pragma unroll
  for (int f = 0; f < 4; ++f) read_b(f, bo0);
#pragma unroll
  for (int f = 0; f < 3; ++f) read_a(f, 0);

  // ---- all K-steps of all tiles of this workgroup, one uninterrupted pipeline.  The host launches
  //      more than one tile per workgroup only when nk is even (the A block of a step is chosen by its
  //      parity, which must continue across the tile boundary) and at least 4.
  float scv0 = scales_from(0);                                     // first tile: waited for here, with the prologue
  float nsa = 1.0f, nsb = 1.0f;                                    // next tile's scales of steps 0..63, one per lane, on their way
  for (;;) {
    set_output(v);
    const bool more = v + (int)gridDim.x < ntiles;
    int kt = 0;
    float sc = 1.0f, sc_prev = 1.0f;
    for (int base = 0; base < nk; base += 64) {
      const float scv = base == 0 ? scv0 : scales_from(base);
      const int end = nk < base + 64 ? nk : base + 64;
      const int steady = end < nk - 2 ? end : nk - 2;              // steps below load only this tile (at most step kt + 2)
      sc = lane_value(scv, 0);
      for (; kt + 1 < steady; kt += 2) {
        const float sc1 = lane_value(scv, (kt + 1) & 63);
        step(I0{}, I0{}, kt, sc, sc_prev);
        const float sc2 = lane_value(scv, (kt + 2) & 63);
        step(I1{}, I0{}, kt + 1, sc1, sc);
        sc_prev = sc1;
        sc = sc2;
      }
      if (end == nk && more && scaled) {
        // The next tile's first register of scales is fetched now and waited for after this tile's
        // stores (asm statements: a load the compiler sees would be waited for with vmcnt(0), which
        // drains the operand pipeline).
        const int t = lane < nk ? lane : nk - 1;
        asm volatile("global_load_dword %0, %1, off" : "=v"(nsa) : "v"(nxt.sa + t) : "memory");
        asm volatile("global_load_dword %0, %1, off" : "=v"(nsb) : "v"(nxt.sb + t) : "memory");
      }
      for (; kt + 1 < end; kt += 2) {                              // the last steps load the next tile's first K-steps
        const float sc1 = lane_value(scv, (kt + 1) & 63);
        step(I0{}, I1{}, kt, sc, sc_prev);
        const float sc2 = lane_value(scv, (kt + 2) & 63);
        step(I1{}, I1{}, kt + 1, sc1, sc);
        sc_prev = sc1;
        sc = sc2;
      }
      if (kt < end) {                                              // odd nk (one tile per workgroup): the very last step
        step(I0{}, I1{}, kt, sc, sc_prev);
        sc_prev = sc;
        ++kt;
      }
    }
#pragma unroll
    for (int t = 0; t < kFD; ++t) fold(7, 4 - kFD + t, (32 - kFD + t) % kNP, sc_prev);
    // the tile is complete: store it while the loads of the next tile's first K-steps are on their way
#pragma unroll
    for (int i = 0; i < 8; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) store_fragment(i, j);
    v += (int)gridDim.x;
    if (v >= ntiles) break;
    // 16 operand loads and 32 stores were issued after the two scale loads; memory operations of a
    // wave complete in order, so at most 48 outstanding means the scales have arrived
    asm volatile("s_waitcnt vmcnt(48)" : "+v"(nsa), "+v"(nsb)::"memory");
    scv0 = scaled ? nsa * nsb : 1.0f;
    cur = nxt;
    nxt = describe(v + (int)gridDim.x);
  }
}

hipError_t launch_gemm_fp8_256(const GemmArgs& g, hipStream_t s) {
  const int ntiles = g.grid_m * g.grid_n;
  const int nk = (int)(g.K / 128);
  const int cus = cu_count();
  // one resident workgroup per CU walks several tiles when the pipeline can continue across tiles
  const bool chain = (nk % 2 == 0) && nk >= 4 && ntiles > cus && (cus % 8 == 0);
  unsigned nwg = (unsigned)(chain ? cus : ntiles);
  hipLaunchKernelGGL(gemm_fp8_256_kernel, dim3(nwg), dim3(512), 0, s, g);
  return hipGetLastError();
}

}  // namespace axe
