// axe_gemm_describe: the Axe layouts (Defs. 2.1 - 2.3 of the paper, plus the swizzle stage) of every
// tile movement of the kernel axe_gemm launches.  Host only.
//
// Nothing here is written down as a finished list of iters.  Each movement is composed with the tile operator
// (Sec. 3.3, Alg. 2: axe_layout_tile) from a small atom and the grids above it, the way Sec. 3.4 matches a
// shared-memory tile as "tiler (x) swizzled atom":
//   LDS image      rows of atoms           (x)  swizzled atom (one period of the key x one K-tile)
//   HBM -> LDS     pieces x wave pairs     (x)  atom of one wave instruction pair (16 rows, swizzle on the lane id)
//   operands       waves (x) fragments in registers (x) MFMA operand fragment
//   accumulators   workgroups (x) waves (x) fragments in registers (x) MFMA accumulator fragment
//   stores         waves (x) fragment pairs in registers (x) exchanged fragment pair
// The atoms' numbers -- key shift, chunks per row, rows per wave instruction, which chunk a lane group reads, which
// columns a lane stores -- are those of csrc/tile_maps.h, which the kernels' address arithmetic uses as well.
//
// Axes: 0 "m" (HBM), 1 "lds" (element address inside one LDS stage), 2 "wg" (row-major tile index),
// 3 "wave", 4 "lane", 5 "reg" (element index inside the lane's fragment / per-thread loop).
#include <string.h>

#include <vector>

#include "../../include/axe.h"
#include "host_layout.h"
#include "tile_maps.h"

namespace {

namespace maps = axe::maps;

enum Axis { M_ = 0, LDS = 1, WG = 2, WAVE = 3, LANE = 4, REG = 5, NAXES = 6 };
const char* const kNames[NAXES] = {"m", "lds", "wg", "wave", "lane", "reg"};

int ilog2(int64_t v) {
  int l = 0;
  while ((int64_t(1) << l) < v) ++l;
  return l;
}

// A layout of a logical (rows, columns) shape that owns its iters.
struct L2 {
  std::vector<axe_iter_t> d, r;
  int64_t off[NAXES] = {0};
  int swz_axis = -1, bits = 0, base = 0, shift = 0;
  int64_t shape[2] = {1, 1};
  L2() {}
  // iters of the row dimension followed by those of the column dimension
  L2(int64_t rows, std::vector<axe_iter_t> dr, int64_t cols, std::vector<axe_iter_t> dc) {
    shape[0] = rows, shape[1] = cols;
    d = dr;
    d.insert(d.end(), dc.begin(), dc.end());
    if (d.empty()) d.push_back(axe_iter_t{1, 1, REG});
  }
  L2& swz(int axis, int b, int ba, int sh) {
    swz_axis = axis, bits = b, base = ba, shift = sh;
    return *this;
  }
  L2& replicas(int64_t e, int64_t s, int axis) {
    if (e > 1) r.push_back(axe_iter_t{e, s, axis});
    return *this;
  }
  // the same layout for the transposed logical shape (columns, rows): the two blocks of iters change places
  L2 transposed() const {
    size_t n_row_iters = 0;                              // the row block: the leading iters whose extents make up shape[0]
    for (int64_t have = 1; have < shape[0]; ++n_row_iters) have *= d[n_row_iters].extent;
    L2 t = *this;
    t.shape[0] = shape[1], t.shape[1] = shape[0];
    t.d.assign(d.begin() + n_row_iters, d.end());
    t.d.insert(t.d.end(), d.begin(), d.begin() + n_row_iters);
    return t;
  }
  axe_layout_t c() const {
    axe_layout_t L;
    memset(&L, 0, sizeof L);
    L.n_axes = NAXES, L.n_d = (int32_t)d.size(), L.d = d.data(), L.n_r = (int32_t)r.size(), L.r = r.empty() ? nullptr : r.data();
    L.offset = off, L.swz_axis = swz_axis, L.swz_bits = bits, L.swz_base = base, L.swz_shift = shift;
    return L;
  }
};

// outer (x) inner (Alg. 2) on two-dimensional shapes; the result admits (rows, columns) = the products of the
// interleaved pairs.
int tile2(const L2& outer, const L2& inner, L2& out) {
  const axe_layout_t a = outer.c(), b = inner.c();
  axe_layout_t t;
  int64_t inter[4];
  alignas(16) char arena[2048];
  if (int rc = axe_layout_tile(&a, 2, outer.shape, &b, inner.shape, &t, inter, arena, sizeof arena)) return rc;
  L2 res;
  res.d.assign(t.d, t.d + t.n_d);
  if (t.n_r) res.r.assign(t.r, t.r + t.n_r);
  for (int x = 0; x < NAXES; ++x) res.off[x] = t.offset ? t.offset[x] : 0;
  res.swz_axis = t.swz_axis, res.bits = t.swz_bits, res.base = t.swz_base, res.shift = t.swz_shift;
  res.shape[0] = inter[0] * inter[1], res.shape[1] = inter[2] * inter[3];
  out = res;
  return AXE_OK;
}

// Kernel geometry: workgroup tile T x TN x BK elements (T rows of A, TN rows of B), wave grid WM x WN,
// MFMA fragment F x F, LDS rows of ROWB bytes made of 16-byte chunks of CE elements.
struct Geo {
  bool big, fp8;
  bool mx;         // fp8 on the matrix cores' scale path (E8M0 scales or none): the 4-wave structure of the bf16 kernel
  bool out32;      // fp32 output: fragments are stored as they are, not in exchanged pairs
  int T, TN, BK, F, ROWB, CE, EB, CH;
  int WM, WN;      // wave grid: wave = WN * wm + wn; A rows are split over wm, B rows over wn
  int64_t b_off;   // element offset of the B block inside one LDS stage
};

Geo geometry(bool big, bool fp8, bool mx, int tile_n, bool out32) {
  Geo g;
  g.big = big;
  g.out32 = out32;
  g.fp8 = fp8;
  g.mx = big && fp8 && mx;
  g.EB = fp8 ? 1 : 2;
  g.CE = maps::kChunkBytes / g.EB;
  g.ROWB = (fp8 || big) ? maps::kLargeRowBytes : 64;
  g.CH = g.ROWB / maps::kChunkBytes;
  g.WM = 2;
  g.WN = (big && fp8 && !g.mx) ? 4 : 2;
  g.F = maps::kFrag;
  g.T = big ? 256 : 64;
  g.TN = tile_n;
  g.BK = g.ROWB / g.EB;
  // 256x256 kernels: five 32 KiB blocks, A in blocks 0 and 1, the B ring starts at block 2
  g.b_off = (int64_t)g.T * g.BK * (big ? 2 : 1);
  return g;
}

// (rows, k) tile of an operand: which thread fetches which element from HBM.
int g2l_threads(const Geo& g, bool is_b, L2& out) {
  const int64_t R = is_b ? g.TN : g.T;
  const int NW = g.WM * g.WN;
  L2 atom, grid;
  if (g.big) {
    // One wave instruction moves kRowsPerLoad rows of 128 bytes straight into LDS, which such a load fills
    // linearly in the lane id: lane 8 lr + lp lands on chunk POSITION lp of row lr, so it fetches the logical chunk
    // lp ^ key(row) -- a swizzle stage on the lane coordinate.  key(row) of row (w + NW i) * 8 + lr takes one bit
    // from the wave id, so the atom is the pair of instructions of waves 2 v, 2 v + 1 (16 rows, one period of the
    // key), stated on the thread id folded into the lane axis: lane coordinate 64 (w % 2) + 8 lr + lp.
    const int RPL = maps::kRowsPerLoad, P = maps::lds_key_period(g.CH);
    atom = L2(P, {{P / RPL, 64, LANE}, {RPL, g.CH, LANE}}, g.BK, {{g.CH, 1, LANE}, {g.CE, 1, REG}});
    atom.swz(LANE, ilog2(g.CH), 0, ilog2(g.CH) + maps::kKeyShift);
    // pieces i = 0 .. NI - 1 of a wave go to consecutive registers, wave pairs to consecutive 128-lane blocks
    const int64_t NI = R / (RPL * NW), pairs = NW / (P / RPL);
    grid = L2(NI * pairs, {{NI, 1, REG}, {pairs, 1, LANE}}, 1, {});
  } else {
    // thread t fetches chunk t (+ 256 p) of the tile in row-major chunk order: a pass of one wave covers 64 / CH rows
    const int RPW = 64 / g.CH, PER = (64 * g.CH) / 256;
    atom = L2(RPW, {{RPW, g.CH, LANE}}, g.BK, {{g.CH, 1, LANE}, {g.CE, 1, REG}});
    grid = L2((int64_t)PER * 4, {{PER, 1, REG}, {4, 1, WAVE}}, 1, {});
  }
  L2 t;
  if (int rc = tile2(grid, atom, t)) return rc;
  out = is_b ? t.transposed() : t;
  return AXE_OK;
}

// (rows, k) tile -> element address inside one LDS stage (A region first, then B): rows of atoms (x) swizzled atom,
// the atom being one period of the key (chunk c of row r at chunk position c ^ key(r)) by one K-tile.
int lds_layout(const Geo& g, bool is_b, L2& out) {
  const int64_t R = is_b ? g.TN : g.T;
  const int P = maps::lds_key_period(g.CH);
  L2 atom(P, {{P, g.BK, LDS}}, g.BK, {{g.BK, 1, LDS}});
  atom.swz(LDS, ilog2(g.CH), ilog2(g.CE), ilog2(g.BK) + maps::kKeyShift);
  L2 rows(R / P, {{R / P, 1, LDS}}, 1, {});
  L2 t;
  if (int rc = tile2(rows, atom, t)) return rc;
  if (is_b) t.off[LDS] += g.b_off;                     // whole periods of the swizzle: the stage is unaffected
  out = is_b ? t.transposed() : t;
  return AXE_OK;
}

// (rows, k) tile -> MFMA operand registers.  Waves form a WM x WN grid (wave = WN wm + wn); A rows are
// split over wm and replicated over wn, B rows the other way round.  Register index = (k sub-step,
// fragment, element): kernels that keep only a few fragments in registers at a time reuse the
// physical registers, the index names the fragment.
int operand_layout(const Geo& g, bool is_b, L2& out) {
  const int WT = is_b ? g.TN / g.WN : g.T / g.WM;      // rows of this operand per wave
  const int NF = WT / g.F;                             // fragments per wave
  const int LG = maps::kLaneGroups;                    // lane groups along k
  // the fragment of one MFMA: row -> lane % 16; which k a lane group holds is tile_maps.h's operand_chunk_*
  L2 frag;
  int KF;                                              // k per MFMA
  if (g.fp8) {
    // v_mfma_f32_16x16x128_f8f6f4: chunk operand_chunk_fp8(h, q) = q + 4 h -> lane group q, registers 16 h .. 16 h + 15
    KF = 2 * LG * g.CE;
    frag = L2(g.F, {{g.F, 1, LANE}}, KF, {{2, g.CE, REG}, {LG, g.F, LANE}, {g.CE, 1, REG}});
  } else {
    // v_mfma_f32_16x16x32: chunk operand_chunk_16bit(s, q) = 4 s + q of K sub-step s -> lane group q, registers 0 .. 7
    KF = LG * g.CE;
    frag = L2(g.F, {{g.F, 1, LANE}}, KF, {{LG, g.F, LANE}, {g.CE, 1, REG}});
  }
  const int KS = g.BK / KF;                            // MFMA k sub-steps per LDS tile
  L2 regs(NF, {{NF, 1, REG}}, KS, {{KS, NF, REG}});
  L2 waves = is_b ? L2(g.WN, {{g.WN, 1, WAVE}}, 1, {}) : L2(g.WM, {{g.WM, g.WN, WAVE}}, 1, {});
  waves.replicas(is_b ? g.WM : g.WN, is_b ? g.WN : 1, WAVE);
  L2 t1, t2;
  if (int rc = tile2(regs, frag, t1)) return rc;
  if (int rc = tile2(waves, t1, t2)) return rc;
  out = is_b ? t2.transposed() : t2;
  return AXE_OK;
}

// MFMA accumulator fragment with the operands swapped: row -> lane % 16; column 4 q + c -> lane group q, register c
L2 acc_fragment(const Geo& g) {
  return L2(g.F, {{g.F, 1, LANE}}, g.F, {{maps::kLaneGroups, g.F, LANE}, {maps::kAccCols, 1, REG}});
}

// (M, N) of the (tile-padded) problem -> wg, wave, lane, reg: the accumulators, innermost first:
//   fragment (16, 16)  (x)  register tile (NFM, NFN)  (x)  wave grid (WM, WN)  (x)  workgroup grid.
int acc_layout(const Geo& g, int64_t grid_m, int64_t grid_n, bool tile_only, L2& out) {
  const int64_t NFM = g.T / g.WM / g.F, NFN = g.TN / g.WN / g.F;
  const L2 levels[3] = {L2(NFM, {{NFM, NFN, REG}}, NFN, {{NFN, 1, REG}}), L2(g.WM, {{g.WM, g.WN, WAVE}}, g.WN, {{g.WN, 1, WAVE}}),
                        L2(grid_m, {{grid_m, grid_n, WG}}, grid_n, {{grid_n, 1, WG}})};
  L2 cur = acc_fragment(g);
  for (int level = 0; level < (tile_only ? 2 : 3); ++level) {
    L2 next;
    if (int rc = tile2(levels[level], cur, next)) return rc;
    cur = next;
  }
  out = cur;
  return AXE_OK;
}

// (T, TN) tile of C -> wave, lane, reg: who stores which element.
int c_store_layout(const Geo& g, L2& out) {
  // The 4-wave 256 x 256 kernels (16-bit inputs, and fp8 on the scale path) pair neighbouring fragments: after an
  // exchange between lane groups (v_permlane16_swap) lane group q stores the 8 consecutive columns that begin at
  // pair_store_col(q) of the 32-column pair: q = 2 h + b -> columns 16 b + 8 h + 4 t + e from register 4 t + e.
  if (g.big && (!g.fp8 || g.mx) && g.TN == 256 && !g.out32) {
    static_assert(maps::pair_store_col(0) == 0 && maps::pair_store_col(1) == 16 && maps::pair_store_col(2) == 8 && maps::pair_store_col(3) == 24,
                  "the exchanged pair below is stated for these first columns");
    const int64_t NFM = g.T / g.WM / g.F, NP = g.TN / g.WN / (2 * g.F);
    L2 pair(g.F, {{g.F, 1, LANE}}, 2 * g.F, {{2, 16, LANE}, {2, 32, LANE}, {2, maps::kAccCols, REG}, {maps::kAccCols, 1, REG}});
    L2 regs(NFM, {{NFM, NP, REG}}, NP, {{NP, 1, REG}});
    L2 waves(g.WM, {{g.WM, g.WN, WAVE}}, g.WN, {{g.WN, 1, WAVE}});
    L2 t1;
    if (int rc = tile2(regs, pair, t1)) return rc;
    return tile2(waves, t1, out);
  }
  // the other kernels store their accumulator fragments as they are: the store map is the accumulator
  // layout of one tile (8 bytes of bf16 per lane and fragment)
  return acc_layout(g, 1, 1, true, out);
}

int build(const Geo& geo, int32_t which, int64_t grid_m, int64_t grid_n, bool acc_tile_only, L2& b) {
  switch (which) {
    case AXE_DESC_A_G2L_THREADS: return g2l_threads(geo, false, b);
    case AXE_DESC_B_G2L_THREADS: return g2l_threads(geo, true, b);
    case AXE_DESC_A_LDS: return lds_layout(geo, false, b);
    case AXE_DESC_B_LDS: return lds_layout(geo, true, b);
    case AXE_DESC_A_OPERAND: return operand_layout(geo, false, b);
    case AXE_DESC_B_OPERAND: return operand_layout(geo, true, b);
    case AXE_DESC_ACC: return acc_layout(geo, grid_m, grid_n, acc_tile_only, b);
    case AXE_DESC_C_STORE: return c_store_layout(geo, b);
    default: return 1;
  }
}

// lay the result out in the caller's arena (unit iters dropped: rule D0)
int emit(const L2& b, const char* who, axe_layout_t* out, int64_t* shape, int32_t* rank, void* arena, size_t arena_bytes) {
  std::vector<axe_iter_t> d;
  for (const axe_iter_t& it : b.d)
    if (it.extent > 1) d.push_back(it);
  if (d.empty()) d.push_back(b.d[0]);
  const size_t need = sizeof(axe_iter_t) * (d.size() + b.r.size()) + sizeof(int64_t) * NAXES + sizeof(char*) * NAXES + 16;
  if (arena_bytes < need) {
    axe::set_error("%s: arena of %zu bytes is too small (%zu needed)", who, arena_bytes, need);
    return AXE_ERANGE;
  }
  char* p = (char*)arena;
  p += (8 - ((uintptr_t)p & 7)) & 7;
  axe_iter_t* dd = (axe_iter_t*)p;
  p += sizeof(axe_iter_t) * d.size();
  axe_iter_t* r = (axe_iter_t*)p;
  p += sizeof(axe_iter_t) * b.r.size();
  int64_t* off = (int64_t*)p;
  p += sizeof(int64_t) * NAXES;
  const char** names = (const char**)p;
  for (size_t i = 0; i < d.size(); ++i) dd[i] = d[i];
  for (size_t i = 0; i < b.r.size(); ++i) r[i] = b.r[i];
  for (int a = 0; a < NAXES; ++a) off[a] = b.off[a], names[a] = kNames[a];
  out->n_axes = NAXES;
  out->axis_names = names;
  out->n_d = (int32_t)d.size();
  out->d = dd;
  out->n_r = (int32_t)b.r.size();
  out->r = b.r.empty() ? nullptr : r;
  out->offset = off;
  out->swz_axis = b.swz_axis;
  out->swz_bits = b.bits;
  out->swz_base = b.base;
  out->swz_shift = b.shift;
  *rank = 2;
  shape[0] = b.shape[0], shape[1] = b.shape[1];
  return AXE_OK;
}

}  // namespace

extern "C" int axe_gemm_describe(const axe_gemm_desc_t* g, int32_t which, axe_layout_t* out, int64_t* shape,
                                 int32_t* rank, void* arena, size_t arena_bytes) {
  if (!g || !out || !shape || !rank || !arena) {
    axe::set_error("axe_gemm_describe: NULL argument");
    return AXE_EINVAL;
  }
  int tile = axe_gemm_tile(g);
  if (tile < 0) return tile;
  if (which < AXE_DESC_A_G2L_THREADS || which > AXE_DESC_C_STORE) {
    axe::set_error("axe_gemm_describe: unknown selector %d", which);
    return AXE_EINVAL;
  }
  const bool big = tile != AXE_TILE_64x64x32;
  const bool mx = g->in_dtype == AXE_FP8_E4M3 && (!g->d_scale_a || g->scale_dtype == AXE_SCALE_E8M0);
  const Geo geo = geometry(big, g->in_dtype == AXE_FP8_E4M3, mx, tile == AXE_TILE_256x224x64 ? 224 : (big ? 256 : 64),
                           g->out_dtype == AXE_F32);
  L2 b;
  if (int rc = build(geo, which, (g->M + geo.T - 1) / geo.T, (g->N + geo.TN - 1) / geo.TN, false, b)) return rc;
  return emit(b, "axe_gemm_describe", out, shape, rank, arena, arena_bytes);
}

// The grouped tile kernels are the dense 256-wide 16-bit kernel at a tile height of 256 or 128 rows: their tile
// movements are the same layouts (a tile's place in the problem depends on the group sizes, which only the
// device knows, so the accumulator layout is that of one tile).
extern "C" int axe_gemm_grouped_describe(const axe_gemm_grouped_desc_t* g, int32_t which, axe_layout_t* out, int64_t* shape,
                                         int32_t* rank, void* arena, size_t arena_bytes) {
  if (!g || !out || !shape || !rank || !arena) {
    axe::set_error("axe_gemm_grouped_describe: NULL argument");
    return AXE_EINVAL;
  }
  const int kernel = axe_gemm_grouped_kernel(g);
  if (kernel < 0) return kernel;
  if (kernel == AXE_GROUPED_STREAM) {
    axe::set_error("axe_gemm_grouped_describe: the streaming kernel keeps no tile in LDS and its maps are not reported "
                   "(lane l holds row l %% 16 and the 16-byte chunks l / 16 and l / 16 + 4 of a 64-wide K-tile of either operand)");
    return AXE_EUNSUPPORTED;
  }
  if (which < AXE_DESC_A_G2L_THREADS || which > AXE_DESC_C_STORE) {
    axe::set_error("axe_gemm_grouped_describe: unknown selector %d", which);
    return AXE_EINVAL;
  }
  if (which == AXE_DESC_C_STORE && g->epilogue != AXE_EPI_NONE) {
    axe::set_error("axe_gemm_grouped_describe: the store map of the gated epilogue (two accumulators per stored element) "
                   "is not a layout of the accumulators and is not reported");
    return AXE_EUNSUPPORTED;
  }
  // fp8 groups on the tile kernel: the 4-wave kernel of the matrix cores' scale path
  Geo geo = g->in_dtype == AXE_FP8_E4M3 ? geometry(true, true, true, 256, false) : geometry(true, false, false, 256, false);
  if (kernel == AXE_GROUPED_TILES_128) geo.T = 128;               // the A blocks in LDS keep their places: b_off stays
  L2 b;
  if (int rc = build(geo, which, 1, 1, true, b)) return rc;
  return emit(b, "axe_gemm_grouped_describe", out, shape, rank, arena, arena_bytes);
}
