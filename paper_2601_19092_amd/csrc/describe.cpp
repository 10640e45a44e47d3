// axe_gemm_describe: the Axe layouts (Defs. 2.1 - 2.3 of the paper, plus the swizzle stage) of every
// tile movement of the kernel axe_gemm launches.  The layouts are composed the way Sec. 3.3 composes
// tiles: register tile (x) lane (x) wave (x) workgroup.  Host only.
//
// Axes: 0 "m" (HBM), 1 "lds" (element address inside one LDS stage), 2 "wg" (row-major tile index),
// 3 "wave", 4 "lane", 5 "reg" (element index inside the lane's fragment / per-thread loop).
#include <string.h>

#include <vector>

#include "../../include/axe.h"
#include "host_layout.h"

namespace {

enum Axis { M_ = 0, LDS = 1, WG = 2, WAVE = 3, LANE = 4, REG = 5, NAXES = 6 };
const char* const kNames[NAXES] = {"m", "lds", "wg", "wave", "lane", "reg"};

struct Builder {
  std::vector<axe_iter_t> d, r;
  int64_t off[NAXES] = {0};
  int swz_axis = -1, bits = 0, base = 0, shift = 0;
  std::vector<int64_t> shape;
  void D(int64_t e, int64_t s, int axis) { d.push_back(axe_iter_t{e, s, axis}); }
  void R(int64_t e, int64_t s, int axis) { r.push_back(axe_iter_t{e, s, axis}); }
  void swz(int axis, int b, int ba, int sh) { swz_axis = axis, bits = b, base = ba, shift = sh; }
};

int ilog2(int64_t v) {
  int l = 0;
  while ((int64_t(1) << l) < v) ++l;
  return l;
}

// Kernel geometry: workgroup tile T x TN x BK elements (T rows of A, TN rows of B), wave grid WM x WN,
// MFMA fragment F x F, LDS rows of ROWB bytes made of 16-byte chunks of CE elements.
struct Geo {
  bool big, fp8;
  bool mx;         // fp8 on the matrix cores' scale path (E8M0 scales or none): the 4-wave structure of the bf16 kernel
  bool out32;      // fp32 output: fragments are stored as they are, not in exchanged pairs
  int T, TN, BK, F, ROWB, CE, EB;
  int WM, WN;      // wave grid: wave = WN * wm + wn; A rows are split over wm, B rows over wn
  int key_shift;   // swizzle key = (row >> key_shift) & (chunks per row - 1)
  int64_t b_off;   // element offset of the B block inside one LDS stage
};

Geo geometry(bool big, bool fp8, bool mx, int tile_n, bool out32) {
  Geo g;
  g.big = big;
  g.out32 = out32;
  g.fp8 = fp8;
  g.mx = big && fp8 && mx;
  g.EB = fp8 ? 1 : 2;
  g.CE = 16 / g.EB;
  g.ROWB = (fp8 || big) ? 128 : 64;
  g.WM = 2;
  g.WN = (big && fp8 && !g.mx) ? 4 : 2;
  g.F = 16;
  if (big) {
    g.T = 256;
  } else {
    g.T = 64;
    g.F = 16;
  }
  g.TN = tile_n;
  g.BK = g.ROWB / g.EB;
  g.key_shift = 1;
  // 256x256 kernels: five 32 KiB blocks, A in blocks 0 and 1, the B ring starts at block 2
  g.b_off = (int64_t)g.T * g.BK * (big ? 2 : 1);
  return g;
}

// (rows, k) tile of an operand: which thread fetches which element from HBM.
int g2l_threads(const Geo& g, bool is_b, Builder& b) {
  const int CH = g.ROWB / 16;                          // chunks per row
  std::vector<axe_iter_t> rows, ks;
  if (g.big) {
    // one wave instruction = 1 KiB = 8 rows of 128 bytes; wave w of NW takes row groups w, w + NW, ...:
    // row = (NW i + w) * 8 + lr, chunk c.  Both operands are loaded straight into LDS, which such a load fills
    // linearly in the lane id, so the swizzle shows up in which chunk a lane fetches: c ^ key(row),
    // key = (4 (w & 1) + (lr >> 1)) & 7.  That key spans the wave id, so the maps are stated on the thread id
    // t = 64 w + lane, folded into the lane axis: key = (t >> 4) & 7.
    const int NW = g.WM * g.WN, NI = (is_b ? g.TN : g.T) / (8 * NW);
    rows = {{NI, g.CE, REG}, {NW, 64, LANE}, {8, CH, LANE}};
    b.swz(LANE, ilog2(CH), 0, ilog2(CH) + g.key_shift);
    ks = {{CH, 1, LANE}, {g.CE, 1, REG}};
  } else {
    // thread t fetches chunk t (+ 256 p): row = 32 p' ..., see kernels_gemm_small.hip
    const int PER = (64 * CH) / 256;                   // chunks per thread
    const int RPW = 64 / CH;                           // rows per wave and pass
    if (PER > 1) rows.push_back({PER, g.CE, REG});
    rows.push_back({4, 1, WAVE});
    rows.push_back({RPW, CH, LANE});
    ks = {{CH, 1, LANE}, {g.CE, 1, REG}};
  }
  if (!is_b) {
    for (auto& it : rows) b.d.push_back(it);
    for (auto& it : ks) b.d.push_back(it);
    b.shape = {g.T, g.BK};
  } else {
    for (auto& it : ks) b.d.push_back(it);
    for (auto& it : rows) b.d.push_back(it);
    b.shape = {g.BK, g.TN};
  }
  return AXE_OK;
}

// (rows, k) tile -> element address inside one LDS stage (A region first, then B).
int lds_layout(const Geo& g, bool is_b, Builder& b) {
  const int CH = g.ROWB / 16;
  if (!is_b) {
    b.D(g.T, g.BK, LDS);
    b.D(g.BK, 1, LDS);
    b.shape = {g.T, g.BK};
  } else {
    b.D(g.BK, 1, LDS);
    b.D(g.TN, g.BK, LDS);
    b.off[LDS] = g.b_off;
    b.shape = {g.BK, g.TN};
  }
  // chunk index ^= (row >> key_shift) & (CH - 1), in element units
  b.swz(LDS, ilog2(CH), ilog2(g.CE), ilog2(g.BK) + g.key_shift);
  return AXE_OK;
}

// (rows, k) tile -> MFMA operand registers.  Waves form a WM x WN grid (wave = WN wm + wn); A rows are
// split over wm and replicated over wn, B rows the other way round.  Register index = (k sub-step,
// fragment, element): kernels that keep only a few fragments in registers at a time reuse the
// physical registers, the index names the fragment.
int operand_layout(const Geo& g, bool is_b, Builder& b) {
  const int WT = is_b ? g.TN / g.WN : g.T / g.WM;      // rows of this operand per wave
  const int NF = WT / g.F;                             // fragments per wave
  const int LG = 64 / g.F;                             // lane groups along k
  const int KPL = g.fp8 ? 32 : 8;                      // k elements per lane per MFMA
  const int KS = g.BK / (LG * KPL);                    // MFMA k sub-steps per LDS tile
  std::vector<axe_iter_t> rows = {{is_b ? g.WN : g.WM, is_b ? 1 : g.WN, WAVE}, {NF, KPL, REG}, {g.F, 1, LANE}};
  std::vector<axe_iter_t> ks;
  if (KS > 1) ks.push_back({KS, (int64_t)NF * KPL, REG});
  if (g.fp8) {
    // the 32 k of a lane are two runs of 16: k = 64 h + 16 (lane / 16) + e sits in register 16 h + e
    ks.push_back({2, 16, REG});
    ks.push_back({LG, g.F, LANE});
    ks.push_back({16, 1, REG});
  } else {
    ks.push_back({LG, g.F, LANE});
    ks.push_back({KPL, 1, REG});
  }
  if (!is_b) {
    for (auto& it : rows) b.d.push_back(it);
    for (auto& it : ks) b.d.push_back(it);
    b.shape = {g.T, g.BK};
  } else {
    for (auto& it : ks) b.d.push_back(it);
    for (auto& it : rows) b.d.push_back(it);
    b.shape = {g.BK, g.TN};
  }
  b.R(is_b ? g.WM : g.WN, is_b ? g.WN : 1, WAVE);
  return AXE_OK;
}

// (M, N) of the (tile-padded) problem -> wg, wave, lane, reg: the accumulators.  Operands are
// swapped in the MFMA, so a lane owns, per 16 x 16 fragment, 4 consecutive columns of one row.
// Not written down but composed with the tile operator (Sec. 3.3, Alg. 2), innermost first:
//   fragment (16, 16)  (x)  register tile (NFM, NFN)  (x)  wave grid (WM, WN)  (x)  workgroup grid.
int acc_layout(const Geo& g, int64_t grid_m, int64_t grid_n, bool tile_only, Builder& b) {
  const int64_t NFM = g.T / g.WM / g.F, NFN = g.TN / g.WN / g.F;
  struct Level {
    axe_iter_t d[3];
    int n;
    int64_t shape[2];
  };
  // row -> lane; column 4 q + c -> lane group q (16 lanes apart), register c
  const Level frag = {{{g.F, 1, LANE}, {64 / g.F, g.F, LANE}, {4, 1, REG}}, 3, {g.F, g.F}};
  const Level outer[3] = {{{{NFM, NFN, REG}, {NFN, 1, REG}}, 2, {NFM, NFN}},
                          {{{g.WM, g.WN, WAVE}, {g.WN, 1, WAVE}}, 2, {g.WM, g.WN}},
                          {{{grid_m, grid_n, WG}, {grid_n, 1, WG}}, 2, {grid_m, grid_n}}};
  auto as_layout = [](const axe_iter_t* d, int n) {
    axe_layout_t L;
    memset(&L, 0, sizeof L);
    L.n_axes = NAXES, L.n_d = n, L.d = d, L.swz_axis = -1;
    return L;
  };
  char arena[2][1024];
  axe_layout_t cur = as_layout(frag.d, frag.n);
  int64_t shape[2] = {frag.shape[0], frag.shape[1]};
  for (int level = 0; level < (tile_only ? 2 : 3); ++level) {
    const axe_layout_t out_l = as_layout(outer[level].d, outer[level].n);
    axe_layout_t next;
    int64_t interleaved[4];
    if (int rc = axe_layout_tile(&out_l, 2, outer[level].shape, &cur, shape, &next, interleaved, arena[level & 1], 1024)) return rc;
    cur = next;                                        // admits (rows, cols) = products of the interleaved pairs as well
    shape[0] = interleaved[0] * interleaved[1];
    shape[1] = interleaved[2] * interleaved[3];
  }
  for (int i = 0; i < cur.n_d; ++i)
    if (cur.d[i].extent > 1 || cur.n_d == 1) b.D(cur.d[i].extent, cur.d[i].stride, cur.d[i].axis);
  b.shape = {shape[0], shape[1]};
  return AXE_OK;
}

// (T, T) tile of C -> wave, lane, reg: who stores which element.
int c_store_layout(const Geo& g, Builder& b) {
  // The 4-wave 256 x 256 kernels (bf16, and fp8 on the scale path) pair neighbouring fragments: after an exchange between lane groups a
  // lane stores 8 consecutive columns (16 bytes).  Column = 128 wn + 32 p + 16 b + 8 h + 4 t + e is
  // stored by lane group 2 h + b from register 8 p + 4 t + e of the fragment row.
  if (g.big && (!g.fp8 || g.mx) && g.TN == 256 && !g.out32) {
    const int NFM = g.T / g.WM / g.F;
    b.D(g.WM, g.WN, WAVE);
    b.D(NFM, 32, REG);
    b.D(g.F, 1, LANE);
    b.D(g.WN, 1, WAVE);
    b.D(4, 8, REG);
    b.D(2, 16, LANE);
    b.D(2, 32, LANE);
    b.D(2, 4, REG);
    b.D(4, 1, REG);
    b.shape = {g.T, g.TN};
    return AXE_OK;
  }
  // the other kernels store their accumulator fragments as they are: the store map is the accumulator
  // layout of one tile (8 bytes of bf16 per lane and fragment)
  return acc_layout(g, 1, 1, true, b);
}

}  // namespace

namespace {
int emit(const Builder& b, const char* who, axe_layout_t* out, int64_t* shape, int32_t* rank, void* arena, size_t arena_bytes);
}

extern "C" int axe_gemm_describe(const axe_gemm_desc_t* g, int32_t which, axe_layout_t* out, int64_t* shape,
                                 int32_t* rank, void* arena, size_t arena_bytes) {
  if (!g || !out || !shape || !rank || !arena) {
    axe::set_error("axe_gemm_describe: NULL argument");
    return AXE_EINVAL;
  }
  int tile = axe_gemm_tile(g);
  if (tile < 0) return tile;
  const bool big = tile != AXE_TILE_64x64x32;
  const bool mx = g->in_dtype == AXE_FP8_E4M3 && (!g->d_scale_a || g->scale_dtype == AXE_SCALE_E8M0);
  const Geo geo = geometry(big, g->in_dtype == AXE_FP8_E4M3, mx, tile == AXE_TILE_256x224x64 ? 224 : (big ? 256 : 64),
                           g->out_dtype == AXE_F32);
  Builder b;
  int rc;
  switch (which) {
    case AXE_DESC_A_G2L_THREADS: rc = g2l_threads(geo, false, b); break;
    case AXE_DESC_B_G2L_THREADS: rc = g2l_threads(geo, true, b); break;
    case AXE_DESC_A_LDS: rc = lds_layout(geo, false, b); break;
    case AXE_DESC_B_LDS: rc = lds_layout(geo, true, b); break;
    case AXE_DESC_A_OPERAND: rc = operand_layout(geo, false, b); break;
    case AXE_DESC_B_OPERAND: rc = operand_layout(geo, true, b); break;
    case AXE_DESC_ACC:
      rc = acc_layout(geo, (g->M + geo.T - 1) / geo.T, (g->N + geo.TN - 1) / geo.TN, false, b);
      break;
    case AXE_DESC_C_STORE: rc = c_store_layout(geo, b); break;
    default:
      axe::set_error("axe_gemm_describe: unknown selector %d", which);
      return AXE_EINVAL;
  }
  if (rc) return rc;
  return emit(b, "axe_gemm_describe", out, shape, rank, arena, arena_bytes);
}

namespace {
// lay the result out in the caller's arena
int emit(const Builder& b, const char* who, axe_layout_t* out, int64_t* shape, int32_t* rank, void* arena, size_t arena_bytes) {
  const size_t need = sizeof(axe_iter_t) * (b.d.size() + b.r.size()) + sizeof(int64_t) * NAXES + sizeof(char*) * NAXES + 16;
  if (arena_bytes < need || b.shape.size() > AXE_MAX_RANK) {
    axe::set_error("%s: arena of %zu bytes is too small (%zu needed)", who, arena_bytes, need);
    return AXE_ERANGE;
  }
  char* p = (char*)arena;
  p += (8 - ((uintptr_t)p & 7)) & 7;
  axe_iter_t* d = (axe_iter_t*)p;
  p += sizeof(axe_iter_t) * b.d.size();
  axe_iter_t* r = (axe_iter_t*)p;
  p += sizeof(axe_iter_t) * b.r.size();
  int64_t* off = (int64_t*)p;
  p += sizeof(int64_t) * NAXES;
  const char** names = (const char**)p;
  for (size_t i = 0; i < b.d.size(); ++i) d[i] = b.d[i];
  for (size_t i = 0; i < b.r.size(); ++i) r[i] = b.r[i];
  for (int a = 0; a < NAXES; ++a) off[a] = b.off[a], names[a] = kNames[a];
  out->n_axes = NAXES;
  out->axis_names = names;
  out->n_d = (int32_t)b.d.size();
  out->d = d;
  out->n_r = (int32_t)b.r.size();
  out->r = b.r.empty() ? nullptr : r;
  out->offset = off;
  out->swz_axis = b.swz_axis;
  out->swz_bits = b.bits;
  out->swz_base = b.base;
  out->swz_shift = b.shift;
  *rank = (int32_t)b.shape.size();
  for (size_t i = 0; i < b.shape.size(); ++i) shape[i] = b.shape[i];
  return AXE_OK;
}
}  // namespace

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
  Geo geo = geometry(true, false, false, 256, false);
  if (kernel == AXE_GROUPED_TILES_128) geo.T = 128;               // the A blocks in LDS keep their places: b_off stays
  Builder b;
  int rc;
  switch (which) {
    case AXE_DESC_A_G2L_THREADS: rc = g2l_threads(geo, false, b); break;
    case AXE_DESC_B_G2L_THREADS: rc = g2l_threads(geo, true, b); break;
    case AXE_DESC_A_LDS: rc = lds_layout(geo, false, b); break;
    case AXE_DESC_B_LDS: rc = lds_layout(geo, true, b); break;
    case AXE_DESC_A_OPERAND: rc = operand_layout(geo, false, b); break;
    case AXE_DESC_B_OPERAND: rc = operand_layout(geo, true, b); break;
    case AXE_DESC_ACC: rc = acc_layout(geo, 1, 1, true, b); break;
    case AXE_DESC_C_STORE:
      if (g->epilogue != AXE_EPI_NONE) {
        axe::set_error("axe_gemm_grouped_describe: the store map of the gated epilogue (two accumulators per stored element) "
                       "is not a layout of the accumulators and is not reported");
        return AXE_EUNSUPPORTED;
      }
      rc = c_store_layout(geo, b);
      break;
    default:
      axe::set_error("axe_gemm_grouped_describe: unknown selector %d", which);
      return AXE_EINVAL;
  }
  if (rc) return rc;
  return emit(b, "axe_gemm_grouped_describe", out, shape, rank, arena, arena_bytes);
}
