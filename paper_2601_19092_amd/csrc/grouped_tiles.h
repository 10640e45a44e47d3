// The tile table of the grouped tile kernels (device code only): which tiles a workgroup owns, worked out on the
// device from the group offsets -- no scratch memory, no host knowledge of the group sizes.
#pragma once
#include <hip/hip_runtime.h>

#include "device_types.h"

namespace axe {

// Tiles of a grouped problem, counted group after group: group e has ceil(rows_e / TM) x grid_n of them
// (row blocks fastest).  Lane t of the calling wave receives the workgroup's t-th tile: its first row, its
// number of rows (0: no such tile), its tile column and its group.  Workgroup ids are dealt round-robin
// to the 8 XCDs, so XCD x takes the x-th eighth of the tile sequence and its 32 workgroups walk it side
// by side: neighbours in the sequence share A rows (same group and row block) or a B panel in that
// XCD's L2.  The offsets are clamped to [0, M], so that whatever they hold no access leaves the buffers.
// t_desc packs rows (bits 0..8), tile column (9..19) and group (20..31): the host admits at most 4096
// groups and 2048 tile columns.
__device__ __forceinline__ int desc_rows(int d) { return d & 511; }
__device__ __forceinline__ int desc_tn(int d) { return (d >> 9) & 2047; }
__device__ __forceinline__ int desc_group(int d) { return (int)((unsigned)d >> 20); }
template <int TM, bool ONE = false>                               // rows of a tile; ONE: a single group of all M rows, no offsets array
__device__ __forceinline__ void group_tiles(const GemmArgs& g, int lane, int& t_row0, int& t_desc) {
  const int G = g.groups, M = (int)g.M, gn = g.grid_n;
  const int* __restrict__ off = g.group_rows;
  int r0 = 0, rows = 0, tg = 0, incl = 0;
  auto chunk = [&](int g0) __attribute__((always_inline)) {         // groups g0 .. g0 + 63, one per lane
    const int gi = g0 + lane;
    int a = 0, b = 0;
    if constexpr (ONE) {
      if (gi == 0) b = M;
    } else if (gi < G) {
      a = off[gi], b = off[gi + 1];
    }
    a = a < 0 ? 0 : (a > M ? M : a);
    b = b < 0 ? 0 : (b > M ? M : b);
    r0 = a;
    rows = b > a ? b - a : 0;
    tg = ((rows + TM - 1) / TM) * gn;
    incl = tg;                                                     // inclusive prefix sum over the lanes
#pragma unroll
    for (int d = 1; d < 64; d <<= 1) {
      const int o = __shfl_up(incl, d, 64);
      if (lane >= d) incl += o;
    }
  };
  int total = 0;
  for (int g0 = 0; g0 < G; g0 += 64) {
    chunk(g0);
    total += __builtin_amdgcn_readlane(incl, 63);
  }
  const int per = (total + 7) >> 3;                                // tiles per XCD
  const int s = (int)(blockIdx.x >> 3) + lane * (int)(gridDim.x >> 3);
  const int u = (int)(blockIdx.x & 7) * per + s;                   // position of this lane's tile in the sequence
  const bool valid = s < per && u < total;
  int f_local = 0, f_rows = 0, f_r0 = 0, f_group = 0, base = 0;
  for (int g0 = 0; g0 < G; g0 += 64) {
    chunk(g0);
    const int excl = incl - tg;
    const int lim = G - g0 < 64 ? G - g0 : 64;
#pragma unroll 1
    for (int l = 0; l < lim; ++l) {
      const int n = __builtin_amdgcn_readlane(tg, l);
      if (n == 0) continue;
      const int local = u - base - __builtin_amdgcn_readlane(excl, l);
      const int lr0 = __builtin_amdgcn_readlane(r0, l), lrows = __builtin_amdgcn_readlane(rows, l);
      if (valid && local >= 0 && local < n) f_local = local, f_rows = lrows, f_r0 = lr0, f_group = g0 + l;
    }
    base += __builtin_amdgcn_readlane(incl, 63);
  }
  // inside a group the row blocks run fastest: the tiles that read one B panel are neighbours in the
  // sequence (they run side by side on one XCD and the second reads the panel from that L2), and the
  // tiles that read one block of A rows are only a group's few row blocks apart
  const int gm = (f_rows + TM - 1) / TM;                           // row blocks of the group (0: the lane found no tile)
  const int tn = gm ? f_local / gm : 0;
  const int tm = f_local - tn * gm;
  t_row0 = f_r0 + tm * TM;
  const int left = f_rows - tm * TM;
  t_desc = (left < TM ? left : TM) | (tn << 9) | (f_group << 20);
}

}  // namespace axe
