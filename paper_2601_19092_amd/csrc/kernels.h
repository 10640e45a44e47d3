// Launch entry points of the kernels (host-callable; defined in the .hip files).
#pragma once
#include <hip/hip_runtime.h>
#include <stdlib.h>

#include "device_types.h"

namespace axe {

hipError_t launch_layout_eval(const EvalDesc& d, int64_t n, const int64_t* idx, int64_t* out, hipStream_t s);
hipError_t launch_relayout_joint(const RelayoutPlan& p, int unit_bytes, const void* src, void* dst, hipStream_t s);
// elem_bytes 1, 2, 4 or 8; every 16-byte chunk of a tile row must be aligned on both sides
hipError_t launch_relayout_transpose(const TransposePlan& p, int elem_bytes, const void* src, void* dst, hipStream_t s);
// tile edge (elements) the transposing kernel uses for an element size
// (measured on 8192 x 8192: rows of 256 - 512 bytes per tile beat 128-byte rows by 10 - 17 %, except for
//  single bytes, where the gather of 16 LDS bytes per store makes a 256 x 256 tile slower)
inline int transpose_tile_edge(int elem_bytes) { return elem_bytes == 8 ? 64 : 128; }
hipError_t launch_relayout_generic(const GenericRelayoutPlan& p, int unit_bytes, const void* src, void* dst,
                                   hipStream_t s);
hipError_t launch_gemm_small(const GemmArgs& g, bool fp8, hipStream_t s);
// Large-tile kernels: 256 x tile_n workgroup tile (tile_n = 256, or 224 for bf16); require
// M % 256 == 0, N % tile_n == 0 and K a multiple of the K step (bf16: 64, fp8: 128).
hipError_t launch_gemm_bf16_256(const GemmArgs& g, hipStream_t s);
// grouped (g.group_rows, g.groups, g.ldg set; g.M = rows of all groups together, any value): N % 256 == 0, K % 64 == 0
hipError_t launch_gemm_bf16_256_grouped(const GemmArgs& g, hipStream_t s);
// two grouped problems, the second reading the first's output, as one launch with tile-level hand-over (Sec. 4.1,
// fused MoE layer); sync = M + 1 words of device memory.  need_extra (tests only) raises the count a wait expects,
// so that with a small spin_limit every wait gives up.
// rows the library's own pair workspace serves, and its address on the current device (no allocation: a __device__ array)
constexpr int64_t kPairStaticRows = int64_t(1) << 20;
hipError_t pair_static_workspace(int32_t** out);
hipError_t launch_pair_sync_clear(int32_t* p, int64_t n, hipStream_t s);   // p[0 .. n) = 0, by a small kernel
hipError_t launch_gemm_bf16_256_grouped_pair(const GemmArgs& g1, const GemmArgs& g2, int32_t* sync, int spin_limit, int need_extra,
                                             hipStream_t s);
// dense with ragged edges through the grouped kernel (g.groups = 1, g.group_rows null): any M, N % 8 == 0, K % 64 == 0
hipError_t launch_gemm_bf16_256_ragged(const GemmArgs& g, hipStream_t s);
// rows of a tile of the grouped tile kernel: 128 unless the groups are large on average (the host knows M, not the
// group sizes) or tile_m says otherwise.  Measured on an MoE layer (128 groups, N = 1536, K = 2048 and N = 2048,
// K = 768): 128-row tiles win by 2 - 11 % up to 64 rows per group on average, draw at 256, and lose 3 - 4 % at 512 and
// 7 - 8 % from 1024 on (AXE_GROUPED_TILE128_ROWS overrides the threshold for experiments).
inline int grouped_tile_rows(int64_t M, int groups, int tile_m) {
  static const int small_avg = [] { const char* v = getenv("AXE_GROUPED_TILE128_ROWS"); return v ? atoi(v) : 384; }();
  if (tile_m) return tile_m == 128 ? 128 : 256;
  return M <= (int64_t)small_avg * groups ? 128 : 256;
}
// The same choice for the fp8 grouped tile kernel (AXE_GROUPED_FP8_TILE128_ROWS overrides the threshold).  Measured on
// the same layer with E8M0 scales (gemm1 + gemm2, us, 256-row against 128-row tiles): 16 rows per group 158 against 136,
// 32 rows 163 against 140, 128 rows 224 against 190, 256 rows 281 against 274, 512 rows 429 against 439, 1024 rows 722
// against 775.
inline int grouped_fp8_tile_rows(int64_t M, int groups, int tile_m) {
  static const int small_avg = [] { const char* v = getenv("AXE_GROUPED_FP8_TILE128_ROWS"); return v ? atoi(v) : 384; }();
  if (tile_m == 128 || tile_m == 256) return tile_m;
  return M <= (int64_t)small_avg * groups ? 128 : 256;
}
// grouped, few rows per group: one workgroup per (group, 128 rows of B), weights streamed once, no LDS
hipError_t launch_gemm_grouped_stream(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_fp8_256(const GemmArgs& g, hipStream_t s);
// fp8 with E8M0 block scales (or none) on the matrix cores' scale path; same shape requirements
hipError_t launch_gemm_fp8_e8m0_256(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_fp8_e8m0_256_grouped(const GemmArgs& g, hipStream_t s);

// Compute units of the current device (host side; asked once per process).
inline int cu_count() {
  static int cus = 0;
  if (!cus) {
    int dev = 0, n = 0;
    if (hipGetDevice(&dev) != hipSuccess || hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n <= 0)
      n = 256;
    cus = n;
  }
  return cus;
}


// Whether two planned grouped problems (the second reading what the first writes) can run as one launch: both on
// the chained tile pipeline with the same tile height, and few enough tiles in the worst case that one workgroup per
// compute unit holds them all (a wave keeps 64 per GEMM) -- the workgroups must all be resident for the waits to end.
inline bool grouped_pair_fusable(const GemmArgs& g1, const GemmArgs& g2) {
  const int cus = cu_count();
  const int tm = grouped_tile_rows(g1.M, g1.groups, g1.tile_m);
  if (g1.fp8 || g2.fp8 || g1.f16 != g2.f16 || g1.M != g2.M || g1.groups != g2.groups || !g1.gated || g2.gated || cus % 8) return false;
  if (tm != grouped_tile_rows(g2.M, g2.groups, g2.tile_m)) return false;
  for (const GemmArgs* g : {&g1, &g2}) {
    const int nk = (int)(g->K / 64);
    if (nk % 2 || nk < 4) return false;
    if ((g->M / tm + g->groups) * (int64_t)g->grid_n > 64 * (int64_t)cus) return false;
  }
  return true;
}

}  // namespace axe
