// Grouped GEMM for few rows per group (an MoE layer at decode batch sizes): bound by streaming the
// experts' weights from HBM once, not by the matrix cores.
//
// The 256 x 256 kernel spends a whole tile (and a whole compute unit) on a group with a handful of
// rows, and a launch has too few such tiles to keep every HBM channel busy.  Here a workgroup owns one
// group and 128 rows of its B image (128 columns of C, or 64 with the gated epilogue); each of its four
// waves owns 32 of them -- two MFMA 16x16x32 operand fragments -- for the whole of K and keeps up to 64
// rows of the group as four accumulator fragments per B fragment.  Nothing is shared between waves, so
// there is no LDS and no barrier: the weights go from HBM straight into the MFMA operand registers,
// each element read once per workgroup, many small workgroups in flight per compute unit.
//
// Tile movements as layouts:
//   HBM -> VGPR (B): lane l of a wave reads, for one 64-wide K-tile, the 16-byte chunks l / 16 and l / 16 + 4
//                    of row l % 16 of a fragment: with weights stored in 256 x 64 blocks a fragment's
//                    16 rows x 128 bytes are 2 contiguous KiB (and a workgroup's 128 rows 16 KiB).
//   HBM -> VGPR (A): the same map on the group's rows (they come from L2: every workgroup of a group
//                    reads the same few rows); rows the group does not have load as zero (buffer bounds).
//   MFMA           : operands swapped (B fragment first), so a lane's accumulator fragment holds 4
//                    consecutive columns of one C row; the k order inside a K-tile (chunks q, q + 4) is
//                    the same for A and B, which is all the sum needs.
//   VGPR -> HBM    : 8 bytes per lane and row fragment; rows past the group's end are not stored.
// Groups with more than 64 rows are handled in passes of 64 (the weights are then read again: the
// host chooses this kernel only when the average group is small).  For a handful of rows per group a
// second variant splits K over the four waves of a workgroup (see the template below).
#include <hip/hip_runtime.h>
#include <stdlib.h>

#include "device_types.h"
#include "gemm_common.h"
#include "kernels.h"

namespace axe {

namespace {
typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
typedef __attribute__((ext_vector_type(2))) unsigned int u32x2;

template <bool F16>
__device__ __forceinline__ f32x4 mfma16(u32x4 a, u32x4 b, f32x4 c) {
  if constexpr (F16) {
    typedef __attribute__((ext_vector_type(8))) _Float16 f16x8;
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(__builtin_bit_cast(f16x8, a), __builtin_bit_cast(f16x8, b), c, 0, 0, 0);
  } else {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(__builtin_bit_cast(bf16x8, a), __builtin_bit_cast(bf16x8, b), c, 0, 0, 0);
  }
}
template <bool F16>
__device__ __forceinline__ uint32_t pack16s(float lo, float hi) {
  if constexpr (F16) {
    typedef __attribute__((ext_vector_type(2))) _Float16 f16x2;
    const f16x2 v = {(_Float16)lo, (_Float16)hi};
    return __builtin_bit_cast(uint32_t, v);
  } else {
    return pack_bf16(lo, hi);
  }
}
}  // namespace

// SPLITK = false: a wave owns 32 rows of B for the whole of K, passes of 64 rows of the group (4 row fragments).
// SPLITK = true, for groups of a handful of rows, where a launch has few workgroups: the workgroup owns
// only 32 rows of B, its four waves take a quarter of K each (4 x as many waves and loads in flight for
// the same weights), passes of 16 rows; the four partial sums meet in LDS and wave 0 adds them in a
// fixed order and stores.
//
// DT = 0 bf16, 1 fp16 (a K-tile is 64 elements, two MFMA 16x16x32 per fragment pair), 2 fp8 e4m3 (a K-tile is 128
// elements = one 128-deep scale block and one MFMA 16x16x128; output bf16).  fp8 with scales: one per row of A
// and K-tile (activations), one per 128 x 128 block of each group's B; a K-tile's product is formed alone and
// folded into the sum with the lane's row scale times the fragment's block scale (fp32, or E8M0 codes decoded
// as 2^(code - 127)).  Here the fold costs nothing: the kernel waits for HBM.
// KS = the number of waves that share one set of 32 B rows and split K among them: 0 = SPLITK off (every wave its
// own rows, all of K), 4 (16-bit inputs) or 2 (fp8, whose K-tiles are twice as deep: with 4 a wave's share of K
// would be too few K-tiles for its pipeline); a workgroup then owns 4 / KS sets of 32 rows.
// MI = row fragments per pass (16 MI rows of the group at a time): 1 or 2 go with split K for groups of a handful
// or a dozen of rows, 4 with whole-K waves for the general case, and 4 with split K for launches with few groups
// (a dense GEMM with few rows is the case of one group), where only the K split yields enough workgroups.
template <int DT, bool GATED, int KS, int MI>
__global__ __launch_bounds__(256) void gemm_grouped_stream_kernel(GemmArgs g) {
  constexpr bool SPLITK = KS != 0;
  constexpr int KW = SPLITK ? KS : 1, SETS = SPLITK ? 4 / KS : 4;   // waves per row set, row sets per workgroup
  constexpr bool F16 = DT == 1, FP8 = DT == 2;
  constexpr int EB = FP8 ? 1 : 2;                                  // bytes per element
  __shared__ float partial[SPLITK ? (4 - SETS) * 64 * 8 * MI : 1]; // SPLITK: the sums of the waves that do not store
  const int lane = threadIdx.x & 63;
  const int w = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6));
  const int M = (int)g.M;
  int e = blockIdx.y;                                              // group
  if (g.compact_groups) {
    // fewer rows than groups (the first tokens of a decode batch): at most M groups have rows, and the launch
    // has one workgroup row per possible non-empty group instead of one per group -- an empty workgroup
    // costs nothing but its dispatch, yet thousands of them cost microseconds.  blockIdx.y = a means the
    // a-th non-empty group: the wave finds it by counting, 64 groups per step.
    const int a = e;
    int seen = 0;
    e = -1;
    for (int g0 = 0; g0 < g.groups && e < 0; g0 += 64) {
      const int gi = g0 + lane;
      bool has = false;
      if (gi < g.groups) {
        int x0 = g.group_rows[gi], x1 = g.group_rows[gi + 1];
        x0 = x0 < 0 ? 0 : (x0 > M ? M : x0);
        x1 = x1 < 0 ? 0 : (x1 > M ? M : x1);
        has = x1 > x0;
      }
      uint64_t m = __ballot(has);
      const int cnt = __popcll(m);
      if (a < seen + cnt) {
        for (int k = a - seen; k > 0; --k) m &= m - 1;             // drop the lower set bits
        e = g0 + (int)__builtin_ctzll(m);
      }
      seen += cnt;
    }
    e = __builtin_amdgcn_readfirstlane(e);
    if (e < 0) return;                                             // fewer non-empty groups than workgroup rows
  }
  int r0 = g.group_rows[e], r1 = g.group_rows[e + 1];
  r0 = r0 < 0 ? 0 : (r0 > M ? M : r0);                             // whatever the offsets hold, no access leaves the buffers
  r1 = r1 < 0 ? 0 : (r1 > M ? M : r1);
  if (r1 <= r0) return;                                            // (the whole workgroup: no barrier is left waiting)
  const int nk = (int)(g.K * EB / 128);                            // K-tiles of 128 bytes per row
  const int kpart = SPLITK ? w % KW : 0, wset = SPLITK ? w / KW : w;
  const int k_lo = (nk * kpart) / KW, k_hi = (nk * (kpart + 1)) / KW;   // this wave's K-tiles
  const int fr = lane & 15, fq = lane >> 4;

  // this wave's 32 rows of the group's B image: rows brow .. brow + 31 (two fragments)
  const int brow = (int)blockIdx.x * (32 * SETS) + wset * 32;
  const int tn = brow >> 8;                                        // 256-row block of the image
  const int64_t b_off = (int64_t)e * g.ldg + (int64_t)(tn >> g.b_tpb_shift) * g.b_blk_stride +
                        ((int64_t)(tn & ((1 << g.b_tpb_shift) - 1)) * 256 + (brow & 255)) * g.ldb;
  const int b_pitch = (int)(g.ldb * EB), b_kstep = g.b_kstep;
  const __amdgpu_buffer_rsrc_t rb =
      __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.B + b_off * EB), 0, 31 * b_pitch + (nk - 1) * b_kstep + 128, 0x00020000);
  const int b_voff = fr * b_pitch + fq * 16;
  const int a_pitch = (int)(g.lda * EB);
  // fp8 block scales: this wave's two fragments lie in one 128-column block of the logical B each (with the gated
  // epilogue fragment 0 is a run of gate columns, fragment 1 the same run of up columns, N / 2 further on)
  const bool scaled = FP8 && g.scale_a != nullptr;
  int sb_idx[2] = {0, 0};
  if (scaled) {
    const int nbn = (int)(g.N / 128);
#pragma unroll
    for (int f = 0; f < 2; ++f) {
      const int col = GATED ? f * (int)(g.N / 2) + (brow >> 1) : brow + 16 * f;
      sb_idx[f] = (e * nbn + col / 128) * g.nkb;
    }
  }
  // A scale is fetched with its K-tile and decoded only when the K-tile is multiplied: touching the loaded
  // word right away would make the wave wait for it -- and for every load issued before it, the next K-tile's
  // data included (measured: 92 instead of 69 us on the layer's first GEMM at 64 tokens).  E8M0 codes come as the
  // aligned 4-byte word that holds them (the host requires such arrays 4-byte aligned and padded to whole words).
  auto scale_word = [&](const float* base, int64_t i) -> uint32_t {
    return g.scale_e8m0 ? ((const uint32_t*)base)[i >> 2] : ((const uint32_t*)base)[i];
  };
  auto scale_value = [&](uint32_t word, int64_t i) -> float {
    return __builtin_bit_cast(float, g.scale_e8m0 ? ((word >> (8 * (int)(i & 3))) & 0xffu) << 23 : word);
  };
  const int a_voff = fr * a_pitch + fq * 16;

  for (int p0 = r0; p0 < r1; p0 += 16 * MI) {                      // passes over the rows of the group
    const int rows = r1 - p0 < 16 * MI ? r1 - p0 : 16 * MI;
    const int nfrag = (rows + 15) >> 4;                            // row fragments that hold any row (wave-uniform)
    const __amdgpu_buffer_rsrc_t ra = __builtin_amdgcn_make_buffer_rsrc((void*)((const uint8_t*)g.A + (int64_t)p0 * g.lda * EB), 0,
                                                                        (rows - 1) * a_pitch + (int)g.K * EB, 0x00020000);
    f32x4 acc[2][MI];
#pragma unroll
    for (int f = 0; f < 2; ++f)
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) acc[f][mi] = f32x4{0.f, 0.f, 0.f, 0.f};

    // one K-tile (64 elements) of a fragment is two 16-byte chunks per lane: q (k = 8 q ..) and q + 4 (k = 32 + 8 q ..)
    u32x4 b[2][2][2], a[2][MI][2];                                 // [buffer][fragment][chunk]
    uint32_t sa_w[2][MI], sb_w[2][2];                              // fp8: the K-tile's scales as loaded, fetched with its data
    int kt_of[2] = {0, 0};
    auto sa_index = [&](int mi, int kt) -> int64_t {
      const int row = mi * 16 + fr < rows ? mi * 16 + fr : rows - 1;            // rows past the end are never stored
      return (int64_t)(p0 + row) * g.nkb + kt;
    };
    auto load = [&](int buf, int kt) __attribute__((always_inline)) {
      if (scaled) {
        kt_of[buf] = kt;
#pragma unroll
        for (int f = 0; f < 2; ++f) sb_w[buf][f] = scale_word(g.scale_b, sb_idx[f] + kt);
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
          if (mi < nfrag) sa_w[buf][mi] = scale_word(g.scale_a, sa_index(mi, kt));
      }
#pragma unroll
      for (int f = 0; f < 2; ++f)
#pragma unroll
        for (int h = 0; h < 2; ++h)
          b[buf][f][h] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(rb, b_voff + f * 16 * b_pitch + h * 64, kt * b_kstep, 0));
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        if (mi < nfrag) {
#pragma unroll
          for (int h = 0; h < 2; ++h)
            a[buf][mi][h] = __builtin_bit_cast(u32x4, __builtin_amdgcn_raw_buffer_load_b128(ra, a_voff + mi * 16 * a_pitch + h * 64, kt * 128, 0));
        }
    };
    auto multiply = [&](int buf) __attribute__((always_inline)) {
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        if (mi < nfrag) {
          if constexpr (FP8) {
            const i32x8 av = {(int)a[buf][mi][0][0], (int)a[buf][mi][0][1], (int)a[buf][mi][0][2], (int)a[buf][mi][0][3],
                              (int)a[buf][mi][1][0], (int)a[buf][mi][1][1], (int)a[buf][mi][1][2], (int)a[buf][mi][1][3]};
#pragma unroll
            for (int f = 0; f < 2; ++f) {
              const i32x8 bv = {(int)b[buf][f][0][0], (int)b[buf][f][0][1], (int)b[buf][f][0][2], (int)b[buf][f][0][3],
                                (int)b[buf][f][1][0], (int)b[buf][f][1][1], (int)b[buf][f][1][2], (int)b[buf][f][1][3]};
              if (scaled) {
                const f32x4 part = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bv, av, f32x4{0.f, 0.f, 0.f, 0.f}, 0, 0, 0, 0, 0, 0);
                const float sc = scale_value(sa_w[buf][mi], sa_index(mi, kt_of[buf])) * scale_value(sb_w[buf][f], sb_idx[f] + kt_of[buf]);
#pragma unroll
                for (int x = 0; x < 4; ++x) acc[f][mi][x] = __builtin_fmaf(sc, part[x], acc[f][mi][x]);
              } else {
                acc[f][mi] = __builtin_amdgcn_mfma_scale_f32_16x16x128_f8f6f4(bv, av, acc[f][mi], 0, 0, 0, 0, 0, 0);
              }
            }
          } else {
#pragma unroll
            for (int h = 0; h < 2; ++h)
#pragma unroll
              for (int f = 0; f < 2; ++f) acc[f][mi] = mfma16<F16>(b[buf][f][h], a[buf][mi][h], acc[f][mi]);
          }
        }
    };
    int kt = k_lo;
    if (kt < k_hi) load(0, kt);
    for (; kt + 2 <= k_hi; kt += 2) {                              // two K-tiles per trip, the next one always on its way
      load(1, kt + 1);
      multiply(0);
      if (kt + 2 < k_hi) load(0, kt + 2);
      multiply(1);
    }
    if (kt < k_hi) multiply(0);                                    // odd number of K-tiles: the last one was loaded into buffer 0

    if constexpr (SPLITK) {
      // the waves with kpart > 0 hand their sums to the wave with kpart = 0 of their row set, which adds them
      // in the order of kpart and stores
      if (kpart) {
#pragma unroll
        for (int mi = 0; mi < MI; ++mi)
#pragma unroll
          for (int f = 0; f < 2; ++f)
#pragma unroll
            for (int x = 0; x < 4; ++x)
              partial[(((wset * (KW - 1) + kpart - 1) * MI + mi) * 8 + f * 4 + x) * 64 + lane] = acc[f][mi][x];
      }
      __syncthreads();
      if (kpart == 0) {
#pragma unroll
        for (int v = 0; v < KW - 1; ++v)
#pragma unroll
          for (int mi = 0; mi < MI; ++mi)
#pragma unroll
            for (int f = 0; f < 2; ++f)
#pragma unroll
              for (int x = 0; x < 4; ++x) acc[f][mi][x] += partial[(((wset * (KW - 1) + v) * MI + mi) * 8 + f * 4 + x) * 64 + lane];
      }
      __syncthreads();                                             // the next pass writes the array again
      if (kpart) continue;
    }

    // ---- store: lane holds columns 4 q .. 4 q + 3 of row 16 mi + fr for each of its two fragments
#pragma unroll
    for (int mi = 0; mi < MI; ++mi) {
      const int row = mi * 16 + fr;
      if (mi < nfrag && row < rows) {
        if constexpr (GATED) {                                     // fragment 0 = gate, fragment 1 = up of the same 16 outputs
          float h[4];
#pragma unroll
          for (int x = 0; x < 4; ++x) {
            const float gate = acc[0][mi][x], up = acc[1][mi][x];
            h[x] = gate * __builtin_amdgcn_rcpf(1.0f + __expf(-gate)) * up;
          }
          uint16_t* c = (uint16_t*)g.C + (int64_t)(p0 + row) * g.ldc + (brow >> 1) + 4 * fq;
          *(u32x2*)c = u32x2{pack16s<F16>(h[0], h[1]), pack16s<F16>(h[2], h[3])};
        } else {
#pragma unroll
          for (int f = 0; f < 2; ++f) {
            uint16_t* c = (uint16_t*)g.C + (int64_t)(p0 + row) * g.ldc + brow + f * 16 + 4 * fq;
            *(u32x2*)c = u32x2{pack16s<F16>(acc[f][mi][0], acc[f][mi][1]), pack16s<F16>(acc[f][mi][2], acc[f][mi][3])};
          }
        }
      }
    }
  }
}

namespace {
template <int SPLIT, int MI>                                       // SPLIT: 0 = whole-K waves, 1 = K split over waves
void launch_stream(const GemmArgs& g, unsigned ny, hipStream_t s) {
  const dim3 block(256);
  constexpr int K16 = SPLIT ? 4 : 0, K8 = SPLIT ? 2 : 0;            // waves per row set: 16-bit inputs, fp8
  const dim3 grid16((unsigned)(g.N / (SPLIT ? 32 : 128)), ny), grid8((unsigned)(g.N / (SPLIT ? 64 : 128)), ny);
  switch ((g.fp8 ? 4 : (g.f16 ? 2 : 0)) + (g.gated ? 1 : 0)) {
    case 0: hipLaunchKernelGGL((gemm_grouped_stream_kernel<0, false, K16, MI>), grid16, block, 0, s, g); break;
    case 1: hipLaunchKernelGGL((gemm_grouped_stream_kernel<0, true, K16, MI>), grid16, block, 0, s, g); break;
    case 2: hipLaunchKernelGGL((gemm_grouped_stream_kernel<1, false, K16, MI>), grid16, block, 0, s, g); break;
    case 3: hipLaunchKernelGGL((gemm_grouped_stream_kernel<1, true, K16, MI>), grid16, block, 0, s, g); break;
    case 4: hipLaunchKernelGGL((gemm_grouped_stream_kernel<2, false, K8, MI>), grid8, block, 0, s, g); break;
    default: hipLaunchKernelGGL((gemm_grouped_stream_kernel<2, true, K8, MI>), grid8, block, 0, s, g); break;
  }
}
}  // namespace

// The host knows the number of rows of all groups together, not the group sizes.  With a handful of rows per group
// on average it takes the variant that splits K over the waves and handles 16 rows per pass; then, up to 16 rows
// per group (24 when K is short), the K split with 32 rows per pass (most groups still fit one pass, and the split
// keeps four times the loads in flight); beyond that, whole-K waves with 64 rows per pass -- unless that launch would have fewer
// than two workgroups per compute unit (few groups: a dense GEMM with few rows is one group), where K is split
// as well.  Measured on an MoE layer of 128 experts, 8 per token (gemm1 + gemm2, us; 16 / 32 rows per pass):
// fp16 at 64 tokens 195 / 194, 96 tokens 207 / 200, 128 tokens 217 / 207, 192 tokens 258 / 220; fp8 at 128 tokens
// 121 / 127, 160 tokens 139 / 132, 256 tokens 183 / 156 (64 rows per pass, whole-K waves: 176); 32 rows per pass with
// the K split against 64 with whole-K waves at 20 / 24 rows per group: K = 768 fp8 56 / 62 against 58 / 62, fp16 92 / 101
// against 94 / 102; K = 2048 fp16 186 / 207 against 184 / 194.
// AXE_GROUPED_SPLITK_ROWS overrides the first bound, AXE_GROUPED_STREAM_VARIANT (1: 16 rows, 2: 32 rows, 3: 64 rows
// with the K split, 4: 64 rows, whole-K waves) the whole choice, for experiments.
hipError_t launch_gemm_grouped_stream(const GemmArgs& g0, hipStream_t s) {
  GemmArgs g = g0;
  g.compact_groups = g.M < g.groups;                               // at most M groups can have rows
  const unsigned ny = (unsigned)(g.compact_groups ? g.M : g.groups);
  static const int avg_env = [] { const char* v = getenv("AXE_GROUPED_SPLITK_ROWS"); return v ? atoi(v) : 0; }();
  static const int force = [] { const char* v = getenv("AXE_GROUPED_STREAM_VARIANT"); return v ? atoi(v) : 0; }();
  const int avg = avg_env > 0 ? avg_env : (g.fp8 ? 8 : 4);
  int variant = force;
  if (variant < 1 || variant > 4) {
    if (g.M <= avg * (int64_t)g.groups) variant = 1;
    else if (g.M <= (g.K <= 1024 ? 24 : 16) * (int64_t)g.groups) variant = 2;
    else if ((g.N / 128) * (int64_t)ny < 2 * cu_count()) variant = 3;
    else variant = 4;
  }
  switch (variant) {
    case 1: launch_stream<1, 1>(g, ny, s); break;
    case 2: launch_stream<1, 2>(g, ny, s); break;
    case 3: launch_stream<1, 4>(g, ny, s); break;
    default: launch_stream<0, 4>(g, ny, s); break;
  }
  return hipGetLastError();
}

}  // namespace axe
