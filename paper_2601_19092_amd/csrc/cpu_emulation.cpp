// Host-memory stand-ins for the integer kernels, used only by the CPU tests of the host logic
// (libaxe_hostcheck.so).  They execute the very plans the host layer hands to the kernels --
// same descriptors, same per-work-item arithmetic -- on ordinary memory, and refuse any address
// outside the buffers the caller declared.  The product library never contains this file.
#include <hip/hip_runtime.h>
#include <string.h>

#include <vector>

#include "device_types.h"
#include "kernels.h"

namespace axe {

static int64_t g_src_bytes = 0, g_dst_bytes = 0;
static int g_violations = 0;
static int g_transposes = 0;      // launches of the transposing relayout since the buffers were declared
static int g_transposes_elem = 0; // ... of which element by element (not in 16-byte chunks)

static int64_t swz_apply(int64_t x, Swz z) { return x ^ (((x >> z.shift) & (int64_t)z.mask) << z.base); }

hipError_t launch_layout_eval(const EvalDesc& d, int64_t n, const int64_t* idx, int64_t* out, hipStream_t) {
  const int64_t per = d.E_R * d.n_axes;
  for (int64_t i = 0; i < n; ++i) {
    int64_t x = idx ? idx[i] : i;
    int64_t* o = out + i * per;
    if (x < 0 || x >= d.E_D) {
      for (int64_t t = 0; t < per; ++t) o[t] = INT64_MIN;
      continue;
    }
    int64_t c[kMaxAxes];
    for (int a = 0; a < kMaxAxes; ++a) c[a] = d.off[a];
    uint64_t rem = (uint64_t)x;
    for (int k = d.n_d - 1; k >= 0; --k) {
      c[d.axis[k]] += (int64_t)(rem % (uint64_t)d.ext[k]) * d.str[k];
      rem /= (uint64_t)d.ext[k];
    }
    for (int64_t t = 0; t < d.E_R; ++t) {
      int64_t r[kMaxAxes];
      memcpy(r, c, sizeof r);
      int64_t tr = t;
      for (int k = d.n_r - 1; k >= 0; --k) {
        r[d.raxis[k]] += (tr % d.rext[k]) * d.rstr[k];
        tr /= d.rext[k];
      }
      for (int a = 0; a < d.n_axes; ++a) o[t * d.n_axes + a] = (a == d.swz_axis) ? swz_apply(r[a], d.swz) : r[a];
    }
  }
  return hipSuccess;
}

static bool move(const char* src, char* dst, int64_t s, int64_t d, int unit) {
  if (s < 0 || (s + 1) * unit > g_src_bytes || d < 0 || (d + 1) * unit > g_dst_bytes) {
    ++g_violations;
    return false;
  }
  memcpy(dst + d * unit, src + s * unit, unit);
  return true;
}

hipError_t launch_relayout_joint(const RelayoutPlan& p, int unit, const void* src_, void* dst_, hipStream_t) {
  const char* src = (const char*)src_;
  char* dst = (char*)dst_;
  for (uint64_t w0 = 0; w0 < p.threads; ++w0) {
    uint32_t w = (uint32_t)w0;
    int64_t s = p.s_off, d = p.d_off;
    for (int k = 0; k < p.n; ++k) {
      uint32_t dig;
      if (p.shift[k] >= 0) {
        dig = w & (p.ext[k] - 1);
        w >>= p.shift[k];
      } else {
        dig = w % p.ext[k];
        w /= p.ext[k];
      }
      s += (int64_t)dig * p.ss[k];
      d += (int64_t)dig * p.ds[k];
    }
    for (int u = 0; u < p.U; ++u) {
      int64_t sa = swz_apply(s + u * p.us, p.s_swz), da = d + u * p.ud;
      for (int64_t t = 0; t < p.E_R; ++t) {
        int64_t tr = t, ra = da;
        for (int k = p.n_r - 1; k >= 0; --k) {
          ra += (tr % p.rext[k]) * p.rstr[k];
          tr /= p.rext[k];
        }
        move(src, dst, sa, swz_apply(ra, p.d_swz), unit);
      }
    }
  }
  return hipSuccess;
}

// Same tiles, same chunk guards and the same addresses as the kernel; a chunk is checked as the 16
// bytes the kernel would touch, on both sides.
hipError_t launch_relayout_transpose(const TransposePlan& p, int eb, const void* src_, void* dst_, hipStream_t) {
  const char* src = (const char*)src_;
  char* dst = (char*)dst_;
  ++g_transposes;
  auto replicas = [&](int64_t a, auto&& f) {                      // every replica address of the destination
    for (int64_t t = 0; t < p.E_R; ++t) {
      int64_t tr = t, ra = a;
      for (int k = p.n_r - 1; k >= 0; --k) {
        ra += (tr % p.rext[k]) * p.rstr[k];
        tr /= p.rext[k];
      }
      f(swz_apply(ra, p.d_swz));
    }
  };
  if (p.elementwise) {                                           // 64 x 64 tiles, element by element
    ++g_transposes_elem;
    const int64_t T = 64;
    for (uint64_t blk = 0; blk < p.blocks; ++blk) {
      uint64_t b = blk;
      const int64_t ts = (int64_t)(b % p.tiles_s);
      b /= p.tiles_s;
      int64_t td = (int64_t)(b % p.tiles_d);
      b /= p.tiles_d;
      if (p.diag > 0) td = (td + ts / p.diag) % p.tiles_d;
      int64_t sb = p.s_off, db = p.d_off;
      for (int k = 0; k < p.n; ++k) {
        sb += (int64_t)(b % p.ext[k]) * p.ss[k];
        db += (int64_t)(b % p.ext[k]) * p.ds[k];
        b /= p.ext[k];
      }
      for (int64_t r = 0; r < T; ++r)
        for (int64_t c = 0; c < T; ++c) {
          const int64_t iD = td * T + r, iS = ts * T + c;
          if (iD >= p.eD || iS >= p.eS) continue;
          const int64_t sa = swz_apply(sb + iD * p.sD + iS, p.s_swz);
          replicas(db + iS * p.dS + iD, [&](int64_t da) { move(src, dst, sa, da, eb); });
        }
    }
    return hipSuccess;
  }
  const int64_t T = transpose_tile_edge(eb), CE = 16 / eb, CPR = T / CE;
  for (uint64_t blk = 0; blk < p.blocks; ++blk) {
    uint64_t b = blk;
    const int64_t ts = (int64_t)(b % p.tiles_s);
    b /= p.tiles_s;
    int64_t td = (int64_t)(b % p.tiles_d);
    b /= p.tiles_d;
    if (p.diag > 0) td = (td + ts / p.diag) % p.tiles_d;
    int64_t sb = p.s_off, db = p.d_off;
    for (int k = 0; k < p.n; ++k) {
      sb += (int64_t)(b % p.ext[k]) * p.ss[k];
      db += (int64_t)(b % p.ext[k]) * p.ds[k];
      b /= p.ext[k];
    }
    std::vector<char> tile((size_t)(T * T * eb), 0);
    std::vector<char> have((size_t)(T * T), 0);
    for (int64_t c = 0; c < T * CPR; ++c) {                       // HBM -> LDS
      const int64_t r = c / CPR, cc = c % CPR, iD = td * T + r, iS = ts * T + cc * CE;
      if (iD >= p.eD || iS >= p.eS) continue;
      const int64_t a = swz_apply(sb + iD * p.sD + iS, p.s_swz) * eb;
      if (a < 0 || a + 16 > g_src_bytes || (a & 15)) {
        ++g_violations;
        continue;
      }
      memcpy(&tile[(size_t)((r * T + cc * CE) * eb)], src + a, 16);
      for (int64_t k = 0; k < CE; ++k) have[(size_t)(r * T + cc * CE + k)] = 1;
    }
    for (int64_t c = 0; c < T * CPR; ++c) {                       // LDS -> HBM
      const int64_t r = c / CPR, cc = c % CPR, iS = ts * T + r, iD = td * T + cc * CE;
      if (iS >= p.eS || iD >= p.eD) continue;
      replicas(db + iS * p.dS + iD, [&](int64_t da) {
        const int64_t a = da * eb;
        if (a < 0 || a + 16 > g_dst_bytes || (a & 15)) {
          ++g_violations;
          return;
        }
        for (int64_t k = 0; k < CE; ++k) {
          if (!have[(size_t)((cc * CE + k) * T + r)]) ++g_violations;   // would store what was never loaded
          memcpy(dst + a + k * eb, &tile[(size_t)(((cc * CE + k) * T + r) * eb)], (size_t)eb);
        }
      });
    }
  }
  return hipSuccess;
}

hipError_t launch_relayout_generic(const GenericRelayoutPlan& p, int unit, const void* src_, void* dst_, hipStream_t) {
  const char* src = (const char*)src_;
  char* dst = (char*)dst_;
  for (int64_t x = 0; x < p.total; ++x) {
    int64_t s = p.s_off, d = p.d_off;
    uint64_t rem = (uint64_t)x;
    for (int k = p.ns - 1; k >= 0; --k) {
      s += (int64_t)(rem % (uint64_t)p.sext[k]) * p.sstr[k];
      rem /= (uint64_t)p.sext[k];
    }
    rem = (uint64_t)x;
    for (int k = p.nd - 1; k >= 0; --k) {
      d += (int64_t)(rem % (uint64_t)p.dext[k]) * p.dstr[k];
      rem /= (uint64_t)p.dext[k];
    }
    for (int64_t t = 0; t < p.E_R; ++t) {
      int64_t tr = t, ra = d;
      for (int k = p.n_r - 1; k >= 0; --k) {
        ra += (tr % p.rext[k]) * p.rstr[k];
        tr /= p.rext[k];
      }
      move(src, dst, swz_apply(s, p.s_swz), swz_apply(ra, p.d_swz), unit);
    }
  }
  return hipSuccess;
}

hipError_t launch_gemm_small(const GemmArgs&, bool, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_bf16_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_bf16_256_grouped(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_bf16_256_ragged(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_pair_sync_clear(int32_t*, int64_t, hipStream_t) { return hipErrorNotSupported; }
hipError_t pair_static_workspace(int32_t**) { return hipErrorNotSupported; }
hipError_t launch_gemm_bf16_256_grouped_pair(const GemmArgs&, const GemmArgs&, int32_t*, int, int, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_grouped_stream(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_fp8_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_fp8_e8m0_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_fp8_e8m0_256_grouped(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace axe

// Test hooks: declare the real sizes of the host buffers (bytes) and read the violation count.
extern "C" void axe_hostcheck_set_buffers(int64_t src_bytes, int64_t dst_bytes) {
  axe::g_src_bytes = src_bytes;
  axe::g_dst_bytes = dst_bytes;
  axe::g_violations = 0;
  axe::g_transposes = 0;
  axe::g_transposes_elem = 0;
}
extern "C" int axe_hostcheck_violations(void) { return axe::g_violations; }
extern "C" int axe_hostcheck_transposes(void) { return axe::g_transposes; }
extern "C" int axe_hostcheck_transposes_elementwise(void) { return axe::g_transposes_elem; }

// ---------------------------------------------------------------------------------------------------------------
// Test hook: a layout axe_gemm_describe reports, evaluated at every point of its tile (through axe_layout_eval and
// the host-memory stand-in above), against the index functions of tile_maps.h that the kernels compute their
// addresses with.  Geometry (tile T x TN x BK, element bytes, waves, wave columns, element offset of the B region in
// an LDS stage, workgroup grid columns for the accumulator layout) comes from the caller.  Returns the number of
// points that differ (0 = the described layout is the kernels' map), or a negative error code.
#include "../../include/axe.h"
#include "tile_maps.h"

extern "C" int axe_hostcheck_describe_vs_tile_maps(const axe_gemm_desc_t* g, int32_t which, int32_t T, int32_t TN, int32_t BK,
                                                   int32_t EB, int32_t NW, int32_t WN, int64_t b_off, int32_t paired_stores) {
  namespace maps = axe::maps;
  enum { M_ = 0, LDS = 1, WG = 2, WAVE = 3, LANE = 4, REG = 5, NAX = 6 };
  axe_layout_t L;
  int64_t shape[AXE_MAX_RANK];
  int32_t rank = 0;
  alignas(16) char arena[4096];
  if (int rc = axe_gemm_describe(g, which, &L, shape, &rank, arena, sizeof arena)) return rc;
  if (rank != 2 || L.n_axes != NAX) return AXE_EINVAL;
  int64_t ER = 1;
  for (int i = 0; i < L.n_r; ++i) ER *= L.r[i].extent;
  const int64_t n = shape[0] * shape[1];
  std::vector<int64_t> pts((size_t)(n * ER * NAX));
  if (int rc = axe_layout_eval(&L, 2, shape, n, nullptr, pts.data(), nullptr)) return rc;
  const int CE = maps::kChunkBytes / EB, CH = BK / CE, WM = NW / WN, F = maps::kFrag;
  const bool big = T > 64, fp8 = EB == 1;
  const bool is_b = which == AXE_DESC_B_G2L_THREADS || which == AXE_DESC_B_LDS || which == AXE_DESC_B_OPERAND;
  int bad = 0;
  for (int64_t x = 0; x < n; ++x) {
    const int64_t u0 = x / shape[1], u1 = x % shape[1];
    const int64_t* p = &pts[(size_t)(x * ER * NAX)];
    int64_t want[NAX] = {0, 0, 0, 0, 0, 0};
    bool replicated = false;
    if (which <= AXE_DESC_B_OPERAND) {
      const int r = (int)(is_b ? u1 : u0), k = (int)(is_b ? u0 : u1);   // row of the operand, k inside the K-tile
      const int chunk = k / CE, e = k % CE;
      if (which == AXE_DESC_A_LDS || which == AXE_DESC_B_LDS) {
        want[LDS] = (is_b ? b_off : 0) + ((int64_t)r * CH + maps::lds_chunk_pos(r, chunk, CH)) * CE + e;
      } else if (which == AXE_DESC_A_G2L_THREADS || which == AXE_DESC_B_G2L_THREADS) {
        if (big) {
          const int RPL = maps::kRowsPerLoad;
          const int w = (r / RPL) % NW, i = r / (RPL * NW), lr = r % RPL;
          if (maps::piece_row(w, i, lr, NW) != r) ++bad;
          want[LANE] = 64 * w + maps::kLargeChunks * lr + maps::lds_chunk_pos(r, chunk, CH);   // thread id: wave folded into the lane axis
          want[REG] = i * CE + e;
        } else {
          const int c = r * CH + chunk, t = c % 256;
          want[WAVE] = t / 64, want[LANE] = t % 64, want[REG] = (c / 256) * CE + e;
        }
      } else {
        const int WT = is_b ? TN / WN : T / WM, NF = WT / F;
        const int wv = r / WT, f = (r % WT) / F, fr = r % F;
        int q = -1, sub = -1;
        for (int s = 0; s < 8 && q < 0; ++s)
          for (int qq = 0; qq < maps::kLaneGroups; ++qq)
            if ((fp8 ? (s < 2 ? maps::operand_chunk_fp8(s, qq) : -1) : maps::operand_chunk_16bit(s, qq)) == chunk) q = qq, sub = s;
        if (q < 0) return AXE_EINVAL;
        want[LANE] = fr + F * q;
        want[REG] = fp8 ? (int64_t)f * 2 * CE + sub * CE + e : ((int64_t)sub * NF + f) * CE + e;
        // the rows are split over one wave dimension and replicated over the other: replica t is wave ...
        replicated = true;
        for (int64_t t = 0; t < ER; ++t) {
          want[WAVE] = is_b ? WN * t + wv : WN * wv + t;
          for (int a = 0; a < NAX; ++a)
            if (p[t * NAX + a] != want[a]) { ++bad; break; }
        }
        if (ER != (is_b ? WM : WN)) ++bad;
      }
    } else {
      const int i = (int)u0, j = (int)u1;                  // element of C (of the padded problem for AXE_DESC_ACC)
      const int gn = (int)(shape[1] / TN);
      const int ti = i % T, tj = j % TN;
      const int WTM = T / WM, WTN = TN / WN, NFN = WTN / F;
      const int wm = ti / WTM, wn = tj / WTN, fi = (ti % WTM) / F, fj = (tj % WTN) / F;
      want[WG] = (int64_t)(i / T) * gn + j / TN;
      want[WAVE] = WN * wm + wn;
      if (which == AXE_DESC_C_STORE && paired_stores) {
        const int cc = tj % (2 * F), pair = (tj % WTN) / (2 * F);
        int q = -1;
        for (int qq = 0; qq < maps::kLaneGroups; ++qq)
          if (cc >= maps::pair_store_col(qq) && cc < maps::pair_store_col(qq) + 2 * maps::kAccCols) q = qq;
        if (q < 0) return AXE_EINVAL;
        want[LANE] = ti % F + F * q;
        want[REG] = ((int64_t)fi * (NFN / 2) + pair) * 2 * maps::kAccCols + (cc - maps::pair_store_col(q));
      } else {
        want[LANE] = ti % F + F * ((tj % F) / maps::kAccCols);
        want[REG] = ((int64_t)fi * NFN + fj) * maps::kAccCols + tj % maps::kAccCols;
      }
    }
    if (!replicated)
      for (int a = 0; a < NAX; ++a)
        if (p[a] != want[a]) { ++bad; break; }
  }
  return bad;
}
