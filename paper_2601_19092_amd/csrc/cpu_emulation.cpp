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
  const int64_t T = transpose_tile_edge(eb), CE = 16 / eb, CPR = T / CE;
  ++g_transposes;
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
      const int64_t a = (sb + iD * p.sD + iS) * eb;
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
      const int64_t a = (db + iS * p.dS + iD) * eb;
      if (a < 0 || a + 16 > g_dst_bytes || (a & 15)) {
        ++g_violations;
        continue;
      }
      for (int64_t k = 0; k < CE; ++k) {
        if (!have[(size_t)((cc * CE + k) * T + r)]) ++g_violations;   // would store what was never loaded
        memcpy(dst + a + k * eb, &tile[(size_t)(((cc * CE + k) * T + r) * eb)], (size_t)eb);
      }
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
hipError_t launch_gemm_grouped_stream(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_fp8_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_fp8_e8m0_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace axe

// Test hooks: declare the real sizes of the host buffers (bytes) and read the violation count.
extern "C" void axe_hostcheck_set_buffers(int64_t src_bytes, int64_t dst_bytes) {
  axe::g_src_bytes = src_bytes;
  axe::g_dst_bytes = dst_bytes;
  axe::g_violations = 0;
  axe::g_transposes = 0;
}
extern "C" int axe_hostcheck_violations(void) { return axe::g_violations; }
extern "C" int axe_hostcheck_transposes(void) { return axe::g_transposes; }
