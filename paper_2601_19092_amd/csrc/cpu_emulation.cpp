// Host-memory stand-ins for the integer kernels, used only by the CPU tests of the host logic
// (libaxe_hostcheck.so).  They execute the very plans the host layer hands to the kernels --
// same descriptors, same per-work-item arithmetic -- on ordinary memory, and refuse any address
// outside the buffers the caller declared.  The product library never contains this file.
#include <hip/hip_runtime.h>
#include <string.h>

#include "device_types.h"
#include "kernels.h"

namespace axe {

static int64_t g_src_bytes = 0, g_dst_bytes = 0;
static int g_violations = 0;

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
hipError_t launch_gemm_fp8_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }

}  // namespace axe

// Test hooks: declare the real sizes of the host buffers (bytes) and read the violation count.
extern "C" void axe_hostcheck_set_buffers(int64_t src_bytes, int64_t dst_bytes) {
  axe::g_src_bytes = src_bytes;
  axe::g_dst_bytes = dst_bytes;
  axe::g_violations = 0;
}
extern "C" int axe_hostcheck_violations(void) { return axe::g_violations; }
