// C ABI of the library: argument validation, layout analysis, kernel choice, launch.
#include <hip/hip_runtime.h>
#include <stdlib.h>
#include <string.h>

#include <algorithm>

#include "../../include/axe.h"
#include "host_layout.h"
#include "kernels.h"

using namespace axe;

namespace {

int hip_fail(hipError_t e, const char* what) {
  set_error("%s: HIP error %d (%s)", what, (int)e, hipGetErrorString(e));
  return AXE_EHIP;
}

int ilog2(int64_t v) {
  int l = 0;
  while ((int64_t(1) << l) < v) ++l;
  return l;
}
bool is_pow2(int64_t v) { return v > 0 && (v & (v - 1)) == 0; }

int env_int(const char* name, int dflt) {
  const char* s = getenv(name);
  return s && *s ? atoi(s) : dflt;
}

}  // namespace

extern "C" {

int32_t axe_version(void) { return 10300; }   // 1.3.0: grouped GEMM, fp16, blocked operands, per-row scales (descriptor fields added)

const char* axe_strerror(int code) {
  switch (code) {
    case AXE_OK: return "ok";
    case AXE_EINVAL: return "invalid argument (violates the definition of an iter / layout)";
    case AXE_ESHAPE: return "shape not admitted by the layout, or inconsistent shapes";
    case AXE_EALIAS: return "destination not injective on the memory axis, or non-memory axis of extent > 1";
    case AXE_ERANGE: return "address outside the declared buffer, or integer overflow";
    case AXE_EUNSUPPORTED: return "layouts outside the supported kernel families";
    case AXE_EHIP: return "HIP runtime failure";
    case AXE_ENOFORM: return "the layout operator's sufficient conditions do not hold";
    case AXE_ETIMEOUT: return "a bounded wait inside a kernel gave up";
    default: return "unknown error code";
  }
}

const char* axe_last_error(void) { return last_error(); }

// ---------------------------------------------------------------------------------------------
int axe_layout_eval(const axe_layout_t* L, int32_t rank, const int64_t* shape, int64_t n, const int64_t* d_flat_idx,
                    int64_t* d_out, void* stream) {
  HLayout h;
  if (int rc = load_layout(L, h, "axe_layout_eval")) return rc;
  if (int rc = check_shape(h, rank, shape, "axe_layout_eval")) return rc;
  if (n < 0) {
    set_error("axe_layout_eval: n = %lld is negative", (long long)n);
    return AXE_EINVAL;
  }
  if (!d_flat_idx && n > h.E_D) {
    set_error("axe_layout_eval: n = %lld exceeds E_D = %lld with implicit indices", (long long)n, (long long)h.E_D);
    return AXE_ERANGE;
  }
  if (n > 0 && !d_out) {
    set_error("axe_layout_eval: d_out is NULL");
    return AXE_EINVAL;
  }
  int64_t per, total;
  if (__builtin_mul_overflow(h.E_R, (int64_t)h.n_axes, &per) || __builtin_mul_overflow(per, n, &total) ||
      total > (INT64_MAX >> 4)) {
    set_error("axe_layout_eval: output size overflows");
    return AXE_ERANGE;
  }
  if (n == 0) return AXE_OK;
  EvalDesc d;
  memset(&d, 0, sizeof d);
  d.n_d = (int)h.D.size();
  d.n_r = (int)h.R.size();
  d.n_axes = h.n_axes;
  d.use32 = h.E_D < (int64_t(1) << 31);
  for (int k = 0; k < d.n_d; ++k) {
    d.ext[k] = h.D[k].e;
    d.str[k] = h.D[k].s;
    d.axis[k] = h.D[k].axis;
    d.shift[k] = is_pow2(h.D[k].e) ? ilog2(h.D[k].e) : -1;
  }
  for (int k = 0; k < d.n_r; ++k) {
    d.rext[k] = h.R[k].e;
    d.rstr[k] = h.R[k].s;
    d.raxis[k] = h.R[k].axis;
  }
  for (int a = 0; a < h.n_axes; ++a) d.off[a] = h.off[a];
  d.swz_axis = h.swz_axis;
  d.swz = Swz{h.swz_axis >= 0 ? (1 << h.swz_bits) - 1 : 0, h.swz_base, h.swz_shift};
  d.E_D = h.E_D;
  d.E_R = h.E_R;
  hipError_t e = launch_layout_eval(d, n, d_flat_idx, d_out, (hipStream_t)stream);
  return e == hipSuccess ? AXE_OK : hip_fail(e, "axe_layout_eval");
}

// ---------------------------------------------------------------------------------------------
// Relayout planning.  The two shard lists are refined to one loop nest (a joint digit system);
// the innermost unit-stride run common to both sides becomes the access width (up to 16 bytes);
// the remaining digits are ordered so that neighbouring threads touch neighbouring memory on at
// least one side, and a per-thread unroll digit is taken along the other side's fastest digit.
int axe_relayout(const axe_layout_t* src, const axe_layout_t* dst, int32_t rank, const int64_t* shape,
                 int32_t elem_bytes, int32_t mem_axis, const void* d_src, int64_t src_elems, void* d_dst,
                 int64_t dst_elems, void* stream) {
  HLayout hs, hd;
  if (int rc = load_layout(src, hs, "axe_relayout(src)")) return rc;
  if (int rc = load_layout(dst, hd, "axe_relayout(dst)")) return rc;
  if (int rc = check_shape(hs, rank, shape, "axe_relayout(src)")) return rc;
  if (int rc = check_shape(hd, rank, shape, "axe_relayout(dst)")) return rc;
  if (!(elem_bytes == 1 || elem_bytes == 2 || elem_bytes == 4 || elem_bytes == 8 || elem_bytes == 16)) {
    set_error("axe_relayout: elem_bytes = %d, must be 1, 2, 4, 8 or 16", elem_bytes);
    return AXE_EINVAL;
  }
  MemLayout ms, md;
  if (int rc = reduce_to_memory(hs, mem_axis, ms, "axe_relayout(src)")) return rc;
  if (int rc = reduce_to_memory(hd, mem_axis, md, "axe_relayout(dst)")) return rc;
  if (int rc = check_range(ms, src_elems, "axe_relayout(src)")) return rc;
  if (int rc = check_range(md, dst_elems, "axe_relayout(dst)")) return rc;
  if (!provably_injective(md)) {
    set_error("axe_relayout(dst): two logical elements may share an address (strides do not nest)");
    return AXE_EALIAS;
  }
  if (!d_src || !d_dst) {
    set_error("axe_relayout: NULL device pointer");
    return AXE_EINVAL;
  }
  if (((uintptr_t)d_src | (uintptr_t)d_dst) % (uintptr_t)elem_bytes) {
    set_error("axe_relayout: buffers are not aligned to the element size");
    return AXE_EINVAL;
  }
  {
    const char* s0 = (const char*)d_src;
    const char* d0 = (const char*)d_dst;
    if (s0 < d0 + dst_elems * elem_bytes && d0 < s0 + src_elems * elem_bytes) {
      set_error("axe_relayout: source and destination buffers overlap");
      return AXE_EINVAL;
    }
  }
  if (md.E_R > (int64_t(1) << 20)) {
    set_error("axe_relayout(dst): %lld replicas", (long long)md.E_R);
    return AXE_EUNSUPPORTED;
  }
  hipStream_t st = (hipStream_t)stream;
  const int64_t E = hs.E_D;

  std::vector<JointIter> J;
  bool joint = joint_refine(ms.D, md.D, J);
  if (!joint) {
    GenericRelayoutPlan p;
    memset(&p, 0, sizeof p);
    p.ns = (int)ms.D.size();
    p.nd = (int)md.D.size();
    for (int k = 0; k < p.ns; ++k) p.sext[k] = ms.D[k].e, p.sstr[k] = ms.D[k].s;
    for (int k = 0; k < p.nd; ++k) p.dext[k] = md.D[k].e, p.dstr[k] = md.D[k].s;
    p.s_off = ms.off;
    p.d_off = md.off;
    p.s_swz = ms.swz;
    p.d_swz = md.swz;
    p.n_r = (int)md.R.size();
    for (int k = 0; k < p.n_r; ++k) p.rext[k] = (int32_t)md.R[k].e, p.rstr[k] = md.R[k].s;
    p.E_R = md.E_R;
    p.total = E;
    hipError_t e = launch_relayout_generic(p, elem_bytes, d_src, d_dst, st);
    return e == hipSuccess ? AXE_OK : hip_fail(e, "axe_relayout");
  }

  // --- transposing case: no digit is contiguous on both sides, but one is contiguous in the source
  //     and another in the destination, and every 16-byte chunk along either is aligned: tiles of
  //     those two digits go through LDS (16-byte accesses on both sides)
  {
    int kS = -1, kD = -1, both = -1;
    for (size_t k = 0; k < J.size(); ++k) {
      if (J[k].e == 1) continue;
      if (J[k].ss == 1 && J[k].ds == 1) both = (int)k;
      else if (J[k].ss == 1) kS = (int)k;
      else if (J[k].ds == 1) kD = (int)k;
    }
    const int64_t ce = elem_bytes <= 8 ? 16 / elem_bytes : 0;
    // the transposing case: tiles of the two digits go through LDS.  Both rows at least 64 bytes long, or the tile
    // is not worth it (the joint loop nest below serves those)
    bool ok = both < 0 && kS >= 0 && kD >= 0 && ce > 0 && md.E_R <= 64 && env_int("AXE_RELAYOUT_TRANSPOSE", 1) != 0 &&
              J[kS].e * elem_bytes >= 64 && J[kD].e * elem_bytes >= 64;
    // ... in whole 16-byte chunks when extents, strides, offsets, replica strides and buffers are chunk multiples and
    // a swizzle stage moves whole chunks; element by element otherwise
    bool chunks = ok;
    if (chunks) {
      chunks = J[kS].e % ce == 0 && J[kD].e % ce == 0 && ms.off % ce == 0 && md.off % ce == 0 &&
               (((uintptr_t)d_src | (uintptr_t)d_dst) & 15) == 0;
      for (size_t k = 0; k < J.size() && chunks; ++k) {
        if ((int)k != kS && J[k].e > 1 && J[k].ss % ce) chunks = false;
        if ((int)k != kD && J[k].e > 1 && J[k].ds % ce) chunks = false;
      }
      for (const HIter& it : md.R)
        if (it.s % ce) chunks = false;
      if (ms.swz.mask && (int64_t(1) << ms.swz.base) % ce) chunks = false;
      if (md.swz.mask && (int64_t(1) << md.swz.base) % ce) chunks = false;
    }
    if (ok) {
      TransposePlan p;
      memset(&p, 0, sizeof p);
      p.elementwise = chunks ? 0 : 1;
      const int64_t T = chunks ? transpose_tile_edge(elem_bytes) : 64;
      p.s_swz = ms.swz, p.d_swz = md.swz;
      p.n_r = (int)md.R.size();
      for (int k = 0; k < p.n_r; ++k) p.rext[k] = (int32_t)md.R[k].e, p.rstr[k] = md.R[k].s;
      p.E_R = md.E_R;
      p.eS = J[kS].e, p.dS = J[kS].ds;
      p.eD = J[kD].e, p.sD = J[kD].ss;
      p.s_off = ms.off, p.d_off = md.off;
      const uint64_t tiles_s = (uint64_t)((p.eS + T - 1) / T), tiles_d = (uint64_t)((p.eD + T - 1) / T);
      uint64_t blocks = tiles_s * tiles_d;
      // outer digits, smallest strides first so that neighbouring workgroups stay close in memory
      std::vector<JointIter> outer;
      for (size_t k = 0; k < J.size(); ++k)
        if ((int)k != kS && (int)k != kD && J[k].e > 1) outer.push_back(J[k]);
      auto mag = [](int64_t x) { return x < 0 ? -x : x; };
      std::stable_sort(outer.begin(), outer.end(), [&](const JointIter& a, const JointIter& b) {
        return std::min(mag(a.ss), mag(a.ds)) < std::min(mag(b.ss), mag(b.ds));
      });
      bool fits = tiles_s < (uint64_t(1) << 31) && tiles_d < (uint64_t(1) << 31) && outer.size() <= (size_t)kMaxJoint;
      for (size_t k = 0; k < outer.size() && fits; ++k) {
        fits = outer[k].e < (int64_t(1) << 31) && blocks < (uint64_t(1) << 31);
        p.ext[k] = (uint32_t)outer[k].e;
        p.ss[k] = outer[k].ss;
        p.ds[k] = outer[k].ds;
        blocks *= (uint64_t)outer[k].e;
      }
      if (fits && blocks < (uint64_t(1) << 31)) {
        p.n = (int)outer.size();
        p.tiles_s = (uint32_t)tiles_s;
        p.tiles_d = (uint32_t)tiles_d;
        p.blocks = blocks;
        const int nt = env_int("AXE_RELAYOUT_NT", -1);
        p.streaming = nt >= 0 ? nt : (2 * E * (int64_t)elem_bytes >= (int64_t(128) << 20));
        p.diag = env_int("AXE_TRANSPOSE_DIAG", 1);
        hipError_t e = launch_relayout_transpose(p, elem_bytes, d_src, d_dst, st);
        return e == hipSuccess ? AXE_OK : hip_fail(e, "axe_relayout");
      }
    }
  }

  // --- vector width: a joint digit with unit stride on both sides
  int unit = elem_bytes;
  int64_t v = 1;
  int vec_k = -1;
  for (size_t k = 0; k < J.size(); ++k)
    if (J[k].ss == 1 && J[k].ds == 1) vec_k = (int)k;
  if (vec_k >= 0) {
    v = 16 / elem_bytes;
    while (v > 1 && (J[vec_k].e % v)) v >>= 1;
    auto fits = [&](int64_t w) {
      for (size_t k = 0; k < J.size(); ++k)
        if ((int)k != vec_k && ((J[k].ss % w) || (J[k].ds % w))) return false;
      for (const HIter& it : md.R)
        if (it.s % w) return false;
      if ((ms.off % w) || (md.off % w)) return false;
      if (ms.swz.mask && (int64_t(1) << ms.swz.base) % w) return false;
      if (md.swz.mask && (int64_t(1) << md.swz.base) % w) return false;
      if (((uintptr_t)d_src | (uintptr_t)d_dst) % (uintptr_t)(w * elem_bytes)) return false;
      return true;
    };
    while (v > 1 && !fits(v)) v >>= 1;
  }
  if (v > 1) {
    int lv = ilog2(v);
    unit = elem_bytes * (int)v;
    for (size_t k = 0; k < J.size(); ++k) {
      if ((int)k == vec_k) {
        J[k].e /= v;
      } else {
        J[k].ss /= v;
        J[k].ds /= v;
      }
    }
    for (HIter& it : md.R) it.s /= v;
    ms.off /= v;
    md.off /= v;
    if (ms.swz.mask) ms.swz.base -= lv, ms.swz.shift -= lv;
    if (md.swz.mask) md.swz.base -= lv, md.swz.shift -= lv;
  }
  J.erase(std::remove_if(J.begin(), J.end(), [](const JointIter& j) { return j.e == 1; }), J.end());

  // --- loop order: fastest digit first, by the smaller of the two |strides|
  auto mag = [](int64_t x) { return x < 0 ? -x : x; };
  std::stable_sort(J.begin(), J.end(), [&](const JointIter& a, const JointIter& b) {
    int64_t ka = std::min(mag(a.ss), mag(a.ds)), kb = std::min(mag(b.ss), mag(b.ds));
    if (ka != kb) return ka < kb;
    return std::max(mag(a.ss), mag(a.ds)) < std::max(mag(b.ss), mag(b.ds));
  });
  // --- unroll digit: the side the thread-fastest non-unit digit does not favour gets its own
  //     fastest digit unrolled inside each thread (so both sides see long contiguous runs)
  int U = 1;
  int64_t us = 0, ud = 0;
  int want_u = env_int("AXE_RELAYOUT_UNROLL", 4);
  if (J.size() >= 2 && want_u > 1) {
    size_t first = (mag(J[0].ss) == 1 && mag(J[0].ds) == 1) ? 1 : 0;   // first digit that favours one side
    if (first < J.size()) {
      bool favours_src = mag(J[first].ss) < mag(J[first].ds);
      int best = -1;
      for (size_t k = first + 1; k < J.size(); ++k) {
        int64_t key = favours_src ? mag(J[k].ds) : mag(J[k].ss);
        int64_t bk = best < 0 ? 0 : (favours_src ? mag(J[best].ds) : mag(J[best].ss));
        if (best < 0 || key < bk) best = (int)k;
      }
      if (best < 0) best = (int)first;
      int u = 1;
      while (u * 2 <= want_u && u * 2 <= 8 && J[best].e % (u * 2) == 0) u *= 2;
      if (u > 1) {
        U = u;
        us = J[best].ss;
        ud = J[best].ds;
        J[best].e /= u;
        J[best].ss *= u;
        J[best].ds *= u;
      }
    }
  }
  J.erase(std::remove_if(J.begin(), J.end(), [](const JointIter& j) { return j.e == 1; }), J.end());

  RelayoutPlan p;
  memset(&p, 0, sizeof p);
  p.n = (int)J.size();
  uint64_t threads = 1;
  for (int k = 0; k < p.n; ++k) {
    if (J[k].e >= (int64_t(1) << 31)) {
      set_error("axe_relayout: digit extent %lld too large", (long long)J[k].e);
      return AXE_EUNSUPPORTED;
    }
    p.ext[k] = (uint32_t)J[k].e;
    p.shift[k] = is_pow2(J[k].e) ? ilog2(J[k].e) : -1;
    p.ss[k] = J[k].ss;
    p.ds[k] = J[k].ds;
    threads *= (uint64_t)J[k].e;
  }
  if (threads >= (uint64_t(1) << 32) || (threads + 255) / 256 >= (uint64_t(1) << 31)) {
    set_error("axe_relayout: %llu work items exceed one launch", (unsigned long long)threads);
    return AXE_EUNSUPPORTED;
  }
  p.U = U;
  p.us = us;
  p.ud = ud;
  p.s_off = ms.off;
  p.d_off = md.off;
  p.s_swz = ms.swz;
  p.d_swz = md.swz;
  p.n_r = (int)md.R.size();
  for (int k = 0; k < p.n_r; ++k) p.rext[k] = (int32_t)md.R[k].e, p.rstr[k] = md.R[k].s;
  p.E_R = md.E_R;
  p.threads = threads;
  // non-temporal accesses once the data cannot stay in the 256 MiB last-level cache anyway
  const int nt = env_int("AXE_RELAYOUT_NT", -1);
  p.streaming = nt >= 0 ? nt : (2 * E * (int64_t)elem_bytes >= (int64_t(128) << 20));
  hipError_t e = launch_relayout_joint(p, unit, d_src, d_dst, st);
  return e == hipSuccess ? AXE_OK : hip_fail(e, "axe_relayout");
}

// ---------------------------------------------------------------------------------------------
// GEMM: recognise the supported family, pick the tile, launch.
namespace {

struct GemmPlan {
  GemmArgs args;
  bool fp8;
  int tile;           // AXE_TILE_*
  bool ragged;        // 256x256 tile on a shape with ragged edges (M, N no multiples of 256)
  int64_t oa, ob, oc; // element offsets of the operands inside their buffers
  int eb, cb;         // bytes per element of A / B and of C
};

// Checks of the device pointers (they change from call to call; everything else of a plan depends on the descriptor
// alone) and the operand addresses.
int bind_gemm_pointers(const axe_gemm_desc_t* g, const void* dA, const void* dB, void* dC, GemmPlan& P) {
  if (!dA || !dB || !dC) {
    set_error("axe_gemm: NULL device pointer");
    return AXE_EINVAL;
  }
  if (((uintptr_t)dA | (uintptr_t)dB | (uintptr_t)dC) & 15) {
    set_error("axe_gemm: device buffers must be 16-byte aligned");
    return AXE_EINVAL;
  }
  const char* c0 = (const char*)dC;
  const char* c1 = c0 + g->c_elems * P.cb;
  const char* a0 = (const char*)dA;
  const char* b0 = (const char*)dB;
  if ((a0 < c1 && c0 < a0 + g->a_elems * P.eb) || (b0 < c1 && c0 < b0 + g->b_elems * P.eb)) {
    set_error("axe_gemm: C overlaps an input buffer");
    return AXE_EINVAL;
  }
  P.args.A = (const char*)dA + P.oa * P.eb;
  P.args.B = (const char*)dB + P.ob * P.eb;
  P.args.C = (char*)dC + P.oc * P.cb;
  return AXE_OK;
}

// The contents of a descriptor as a flat run of words: what a plan depends on, device pointers aside (of the scale
// pointers only whether they are given and their alignment matter).  False when the descriptor is malformed in a way
// that makes its arrays unreadable: the planner then reports the error.
constexpr int kKeyWords = 24 + 3 * (12 + 3 * (AXE_MAX_D + AXE_MAX_R) + AXE_MAX_AXES);
struct PlanKey {
  int64_t w[kKeyWords];
  int n = 0;
  void put(int64_t v) { w[n++] = v; }
};
bool key_of_layout(const axe_layout_t& L, PlanKey& k) {
  if (L.n_axes < 1 || L.n_axes > AXE_MAX_AXES || L.n_d < 1 || L.n_d > AXE_MAX_D || L.n_r < 0 || L.n_r > AXE_MAX_R || !L.d ||
      (L.n_r && !L.r))
    return false;
  k.put(L.n_axes), k.put(L.n_d), k.put(L.n_r);
  for (int i = 0; i < L.n_d; ++i) k.put(L.d[i].extent), k.put(L.d[i].stride), k.put(L.d[i].axis);
  for (int i = 0; i < L.n_r; ++i) k.put(L.r[i].extent), k.put(L.r[i].stride), k.put(L.r[i].axis);
  for (int a = 0; a < L.n_axes; ++a) k.put(L.offset ? L.offset[a] : 0);
  k.put(L.swz_axis), k.put(L.swz_bits), k.put(L.swz_base), k.put(L.swz_shift);
  return true;
}
bool key_of_gemm(const axe_gemm_desc_t* g, PlanKey& k) {
  k.n = 0;
  k.put(g->M), k.put(g->N), k.put(g->K), k.put(g->in_dtype), k.put(g->out_dtype), k.put(g->mem_axis);
  k.put(g->a_elems), k.put(g->b_elems), k.put(g->c_elems), k.put(g->scale_block), k.put(g->tile_hint), k.put(g->scale_dtype);
  k.put(g->scale_a_rows), k.put(g->d_scale_a != nullptr), k.put(g->d_scale_b != nullptr);
  k.put((int64_t)(((uintptr_t)g->d_scale_a | (uintptr_t)g->d_scale_b) & 3));
  return key_of_layout(g->A, k) && key_of_layout(g->B, k) && key_of_layout(g->C, k);
}

// A 2-D operand whose canonical memory layout is "unit stride along `inner`, pitch along
// `outer`": returns pitch and offset.  `outer_first` tells which logical dim comes first.
int strided_2d(const axe_layout_t* L, int mem_axis, int64_t d0, int64_t d1, bool inner_is_dim1, int64_t elems,
               const char* what, int64_t* pitch, int64_t* offset) {
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  int64_t shape[2] = {d0, d1};
  if (int rc = check_shape(h, 2, shape, what)) return rc;
  MemLayout m;
  if (int rc = reduce_to_memory(h, mem_axis, m, what)) return rc;
  if (!m.R.empty()) {
    set_error("%s: replicated GEMM operands are not supported", what);
    return AXE_EUNSUPPORTED;
  }
  if (m.swz.mask) {
    set_error("%s: swizzled HBM operands are not supported by axe_gemm", what);
    return AXE_EUNSUPPORTED;
  }
  if (int rc = check_range(m, elems, what)) return rc;
  const int64_t inner = inner_is_dim1 ? d1 : d0, outer = inner_is_dim1 ? d0 : d1;
  // canonical forms accepted: [(outer, pitch), (inner, 1)] in logical order (or swapped when the
  // inner dim is logical dim 0), or a single merged iter (outer*inner, 1) when pitch == inner
  std::vector<HIter>& D = m.D;
  int64_t p = 0;
  bool ok = false;
  if (D.empty()) {
    ok = (d0 == 1 && d1 == 1);
    p = inner;
  } else if (D.size() == 1) {
    if (D[0].s == 1 && D[0].e == d0 * d1 && (outer == 1 || inner_is_dim1)) ok = true, p = inner;      // contiguous
    else if (inner == 1 && D[0].e == outer) ok = true, p = D[0].s;
    else if (outer == 1 && D[0].e == inner && D[0].s == 1) ok = true, p = inner;
  } else if (D.size() == 2) {
    const HIter& a = D[0];
    const HIter& b = D[1];
    if (inner_is_dim1 && a.e == d0 && b.e == d1 && b.s == 1) ok = true, p = a.s;
    if (!inner_is_dim1 && a.e == d0 && b.e == d1 && a.s == 1) ok = true, p = b.s;
  }
  if (!ok || p < inner) {
    set_error("%s: layout is not a pitched matrix with unit stride along the %s dimension", what,
              inner_is_dim1 ? "second" : "first");
    return AXE_EUNSUPPORTED;
  }
  *pitch = p;
  *offset = m.off;
  return AXE_OK;
}


// An input operand that is not a plain pitched matrix may still be a blocked one (Sec. 3.3: a tile product
// of a grid of blocks and a block): grouped by its logical shape (Alg. 1), the k block is
// [(K / 64, kt_stride), (64, 1)] (64-wide K-tiles stored kt_stride elements apart) and / or the row block is
// [(R / rb, rb_stride), (rb, pitch)].  kt_stride = 0 / rb = 0 in the result mean "not split".
struct Operand2D {
  int64_t pitch, off, kt_stride, rb, rb_stride;
};

int blocked_2d(const axe_layout_t* L, int mem_axis, int64_t d0, int64_t d1, bool k_is_dim1, int64_t elems, const char* what,
               Operand2D* out) {
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  const int64_t shape[2] = {d0, d1};
  if (int rc = check_shape(h, 2, shape, what)) return rc;
  MemLayout m;
  if (int rc = reduce_to_memory(h, mem_axis, m, what)) return rc;
  if (!m.R.empty() || m.swz.mask) {
    set_error("%s: replicated or swizzled GEMM operands are not supported", what);
    return AXE_EUNSUPPORTED;
  }
  if (int rc = check_range(m, elems, what)) return rc;
  axe_layout_t grouped;
  int32_t block_end[2];
  alignas(16) char arena[2048];
  if (int rc = axe_layout_group(L, 2, shape, &grouped, block_end, arena, sizeof arena)) return rc;
  std::vector<HIter> blk[2];
  for (int b = 0, first = 0; b < 2; first = block_end[b++]) {
    for (int i = first; i < block_end[b]; ++i)
      if (grouped.d[i].axis == mem_axis) blk[b].push_back(HIter{grouped.d[i].extent, grouped.d[i].stride, mem_axis});
    canon_D(blk[b]);
    for (const HIter& it : blk[b])
      if (it.s <= 0) {
        set_error("%s: negative strides are not supported", what);
        return AXE_EUNSUPPORTED;
      }
  }
  const std::vector<HIter>& kb = blk[k_is_dim1 ? 1 : 0];
  const std::vector<HIter>& rb = blk[k_is_dim1 ? 0 : 1];
  const int64_t K = k_is_dim1 ? d1 : d0, Rn = k_is_dim1 ? d0 : d1;
  Operand2D o = {0, m.off, 0, 0, 0};
  bool ok = true;
  if (kb.empty()) ok = K == 1;
  else if (kb.size() == 1) ok = kb[0].s == 1 && kb[0].e == K;
  else if (kb.size() == 2) ok = kb[1].s == 1 && kb[1].e == 64 && kb[0].e * 64 == K, o.kt_stride = kb[0].s;
  else ok = false;
  if (rb.empty()) o.pitch = K;
  else if (rb.size() == 1) o.pitch = rb[0].s;
  else if (rb.size() == 2) o.pitch = rb[1].s, o.rb = rb[1].e, o.rb_stride = rb[0].s;
  else ok = false;
  if (ok && rb.size() == 1 && rb[0].e != Rn) ok = false;
  if (!ok || o.pitch < (o.kt_stride ? 64 : K)) {
    set_error("%s: layout is neither a pitched matrix with unit stride along k nor a blocked one "
              "((K/64, s)(64, 1) along k, (R/rb, S)(rb, pitch) along the other dimension)", what);
    return AXE_EUNSUPPORTED;
  }
  *out = o;
  return AXE_OK;
}

int plan_gemm(const axe_gemm_desc_t* g, const void* dA, const void* dB, void* dC, GemmPlan& P, bool need_ptrs) {
  if (!g) {
    set_error("axe_gemm: descriptor is NULL");
    return AXE_EINVAL;
  }
  if (g->M <= 0 || g->N <= 0 || g->K <= 0) {
    set_error("axe_gemm: M, N, K must be positive");
    return AXE_EINVAL;
  }
  if (g->in_dtype != AXE_BF16 && g->in_dtype != AXE_FP8_E4M3 && g->in_dtype != AXE_F16) {
    set_error("axe_gemm: in_dtype %d unknown", g->in_dtype);
    return AXE_EINVAL;
  }
  if (g->out_dtype != AXE_F32 && g->out_dtype != AXE_BF16 && g->out_dtype != AXE_F16) {
    set_error("axe_gemm: out_dtype %d unknown", g->out_dtype);
    return AXE_EINVAL;
  }
  const bool f16 = g->in_dtype == AXE_F16;
  if (g->out_dtype != AXE_F32 && (g->out_dtype == AXE_F16) != f16) {
    set_error("axe_gemm: a 16-bit output has the type that goes with the inputs (fp16 for fp16, bf16 for bf16 and fp8)");
    return AXE_EUNSUPPORTED;
  }
  const bool fp8 = g->in_dtype == AXE_FP8_E4M3;
  const int eb = fp8 ? 1 : 2, ob = g->out_dtype == AXE_F32 ? 4 : 2;
  if ((g->d_scale_a == nullptr) != (g->d_scale_b == nullptr)) {
    set_error("axe_gemm: scales must be given for both operands or neither");
    return AXE_EINVAL;
  }
  if (g->scale_dtype != AXE_SCALE_F32 && g->scale_dtype != AXE_SCALE_E8M0) {
    set_error("axe_gemm: unknown scale_dtype %d", g->scale_dtype);
    return AXE_EINVAL;
  }
  if (g->d_scale_a && g->scale_dtype == AXE_SCALE_E8M0 && (((uintptr_t)g->d_scale_a | (uintptr_t)g->d_scale_b) & 3)) {
    set_error("axe_gemm: E8M0 scale arrays must be 4-byte aligned");
    return AXE_EINVAL;
  }
  if (g->scale_a_rows != 0 && g->scale_a_rows != 1 && g->scale_a_rows != 128) {
    set_error("axe_gemm: scale_a_rows must be 0, 1 or 128");
    return AXE_EINVAL;
  }
  const bool row_scaled = g->d_scale_a && g->scale_a_rows == 1;
  if (g->d_scale_a && (!fp8 || g->scale_block != 128)) {
    set_error("axe_gemm: block scales need in_dtype fp8 and scale_block 128");
    return AXE_EUNSUPPORTED;
  }
  int64_t lda, ldb, ldc, oa, ob_, oc;
  Operand2D opa, opb;
  if (int rc = blocked_2d(&g->A, g->mem_axis, g->M, g->K, true, g->a_elems, "axe_gemm(A)", &opa)) return rc;
  if (int rc = blocked_2d(&g->B, g->mem_axis, g->K, g->N, false, g->b_elems, "axe_gemm(B)", &opb)) return rc;
  if (int rc = strided_2d(&g->C, g->mem_axis, g->M, g->N, true, g->c_elems, "axe_gemm(C)", &ldc, &oc)) return rc;
  lda = opa.pitch, ldb = opb.pitch, oa = opa.off, ob_ = opb.off;
  // blocked operands: the 256-tile bf16 kernel only, row blocks a power-of-two number of tiles high
  const bool blocked = opa.kt_stride || opa.rb || opb.kt_stride || opb.rb;
  auto block_ok = [&](const Operand2D& o) {
    if (o.rb && (o.rb % 256 || !is_pow2(o.rb / 256) || o.rb_stride % 8)) return false;
    if (o.kt_stride && (o.kt_stride % 8 || (g->K / 64) * o.kt_stride * 2 >= (int64_t(1) << 30))) return false;
    return true;
  };
  const int64_t vec = 16 / eb;
  if ((g->K % vec) || (lda % vec) || (ldb % vec) || (oa % vec) || (ob_ % vec)) {
    set_error("axe_gemm: K, leading dimensions and offsets of A and B must be multiples of %lld elements (16 bytes)",
              (long long)vec);
    return AXE_EUNSUPPORTED;
  }
  if ((oc * ob) % 16) {
    set_error("axe_gemm: offset of C must keep 16-byte alignment");
    return AXE_EUNSUPPORTED;
  }
  memset(&P.args, 0, sizeof P.args);
  P.fp8 = fp8;
  P.oa = oa, P.ob = ob_, P.oc = oc, P.eb = eb, P.cb = ob;
  if (need_ptrs) {
    if (int rc = bind_gemm_pointers(g, dA, dB, dC, P)) return rc;
  }
  P.args.M = g->M;
  P.args.N = g->N;
  P.args.K = g->K;
  P.args.lda = lda;
  P.args.ldb = ldb;
  P.args.ldc = ldc;
  P.args.scale_a = (const float*)g->d_scale_a;
  P.args.scale_b = (const float*)g->d_scale_b;
  P.args.scale_e8m0 = g->d_scale_a && g->scale_dtype == AXE_SCALE_E8M0;
  P.args.scale_a_rows = row_scaled ? 1 : 128;
  P.args.nkb = (int32_t)((g->K + 127) / 128);
  P.args.out_bf16 = g->out_dtype != AXE_F32;
  P.args.f16 = f16;
  const int64_t bk = fp8 ? 128 : 64;
  // the large-tile kernels address a tile's 256 rows through 32-bit buffer offsets
  const bool pitch_ok = 256 * lda * eb < (int64_t(1) << 31) && 256 * ldb * eb < (int64_t(1) << 31);
  const bool big_common = (g->M % 256 == 0) && (g->K % bk == 0) && (ldc % 8 == 0) && P.args.out_bf16 && pitch_ok;
  // 16-bit inputs: the 256x256 tile also stores fp32 (a wave's part of C is addressed through 32-bit byte offsets)
  const bool big_f32 = !fp8 && !P.args.out_bf16 && (g->M % 256 == 0) && (g->N % 256 == 0) && (g->K % 64 == 0) && (ldc % 4 == 0) &&
                       pitch_ok && 256 * ldc * 4 < (int64_t(1) << 31);
  const bool big_ok = (big_common && (g->N % 256 == 0)) || big_f32;
  // bf16 only: 224 columns per tile (7 fragments per wave instead of 8)
  const bool n224_ok = big_common && !fp8 && !f16 && (g->N % 224 == 0);
  // 16-bit inputs: the 256x256 tile also on edges that do not fill a tile (a lane stores 8 columns at once; a wave's
  // part of C and the tile's part of B are addressed through 32-bit offsets; tile columns are counted in 11 bits)
  const int64_t cvec = P.args.out_bf16 ? 8 : 4;                    // columns a lane stores at once
  const bool ragged_ok = !fp8 && (g->K % 64 == 0) && (g->N % cvec == 0) && (ldc % cvec == 0) && pitch_ok &&
                         256 * ldc * ob < (int64_t(1) << 31) && g->N <= 2048 * 256 && g->M < (int64_t(1) << 31);
  int tile = g->tile_hint;
  if (row_scaled) {
    // one scale per row of A: the 64 x 64 kernel folds it per lane (fp32 or E8M0); the 256 x 256 kernel on the matrix
    // cores' scale path takes E8M0 row codes a window of 8 K-tiles at a time
    const bool rows_big = big_ok && P.args.scale_e8m0 && g->M * (int64_t)P.args.nkb < (int64_t(1) << 30);
    if (tile == AXE_TILE_256x256x64 && !rows_big) {
      set_error("axe_gemm: one scale per row of A on the 256x256 tile needs E8M0 scales, K a multiple of 128 and M, N multiples of 256");
      return AXE_EUNSUPPORTED;
    }
    if (tile != AXE_TILE_AUTO && tile != AXE_TILE_64x64x32 && tile != AXE_TILE_256x256x64) {
      set_error("axe_gemm: one scale per row of A is served by the 64x64 and the 256x256 kernels");
      return AXE_EUNSUPPORTED;
    }
    if (tile == AXE_TILE_AUTO && !rows_big) tile = AXE_TILE_64x64x32;
  }
  if (blocked) {
    if (fp8 || !big_ok || !block_ok(opa) || !block_ok(opb) || (tile != AXE_TILE_AUTO && tile != AXE_TILE_256x256x64)) {
      set_error("axe_gemm: blocked operands need the 16-bit 256x256 tile (M, N multiples of 256, K of 64), "
                "row blocks of 256 x 2^n rows and strides that are multiples of 16 bytes");
      return AXE_EUNSUPPORTED;
    }
    tile = AXE_TILE_256x256x64;
  }
  if (tile == AXE_TILE_AUTO) {
    tile = big_ok ? AXE_TILE_256x256x64 : (n224_ok ? AXE_TILE_256x224x64 : AXE_TILE_64x64x32);
    // 16-bit inputs: the large tile only once the 64 x 64 tiles of C would take more than about four rounds on the
    // chip (measured, bf16, K = 1024 .. 4096: 768 x 768 12 vs 27 us, 1000 x 1000 12 vs 27 us, 2000 x 2000 41 vs 47 us,
    // 4000 x 4000 388 vs 107 us -- a single large tile takes 27 - 47 us on its own, the small tiles' time grows
    // with M x N); with ragged edges as well as without
    static const int64_t large_min = [] { const char* v = getenv("AXE_LARGE_TILE_MIN_ELEMS"); return v ? atoll(v) : int64_t(5) << 20; }();
    // (fp8: the 64 x 64 kernel is slower per tile; measured crossover near 1024 x 1024 -- 256^3: 8 vs 14 us,
    //  1024^3: 19 vs 20 us, 2048^3: 91 vs 30 us)
    const bool large = g->M * g->N >= (fp8 ? std::min<int64_t>(large_min, int64_t(1) << 20) : large_min);
    if (!large) tile = AXE_TILE_64x64x32;
    if (tile == AXE_TILE_64x64x32 && ragged_ok && large) tile = AXE_TILE_256x256x64;
    if (big_ok && n224_ok && tile != AXE_TILE_64x64x32) {
      // both fit: the launch runs ceil(tiles / compute units) rounds of tiles one after the other,
      // each as long as the tile is wide; take the narrower tile when that is shorter in total
      const int64_t cus = axe::cu_count(), gm = g->M / 256;
      const int64_t t256 = (gm * (g->N / 256) + cus - 1) / cus * 256, t224 = (gm * (g->N / 224) + cus - 1) / cus * 224;
      if (t224 < t256) tile = AXE_TILE_256x224x64;
    }
  }
  P.ragged = tile == AXE_TILE_256x256x64 && !big_ok && !blocked && ragged_ok;
  if (tile == AXE_TILE_256x256x64 && !big_ok && !P.ragged) {
    set_error("axe_gemm: the 256x256 tile needs K a multiple of %lld, row pitches below 2^31 / 256 bytes and M, N multiples "
              "of 256 (16-bit inputs: any M, N a multiple of 8, or of 4 with an fp32 output, which goes with 16-bit inputs only)",
              (long long)bk);
    return AXE_EUNSUPPORTED;
  }
  if (tile == AXE_TILE_256x224x64 && !n224_ok) {
    set_error("axe_gemm: the 256x224 tile needs bf16 inputs, M a multiple of 256, N of 224, K of 64, bf16 output and "
              "row pitches below 2^31 / 256 bytes");
    return AXE_EUNSUPPORTED;
  }
  if (tile != AXE_TILE_256x256x64 && tile != AXE_TILE_256x224x64 && tile != AXE_TILE_64x64x32) {
    set_error("axe_gemm: unknown tile_hint %d", tile);
    return AXE_EINVAL;
  }
  P.tile = tile;
  const int64_t bm = tile == AXE_TILE_64x64x32 ? 64 : 256;
  const int64_t bn = tile == AXE_TILE_64x64x32 ? 64 : (tile == AXE_TILE_256x224x64 ? 224 : 256);
  P.args.grid_m = (int32_t)((g->M + bm - 1) / bm);
  P.args.grid_n = (int32_t)((g->N + bn - 1) / bn);
  P.args.tile_n = (int32_t)bn;
  P.args.a_kstep = (int32_t)(opa.kt_stride ? opa.kt_stride * eb : 64 * eb);
  P.args.b_kstep = (int32_t)(opb.kt_stride ? opb.kt_stride * eb : 64 * eb);
  P.args.a_tpb_shift = opa.rb ? ilog2(opa.rb / 256) : 0;
  P.args.b_tpb_shift = opb.rb ? ilog2(opb.rb / 256) : 0;
  P.args.a_blk_stride = opa.rb ? opa.rb_stride : bm * lda;
  P.args.b_blk_stride = opb.rb ? opb.rb_stride : bn * ldb;
  if (P.ragged) P.args.groups = 1, P.args.tile_m = 256;            // one group of all rows, no offsets array
  if (P.args.grid_m > 65535) {
    set_error("axe_gemm: M too large for one launch");
    return AXE_EUNSUPPORTED;
  }
  return AXE_OK;
}


// B of a grouped GEMM, logical (G, K, N): grouped by that shape (Alg. 1) the group block must be one iter
// on the memory axis (one stride between groups); the k and n blocks are those of a pitched or blocked
// matrix (blocked_2d above).
// gated: logical column n = h * (N / 2) + 16 f + i (h = 0: gate, 1: up) must sit in memory row 32 f + 16 h + i of
// the group's image -- n block [(2, 16 p), (N / 32, 32 p), (16, p)], or with 256-row blocks
// [(2, 16 p), (N / 256, S), (8, 32 p), (16, p)] -- which the result then describes as that image's rows.
int grouped_b(const axe_layout_t* L, int mem_axis, int64_t G, int64_t K, int64_t N, int64_t elems, bool gated, int64_t* ldg,
              Operand2D* out) {
  const char* what = "axe_gemm_grouped(B)";
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  const int64_t shape[3] = {G, K, N};
  if (int rc = check_shape(h, 3, shape, what)) return rc;
  MemLayout m;
  if (int rc = reduce_to_memory(h, mem_axis, m, what)) return rc;
  if (!m.R.empty() || m.swz.mask) {
    set_error("%s: replicated or swizzled operands are not supported", what);
    return AXE_EUNSUPPORTED;
  }
  if (int rc = check_range(m, elems, what)) return rc;
  axe_layout_t grouped;
  int32_t block_end[3];
  alignas(16) char arena[2048];
  if (int rc = axe_layout_group(L, 3, shape, &grouped, block_end, arena, sizeof arena)) return rc;
  std::vector<HIter> blk[3];
  for (int b = 0, first = 0; b < 3; first = block_end[b++]) {
    for (int i = first; i < block_end[b]; ++i)
      if (grouped.d[i].axis == mem_axis) blk[b].push_back(HIter{grouped.d[i].extent, grouped.d[i].stride, mem_axis});
    canon_D(blk[b]);                                               // D0, D1 inside the block
    for (const HIter& it : blk[b])
      if (it.s <= 0) {
        set_error("%s: negative strides are not supported", what);
        return AXE_EUNSUPPORTED;
      }
  }
  if (blk[0].size() > 1) {
    set_error("%s: the groups are not a single stride apart", what);
    return AXE_EUNSUPPORTED;
  }
  *ldg = blk[0].empty() ? 0 : blk[0][0].s;
  Operand2D o = {0, m.off, 0, 0, 0};
  const std::vector<HIter>&kb = blk[1], &nb = blk[2];
  bool ok = true;
  if (kb.empty()) ok = K == 1;
  else if (kb.size() == 1) ok = kb[0].s == 1;
  else if (kb.size() == 2) ok = kb[1].s == 1 && kb[1].e == 64, o.kt_stride = kb[0].s;
  else ok = false;
  if (gated) {
    const size_t n = nb.size();
    const int64_t p = n ? nb[n - 1].s : 0;
    if ((n != 3 && n != 4) || nb[0].e != 2 || nb[0].s != 16 * p || nb[n - 1].e != 16 || nb[n - 2].s != 32 * p ||
        (n == 4 && nb[2].e != 8)) {
      set_error("%s: the gated epilogue needs gate and up columns interleaved in runs of 16 rows: n block "
                "(2, 16 p)(N/32, 32 p)(16, p) or, in 256-row blocks, (2, 16 p)(N/256, S)(8, 32 p)(16, p)", what);
      return AXE_EUNSUPPORTED;
    }
    o.pitch = p;
    if (n == 4) o.rb = 256, o.rb_stride = nb[1].s;
  } else if (nb.empty()) o.pitch = K;
  else if (nb.size() == 1) o.pitch = nb[0].s;
  else if (nb.size() == 2) o.pitch = nb[1].s, o.rb = nb[1].e, o.rb_stride = nb[0].s;
  else ok = false;
  if (!ok || o.pitch < (o.kt_stride ? 64 : K)) {
    set_error("%s: each group's matrix must be column-major (unit stride along k) or blocked "
              "((K/64, s)(64, 1) along k, (N/rb, S)(rb, pitch) along n)", what);
    return AXE_EUNSUPPORTED;
  }
  *out = o;
  return AXE_OK;
}

int plan_gemm_grouped(const axe_gemm_grouped_desc_t* g, const void* dA, const void* dB, void* dC, const int32_t* rows,
                      GemmArgs& a, bool need_ptrs) {
  const char* fn = "axe_gemm_grouped";
  if (!g) {
    set_error("%s: descriptor is NULL", fn);
    return AXE_EINVAL;
  }
  if (g->M <= 0 || g->N <= 0 || g->K <= 0 || g->G <= 0) {
    set_error("%s: M, N, K, G must be positive", fn);
    return AXE_EINVAL;
  }
  const bool fp8 = g->in_dtype == AXE_FP8_E4M3 && g->out_dtype == AXE_BF16;
  if (!((g->in_dtype == AXE_BF16 && g->out_dtype == AXE_BF16) || (g->in_dtype == AXE_F16 && g->out_dtype == AXE_F16) || fp8)) {
    set_error("%s: bf16 inputs with bf16 output, fp16 inputs with fp16 output, or fp8 inputs with bf16 output", fn);
    const bool known = (g->in_dtype >= AXE_BF16 && g->in_dtype <= AXE_F16 && g->in_dtype != AXE_F32) &&
                       (g->out_dtype == AXE_BF16 || g->out_dtype == AXE_F32 || g->out_dtype == AXE_F16);
    return known ? AXE_EUNSUPPORTED : AXE_EINVAL;
  }
  int64_t lda, ldb, ldc, ldg, oa, ob, oc;
  Operand2D opb;
  if (int rc = strided_2d(&g->A, g->mem_axis, g->M, g->K, true, g->a_elems, "axe_gemm_grouped(A)", &lda, &oa)) return rc;
  if (g->epilogue != AXE_EPI_NONE && g->epilogue != AXE_EPI_SWIGLU) {
    set_error("%s: unknown epilogue %d", fn, g->epilogue);
    return AXE_EINVAL;
  }
  if (g->kernel_hint < AXE_GROUPED_AUTO || g->kernel_hint > AXE_GROUPED_TILES_128) {
    set_error("%s: unknown kernel_hint %d", fn, g->kernel_hint);
    return AXE_EINVAL;
  }
  const bool gated = g->epilogue == AXE_EPI_SWIGLU;
  const int64_t NC = gated ? g->N / 2 : g->N;                      // columns of C
  if (int rc = grouped_b(&g->B, g->mem_axis, g->G, g->K, g->N, g->b_elems, gated, &ldg, &opb)) return rc;
  ldb = opb.pitch, ob = opb.off;
  if ((opb.rb && (opb.rb % 256 || !is_pow2(opb.rb / 256) || opb.rb_stride % 8)) ||
      (opb.kt_stride && (opb.kt_stride % 8 || (g->K / 64) * opb.kt_stride * 2 >= (int64_t(1) << 30)))) {
    set_error("%s: a blocked B needs row blocks of 256 x 2^n columns of C and strides that are multiples of 16 bytes", fn);
    return AXE_EUNSUPPORTED;
  }
  if (int rc = strided_2d(&g->C, g->mem_axis, g->M, NC, true, g->c_elems, "axe_gemm_grouped(C)", &ldc, &oc)) return rc;
  const int eb = fp8 ? 1 : 2;
  const int64_t vec = 16 / eb;
  if ((g->K % vec) || (lda % vec) || (ldb % vec) || (ldg % vec) || (oa % vec) || (ob % vec) || (oc % 8) || (ldc % 8)) {
    set_error("%s: K, leading dimensions, the group stride and offsets must be multiples of 16 bytes", fn);
    return AXE_EUNSUPPORTED;
  }
  if ((g->d_scale_a == nullptr) != (g->d_scale_b == nullptr) || (g->d_scale_a && !fp8) ||
      (g->scale_dtype != AXE_SCALE_F32 && g->scale_dtype != AXE_SCALE_E8M0)) {
    set_error("%s: block scales come in pairs, with fp8 inputs only, as fp32 or E8M0", fn);
    return AXE_EINVAL;
  }
  if (g->d_scale_a && g->scale_dtype == AXE_SCALE_E8M0 && (((uintptr_t)g->d_scale_a | (uintptr_t)g->d_scale_b) & 3)) {
    set_error("%s: E8M0 scale arrays must be 4-byte aligned", fn);
    return AXE_EINVAL;
  }
  const bool tiles_forced = g->kernel_hint == AXE_GROUPED_TILES || g->kernel_hint == AXE_GROUPED_TILES_256 || g->kernel_hint == AXE_GROUPED_TILES_128;
  if (fp8 && (g->K % 128 || opb.kt_stride || opb.rb)) {
    set_error("%s: fp8 inputs need K a multiple of 128 and each B[e] column-major (not blocked)", fn);
    return AXE_EUNSUPPORTED;
  }
  // fp8 on the tile kernel (the matrix cores' scale path, tiles of 256 or 128 rows): E8M0 scales or none; with the gated
  // epilogue the gate and the up half must each be whole 128-wide scale blocks; the row codes are addressed in 32 bits
  const bool fp8_tiles_ok = fp8 && (!g->d_scale_a || (g->scale_dtype == AXE_SCALE_E8M0 && (!gated || (g->N / 2) % 128 == 0) &&
                                                       g->M * ((g->K + 127) / 128) >= 8 && g->M * ((g->K + 127) / 128) < (int64_t(1) << 30)));
  if (fp8 && tiles_forced && !fp8_tiles_ok) {
    set_error("%s: the fp8 tile kernel takes E8M0 scales or none (gated: N / 2 a multiple of 128)", fn);
    return AXE_EUNSUPPORTED;
  }
  if (g->G > 4096 || g->N % 256 || g->N / 256 > 2048 || g->K % 64 || g->M >= (int64_t(1) << 31) ||
      256 * lda * eb >= (int64_t(1) << 31) || 256 * ldb * eb >= (int64_t(1) << 31) || 128 * ldc * 2 >= (int64_t(1) << 31)) {
    set_error("%s: needs G <= 4096, N a multiple of 256 (at most 2048 tile columns), K a multiple of 64, M < 2^31 and "
              "row pitches below 2^31 / 256 bytes", fn);
    return AXE_EUNSUPPORTED;
  }
  if ((g->M / 256 + g->G) * (g->N / 256) > (int64_t(1) << 24)) {
    set_error("%s: too many tiles for one launch", fn);
    return AXE_EUNSUPPORTED;
  }
  if (need_ptrs) {
    if (!dA || !dB || !dC || !rows) {
      set_error("%s: NULL device pointer", fn);
      return AXE_EINVAL;
    }
    if ((((uintptr_t)dA | (uintptr_t)dB | (uintptr_t)dC) & 15) || ((uintptr_t)rows & 3)) {
      set_error("%s: device buffers must be 16-byte aligned (group_rows: 4-byte)", fn);
      return AXE_EINVAL;
    }
    const char* c0 = (const char*)dC;
    const char* c1 = c0 + g->c_elems * 2;
    const char* a0 = (const char*)dA;
    const char* b0 = (const char*)dB;
    const char* r0 = (const char*)rows;
    if ((a0 < c1 && c0 < a0 + g->a_elems * eb) || (b0 < c1 && c0 < b0 + g->b_elems * eb) ||
        (r0 < c1 && c0 < r0 + (g->G + 1) * 4)) {
      set_error("%s: C overlaps an input buffer", fn);
      return AXE_EINVAL;
    }
  }
  memset(&a, 0, sizeof a);
  a.A = (const char*)dA + oa * eb;
  a.B = (const char*)dB + ob * eb;
  a.C = (char*)dC + oc * 2;
  a.M = g->M, a.N = g->N, a.K = g->K;
  a.lda = lda, a.ldb = ldb, a.ldc = ldc, a.ldg = ldg;
  a.out_bf16 = 1;
  a.f16 = g->in_dtype == AXE_F16;
  a.fp8 = fp8;
  a.scale_a = (const float*)g->d_scale_a;
  a.scale_b = (const float*)g->d_scale_b;
  a.scale_e8m0 = g->d_scale_a && g->scale_dtype == AXE_SCALE_E8M0;
  a.nkb = (int32_t)((g->K + 127) / 128);
  a.grid_m = 0;
  a.grid_n = (int32_t)(g->N / 256);
  a.tile_n = 256;
  a.a_kstep = 128;
  a.b_kstep = (int32_t)(opb.kt_stride ? opb.kt_stride * 2 : 128);
  a.b_tpb_shift = opb.rb ? ilog2(opb.rb / 256) : 0;
  a.a_blk_stride = 256 * lda;
  a.b_blk_stride = opb.rb ? opb.rb_stride : 256 * ldb;
  a.group_rows = rows;
  a.groups = g->G;
  a.gated = gated;
  a.tile_m = g->kernel_hint == AXE_GROUPED_TILES_256 ? 256 : (g->kernel_hint == AXE_GROUPED_TILES_128 ? 128 : 0);
  if (fp8 && !fp8_tiles_ok) a.tile_m = -1;                         // -1: only the streaming kernel serves this problem
  return AXE_OK;
}

// Which kernel a planned grouped problem goes to: the streaming kernel while the groups average few rows, then the
// tile kernels.  The crossover depends on K -- a tile's fixed costs (tile table, prologue, stores) weigh more when its
// K loop is short -- and was measured on the two GEMMs of an MoE layer (128 groups; gemm1: K = 2048, gemm2: K = 768;
// streaming kernel against tiles, us): fp16 gemm1 at 12 rows per group 148 against 152, at 16 rows 165 against 152;
// fp16 gemm2 at 16 rows 84 against 88, at 20 rows 92 against 90; fp8 (tiles of 128 rows) gemm1 at 6 rows 78 against 84,
// at 8 rows 84 against 85, at 10 rows 91 against 85; fp8 gemm2 at 12 rows 44 against 49, at 16 rows 50 against 50, at
// 20 rows 55 against 50.  Far from the crossover (fp8 layer): 4 rows per group 104 against 151, 256 rows 1373 against 274.
bool grouped_goes_to_stream(const axe_gemm_grouped_desc_t* g, const GemmArgs& a) {
  if (g->kernel_hint == AXE_GROUPED_STREAM) return true;
  if (a.fp8 && a.tile_m < 0) return true;
  if (g->kernel_hint != AXE_GROUPED_AUTO) return false;            // tiles asked for
  const bool short_k = g->K <= 1024;
  int64_t rows = a.fp8 ? (short_k ? 15 : 8) : (short_k ? 19 : 13);
  if (a.fp8) {
    static const int64_t min_rows = [] { const char* v = getenv("AXE_GROUPED_FP8_TILE_ROWS"); return v ? atoll(v) : int64_t(0); }();
    if (min_rows > 0) rows = min_rows - 1;
  }
  return g->M <= rows * (int64_t)g->G;
}

}  // namespace

int axe_gemm_grouped(const axe_gemm_grouped_desc_t* g, const void* d_A, const void* d_B, void* d_C,
                     const int32_t* d_group_rows, void* stream) {
  GemmArgs a;
  if (int rc = plan_gemm_grouped(g, d_A, d_B, d_C, d_group_rows, a, true)) return rc;
  hipError_t e = grouped_goes_to_stream(g, a) ? launch_gemm_grouped_stream(a, (hipStream_t)stream)
                 : a.fp8                      ? launch_gemm_fp8_e8m0_256_grouped(a, (hipStream_t)stream)
                                              : launch_gemm_bf16_256_grouped(a, (hipStream_t)stream);
  return e == hipSuccess ? AXE_OK : hip_fail(e, "axe_gemm_grouped");
}

// Chosen kernel, for tests and tools: AXE_GROUPED_STREAM, AXE_GROUPED_TILES_256 or AXE_GROUPED_TILES_128, or a negative error.
int axe_gemm_grouped_kernel(const axe_gemm_grouped_desc_t* g) {
  GemmArgs a;
  if (int rc = plan_gemm_grouped(g, nullptr, nullptr, nullptr, nullptr, a, false)) return rc;
  if (grouped_goes_to_stream(g, a)) return AXE_GROUPED_STREAM;
  if (a.fp8) return grouped_fp8_tile_rows(a.M, a.groups, a.tile_m) == 128 ? AXE_GROUPED_TILES_128 : AXE_GROUPED_TILES_256;
  return grouped_tile_rows(a.M, a.groups, a.tile_m) == 128 ? AXE_GROUPED_TILES_128 : AXE_GROUPED_TILES_256;
}

int axe_gemm_grouped_check(const axe_gemm_grouped_desc_t* g) {
  GemmArgs a;
  return plan_gemm_grouped(g, nullptr, nullptr, nullptr, nullptr, a, false);
}

namespace {
// The two problems of axe_gemm_grouped_pair, planned: the second must read exactly what the first writes.
int plan_grouped_pair(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2, const void* dA, const void* dB1, void* dH,
                      const void* dB2, void* dC, const int32_t* rows, GemmArgs& a1, GemmArgs& a2, bool need_ptrs) {
  const char* fn = "axe_gemm_grouped_pair";
  // (a placeholder keeps the address arithmetic of the two plans comparable when no pointers are given)
  void* h = need_ptrs ? dH : (void*)(uintptr_t)4096;
  if (int rc = plan_gemm_grouped(g1, need_ptrs ? dA : nullptr, need_ptrs ? dB1 : nullptr, h, rows, a1, need_ptrs)) return rc;
  if (int rc = plan_gemm_grouped(g2, h, need_ptrs ? dB2 : nullptr, need_ptrs ? dC : nullptr, rows, a2, need_ptrs)) return rc;
  const int64_t NC1 = g1->epilogue == AXE_EPI_SWIGLU ? g1->N / 2 : g1->N;
  if (g1->M != g2->M || g1->G != g2->G || g2->K != NC1 || g1->out_dtype != g2->in_dtype || g1->c_elems != g2->a_elems ||
      a1.C != a2.A || a1.ldc != a2.lda) {
    set_error("%s: the second problem's A must be the first problem's C: same M, G, element type, element count, layout, and K2 = "
              "columns of C1", fn);
    return AXE_EINVAL;
  }
  if (need_ptrs) {
    // in one launch tiles of the second problem are stored while tiles of the first still read their inputs: the
    // outputs (H, C) must be disjoint from each other and from every input of either problem
    const int eb1 = g1->in_dtype == AXE_FP8_E4M3 ? 1 : 2, eb2 = g2->in_dtype == AXE_FP8_E4M3 ? 1 : 2;
    struct Span { const char* lo; int64_t bytes; };
    const Span in[] = {{(const char*)dA, g1->a_elems * eb1}, {(const char*)dB1, g1->b_elems * eb1}, {(const char*)dB2, g2->b_elems * eb2},
                       {(const char*)rows, (int64_t)(g1->G + 1) * 4}};
    const Span outp[] = {{(const char*)dH, g1->c_elems * 2}, {(const char*)dC, g2->c_elems * 2}};
    auto meet = [](const Span& a, const Span& b) { return a.lo < b.lo + b.bytes && b.lo < a.lo + a.bytes; };
    bool bad = meet(outp[0], outp[1]);
    for (const Span& i : in)
      for (const Span& o : outp) bad = bad || meet(i, o);
    if (bad) {
      set_error("%s: H and C must be disjoint from each other and from A, B1, B2 and group_rows", fn);
      return AXE_EINVAL;
    }
  }
  return AXE_OK;
}

// The second GEMM of a pair: with 16-bit inputs and no hint of its own it follows the first onto the tile kernels (its
// own crossover lies a few rows per group higher, but the shared launch is worth more: fp16 layer at 16 rows per group
// 232 us fused against 152 + 84), so that the pair runs the same kernels with and without a workspace.
bool pair_second_goes_to_stream(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2, const GemmArgs& a1, const GemmArgs& a2) {
  if (g2->kernel_hint == AXE_GROUPED_AUTO && !a2.fp8 && !grouped_goes_to_stream(g1, a1)) return false;
  return grouped_goes_to_stream(g2, a2);
}

bool pair_runs_fused(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2, const GemmArgs& a1, const GemmArgs& a2) {
  // (rows of the intermediate matrix start on 128-byte lines: no cache line then holds rows of two row blocks, or
  //  columns of two tiles of the first GEMM)
  return !grouped_goes_to_stream(g1, a1) && !pair_second_goes_to_stream(g1, g2, a1, a2) && grouped_pair_fusable(a1, a2) &&
         (a1.ldc * 2) % 128 == 0 && ((uintptr_t)a1.C & 127) == 0 && env_int("AXE_GROUPED_PAIR_FUSE", 1) != 0;
}
}  // namespace

int axe_gemm_grouped_pair(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2, const void* d_A, const void* d_B1,
                          void* d_H, const void* d_B2, void* d_C, const int32_t* d_group_rows, int32_t* d_sync, int64_t sync_elems,
                          void* stream) {
  GemmArgs a1, a2;
  if (int rc = plan_grouped_pair(g1, g2, d_A, d_B1, d_H, d_B2, d_C, d_group_rows, a1, a2, true)) return rc;
  if (d_sync && (sync_elems < g1->M + 1 || ((uintptr_t)d_sync & 3))) {
    set_error("axe_gemm_grouped_pair: d_sync needs M + 1 = %lld 4-byte words, 4-byte aligned", (long long)(g1->M + 1));
    return AXE_EINVAL;
  }
  if (d_sync) {
    const char* s0 = (const char*)d_sync;
    const char* s1 = s0 + (g1->M + 1) * 4;
    auto meets = [&](const void* p, int64_t bytes) { return (const char*)p < s1 && s0 < (const char*)p + bytes; };
    const int eb1 = g1->in_dtype == AXE_FP8_E4M3 ? 1 : 2, eb2 = g2->in_dtype == AXE_FP8_E4M3 ? 1 : 2;
    if (meets(d_A, g1->a_elems * eb1) || meets(d_B1, g1->b_elems * eb1) || meets(d_B2, g2->b_elems * eb2) || meets(d_H, g1->c_elems * 2) ||
        meets(d_C, g2->c_elems * 2) || meets(d_group_rows, (int64_t)(g1->G + 1) * 4)) {
      set_error("axe_gemm_grouped_pair: d_sync overlaps an operand");
      return AXE_EINVAL;
    }
  }
  hipStream_t st = (hipStream_t)stream;
  if (d_sync && pair_runs_fused(g1, g2, a1, a2)) {
    hipError_t e = launch_gemm_bf16_256_grouped_pair(a1, a2, d_sync, env_int("AXE_GROUPED_PAIR_POLLS", 1 << 20),
                                                     env_int("AXE_GROUPED_PAIR_TEST_NEVER", 0) ? 1 : 0, st);
    return e == hipSuccess ? AXE_OK : hip_fail(e, "axe_gemm_grouped_pair");
  }
  if (d_sync)                                                      // the status word answers for this call too
    if (hipError_t e = launch_pair_sync_clear(d_sync + g1->M, 1, st); e != hipSuccess) return hip_fail(e, "axe_gemm_grouped_pair");
  for (int i = 0; i < 2; ++i) {                                    // one after the other, on the stream
    const axe_gemm_grouped_desc_t* g = i ? g2 : g1;
    const GemmArgs& a = i ? a2 : a1;
    const bool streams = i ? pair_second_goes_to_stream(g1, g2, a1, a2) : grouped_goes_to_stream(g1, a1);
    hipError_t e = streams ? launch_gemm_grouped_stream(a, st)
                   : a.fp8 ? launch_gemm_fp8_e8m0_256_grouped(a, st)
                           : launch_gemm_bf16_256_grouped(a, st);
    if (e != hipSuccess) return hip_fail(e, "axe_gemm_grouped_pair");
  }
  return AXE_OK;
}

int axe_gemm_grouped_pair_static(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2, const void* d_A,
                                 const void* d_B1, void* d_H, const void* d_B2, void* d_C, const int32_t* d_group_rows, void* stream) {
  if (g1 && g1->M > kPairStaticRows) {
    set_error("axe_gemm_grouped_pair_static: M = %lld rows, the library's workspace serves at most %lld (use axe_gemm_grouped_pair "
              "with a workspace of your own)", (long long)g1->M, (long long)kPairStaticRows);
    return AXE_EUNSUPPORTED;
  }
  int32_t* ws = nullptr;
  if (hipError_t e = pair_static_workspace(&ws); e != hipSuccess) return hip_fail(e, "axe_gemm_grouped_pair_static");
  return axe_gemm_grouped_pair(g1, g2, d_A, d_B1, d_H, d_B2, d_C, d_group_rows, ws, kPairStaticRows + 1, stream);
}

int axe_gemm_grouped_pair_fused(const axe_gemm_grouped_desc_t* g1, const axe_gemm_grouped_desc_t* g2) {
  GemmArgs a1, a2;
  if (int rc = plan_grouped_pair(g1, g2, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, a1, a2, false)) return rc;
  return pair_runs_fused(g1, g2, a1, a2) ? 1 : 0;
}

int axe_gemm_grouped_pair_status(const int32_t* d_sync, int64_t M, void* stream) {
  if (M <= 0 || (!d_sync && M > kPairStaticRows)) {
    set_error("axe_gemm_grouped_pair_status: M must be positive (and within the library's workspace when d_sync is NULL)");
    return AXE_EINVAL;
  }
  if (!d_sync) {                                                   // the library's own workspace on the current device
    int32_t* ws = nullptr;
    if (hipError_t e = pair_static_workspace(&ws); e != hipSuccess) return hip_fail(e, "axe_gemm_grouped_pair_status");
    d_sync = ws;
  }
  int32_t gave_up = 0;
  hipError_t e = hipMemcpyAsync(&gave_up, d_sync + M, sizeof gave_up, hipMemcpyDeviceToHost, (hipStream_t)stream);
  if (e == hipSuccess) e = hipStreamSynchronize((hipStream_t)stream);
  if (e != hipSuccess) return hip_fail(e, "axe_gemm_grouped_pair_status");
  if (gave_up) {
    set_error("axe_gemm_grouped_pair: %d waits for rows of the first GEMM gave up; the rows of C they cover are invalid", gave_up);
    return AXE_ETIMEOUT;
  }
  return AXE_OK;
}

int axe_gemm(const axe_gemm_desc_t* g, const void* d_A, const void* d_B, void* d_C, void* stream) {
  // The plan of the last descriptor this thread launched is kept: a caller that launches the same GEMM again (same
  // shape, types and layouts, compared word by word; other buffers are fine) skips the layout analysis -- a few
  // microseconds, as much as a small problem's kernel takes.
  static thread_local PlanKey last_key;
  static thread_local GemmPlan last_plan;
  static thread_local bool have_last = false;
  GemmPlan P;
  PlanKey key;
  const bool keyed = g && key_of_gemm(g, key);
  if (keyed && have_last && key.n == last_key.n && memcmp(key.w, last_key.w, sizeof(int64_t) * key.n) == 0) {
    P = last_plan;
    P.args.scale_a = (const float*)g->d_scale_a;
    P.args.scale_b = (const float*)g->d_scale_b;
    if (int rc = bind_gemm_pointers(g, d_A, d_B, d_C, P)) return rc;
  } else {
    if (int rc = plan_gemm(g, d_A, d_B, d_C, P, true)) return rc;
    if (keyed) last_key = key, last_plan = P, have_last = true;
  }
  hipError_t e;
  if (P.tile == AXE_TILE_256x256x64 || P.tile == AXE_TILE_256x224x64)
    e = !P.fp8 ? (P.ragged ? launch_gemm_bf16_256_ragged(P.args, (hipStream_t)stream) : launch_gemm_bf16_256(P.args, (hipStream_t)stream))
        // power-of-two scales (or none) ride on the matrix cores' scale operands; arbitrary fp32 scales are folded on the vector ALU
        : (P.args.scale_e8m0 || !P.args.scale_a ? launch_gemm_fp8_e8m0_256(P.args, (hipStream_t)stream)
                                                : launch_gemm_fp8_256(P.args, (hipStream_t)stream));
  else
    e = launch_gemm_small(P.args, P.fp8, (hipStream_t)stream);
  return e == hipSuccess ? AXE_OK : hip_fail(e, "axe_gemm");
}

// Chosen kernel, for tests and tools: returns AXE_TILE_* or a negative error.
int axe_gemm_tile(const axe_gemm_desc_t* g) {
  GemmPlan P;
  if (int rc = plan_gemm(g, nullptr, nullptr, nullptr, P, false)) return rc;
  return P.tile;
}

}  // extern "C"
