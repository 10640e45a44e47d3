#include "host_layout.h"

#include <stdarg.h>
#include <stdio.h>

#include <algorithm>

namespace axe {

static thread_local char g_err[512] = "";

void set_error(const char* fmt, ...) {
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(g_err, sizeof g_err, fmt, ap);
  va_end(ap);
}
const char* last_error() { return g_err; }

static bool mul_ok(int64_t a, int64_t b, int64_t* r) { return !__builtin_mul_overflow(a, b, r); }
static bool add_ok(int64_t a, int64_t b, int64_t* r) { return !__builtin_add_overflow(a, b, r); }

int load_layout(const axe_layout_t* L, HLayout& out, const char* what) {
  if (!L) {
    set_error("%s: layout pointer is NULL", what);
    return AXE_EINVAL;
  }
  if (L->n_axes < 1 || L->n_axes > AXE_MAX_AXES) {
    set_error("%s: n_axes = %d outside 1..%d", what, L->n_axes, AXE_MAX_AXES);
    return AXE_EINVAL;
  }
  if (L->n_d < 1 || L->n_d > AXE_MAX_D || !L->d) {
    set_error("%s: a layout needs 1..%d sharded iters (Def. 2.2), got %d", what, AXE_MAX_D, L->n_d);
    return AXE_EINVAL;
  }
  if (L->n_r < 0 || L->n_r > AXE_MAX_R || (L->n_r > 0 && !L->r)) {
    set_error("%s: n_r = %d outside 0..%d or r is NULL", what, L->n_r, AXE_MAX_R);
    return AXE_EINVAL;
  }
  out = HLayout();
  out.n_axes = L->n_axes;
  auto take = [&](const axe_iter_t& it, const char* part, int k, std::vector<HIter>& dst, int64_t& prod) -> int {
    if (it.extent <= 0) {
      set_error("%s: %s iter %d has extent %lld (must be > 0, Def. 2.1)", what, part, k, (long long)it.extent);
      return AXE_EINVAL;
    }
    if (it.stride == 0) {
      set_error("%s: %s iter %d has stride 0 (Def. 2.1)", what, part, k);
      return AXE_EINVAL;
    }
    if (it.axis < 0 || it.axis >= L->n_axes) {
      set_error("%s: %s iter %d names axis %d, outside 0..%d", what, part, k, it.axis, L->n_axes - 1);
      return AXE_EINVAL;
    }
    if (!mul_ok(prod, it.extent, &prod)) {
      set_error("%s: product of %s extents overflows int64", what, part);
      return AXE_ERANGE;
    }
    int64_t reach;
    if (!mul_ok(it.extent - 1, it.stride, &reach)) {
      set_error("%s: %s iter %d: (extent-1)*stride overflows int64", what, part, k);
      return AXE_ERANGE;
    }
    dst.push_back(HIter{it.extent, it.stride, it.axis});
    return AXE_OK;
  };
  for (int k = 0; k < L->n_d; ++k)
    if (int rc = take(L->d[k], "D", k, out.D, out.E_D)) return rc;
  for (int k = 0; k < L->n_r; ++k)
    if (int rc = take(L->r[k], "R", k, out.R, out.E_R)) return rc;
  for (int a = 0; a < L->n_axes; ++a) out.off[a] = L->offset ? L->offset[a] : 0;
  if (L->swz_axis >= 0) {
    if (L->swz_axis >= L->n_axes || L->swz_bits < 0 || L->swz_base < 0 || L->swz_shift < 0 ||
        L->swz_base + L->swz_bits > L->swz_shift || L->swz_shift + L->swz_bits > 62 || L->swz_bits > 30) {
      set_error("%s: bad swizzle (axis %d, bits %d, base %d, shift %d): need base + bits <= shift", what,
                L->swz_axis, L->swz_bits, L->swz_base, L->swz_shift);
      return AXE_EINVAL;
    }
    if (L->swz_bits > 0) {
      out.swz_axis = L->swz_axis;
      out.swz_bits = L->swz_bits;
      out.swz_base = L->swz_base;
      out.swz_shift = L->swz_shift;
    }
  }
  return AXE_OK;
}

int check_shape(const HLayout& L, int32_t rank, const int64_t* shape, const char* what) {
  if (rank < 1 || rank > AXE_MAX_RANK || !shape) {
    set_error("%s: rank %d outside 1..%d or shape is NULL", what, rank, AXE_MAX_RANK);
    return AXE_EINVAL;
  }
  int64_t p = 1;
  for (int i = 0; i < rank; ++i) {
    if (shape[i] <= 0) {
      set_error("%s: shape[%d] = %lld must be positive", what, i, (long long)shape[i]);
      return AXE_EINVAL;
    }
    if (!mul_ok(p, shape[i], &p)) {
      set_error("%s: shape product overflows", what);
      return AXE_ERANGE;
    }
  }
  if (p != L.E_D) {
    set_error("%s: shape is not admitted: prod(shape) = %lld but E_D = %lld", what, (long long)p, (long long)L.E_D);
    return AXE_ESHAPE;
  }
  return AXE_OK;
}

void canon_D(std::vector<HIter>& D) {
  std::vector<HIter> cur;
  for (const HIter& it : D)
    if (it.e != 1) cur.push_back(it);                       // D0
  bool changed = true;
  while (changed) {
    changed = false;
    for (size_t i = 0; i + 1 < cur.size(); ++i) {
      int64_t chain;
      if (cur[i].axis == cur[i + 1].axis && mul_ok(cur[i + 1].e, cur[i + 1].s, &chain) && cur[i].s == chain) {
        cur[i] = HIter{cur[i].e * cur[i + 1].e, cur[i + 1].s, cur[i].axis};   // D1
        cur.erase(cur.begin() + i + 1);
        changed = true;
        break;
      }
    }
  }
  D.swap(cur);
}

int reduce_to_memory(const HLayout& L, int mem_axis, MemLayout& out, const char* what) {
  if (mem_axis < 0 || mem_axis >= L.n_axes) {
    set_error("%s: memory axis %d outside 0..%d", what, mem_axis, L.n_axes - 1);
    return AXE_EINVAL;
  }
  out = MemLayout();
  for (const HIter& it : L.D) {
    if (it.axis != mem_axis) {
      if (it.e > 1) {
        set_error("%s: D iter of extent %lld on non-memory axis %d: one GPU holds the whole tensor", what,
                  (long long)it.e, it.axis);
        return AXE_EALIAS;
      }
      continue;
    }
    out.D.push_back(it);
  }
  for (const HIter& it : L.R) {
    if (it.e == 1) continue;                                 // C0
    if (it.axis != mem_axis) {
      set_error("%s: replica iter of extent %lld on non-memory axis %d", what, (long long)it.e, it.axis);
      return AXE_EALIAS;
    }
    out.R.push_back(it);
  }
  canon_D(out.D);
  out.off = L.off[mem_axis];
  out.E_D = L.E_D;
  out.E_R = 1;
  for (const HIter& it : out.R) out.E_R *= it.e;
  if (L.swz_axis == mem_axis) out.swz = Swz{(1 << L.swz_bits) - 1, L.swz_base, L.swz_shift};
  // address range before the swizzle
  int64_t lo = out.off, hi = out.off;
  auto widen = [&](const HIter& it) -> bool {
    int64_t reach;
    if (!mul_ok(it.e - 1, it.s, &reach)) return false;
    return reach < 0 ? add_ok(lo, reach, &lo) : add_ok(hi, reach, &hi);
  };
  for (const HIter& it : out.D)
    if (!widen(it)) goto overflow;
  for (const HIter& it : out.R)
    if (!widen(it)) goto overflow;
  if (out.swz.mask) {
    if (lo < 0) {
      set_error("%s: swizzle applied to a negative coordinate (lowest address %lld)", what, (long long)lo);
      return AXE_ERANGE;
    }
    // the XOR only changes bits base .. base+bits-1, so an address stays inside its aligned
    // block of 2^(base+bits) coordinates: widen the range to whole blocks
    int64_t blk = (((int64_t)out.swz.mask + 1) << out.swz.base) - 1;
    lo = lo & ~blk;
    hi = hi | blk;
  }
  out.lo = lo;
  out.hi = hi;
  return AXE_OK;
overflow:
  set_error("%s: address range overflows int64", what);
  return AXE_ERANGE;
}

int check_range(const MemLayout& L, int64_t elems, const char* what) {
  if (elems < 0) {
    set_error("%s: negative buffer size", what);
    return AXE_EINVAL;
  }
  if (L.lo < 0 || L.hi >= elems) {
    set_error("%s: addresses span [%lld, %lld] but the buffer holds %lld elements", what, (long long)L.lo,
              (long long)L.hi, (long long)elems);
    return AXE_ERANGE;
  }
  return AXE_OK;
}

bool provably_injective(const MemLayout& L) {
  // shard and replica iters together: every (logical element, replica) pair needs an address of its own,
  // e.g. D = [(4, 1)], R = [(2, 2)] writes address 2 from element 0 (replica 1) and from element 2 (replica 0)
  std::vector<HIter> v = L.D;
  v.insert(v.end(), L.R.begin(), L.R.end());
  std::sort(v.begin(), v.end(), [](const HIter& a, const HIter& b) {
    int64_t x = a.s < 0 ? -a.s : a.s, y = b.s < 0 ? -b.s : b.s;
    return x < y;
  });
  __int128 reach = 0;                                        // span - 1 of all smaller-stride iters
  for (const HIter& it : v) {
    __int128 s = it.s < 0 ? -(__int128)it.s : (__int128)it.s;
    if (s <= reach) return false;
    reach += s * (it.e - 1);
  }
  return true;
}

bool joint_refine(const std::vector<HIter>& s, const std::vector<HIter>& d, std::vector<JointIter>& out) {
  out.clear();
  size_t i = 0, j = 0;
  int64_t a = s.empty() ? 1 : s[0].e, b = d.empty() ? 1 : d[0].e;
  while (i < s.size() && j < d.size()) {
    if (a == b) {
      out.push_back(JointIter{a, s[i].s, d[j].s});
      ++i;
      ++j;
      if (i < s.size()) a = s[i].e;
      if (j < d.size()) b = d[j].e;
    } else if (a > b) {
      if (a % b) return false;
      int64_t ss;
      if (!mul_ok(s[i].s, a / b, &ss)) return false;
      out.push_back(JointIter{b, ss, d[j].s});
      a /= b;
      ++j;
      if (j < d.size()) b = d[j].e; else return false;
    } else {
      if (b % a) return false;
      int64_t ds;
      if (!mul_ok(d[j].s, b / a, &ds)) return false;
      out.push_back(JointIter{a, s[i].s, ds});
      b /= a;
      ++i;
      if (i < s.size()) a = s[i].e; else return false;
    }
  }
  return i == s.size() && j == d.size() && out.size() <= (size_t)kMaxJoint;
}

}  // namespace axe
