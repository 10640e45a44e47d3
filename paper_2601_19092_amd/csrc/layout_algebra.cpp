// Host-side layout algebra behind the C ABI (Sec. 3.3 and Apps. A - F of the paper): span,
// canonical forms, group-by-shape, tile (Kronecker product), direct sum, tile-of and slice.  Pure
// integer bookkeeping on (D, R, O); nothing here touches the GPU.
//
// Failure of an operator's sufficient conditions (the paper's FAILURE / FAIL outcomes) is reported
// as AXE_ENOFORM: the inputs are valid layouts, the operator just has no answer of the required form.
#include <string.h>

#include <algorithm>
#include <numeric>
#include <vector>

#include "../../include/axe.h"
#include "host_layout.h"

using namespace axe;

namespace {

typedef std::vector<HIter> Iters;

bool mul_ok(int64_t a, int64_t b, int64_t* r) { return !__builtin_mul_overflow(a, b, r); }
bool add_ok(int64_t a, int64_t b, int64_t* r) { return !__builtin_add_overflow(a, b, r); }
int64_t iabs(int64_t v) { return v < 0 ? -v : v; }

int overflow(const char* what) {
  set_error("%s: integer overflow", what);
  return AXE_ERANGE;
}

// ---- span (Sec. 2.3; closed form of App. C): per axis 1 + sum |s| (e - 1) over D and R; O does not enter
int span_of(const HLayout& L, int64_t* sp, const char* what) {
  for (int a = 0; a < L.n_axes; ++a) sp[a] = 1;
  for (const Iters* part : {&L.D, &L.R})
    for (const HIter& it : *part) {
      int64_t reach;
      if (!mul_ok(iabs(it.s), it.e - 1, &reach) || !add_ok(sp[it.axis], reach, &sp[it.axis])) return overflow(what);
    }
  return AXE_OK;
}

// ---- (O, R) rules of App. A: C0 drops unit iters, C1 makes strides positive (the reach of the
//      negative iter moves into O), C2 absorbs an iter whose stride is q times another's with
//      1 <= q <= that other's extent.  R is a multiset: the result is sorted by (axis, stride, extent).
int canon_replicas(Iters& R, int64_t* off, const char* what) {
  Iters cur;
  for (HIter it : R) {
    if (it.e == 1) continue;                                                   // C0
    if (it.s < 0) {                                                            // C1
      int64_t reach;
      if (!mul_ok(it.e - 1, it.s, &reach) || !add_ok(off[it.axis], reach, &off[it.axis])) return overflow(what);
      it.s = -it.s;
    }
    cur.push_back(it);
  }
  auto by_stride = [](const HIter& a, const HIter& b) {
    return a.axis != b.axis ? a.axis < b.axis : (a.s != b.s ? a.s < b.s : a.e < b.e);
  };
  for (bool merged = true; merged;) {                                          // C2, to a fixpoint
    merged = false;
    std::sort(cur.begin(), cur.end(), by_stride);
    for (size_t fine = 0; fine < cur.size() && !merged; ++fine)
      for (size_t coarse = 0; coarse < cur.size() && !merged; ++coarse) {
        if (coarse == fine || cur[coarse].axis != cur[fine].axis || cur[coarse].s % cur[fine].s) continue;
        const int64_t q = cur[coarse].s / cur[fine].s;
        if (q < 1 || q > cur[fine].e) continue;
        int64_t grown;                                                         // e_fine + q (e_coarse - 1)
        if (!mul_ok(q, cur[coarse].e - 1, &grown) || !add_ok(grown, cur[fine].e, &grown)) return overflow(what);
        cur[fine].e = grown;
        cur.erase(cur.begin() + coarse);
        merged = true;
      }
  }
  std::sort(cur.begin(), cur.end(), by_stride);
  R.swap(cur);
  return AXE_OK;
}

// ---- gap condition of App. A on sign-normalised replicas: per axis, strides increasing,
//      sigma_{k+1} > E_k sigma_k (then distinct replica digits give distinct coordinates)
bool gap_holds(Iters R) {
  std::sort(R.begin(), R.end(), [](const HIter& a, const HIter& b) { return a.axis != b.axis ? a.axis < b.axis : a.s < b.s; });
  for (size_t k = 0; k + 1 < R.size(); ++k) {
    if (R[k].axis != R[k + 1].axis) continue;
    int64_t reach;
    if (!mul_ok(R[k].e, R[k].s, &reach) || !(R[k + 1].s > reach)) return false;
  }
  return true;
}

// ---- Group-By-Shape (App. B, Alg. 1): cut D, left to right, into consecutive blocks whose extent
//      products are shape[0], shape[1], ...; an iter that straddles a boundary is split
//      (e, s, a) -> (g, (e / g) s, a)(e / g, s, a) with g = gcd(e, what the block still needs).
int group_by_shape(const Iters& D, int rank, const int64_t* shape, std::vector<Iters>& blocks, const char* what) {
  blocks.assign(rank, Iters());
  Iters src(D);
  size_t next = 0;
  for (int b = 0; b < rank; ++b) {
    int64_t have = 1;
    while (have < shape[b]) {
      if (next == src.size()) {
        set_error("%s: the iters run out before block %d (extent %lld) is complete", what, b, (long long)shape[b]);
        return AXE_ENOFORM;
      }
      HIter& it = src[next];
      const int64_t need = shape[b] / have, g = std::gcd(it.e, need);
      if (it.e == 1) {                                       // a unit iter completes nothing; it stays in this block
        blocks[b].push_back(it);
        ++next;
        continue;
      }
      if (g == 1) {
        set_error("%s: iter (%lld, %lld) cannot be split to complete block %d of extent %lld", what, (long long)it.e,
                  (long long)it.s, b, (long long)shape[b]);
        return AXE_ENOFORM;
      }
      const int64_t rest = it.e / g;
      int64_t outer_stride;
      if (!mul_ok(rest, it.s, &outer_stride)) return overflow(what);
      blocks[b].push_back(HIter{g, outer_stride, it.axis});
      have *= g;
      if (rest > 1) it.e = rest;
      else ++next;
    }
    if (have != shape[b]) {
      set_error("%s: block %d overshoots its extent %lld", what, b, (long long)shape[b]);
      return AXE_ENOFORM;
    }
    while (next < src.size() && src[next].e == 1) blocks[b].push_back(src[next++]);   // trailing unit iters stay here
  }
  if (next != src.size()) {
    set_error("%s: iters are left over after the last block", what);
    return AXE_ENOFORM;
  }
  return AXE_OK;
}

int check_shapes(const HLayout& L, int rank, const int64_t* shape, const char* what) { return check_shape(L, rank, shape, what); }

// A swizzled operand takes part in an operator only where the stage provably commutes with it.
int no_swizzle(const HLayout& L, const char* what) {
  if (L.swz_axis < 0) return AXE_OK;
  set_error("%s: the operator acts on (D, R, O); this operand carries a swizzle stage", what);
  return AXE_EUNSUPPORTED;
}

// ---- writes a host layout into the caller's arena
int emit(const HLayout& L, const axe_layout_t* names_from, axe_layout_t* out, void* arena, size_t arena_bytes, const char* what) {
  if (L.D.empty() || L.D.size() > AXE_MAX_D || L.R.size() > AXE_MAX_R) {
    set_error("%s: the result has %zu sharded and %zu replica iters; a layout carries 1..%d and 0..%d", what, L.D.size(),
              L.R.size(), AXE_MAX_D, AXE_MAX_R);
    return AXE_ERANGE;
  }
  const size_t need = sizeof(axe_iter_t) * (L.D.size() + L.R.size()) + sizeof(int64_t) * L.n_axes + 16;
  if (!arena || arena_bytes < need) {
    set_error("%s: arena of %zu bytes is too small (%zu needed)", what, arena_bytes, need);
    return AXE_ERANGE;
  }
  char* p = (char*)arena;
  p += (8 - ((uintptr_t)p & 7)) & 7;
  axe_iter_t* d = (axe_iter_t*)p;
  p += sizeof(axe_iter_t) * L.D.size();
  axe_iter_t* r = (axe_iter_t*)p;
  p += sizeof(axe_iter_t) * L.R.size();
  int64_t* off = (int64_t*)p;
  for (size_t i = 0; i < L.D.size(); ++i) d[i] = axe_iter_t{L.D[i].e, L.D[i].s, L.D[i].axis};
  for (size_t i = 0; i < L.R.size(); ++i) r[i] = axe_iter_t{L.R[i].e, L.R[i].s, L.R[i].axis};
  for (int a = 0; a < L.n_axes; ++a) off[a] = L.off[a];
  out->n_axes = L.n_axes;
  out->axis_names = names_from ? names_from->axis_names : nullptr;
  out->n_d = (int32_t)L.D.size();
  out->d = d;
  out->n_r = (int32_t)L.R.size();
  out->r = L.R.empty() ? nullptr : r;
  out->offset = off;
  out->swz_axis = L.swz_axis;
  out->swz_bits = L.swz_bits;
  out->swz_base = L.swz_base;
  out->swz_shift = L.swz_shift;
  return AXE_OK;
}

// D must never be empty (Def. 2.2): a unit iter on `axis` stands for the empty product
void keep_one(Iters& D, int axis) {
  if (D.empty()) D.push_back(HIter{1, 1, axis});
}

int load_pair(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B, const int64_t* SB, HLayout& a,
              HLayout& b, const char* what) {
  if (int rc = load_layout(A, a, what)) return rc;
  if (int rc = load_layout(B, b, what)) return rc;
  if (a.n_axes != b.n_axes) {
    set_error("%s: the operands name %d and %d axes; they must share one axis list", what, a.n_axes, b.n_axes);
    return AXE_EINVAL;
  }
  if (int rc = check_shapes(a, rank, SA, what)) return rc;
  return check_shapes(b, rank, SB, what);
}

// Shared body of tile (scaled = true, Alg. 2) and direct sum (scaled = false, App. F):
// blocks of A and of B interleaved dimension by dimension, A's strides, replicas and offset
// multiplied by the span of B when scaled.
int combine(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B, const int64_t* SB, bool scaled,
            axe_layout_t* out, int64_t* shape_out, void* arena, size_t arena_bytes, const char* what) {
  if (!out || !shape_out) {
    set_error("%s: NULL argument", what);
    return AXE_EINVAL;
  }
  HLayout a, b;
  if (int rc = load_pair(A, rank, SA, B, SB, a, b, what)) return rc;
  if (int rc = no_swizzle(a, what)) return rc;
  int64_t w[AXE_MAX_AXES];
  if (int rc = span_of(b, w, what)) return rc;
  if (!scaled)
    for (int x = 0; x < b.n_axes; ++x) w[x] = 1;
  if (b.swz_axis >= 0) {
    // B's swizzle stage reads and writes only the bits below 2^(shift + bits) of the coordinate: it
    // commutes with adding A's part when everything A adds on that axis is a multiple of that period
    // (Sec. 3.4: the swizzled atom is the innermost layout, the tiler steps over whole atoms).
    if (!scaled) return no_swizzle(b, what);
    const int64_t period = int64_t(1) << (b.swz_shift + b.swz_bits);
    bool whole = true;
    int64_t v;
    for (const Iters* part : {&a.D, &a.R})
      for (const HIter& it : *part)
        if (it.axis == b.swz_axis && (!mul_ok(it.s, w[it.axis], &v) || v % period)) whole = false;
    if (!mul_ok(a.off[b.swz_axis], w[b.swz_axis], &v) || v % period) whole = false;
    if (!whole) {
      set_error("%s: A does not step over whole swizzle periods (%lld) of B on the swizzled axis", what, (long long)period);
      return AXE_EUNSUPPORTED;
    }
  }
  std::vector<Iters> ga, gb;
  if (int rc = group_by_shape(a.D, rank, SA, ga, what)) return rc;
  if (int rc = group_by_shape(b.D, rank, SB, gb, what)) return rc;
  HLayout t;
  t.n_axes = a.n_axes;
  auto scale = [&](HIter it, HIter& o) { o = it; return mul_ok(it.s, w[it.axis], &o.s); };
  for (int i = 0; i < rank; ++i) {
    for (const HIter& it : ga[i]) {
      HIter o;
      if (!scale(it, o)) return overflow(what);
      t.D.push_back(o);
    }
    t.D.insert(t.D.end(), gb[i].begin(), gb[i].end());
    shape_out[2 * i] = SA[i];
    shape_out[2 * i + 1] = SB[i];
  }
  for (const HIter& it : a.R) {
    HIter o;
    if (!scale(it, o)) return overflow(what);
    t.R.push_back(o);
  }
  t.R.insert(t.R.end(), b.R.begin(), b.R.end());
  for (int x = 0; x < t.n_axes; ++x) {
    int64_t oa;
    if (!mul_ok(a.off[x], w[x], &oa) || !add_ok(oa, b.off[x], &t.off[x])) return overflow(what);
  }
  t.swz_axis = b.swz_axis, t.swz_bits = b.swz_bits, t.swz_base = b.swz_base, t.swz_shift = b.swz_shift;
  keep_one(t.D, a.D[0].axis);
  return emit(t, A, out, arena, arena_bytes, what);
}

// Region [begin, begin + size) of one grouped block (Alg. 4), as iters slow -> fast.  The constant
// part (the image of `begin`) is added to the offset by the caller.
int slice_block(const Iters& block, int64_t begin, int64_t size, Iters& out, const char* what) {
  Iters blk(block);
  canon_D(blk);
  const int m = (int)blk.size();
  std::vector<int64_t> digit(m);
  int64_t rest = begin;
  for (int j = m - 1; j >= 0; --j) digit[j] = rest % blk[j].e, rest /= blk[j].e;
  // greedy peel: fast digits the region covers completely stay as they are
  int k = m - 1;
  Iters whole;
  while (k >= 0 && digit[k] == 0 && size % blk[k].e == 0) {
    whole.insert(whole.begin(), blk[k]);
    size /= blk[k].e;
    --k;
  }
  if (k < 0) {
    if (size != 1) {
      set_error("%s: the region is larger than its block", what);
      return AXE_ENOFORM;
    }
    out = whole;
    return AXE_OK;
  }
  if (digit[k] + size <= blk[k].e) {                         // no wrap: a run of `size` values of digit k
    out.assign(1, HIter{size, blk[k].s, blk[k].axis});
  } else if (size % 2 == 0 && digit[k] + size / 2 == blk[k].e) {
    // symmetric single wrap: two runs of c = size / 2, the second after one carry into digit k - 1
    const int64_t c = size / 2;
    if (k == 0 || digit[k - 1] + 1 > blk[k - 1].e - 1) {     // the carry must not wrap digit k - 1 in turn
      set_error("%s: the wrap-around carry leaves the block", what);
      return AXE_ENOFORM;
    }
    if (blk[k - 1].axis != blk[k].axis) {
      set_error("%s: the wrap-around carry crosses axes", what);
      return AXE_ENOFORM;
    }
    int64_t back, jump;
    if (!mul_ok(blk[k].e - c, blk[k].s, &back) || !add_ok(blk[k - 1].s, -back, &jump)) return overflow(what);
    if (jump == 0) {
      set_error("%s: the two runs of the wrapped region coincide", what);
      return AXE_ENOFORM;
    }
    out = {HIter{2, jump, blk[k].axis}, HIter{c, blk[k].s, blk[k].axis}};
  } else {
    set_error("%s: the region fits neither the no-wrap nor the symmetric one-wrap form", what);
    return AXE_ENOFORM;
  }
  out.insert(out.end(), whole.begin(), whole.end());
  return AXE_OK;
}

}  // namespace

extern "C" {

int axe_layout_span(const axe_layout_t* L, int64_t* span) {
  HLayout h;
  if (int rc = load_layout(L, h, "axe_layout_span")) return rc;
  if (!span) {
    set_error("axe_layout_span: NULL argument");
    return AXE_EINVAL;
  }
  return span_of(h, span, "axe_layout_span");
}

int axe_layout_canonicalize(const axe_layout_t* L, axe_layout_t* out, void* arena, size_t arena_bytes) {
  const char* what = "axe_layout_canonicalize";
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  if (!out) {
    set_error("%s: NULL argument", what);
    return AXE_EINVAL;
  }
  const int first_axis = h.D[0].axis;
  canon_D(h.D);
  keep_one(h.D, first_axis);
  if (int rc = canon_replicas(h.R, h.off, what)) return rc;
  return emit(h, L, out, arena, arena_bytes, what);
}

int axe_layout_gap_condition(const axe_layout_t* L) {
  const char* what = "axe_layout_gap_condition";
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  if (int rc = canon_replicas(h.R, h.off, what)) return rc;
  return gap_holds(h.R) ? 1 : 0;
}

int axe_layout_equal(const axe_layout_t* A, const axe_layout_t* B) {
  const char* what = "axe_layout_equal";
  HLayout a, b;
  if (int rc = load_layout(A, a, what)) return rc;
  if (int rc = load_layout(B, b, what)) return rc;
  if (a.n_axes != b.n_axes) return 0;
  canon_D(a.D);
  canon_D(b.D);
  if (int rc = canon_replicas(a.R, a.off, what)) return rc;
  if (int rc = canon_replicas(b.R, b.off, what)) return rc;
  auto same = [](const Iters& x, const Iters& y) {
    if (x.size() != y.size()) return false;
    for (size_t i = 0; i < x.size(); ++i)
      if (x[i].e != y[i].e || x[i].s != y[i].s || x[i].axis != y[i].axis) return false;
    return true;
  };
  if (!same(a.D, b.D) || !same(a.R, b.R)) return 0;
  for (int x = 0; x < a.n_axes; ++x)
    if (a.off[x] != b.off[x]) return 0;
  if (a.swz_axis != b.swz_axis) return 0;
  if (a.swz_axis >= 0 && (a.swz_bits != b.swz_bits || a.swz_base != b.swz_base || a.swz_shift != b.swz_shift)) return 0;
  return 1;
}

int axe_layout_group(const axe_layout_t* L, int32_t rank, const int64_t* shape, axe_layout_t* out, int32_t* block_end,
                     void* arena, size_t arena_bytes) {
  const char* what = "axe_layout_group";
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  if (int rc = check_shapes(h, rank, shape, what)) return rc;
  if (!out || !block_end) {
    set_error("%s: NULL argument", what);
    return AXE_EINVAL;
  }
  std::vector<Iters> blocks;
  if (int rc = group_by_shape(h.D, rank, shape, blocks, what)) return rc;
  const int first_axis = h.D[0].axis;
  h.D.clear();
  for (int i = 0; i < rank; ++i) {
    h.D.insert(h.D.end(), blocks[i].begin(), blocks[i].end());
    block_end[i] = (int32_t)h.D.size();
  }
  keep_one(h.D, first_axis);
  return emit(h, L, out, arena, arena_bytes, what);
}

int axe_layout_tile(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B, const int64_t* SB,
                    axe_layout_t* out, int64_t* shape_out, void* arena, size_t arena_bytes) {
  return combine(A, rank, SA, B, SB, true, out, shape_out, arena, arena_bytes, "axe_layout_tile");
}

int axe_layout_direct_sum(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B, const int64_t* SB,
                          axe_layout_t* out, int64_t* shape_out, void* arena, size_t arena_bytes) {
  return combine(A, rank, SA, B, SB, false, out, shape_out, arena, arena_bytes, "axe_layout_direct_sum");
}

int axe_layout_flatten(const axe_layout_t* L, const int64_t* pitch, int32_t to_axis, axe_layout_t* out, void* arena,
                       size_t arena_bytes) {
  const char* what = "axe_layout_flatten";
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  if (!pitch || !out || to_axis < 0 || to_axis >= h.n_axes) {
    set_error("%s: NULL argument or to_axis out of range", what);
    return AXE_EINVAL;
  }
  if (int rc = no_swizzle(h, what)) return rc;
  auto move = [&](HIter& it) -> int {
    if (pitch[it.axis] == 0 && it.e > 1) {
      set_error("%s: pitch 0 for axis %d, which carries an iter of extent %lld", what, it.axis, (long long)it.e);
      return AXE_EINVAL;
    }
    if (pitch[it.axis] && !mul_ok(it.s, pitch[it.axis], &it.s)) return overflow(what);
    it.axis = to_axis;
    return AXE_OK;
  };
  for (HIter& it : h.D)
    if (int rc = move(it)) return rc;
  for (HIter& it : h.R)
    if (int rc = move(it)) return rc;
  int64_t off = 0;
  for (int a = 0; a < h.n_axes; ++a) {
    int64_t t;
    if (!mul_ok(h.off[a], pitch[a], &t) || !add_ok(off, t, &off)) return overflow(what);
    h.off[a] = 0;
  }
  h.off[to_axis] = off;
  return emit(h, L, out, arena, arena_bytes, what);
}

int axe_layout_tile_of(const axe_layout_t* A, int32_t rank, const int64_t* SA, const axe_layout_t* B, const int64_t* SB,
                       axe_layout_t* out, int64_t* shape_out, void* arena, size_t arena_bytes) {
  const char* what = "axe_layout_tile_of";
  if (!out || !shape_out) {
    set_error("%s: NULL argument", what);
    return AXE_EINVAL;
  }
  HLayout a, b;
  if (int rc = load_pair(A, rank, SA, B, SB, a, b, what)) return rc;
  if (int rc = no_swizzle(a, what)) return rc;
  if (int rc = no_swizzle(b, what)) return rc;
  for (int i = 0; i < rank; ++i)
    if (SA[i] % SB[i]) {
      set_error("%s: S_B[%d] = %lld does not divide S_A[%d] = %lld", what, i, (long long)SB[i], i, (long long)SA[i]);
      return AXE_ENOFORM;
    }
  int64_t w[AXE_MAX_AXES];
  if (int rc = span_of(b, w, what)) return rc;
  std::vector<Iters> ga, gb;
  if (int rc = group_by_shape(a.D, rank, SA, ga, what)) return rc;
  if (int rc = group_by_shape(b.D, rank, SB, gb, what)) return rc;
  HLayout c;
  c.n_axes = a.n_axes;
  for (int i = 0; i < rank; ++i) {
    // In C (x) B the block of dimension i is C's block, span-scaled, followed by B's block.  Both
    // sides are normalised (D0, D1) first, so B's iters must reappear at the end of A's block;
    // where the last iter of the scaled C chained into B's first (rule D1 fused them) it is split again.
    Iters blkA(ga[i]), blkB(gb[i]);
    canon_D(blkA);
    canon_D(blkB);
    for (size_t q = blkB.size(); q-- > 0;) {
      if (blkA.empty()) {
        set_error("%s: dimension %d of A is shorter than B's block", what, i);
        return AXE_ENOFORM;
      }
      HIter& last = blkA.back();
      const HIter& want = blkB[q];
      if (last.axis != want.axis || last.s != want.s || last.e % want.e) {
        set_error("%s: dimension %d of A does not end with B's block", what, i);
        return AXE_ENOFORM;
      }
      if (last.e == want.e) {
        blkA.pop_back();
      } else if (q == 0) {                                   // fused by D1: (e_c e_b, s_b) = (e_c, e_b s_b)(e_b, s_b)
        last.e /= want.e;
        if (!mul_ok(want.e, want.s, &last.s)) return overflow(what);
      } else {
        set_error("%s: dimension %d of A does not end with B's block", what, i);
        return AXE_ENOFORM;
      }
    }
    int64_t have = 1;
    for (const HIter& it : blkA) {
      if (it.s % w[it.axis]) {
        set_error("%s: an outer iter of dimension %d has stride %lld, not a multiple of B's span %lld", what, i,
                  (long long)it.s, (long long)w[it.axis]);
        return AXE_ENOFORM;
      }
      c.D.push_back(HIter{it.e, it.s / w[it.axis], it.axis});
      have *= it.e;
    }
    shape_out[i] = SA[i] / SB[i];
    if (have != shape_out[i]) {
      set_error("%s: the recovered block of dimension %d has extent %lld, not %lld", what, i, (long long)have,
                (long long)shape_out[i]);
      return AXE_ENOFORM;
    }
  }
  // replicas: those of B must be present in A; what remains are C's, span-scaled
  Iters ra(a.R), rb(b.R);
  for (const HIter& it : rb) {
    auto hit = std::find_if(ra.begin(), ra.end(), [&](const HIter& x) { return x.e == it.e && x.s == it.s && x.axis == it.axis; });
    if (hit == ra.end()) {
      set_error("%s: a replica iter of B does not occur in A", what);
      return AXE_ENOFORM;
    }
    ra.erase(hit);
  }
  for (const HIter& it : ra) {
    if (it.s % w[it.axis]) {
      set_error("%s: a replica iter of A is neither B's nor span-scaled", what);
      return AXE_ENOFORM;
    }
    c.R.push_back(HIter{it.e, it.s / w[it.axis], it.axis});
  }
  for (int x = 0; x < c.n_axes; ++x) {
    const int64_t diff = a.off[x] - b.off[x];
    if (diff % w[x]) {
      set_error("%s: the offsets differ by %lld on axis %d, not a multiple of B's span %lld", what, (long long)diff, x,
                (long long)w[x]);
      return AXE_ENOFORM;
    }
    c.off[x] = diff / w[x];
  }
  keep_one(c.D, a.D[0].axis);
  return emit(c, A, out, arena, arena_bytes, what);
}

int axe_layout_slice(const axe_layout_t* L, int32_t rank, const int64_t* shape, const int64_t* begin, const int64_t* size,
                     axe_layout_t* out, void* arena, size_t arena_bytes) {
  const char* what = "axe_layout_slice";
  HLayout h;
  if (int rc = load_layout(L, h, what)) return rc;
  if (int rc = check_shapes(h, rank, shape, what)) return rc;
  if (!begin || !size || !out) {
    set_error("%s: NULL argument", what);
    return AXE_EINVAL;
  }
  for (int i = 0; i < rank; ++i)
    if (begin[i] < 0 || size[i] < 1 || begin[i] > shape[i] - size[i]) {
      set_error("%s: region [%lld, %lld + %lld) leaves dimension %d of extent %lld", what, (long long)begin[i],
                (long long)begin[i], (long long)size[i], i, (long long)shape[i]);
      return AXE_ESHAPE;
    }
  std::vector<Iters> blocks;
  if (int rc = group_by_shape(h.D, rank, shape, blocks, what)) return rc;
  HLayout s;
  s.n_axes = h.n_axes;
  s.R = h.R;
  memcpy(s.off, h.off, sizeof s.off);
  // the swizzle stage acts on D + R + O, whatever produced it: it is kept as it is
  s.swz_axis = h.swz_axis, s.swz_bits = h.swz_bits, s.swz_base = h.swz_base, s.swz_shift = h.swz_shift;
  for (int i = 0; i < rank; ++i) {
    Iters part;
    if (int rc = slice_block(blocks[i], begin[i], size[i], part, what)) return rc;
    s.D.insert(s.D.end(), part.begin(), part.end());
    // image of begin[i] under this block goes into the offset
    int64_t rest = begin[i];
    for (size_t j = blocks[i].size(); j-- > 0;) {
      const HIter& it = blocks[i][j];
      int64_t step;
      if (!mul_ok(rest % it.e, it.s, &step) || !add_ok(s.off[it.axis], step, &s.off[it.axis])) return overflow(what);
      rest /= it.e;
    }
    // every dimension keeps at least one iter, so that the result still admits `size` block by block
    if (part.empty()) s.D.push_back(HIter{1, 1, blocks[i].empty() ? h.D[0].axis : blocks[i].back().axis});
  }
  return emit(s, L, out, arena, arena_bytes, what);
}

}  // extern "C"
