// Host-side layout analysis: validation (Defs. 2.1 / 2.2), reduction to the memory axis of one
// GPU, canonicalisation rules D0 / D1 (App. A), address range and injectivity tests, and the
// common refinement of two shard lists that drives the relayout loop nest.
#pragma once
#include <stdint.h>

#include <vector>

#include "../../include/axe.h"
#include "device_types.h"

namespace axe {

struct HIter {
  int64_t e, s;
  int axis;
};

struct HLayout {
  int n_axes = 0;
  std::vector<HIter> D, R;
  int64_t off[AXE_MAX_AXES] = {0};
  int swz_axis = -1, swz_bits = 0, swz_base = 0, swz_shift = 0;
  int64_t E_D = 1, E_R = 1;
};

// Layout restricted to the memory axis (one GPU): D after D0 / D1, replicas, offset, swizzle.
struct MemLayout {
  std::vector<HIter> D;      // canonical; may be empty when E_D == 1
  std::vector<HIter> R;      // extent > 1 only
  int64_t off = 0;
  Swz swz = {0, 0, 0};
  int64_t E_D = 1, E_R = 1;
  int64_t lo = 0, hi = 0;    // inclusive address range over all x and replicas (after swizzle)
};

struct JointIter {
  int64_t e, ss, ds;
};

void set_error(const char* fmt, ...);
const char* last_error();

// AXE_EINVAL on any violation of the definitions; fills E_D / E_R (AXE_ERANGE on overflow).
int load_layout(const axe_layout_t* L, HLayout& out, const char* what);
// AXE_ESHAPE unless prod(shape) == E_D.
int check_shape(const HLayout& L, int32_t rank, const int64_t* shape, const char* what);
// Drops unit iters on other axes; AXE_EALIAS if another axis has extent > 1.  Canonicalises D.
int reduce_to_memory(const HLayout& L, int mem_axis, MemLayout& out, const char* what);
// AXE_ERANGE unless every address lies in [0, elems).
int check_range(const MemLayout& L, int64_t elems, const char* what);
// Sufficient test that no two (logical element, replica) pairs share an address on the memory axis:
// the strides of the shard and replica iters together nest.
bool provably_injective(const MemLayout& L);
void canon_D(std::vector<HIter>& D);
// Common refinement of two digit systems with equal total extent; false if none exists.
bool joint_refine(const std::vector<HIter>& s, const std::vector<HIter>& d, std::vector<JointIter>& out);

}  // namespace axe
