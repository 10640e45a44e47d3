// Launch entry points of the kernels (host-callable; defined in the .hip files).
#pragma once
#include <hip/hip_runtime.h>

#include "device_types.h"

namespace axe {

hipError_t launch_layout_eval(const EvalDesc& d, int64_t n, const int64_t* idx, int64_t* out, hipStream_t s);
hipError_t launch_relayout_joint(const RelayoutPlan& p, int unit_bytes, const void* src, void* dst, hipStream_t s);
hipError_t launch_relayout_generic(const GenericRelayoutPlan& p, int unit_bytes, const void* src, void* dst,
                                   hipStream_t s);
hipError_t launch_gemm_small(const GemmArgs& g, bool fp8, hipStream_t s);
// Large-tile kernels: 256 x tile_n workgroup tile (tile_n = 256, or 224 for bf16); require
// M % 256 == 0, N % tile_n == 0 and K a multiple of the K step (bf16: 64, fp8: 128).
hipError_t launch_gemm_bf16_256(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_fp8_256(const GemmArgs& g, hipStream_t s);

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

}  // namespace axe
