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
// Large-tile kernels: 256 x 256 workgroup tile; require M % 256 == 0, N % 256 == 0 and K a
// multiple of the K step (bf16: 32, fp8: 128).
hipError_t launch_gemm_bf16_256(const GemmArgs& g, hipStream_t s);
hipError_t launch_gemm_fp8_256(const GemmArgs& g, hipStream_t s);

}  // namespace axe
