#include <hip/hip_runtime.h>
#include "device_types.h"
#include "kernels.h"
namespace axe {
hipError_t launch_gemm_bf16_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_fp8_256(const GemmArgs&, hipStream_t) { return hipErrorNotSupported; }
}
