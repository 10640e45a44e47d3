#include "../../include/axe.h"
#include "host_layout.h"
extern "C" int axe_gemm_describe(const axe_gemm_desc_t*, int32_t, axe_layout_t*, int64_t*, int32_t*, void*, size_t) {
  axe::set_error("axe_gemm_describe: not built yet");
  return AXE_EUNSUPPORTED;
}
