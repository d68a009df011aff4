// Many-row (prefill) routed LoRA linear on row-major bf16 weights: matrix-core GEMM tiles staged
// through LDS.  Placeholder until the tiled kernel lands: reports "not covered" so that callers
// take the any-shape path.
#include "common.h"

namespace milora {

bool prefill_supported(int64_t, int, int, const void*, const void*, const void*) { return false; }

int routed_linear_prefill(const bf16_t*, int64_t, int, int, const int32_t*, const bf16_t*, const bf16_t*,
                          const AdapterView&, int, const int32_t*, const uint8_t*, int, const float*, bf16_t*,
                          hipStream_t) {
  return MILORA_EUNSUPPORTED;
}

}  // namespace milora
