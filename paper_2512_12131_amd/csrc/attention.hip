// Causal multi-head attention for the decoder block (placeholder until the kernels land).
#include "common.h"
namespace lrb {
hipError_t attention_fwd_bf16(const void*, const void*, const void*, void*, float*, int64_t, int, int, int, int, int,
                              hipStream_t) { return hipErrorNotSupported; }
size_t attention_bwd_ws_bytes(int, int, int, int) { return 0; }
hipError_t attention_bwd_bf16(const void*, const void*, const void*, const void*, const void*, const float*, void*,
                              void*, void*, int64_t, int, int, int, int, int, void*, hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace lrb
