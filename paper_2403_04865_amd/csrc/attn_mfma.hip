// bf16 MFMA attention for gfx950 (placeholder until the tiled kernels land: reports "not available").
#include "slide_internal.h"

namespace sl {
bool attn_mfma_ok(int, int) { return false; }
hipError_t launch_attn_fwd_mfma(const void*, void*, float*, long long, int, int, int, hipStream_t) {
  return hipErrorNotSupported;
}
hipError_t launch_attn_bwd_mfma(const void*, const void*, const float*, const void*, void*, long long, int, int, int,
                                hipStream_t) {
  return hipErrorNotSupported;
}
}  // namespace sl
