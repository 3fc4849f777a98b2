// bf16 MFMA GEMMs for gfx950 (placeholder until the tiled kernels land: reports "not available").
#include "gemm_epi.h"

namespace sl {
bool gemm_nt_mfma_ok(const GemmNT&) { return false; }
bool gemm_tn_mfma_ok(const GemmTN&) { return false; }
hipError_t launch_gemm_nt_mfma(const GemmNT&, hipStream_t) { return hipErrorNotSupported; }
hipError_t launch_gemm_tn_mfma(const GemmTN&, hipStream_t) { return hipErrorNotSupported; }
}  // namespace sl
