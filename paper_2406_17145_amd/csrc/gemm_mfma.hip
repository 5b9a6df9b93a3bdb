// Branch-grouped bf16 GEMM on the CDNA4 matrix cores (placeholder until the
// MFMA kernels land: reports every problem as unsupported, so the planner
// routes all GEMMs to the generic kernel).
#include "device_utils.h"

namespace gpp {
bool gemm_mfma_supported(const GemmProb &) { return false; }
int gemm_mfma_tiles(int, int, int, int, int *tiles_n) {
  if (tiles_n) *tiles_n = 0;
  return 0;
}
void launch_gemm_mfma(const GemmProb *, int, int, int, int, hipStream_t) {}
}  // namespace gpp
