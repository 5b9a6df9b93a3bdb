// Backward-weight GEMM  dW[n,k] (+)= sum_m dZ[m,n] X[m,k]  for SMALL weight matrices and MANY rows
// (the MLPs of a large micro-batch): there are too few output tiles to fill the chip and each tile
// has a long contraction, so the contraction is split inside the workgroup.
//
// A workgroup owns a 64 x 64 tile of dW; its eight waves each take a contiguous slice of the rows m
// and run without workgroup barriers: 64-row steps fetched with coalesced 16-byte buffer loads, kept
// two steps ahead in registers, staged in a wave-private LDS tile and read with the transposing LDS
// read (both operands have the contraction index as their row).  The eight partial tiles meet in LDS
// and are added in wave order.  Tiles of the first column block also produce the bias gradient
// db[n] = sum_m dZ[m,n] from the dZ tiles they stage.  The old gradient values are requested before
// the k-loop so that their round trip overlaps it.
#include "gemm_dw_ksplit_body.h"

namespace gpp {

int gemm_dw_ksplit_blocks(int M, int N) { return cdiv(M, KS_T) * cdiv(N, KS_T); }

__global__ __launch_bounds__(64 * KS_NW) void k_gemm_dw_ksplit(const GemmProb *__restrict__ probs, int n, int accumulate_dw) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[KS_LDS_BYTES];
  const int pi = find_prob(probs, n, blockIdx.x);
  const GemmProb p = probs[pi];
  gemm_dw_ksplit_body(p, blockIdx.x - p.blk_begin, lds_raw, accumulate_dw);
}

void launch_gemm_dw_ksplit(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_gemm_dw_ksplit, dim3(total_blocks), dim3(64 * KS_NW), 0, s, probs, n, accumulate_dw);
}

}  // namespace gpp
