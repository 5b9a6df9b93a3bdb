// Branch-grouped bf16 GEMM on the CDNA4 matrix cores: the stand-alone kernel around the tile body.
// One launch covers every independent branch of a topological level: the workgroup index is first
// spread XCD-aware (consecutive tiles of a problem land on one XCD and share its L2), then mapped to
// (problem, tile) through the records' workgroup prefix sums.
#include "gemm_tile_body.h"

namespace gpp {

struct TileCfg {
  int bm, bn;
};

template <int FORM, int BM, int BN>
__global__ __launch_bounds__(256) void k_gemm_mfma(const GemmProb *__restrict__ probs, int n, int total_blocks,
                                                   int accumulate_dw, ExtPtrs ext) {
  __shared__ __attribute__((aligned(16))) uint16_t lds[TileLds<FORM, BM, BN>::ELEMS];
  // XCD-aware spreading: hardware deals consecutive workgroup ids round-robin over the 8 XCDs;
  // give each XCD one contiguous range of tiles instead
  int bid = blockIdx.x;
  {
    const int xcd = bid & 7, idx = bid >> 3, per = total_blocks >> 3, rem = total_blocks & 7;
    bid = xcd * per + min(xcd, rem) + idx;
  }
  const int pi = find_prob(probs, n, bid);
  const GemmProb p = probs[pi];
  gemm_tile_body<FORM, BM, BN, true>(p, bid - p.blk_begin, threadIdx.x, lds, accumulate_dw, ext);
}

// ---- host side -------------------------------------------------------------------------
static TileCfg pick_cfg(int form, int M, int N) {
  (void)form;
  TileCfg c;
  c.bm = M > 64 ? 128 : 64;
  c.bn = N > 64 ? 128 : 64;
  if (c.bm != c.bn) c.bm = c.bn = (M > 64 && N > 64) ? 128 : 64;
  return c;
}

bool gemm_mfma_supported(const GemmProb &p) {
  if (p.in_dtype != DT_BF16) return false;
  if (((uintptr_t)p.A | (uintptr_t)p.B) & 15) return false;
  if ((p.lda | p.ldb) & 7) return false;
  if (p.M <= 0 || p.N <= 0 || p.K <= 0) return false;
  return true;
}

// A launch uses one tile shape for all of its problems: the planner asks for it with the largest
// M and N of the group, then counts each problem's workgroups for that shape.
int gemm_mfma_group_tile(int form, int maxM, int maxN) {
  TileCfg c = pick_cfg(form, maxM, maxN);
  return c.bm;  // square shapes only: 64 or 128
}
int gemm_mfma_tiles_for(int tile, int M, int N, int *tiles_n) {
  if (tiles_n) *tiles_n = cdiv(N, tile);
  return cdiv(M, tile) * cdiv(N, tile);
}
// floats of one split's partial tile (the tile plus one row of bias-gradient partials)
int gemm_mfma_partial_floats(int tile) { return tile * tile + tile; }
// Split factor for a problem of a launch whose unsplit tiles add up to `launch_tiles`: aim at a few
// workgroups per CU, keep every slice long enough that the partial tiles (written and read once,
// fp32) do not exceed the operand bytes the slice streams.
int gemm_mfma_pick_split(int tile, int launch_tiles, int rows_in_tile, int K) {
  if (launch_tiles >= 512) return 1;
  int want = (1024 + launch_tiles - 1) / launch_tiles;
  int min_slice = 2 * (rows_in_tile < tile ? rows_in_tile : tile);
  if (min_slice < 2 * BK) min_slice = 2 * BK;
  int cap = K / min_slice;
  if (cap < 1) cap = 1;
  int s = want < cap ? want : cap;
  return s > 32 ? 32 : s;
}

template <int FORM>
static void launch_form(const GemmProb *probs, int n, int blocks, int acc, int tile, const ExtPtrs &ext, hipStream_t s) {
  if (tile == 128)
    hipLaunchKernelGGL((k_gemm_mfma<FORM, 128, 128>), dim3(blocks), dim3(256), 0, s, probs, n, blocks, acc, ext);
  else
    hipLaunchKernelGGL((k_gemm_mfma<FORM, 64, 64>), dim3(blocks), dim3(256), 0, s, probs, n, blocks, acc, ext);
}

void launch_gemm_mfma(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int form, int tile,
                      const ExtPtrs &ext, hipStream_t s) {
  if (total_blocks <= 0) return;
  if (form == FORM_FWD) launch_form<FORM_FWD>(probs, n, total_blocks, accumulate_dw, tile, ext, s);
  else if (form == FORM_DX) launch_form<FORM_DX>(probs, n, total_blocks, accumulate_dw, tile, ext, s);
  else launch_form<FORM_DW>(probs, n, total_blocks, accumulate_dw, tile, ext, s);
}

}  // namespace gpp
