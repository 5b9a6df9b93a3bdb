// Branch-grouped GEMM, generic variant: fp32 FMA on LDS-staged 64x64x16 tiles.
// It serves the fp32 numeric mode and any bf16 problem whose pointers or
// leading dimensions do not meet the MFMA kernels' alignment rules.  One
// launch covers every independent branch of a topological level; a workgroup
// locates its problem through the records' workgroup prefix sums.
#include "device_utils.h"

namespace gpp {

constexpr int GT = 64;   // tile edge
constexpr int GK = 16;   // contraction step

int gemm_generic_tiles(int M, int N, int *tiles_n) {
  int tm = (M + GT - 1) / GT, tn = (N + GT - 1) / GT;
  if (tiles_n) *tiles_n = tn;
  return tm * tn;
}

template <typename T>
__global__ __launch_bounds__(256) void k_gemm_generic(const GemmProb *__restrict__ probs, int n,
                                                       int accumulate_dw) {
  __shared__ float As[GK][GT + 4];
  __shared__ float Bs[GK][GT + 4];
  const int pi = find_prob(probs, n, blockIdx.x);
  const GemmProb p = probs[pi];
  const int tile = blockIdx.x - p.blk_begin;
  const int m0 = (tile / p.tiles_n) * GT, n0 = (tile % p.tiles_n) * GT;
  const int t = threadIdx.x, tx = t & 15, ty = t >> 4;

  // element strides of the logical operands A(i, kk) [M x K] and B(kk, j) [K x N]
  int64_t sai, sak, sbk, sbj;
  if (p.form == FORM_FWD) {
    sai = p.lda; sak = 1; sbk = 1; sbj = p.ldb;
  } else if (p.form == FORM_DX) {
    sai = p.lda; sak = 1; sbk = p.ldb; sbj = 1;
  } else {
    sai = 1; sak = p.lda; sbk = p.ldb; sbj = 1;
  }
  const T *A = (const T *)p.A;
  const T *B = (const T *)p.B;

  float acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = 0.0f;

  for (int k0 = 0; k0 < p.K; k0 += GK) {
#pragma unroll
    for (int r = 0; r < 4; ++r) {
      int e = t + 256 * r, ii, kk;
      if (sak == 1) { kk = e & 15; ii = e >> 4; } else { ii = e & 63; kk = e >> 6; }
      float v = 0.0f;
      if (m0 + ii < p.M && k0 + kk < p.K) v = to_f32<T>(A[(int64_t)(m0 + ii) * sai + (int64_t)(k0 + kk) * sak]);
      As[kk][ii] = v;
      int jj;
      if (sbk == 1) { kk = e & 15; jj = e >> 4; } else { jj = e & 63; kk = e >> 6; }
      v = 0.0f;
      if (n0 + jj < p.N && k0 + kk < p.K) v = to_f32<T>(B[(int64_t)(k0 + kk) * sbk + (int64_t)(n0 + jj) * sbj]);
      Bs[kk][jj] = v;
    }
    __syncthreads();
#pragma unroll
    for (int kk = 0; kk < GK; ++kk) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[kk][ty + 16 * i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[kk][tx + 16 * j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }

#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = m0 + ty + 16 * i;
    if (row >= p.M) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      const int col = n0 + tx + 16 * j;
      if (col >= p.N) continue;
      float v = acc[i][j];
      const int64_t ci = (int64_t)row * p.ldc + col;
      if (p.form == FORM_FWD) {
        if (p.bias) v += p.bias[col];
        if (p.aux) store_from_f32(p.aux, p.aux_dtype, (int64_t)row * p.ldaux + col, act_stash(v, p.act));
        v = act_apply(v, p.act);
        if (p.res) v += load_as_f32(p.res, p.res_dtype, (int64_t)row * p.ldres + col);
        store_from_f32(p.C, p.c_dtype, ci, v);
      } else if (p.form == FORM_DX) {
        if (p.res) v += load_as_f32(p.res, p.res_dtype, (int64_t)row * p.ldres + col);
        if (p.act != ACT_NONE) v *= act_grad(load_as_f32(p.aux, p.aux_dtype, (int64_t)row * p.ldaux + col), p.act);
        store_from_f32(p.C, p.c_dtype, ci, v);
      } else {
        float *c = (float *)p.C;
        c[ci] = accumulate_dw ? c[ci] + v : v;
      }
    }
  }
}

void launch_gemm_generic(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int in_dtype,
                         hipStream_t s) {
  if (total_blocks <= 0) return;
  if (in_dtype == DT_BF16)
    hipLaunchKernelGGL(k_gemm_generic<uint16_t>, dim3(total_blocks), dim3(256), 0, s, probs, n, accumulate_dw);
  else
    hipLaunchKernelGGL(k_gemm_generic<float>, dim3(total_blocks), dim3(256), 0, s, probs, n, accumulate_dw);
}

}  // namespace gpp
