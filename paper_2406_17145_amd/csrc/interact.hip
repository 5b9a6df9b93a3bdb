// Pairwise-dot feature interaction of a DLRM-shaped stage (forward and backward),
// grouped over operators; one workgroup per sample with the F vectors in LDS.
#include "device_utils.h"

namespace gpp {

// ------------------------------------------------------------------ pairwise-dot interaction
// one workgroup per sample; the F vectors sit in LDS
__device__ __forceinline__ void term_to_pair(int t, int &i, int &j) {
  i = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)t)) * 0.5f);
  while (i * (i - 1) / 2 > t) --i;
  while ((i + 1) * i / 2 <= t) ++i;
  j = t - i * (i - 1) / 2;
}

__global__ __launch_bounds__(256) void k_interact_fwd(const InteractProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const InteractProb p = probs[pi];
  const int s = blockIdx.x - p.blk_begin;
  const int st = p.d + 1;
  for (int e = threadIdx.x; e < p.F * p.d; e += 256)
    lds[(e / p.d) * st + (e % p.d)] = load_as_f32(p.x, p.x_dtype, (int64_t)s * p.ld_x + e);
  __syncthreads();
  for (int c = threadIdx.x; c < p.d; c += 256) store_from_f32(p.y, p.y_dtype, (int64_t)s * p.ld_y + c, lds[c]);
  const int terms = p.F * (p.F - 1) / 2;
  for (int t = threadIdx.x; t < terms; t += 256) {
    int i, j;
    term_to_pair(t, i, j);
    float a = 0.0f;
    for (int c = 0; c < p.d; ++c) a += lds[i * st + c] * lds[j * st + c];
    store_from_f32(p.y, p.y_dtype, (int64_t)s * p.ld_y + p.d + t, a);
  }
}

__global__ __launch_bounds__(256) void k_interact_bwd(const InteractProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const InteractProb p = probs[pi];
  const int s = blockIdx.x - p.blk_begin;
  const int st = p.d + 1;
  float *T = lds;
  float *G = lds + p.F * st;  // symmetric F x F, zero diagonal
  for (int e = threadIdx.x; e < p.F * p.d; e += 256)
    T[(e / p.d) * st + (e % p.d)] = load_as_f32(p.x, p.x_dtype, (int64_t)s * p.ld_x + e);
  for (int e = threadIdx.x; e < p.F; e += 256) G[e * p.F + e] = 0.0f;
  const int terms = p.F * (p.F - 1) / 2;
  for (int t = threadIdx.x; t < terms; t += 256) {
    int i, j;
    term_to_pair(t, i, j);
    float g = load_as_f32(p.dy, p.dy_dtype, (int64_t)s * p.ld_dy + p.d + t);
    G[i * p.F + j] = g;
    G[j * p.F + i] = g;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < p.F * p.d; e += 256) {
    const int i = e / p.d, c = e % p.d;
    float a = i == 0 ? load_as_f32(p.dy, p.dy_dtype, (int64_t)s * p.ld_dy + c) : 0.0f;
    for (int j = 0; j < p.F; ++j) a += G[i * p.F + j] * T[j * st + c];
    store_from_f32(p.y, p.y_dtype, (int64_t)s * p.ld_y + e, a);
  }
}

static size_t interact_lds(int F, int d) { return ((size_t)F * (d + 1) + (size_t)F * F) * sizeof(float); }
void launch_interact_fwd(const InteractProb *probs, int n, int total_blocks, int maxF, int maxd, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_interact_fwd, dim3(total_blocks), dim3(256), interact_lds(maxF, maxd), s, probs, n);
}
void launch_interact_bwd(const InteractProb *probs, int n, int total_blocks, int maxF, int maxd, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_interact_bwd, dim3(total_blocks), dim3(256), interact_lds(maxF, maxd), s, probs, n);
}
size_t interact_lds_bytes(int F, int d) { return interact_lds(F, d); }

}  // namespace gpp
