// Pairwise-dot feature interaction of a DLRM-shaped stage (forward and backward),
// grouped over operators; one workgroup per sample with the F vectors in LDS.
#include <algorithm>

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

// ---- vector bodies: rows of whole, aligned 16-byte chunks, one storage type for x / y / dy.  The type
// is a template parameter, so that the loads of a phase are requested together (a run-time type test in
// front of every load is a branch, and a wave waits for its earlier loads at a branch).
template <int DT>
__device__ __forceinline__ void ld8(const void *base, int64_t i, float (&v)[8]) {
  if (DT == DT_BF16) {
    const uint4 u = *(const uint4 *)((const uint16_t *)base + i);
    const uint32_t w[4] = {u.x, u.y, u.z, u.w};
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      v[2 * e] = __uint_as_float(w[e] << 16);
      v[2 * e + 1] = __uint_as_float(w[e] & 0xffff0000u);
    }
  } else {
    const float4 a = *(const float4 *)((const float *)base + i), b = *(const float4 *)((const float *)base + i + 4);
    v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
  }
}
template <int DT>
__device__ __forceinline__ void st8(void *base, int64_t i, const float (&v)[8]) {
  if (DT == DT_BF16) {
    uint4 u;
    u.x = (uint32_t)f32_to_bf16_bits(v[0]) | ((uint32_t)f32_to_bf16_bits(v[1]) << 16);
    u.y = (uint32_t)f32_to_bf16_bits(v[2]) | ((uint32_t)f32_to_bf16_bits(v[3]) << 16);
    u.z = (uint32_t)f32_to_bf16_bits(v[4]) | ((uint32_t)f32_to_bf16_bits(v[5]) << 16);
    u.w = (uint32_t)f32_to_bf16_bits(v[6]) | ((uint32_t)f32_to_bf16_bits(v[7]) << 16);
    *(uint4 *)((uint16_t *)base + i) = u;
  } else {
    *(float4 *)((float *)base + i) = make_float4(v[0], v[1], v[2], v[3]);
    *(float4 *)((float *)base + i + 4) = make_float4(v[4], v[5], v[6], v[7]);
  }
}
constexpr int INT_GP = 32;          // row stride of the F x F gradient matrix in the vector backward body
constexpr int INT_MAX_CHUNKS = 4;   // 8-element chunks of the F x d block per thread: F * d <= 8192
__device__ __forceinline__ bool interact_vec_ok(const InteractProb &p, bool bwd) {
  if ((p.d & 7) || p.F * p.d > 256 * 8 * INT_MAX_CHUNKS) return false;
  if ((p.ld_x & 7) || ((uintptr_t)p.x & 15)) return false;
  if (bwd && ((p.ld_y & 7) || ((uintptr_t)p.y & 15) || p.F > INT_GP)) return false;   // G in rows of INT_GP
  return true;
}
// the F x d block of sample s into LDS rows of stride d + 4 floats: rows stay 16-byte aligned, and sixteen
// consecutive rows read with 16-byte reads fall into sixteen different groups of four banks
__device__ __forceinline__ int interact_stride(int d) { return d + 4; }
template <int DT>
__device__ __forceinline__ void interact_stage_x(const InteractProb &p, int s, float *T, int st) {
  const int chunks = (p.F * p.d) >> 3;
  float v[INT_MAX_CHUNKS][8];
#pragma unroll
  for (int u = 0; u < INT_MAX_CHUNKS; ++u) {
    const int q = threadIdx.x + 256 * u;
    ld8<DT>(p.x, (int64_t)s * p.ld_x + 8 * (q < chunks ? q : 0), v[u]);
  }
#pragma unroll
  for (int u = 0; u < INT_MAX_CHUNKS; ++u) {
    const int q = threadIdx.x + 256 * u;
    if (q < chunks) {
      const int row = (8 * q) / p.d, col = 8 * q - row * p.d;
      float4 *dst = (float4 *)(T + row * st + col);
      dst[0] = make_float4(v[u][0], v[u][1], v[u][2], v[u][3]);
      dst[1] = make_float4(v[u][4], v[u][5], v[u][6], v[u][7]);
    }
  }
}
// A thread per dot product, four columns per pair of 16-byte LDS reads, summed in column order.  (One 4-byte
// read per operand and column was two LDS instructions per multiply-add: 18 us for 2048 samples of 27 x 128.)
template <int DT>
__device__ __forceinline__ void interact_fwd_vec(const InteractProb &p, int s, float *lds) {
  const int st = interact_stride(p.d);
  interact_stage_x<DT>(p, s, lds, st);
  __syncthreads();
  for (int c = threadIdx.x; c < p.d; c += 256) store_from_f32(p.y, DT, (int64_t)s * p.ld_y + c, lds[c]);
  const int terms = p.F * (p.F - 1) / 2;
  for (int t = threadIdx.x; t < terms; t += 256) {
    int i, j;
    term_to_pair(t, i, j);
    const float4 *xi = (const float4 *)(lds + i * st), *xj = (const float4 *)(lds + j * st);
    float a = 0.0f;
    for (int c = 0; c < (p.d >> 2); ++c) {
      const float4 u = xi[c], v = xj[c];
      a += u.x * v.x;
      a += u.y * v.y;
      a += u.z * v.z;
      a += u.w * v.w;
    }
    store_from_f32(p.y, DT, (int64_t)s * p.ld_y + p.d + t, a);
  }
}
// Backward: dT[i][c] = sum_j G[i][j] T[j][c] (+ the pass-through of vector 0), G the symmetric matrix of the
// dot-product gradients with a zero diagonal.  COLS: the vector width d when it divides 256 (64, 128, 256), else 0.
// With COLS a thread owns one column c and the rows i = g, g + 256 / d, ...: it keeps its column of T in
// registers (F <= 32 values) and reads G four entries at a time; a wave covers 64 columns of ONE row, so those
// reads are the same address for all its lanes.  About one LDS instruction per six multiply-adds instead of two
// per multiply-add (34 -> ~12 us for 2048 samples of 27 x 128).  Sums run over j in ascending order either way.
template <int DT, int COLS>
__device__ __forceinline__ void interact_bwd_vec(const InteractProb &p, int s, float *lds) {
  const int st = interact_stride(p.d);
  float *T = lds;
  float *G = lds + p.F * st;  // symmetric F x F in rows of INT_GP, zero diagonal
  const int terms = p.F * (p.F - 1) / 2;
  // the gradients of the dot products (their offset d + t is not chunk-aligned: element loads), all
  // of a thread's requested before the block of x is staged
  constexpr int GT = 4;
  float g[GT];
#pragma unroll
  for (int u = 0; u < GT; ++u) {
    const int t = threadIdx.x + 256 * u;
    g[u] = load_as_f32(p.dy, DT, (int64_t)s * p.ld_dy + p.d + (t < terms ? t : 0));
  }
  interact_stage_x<DT>(p, s, T, st);
  for (int e = threadIdx.x; e < p.F; e += 256) G[e * INT_GP + e] = 0.0f;
#pragma unroll
  for (int u = 0; u < GT; ++u) {
    const int t = threadIdx.x + 256 * u;
    if (t < terms) {
      int i, j;
      term_to_pair(t, i, j);
      G[i * INT_GP + j] = g[u];
      G[j * INT_GP + i] = g[u];
    }
  }
  for (int t = threadIdx.x + 256 * GT; t < terms; t += 256) {   // more than 1024 terms (F > 45)
    int i, j;
    term_to_pair(t, i, j);
    const float gv = load_as_f32(p.dy, DT, (int64_t)s * p.ld_dy + p.d + t);
    G[i * INT_GP + j] = gv;
    G[j * INT_GP + i] = gv;
  }
  __syncthreads();
  if (COLS > 0) {
    const int c = threadIdx.x % COLS, g0 = threadIdx.x / COLS;
    float tc[INT_GP];
#pragma unroll
    for (int j = 0; j < INT_GP; ++j) tc[j] = j < p.F ? T[j * st + c] : 0.0f;
    const float pass = load_as_f32(p.dy, DT, (int64_t)s * p.ld_dy + c);
    for (int i = g0; i < p.F; i += 256 / COLS) {
      float a = i == 0 ? pass : 0.0f;
      const float4 *gr = (const float4 *)(G + i * INT_GP);
#pragma unroll
      for (int q = 0; q < INT_GP / 4; ++q) {
        const float4 gv = gr[q];
        if (4 * q + 0 < p.F) a += gv.x * tc[4 * q + 0];
        if (4 * q + 1 < p.F) a += gv.y * tc[4 * q + 1];
        if (4 * q + 2 < p.F) a += gv.z * tc[4 * q + 2];
        if (4 * q + 3 < p.F) a += gv.w * tc[4 * q + 3];
      }
      store_from_f32(p.y, DT, (int64_t)s * p.ld_y + (int64_t)i * p.d + c, a);
    }
    return;
  }
  // a thread per element, consecutive columns in consecutive lanes (LDS reads without bank conflicts)
  for (int e = threadIdx.x; e < p.F * p.d; e += 256) {
    const int i = e / p.d, c = e - i * p.d;
    float a = i == 0 ? load_as_f32(p.dy, DT, (int64_t)s * p.ld_dy + c) : 0.0f;
    for (int j = 0; j < p.F; ++j) a += G[i * INT_GP + j] * T[j * st + c];
    store_from_f32(p.y, DT, (int64_t)s * p.ld_y + e, a);
  }
}
template <int DT>
__device__ __forceinline__ void interact_bwd_pick(const InteractProb &p, int s, float *lds) {
  if (p.F <= INT_GP && p.d == 64) return interact_bwd_vec<DT, 64>(p, s, lds);
  if (p.F <= INT_GP && p.d == 128) return interact_bwd_vec<DT, 128>(p, s, lds);
  if (p.F <= INT_GP && p.d == 256) return interact_bwd_vec<DT, 256>(p, s, lds);
  return interact_bwd_vec<DT, 0>(p, s, lds);
}

__global__ __launch_bounds__(256) void k_interact_fwd(const InteractProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const InteractProb p = probs[pi];
  const int s = blockIdx.x - p.blk_begin;
  if (interact_vec_ok(p, false) && p.x_dtype == p.y_dtype) {
    if (p.x_dtype == DT_BF16) return interact_fwd_vec<DT_BF16>(p, s, lds);
    if (p.x_dtype == DT_F32) return interact_fwd_vec<DT_F32>(p, s, lds);
  }
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
  if (interact_vec_ok(p, true) && p.x_dtype == p.y_dtype && p.x_dtype == p.dy_dtype && (p.ld_dy & 7) == 0 &&
      ((uintptr_t)p.dy & 15) == 0) {
    if (p.x_dtype == DT_BF16) return interact_bwd_pick<DT_BF16>(p, s, lds);
    if (p.x_dtype == DT_F32) return interact_bwd_pick<DT_F32>(p, s, lds);
  }
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

// rows of d + 4 (vector bodies; the scalar bodies use d + 1) and a gradient matrix of max(F, 32) x max(F, 32)
static size_t interact_lds(int F, int d) { return ((size_t)F * (d + 4) + (size_t)std::max(F, 32) * std::max(F, 32)) * sizeof(float); }
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
