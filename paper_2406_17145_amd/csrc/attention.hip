// Multi-head softmax attention for the transformer branches, forward and
// backward, grouped over all branches of a level.  Per (sample, head):
//   P = softmax_rows(Q K^T / sqrt(dh)),  O = P V
//   dV = P^T dO, dP = dO V^T, dS = P * (dP - rowsum(dO * O)), dQ = dS K / sqrt(dh), dK = dS^T Q / sqrt(dh)
// The forward keeps only the row log-sum-exp; the backward recomputes P from it.
// Row-parallel reference variant: one wavefront per query row (forward, dQ) or
// per key row (dK, dV); scores live in LDS.  Deterministic: no atomics.
#include "device_utils.h"

namespace gpp {

constexpr int ATT_MAX_SEQ = 1536;  // LDS: 4 waves * (2*seq + 256) floats must stay under 64 KB

int attn_blocks(int batch, int heads, int seq) { return batch * heads * ((seq + 3) / 4); }

struct RowCtx {
  int b, h, row;
  bool valid;
};
__device__ __forceinline__ RowCtx row_ctx(const AttnProb &p, int blk) {
  const int rb = (p.seq + 3) / 4;
  const int bh = blk / rb;
  RowCtx c;
  c.b = bh / p.heads;
  c.h = bh % p.heads;
  c.row = (blk % rb) * 4 + (threadIdx.x >> 6);
  c.valid = c.row < p.seq;
  return c;
}

// dot product of two dh-long rows held in global memory; lanes each own whole rows
__device__ __forceinline__ float row_dot(const void *a, int64_t ao, const float *q_lds, int dh, int dtype) {
  float s = 0.0f;
  for (int c = 0; c < dh; ++c) s += q_lds[c] * load_as_f32(a, dtype, ao + c);
  return s;
}

__global__ __launch_bounds__(256) void k_attn_fwd(const AttnProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const AttnProb p = probs[pi];
  const RowCtx rc = row_ctx(p, blockIdx.x - p.blk_begin);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float *sc = lds + (size_t)w * (p.seq + 128);
  float *qv = sc + p.seq;
  if (!rc.valid) return;
  const int d = p.heads * p.dh;
  const float scale = rsqrtf((float)p.dh);
  const int64_t base = (int64_t)rc.b * p.seq;
  const int64_t qo = (base + rc.row) * p.ld_qkv + rc.h * p.dh;
  for (int c = lane; c < p.dh; c += 64) qv[c] = load_as_f32(p.qkv, p.dtype, qo + c) * scale;
  __builtin_amdgcn_wave_barrier();
  float m = -INFINITY;
  for (int j = lane; j < p.seq; j += 64) {
    float s = row_dot(p.qkv, (base + j) * p.ld_qkv + d + rc.h * p.dh, qv, p.dh, p.dtype);
    sc[j] = s;
    m = fmaxf(m, s);
  }
  m = wave_max(m);
  float se = 0.0f;
  for (int j = lane; j < p.seq; j += 64) {
    float e = __expf(sc[j] - m);
    sc[j] = e;
    se += e;
  }
  se = wave_sum(se);
  const float inv = 1.0f / se;
  __builtin_amdgcn_wave_barrier();
  for (int c = lane; c < p.dh; c += 64) {
    float o = 0.0f;
    for (int j = 0; j < p.seq; ++j) o += sc[j] * load_as_f32(p.qkv, p.dtype, (base + j) * p.ld_qkv + 2 * d + rc.h * p.dh + c);
    store_from_f32(p.out, p.out_dtype, (base + rc.row) * p.ld_out + rc.h * p.dh + c, o * inv);
  }
  if (lane == 0) p.lse[((int64_t)rc.b * p.heads + rc.h) * p.seq + rc.row] = m + __logf(se);
}

// dQ for one query row per wave; also writes delta = rowsum(dO * O)
__global__ __launch_bounds__(256) void k_attn_bwd_dq(const AttnProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const AttnProb p = probs[pi];
  const RowCtx rc = row_ctx(p, blockIdx.x - p.blk_begin);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float *ds = lds + (size_t)w * (p.seq + 256);
  float *qv = ds + p.seq;
  float *dov = qv + 128;
  if (!rc.valid) return;
  const int d = p.heads * p.dh;
  const float scale = rsqrtf((float)p.dh);
  const int64_t base = (int64_t)rc.b * p.seq;
  const int64_t stat = ((int64_t)rc.b * p.heads + rc.h) * p.seq + rc.row;
  float dl = 0.0f;
  for (int c = lane; c < p.dh; c += 64) {
    qv[c] = load_as_f32(p.qkv, p.dtype, (base + rc.row) * p.ld_qkv + rc.h * p.dh + c) * scale;
    float g = load_as_f32(p.dout, p.out_dtype, (base + rc.row) * p.ld_dout + rc.h * p.dh + c);
    dov[c] = g;
    dl += g * load_as_f32(p.o, p.out_dtype, (base + rc.row) * p.ld_o + rc.h * p.dh + c);
  }
  dl = wave_sum(dl);
  if (lane == 0) p.delta[stat] = dl;
  const float lse = p.lse[stat];
  __builtin_amdgcn_wave_barrier();
  for (int j = lane; j < p.seq; j += 64) {
    float s = row_dot(p.qkv, (base + j) * p.ld_qkv + d + rc.h * p.dh, qv, p.dh, p.dtype);
    float dp = row_dot(p.qkv, (base + j) * p.ld_qkv + 2 * d + rc.h * p.dh, dov, p.dh, p.dtype);
    ds[j] = __expf(s - lse) * (dp - dl);
  }
  __builtin_amdgcn_wave_barrier();
  for (int c = lane; c < p.dh; c += 64) {
    float a = 0.0f;
    for (int j = 0; j < p.seq; ++j) a += ds[j] * load_as_f32(p.qkv, p.dtype, (base + j) * p.ld_qkv + d + rc.h * p.dh + c);
    store_from_f32(p.out, p.grad_dtype, (base + rc.row) * p.ld_out + rc.h * p.dh + c, a * scale);
  }
}

// dK and dV for one key row per wave
__global__ __launch_bounds__(256) void k_attn_bwd_dkv(const AttnProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const AttnProb p = probs[pi];
  const RowCtx rc = row_ctx(p, blockIdx.x - p.blk_begin);
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float *ds = lds + (size_t)w * (2 * p.seq + 256);
  float *pr = ds + p.seq;
  float *kv = pr + p.seq;
  float *vv = kv + 128;
  if (!rc.valid) return;
  const int d = p.heads * p.dh;
  const float scale = rsqrtf((float)p.dh);
  const int64_t base = (int64_t)rc.b * p.seq;
  const int64_t stat0 = ((int64_t)rc.b * p.heads + rc.h) * p.seq;
  for (int c = lane; c < p.dh; c += 64) {
    kv[c] = load_as_f32(p.qkv, p.dtype, (base + rc.row) * p.ld_qkv + d + rc.h * p.dh + c) * scale;
    vv[c] = load_as_f32(p.qkv, p.dtype, (base + rc.row) * p.ld_qkv + 2 * d + rc.h * p.dh + c);
  }
  __builtin_amdgcn_wave_barrier();
  for (int i = lane; i < p.seq; i += 64) {
    float s = row_dot(p.qkv, (base + i) * p.ld_qkv + rc.h * p.dh, kv, p.dh, p.dtype);
    float dp = row_dot(p.dout, (base + i) * p.ld_dout + rc.h * p.dh, vv, p.dh, p.out_dtype);
    float pij = __expf(s - p.lse[stat0 + i]);
    pr[i] = pij;
    ds[i] = pij * (dp - p.delta[stat0 + i]);
  }
  __builtin_amdgcn_wave_barrier();
  for (int c = lane; c < p.dh; c += 64) {
    float dk = 0.0f, dv = 0.0f;
    for (int i = 0; i < p.seq; ++i) {
      dk += ds[i] * load_as_f32(p.qkv, p.dtype, (base + i) * p.ld_qkv + rc.h * p.dh + c);
      dv += pr[i] * load_as_f32(p.dout, p.out_dtype, (base + i) * p.ld_dout + rc.h * p.dh + c);
    }
    store_from_f32(p.out, p.grad_dtype, (base + rc.row) * p.ld_out + d + rc.h * p.dh + c, dk * scale);
    store_from_f32(p.out, p.grad_dtype, (base + rc.row) * p.ld_out + 2 * d + rc.h * p.dh + c, dv);
  }
}

void launch_attn_fwd(const AttnProb *probs, int n, int total_blocks, int max_seq, hipStream_t s) {
  if (total_blocks <= 0) return;
  size_t sh = 4 * (size_t)(max_seq + 128) * sizeof(float);
  hipLaunchKernelGGL(k_attn_fwd, dim3(total_blocks), dim3(256), sh, s, probs, n);
}
void launch_attn_bwd_dq(const AttnProb *probs, int n, int total_blocks, int max_seq, hipStream_t s) {
  if (total_blocks <= 0) return;
  size_t sh = 4 * (size_t)(max_seq + 256) * sizeof(float);
  hipLaunchKernelGGL(k_attn_bwd_dq, dim3(total_blocks), dim3(256), sh, s, probs, n);
}
void launch_attn_bwd_dkv(const AttnProb *probs, int n, int total_blocks, int max_seq, hipStream_t s) {
  if (total_blocks <= 0) return;
  size_t sh = 4 * (size_t)(2 * max_seq + 256) * sizeof(float);
  hipLaunchKernelGGL(k_attn_bwd_dkv, dim3(total_blocks), dim3(256), sh, s, probs, n);
}
int attn_max_seq() { return ATT_MAX_SEQ; }

}  // namespace gpp
