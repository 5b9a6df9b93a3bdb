// Grouped non-GEMM kernels of a stage: 2-D copy / convert / accumulate and
// activation backward, bias-gradient column sums, LayerNorm forward/backward,
// sequence mean-pool, loss heads.  All are bound by HBM traffic; every launch
// covers all branches of one topological level.
#include "device_utils.h"

namespace gpp {

// ------------------------------------------------------------------ elt
constexpr int ELT_PER_BLOCK = 2048;
int elt_blocks(int rows, int cols) {
  int64_t e = (int64_t)rows * cols;
  return (int)((e + ELT_PER_BLOCK - 1) / ELT_PER_BLOCK);
}

// Plain copy / conversion (no addend, no derivative) with the storage types as template parameters and
// every load of a thread requested before its first store: a run-time type test or a bounds branch in
// front of each load makes the wave wait for the previous load, and the copy then pays one memory
// latency per element instead of one per thread.  Elements beyond the end re-read the last element.
template <int SD, int DD>
__device__ __forceinline__ void elt_copy_body(const EltProb &p, const void *src, void *dst, uint32_t base, uint32_t total) {
  constexpr int IT = ELT_PER_BLOCK / 256;
  float v[IT];
  uint32_t di[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const uint32_t e = min(base + it * 256 + threadIdx.x, total - 1);
    const uint32_t r = e / (uint32_t)p.cols, c = e - r * (uint32_t)p.cols;
    const int64_t si = (int64_t)r * p.ld_src + c;
    di[it] = r * (uint32_t)p.ld_dst + c;
    v[it] = SD == DT_BF16 ? bf16_bits_to_f32(((const uint16_t *)src)[si]) : ((const float *)src)[si];
  }
#pragma unroll
  for (int it = 0; it < IT; ++it)
    if (base + it * 256 + threadIdx.x < total) {
      if (DD == DT_BF16) ((uint16_t *)dst)[di[it]] = f32_to_bf16_bits(v[it]);
      else ((float *)dst)[di[it]] = v[it];
    }
}

// Same-type copy whose rows are whole 16-byte chunks (columns, leading dimensions and base addresses multiples
// of 16 bytes): a thread moves 16 bytes per load instead of one element (the 16 MB input copy of the
// transformer stage: 59 -> 13 us).  Same block -> element range as the element-wise body.
template <int ES>
__device__ __forceinline__ void elt_copy_vec_body(const EltProb &p, const void *src, void *dst, uint32_t base, uint32_t total) {
  constexpr int EPC = 16 / ES, IT = ELT_PER_BLOCK / EPC / 256;
  typedef __attribute__((ext_vector_type(4))) uint32_t u4;
  u4 v[IT];
  int64_t di[IT];
#pragma unroll
  for (int it = 0; it < IT; ++it) {
    const uint32_t e = min(base + (it * 256 + threadIdx.x) * EPC, total - EPC);
    const uint32_t r = e / (uint32_t)p.cols, c = e - r * (uint32_t)p.cols;
    di[it] = ((int64_t)r * p.ld_dst + c) * ES;
    v[it] = *(const u4 *)((const char *)src + ((int64_t)r * p.ld_src + c) * ES);
  }
#pragma unroll
  for (int it = 0; it < IT; ++it)
    if (base + (it * 256 + threadIdx.x) * EPC < total) *(u4 *)((char *)dst + di[it]) = v[it];
}
__device__ __forceinline__ bool elt_vec_ok(const EltProb &p, const void *src, const void *dst, int es) {
  const int epc = 16 / es;
  return p.cols % epc == 0 && p.ld_src % epc == 0 && p.ld_dst % epc == 0 && (((uintptr_t)src | (uintptr_t)dst) & 15) == 0;
}

__global__ __launch_bounds__(256) void k_elt(const EltProb *__restrict__ probs, int n, ExtPtrs ext) {
  const int pi = find_prob(probs, n, blockIdx.x);
  const EltProb p = probs[pi];
  const void *src = p.ext_src >= 0 ? ext.p[p.ext_src] : p.src;
  void *dst = p.ext_dst >= 0 ? ext.p[p.ext_dst] : p.dst;
  if (!src || !dst) return;
  const int64_t total = (int64_t)p.rows * p.cols;
  const int64_t base = (int64_t)(blockIdx.x - p.blk_begin) * ELT_PER_BLOCK;
  if (p.mode == 0 && !p.addend && p.src_dtype != DT_I32 && p.dst_dtype != DT_I32 && total < (1ll << 31) &&
      (int64_t)p.rows * p.ld_dst < (1ll << 32)) {
    const bool sb = p.src_dtype == DT_BF16, db = p.dst_dtype == DT_BF16;
    if (sb && db && elt_vec_ok(p, src, dst, 2)) return elt_copy_vec_body<2>(p, src, dst, (uint32_t)base, (uint32_t)total);
    if (!sb && !db && elt_vec_ok(p, src, dst, 4)) return elt_copy_vec_body<4>(p, src, dst, (uint32_t)base, (uint32_t)total);
    if (sb && db) return elt_copy_body<DT_BF16, DT_BF16>(p, src, dst, (uint32_t)base, (uint32_t)total);
    if (sb) return elt_copy_body<DT_BF16, DT_F32>(p, src, dst, (uint32_t)base, (uint32_t)total);
    if (db) return elt_copy_body<DT_F32, DT_BF16>(p, src, dst, (uint32_t)base, (uint32_t)total);
    return elt_copy_body<DT_F32, DT_F32>(p, src, dst, (uint32_t)base, (uint32_t)total);
  }
#pragma unroll
  for (int it = 0; it < ELT_PER_BLOCK / 256; ++it) {
    const int64_t e = base + it * 256 + threadIdx.x;
    if (e >= total) break;
    const int r = (int)(e / p.cols), c = (int)(e - (int64_t)r * p.cols);
    const int64_t si = (int64_t)r * p.ld_src + c, di = (int64_t)r * p.ld_dst + c;
    if (p.src_dtype == DT_I32) {
      ((int32_t *)dst)[di] = ((const int32_t *)src)[si];
      continue;
    }
    if (p.mode == 1) {
      float g = load_as_f32(dst, p.dst_dtype, di);
      store_from_f32(dst, p.dst_dtype, di, g * act_grad(load_as_f32(src, p.src_dtype, si), p.act));
    } else {
      float v = load_as_f32(src, p.src_dtype, si);
      if (p.addend) v += load_as_f32(p.addend, p.add_dtype, (int64_t)r * p.ld_add + c);
      store_from_f32(dst, p.dst_dtype, di, v);
    }
  }
}

void launch_elt(const EltProb *probs, int n, int total_blocks, const ExtPtrs &ext, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_elt, dim3(total_blocks), dim3(256), 0, s, probs, n, ext);
}

__global__ __launch_bounds__(256) void k_fill_zero(uint32_t *p, size_t words) {
  size_t i = (size_t)blockIdx.x * 256 + threadIdx.x;
  const size_t stride = (size_t)gridDim.x * 256;
  for (; i < words; i += stride) p[i] = 0u;
}
void launch_fill_zero(void *ptr, size_t bytes, hipStream_t s) {
  size_t words = bytes / 4;
  if (!words) return;
  int blocks = (int)((words + 256 * 16 - 1) / (256 * 16));
  if (blocks > 8192) blocks = 8192;
  hipLaunchKernelGGL(k_fill_zero, dim3(blocks), dim3(256), 0, s, (uint32_t *)ptr, words);
}

// ------------------------------------------------------------------ column sums
int colsum_blocks(int cols) { return (cols + 63) / 64; }

__global__ __launch_bounds__(256) void k_colsum(const ColsumProb *__restrict__ probs, int n, int accumulate) {
  __shared__ float red[4][64];
  const int pi = find_prob(probs, n, blockIdx.x);
  const ColsumProb p = probs[pi];
  const int c = (blockIdx.x - p.blk_begin) * 64 + (threadIdx.x & 63);
  const int rg = threadIdx.x >> 6;
  float s = 0.0f;
  if (c < p.cols)
    for (int r = rg; r < p.rows; r += 4) s += load_as_f32(p.src, p.dtype, (int64_t)r * p.ld + c);
  red[rg][threadIdx.x & 63] = s;
  __syncthreads();
  if (rg == 0 && c < p.cols) {
    float v = (red[0][threadIdx.x] + red[1][threadIdx.x]) + (red[2][threadIdx.x] + red[3][threadIdx.x]);
    p.out[c] = accumulate ? p.out[c] + v : v;
  }
}
void launch_colsum(const ColsumProb *probs, int n, int total_blocks, int accumulate, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_colsum, dim3(total_blocks), dim3(256), 0, s, probs, n, accumulate);
}

// ------------------------------------------------------------------ LayerNorm
constexpr int LNF_RPW = 4;     // rows per wave of the forward kernels
int ln_rows_per_block() { return 4 * LNF_RPW; }
constexpr int LNP_COLS = 16, LNP_GROUPS = 16;      // columns and row groups of a parameter-gradient workgroup
int ln_param_blocks(int d) { return (d + LNP_COLS - 1) / LNP_COLS; }

__global__ __launch_bounds__(256) void k_ln_fwd(const LnProb *__restrict__ probs, int n) {
  const int pi = find_prob(probs, n, blockIdx.x);
  const LnProb p = probs[pi];
  const int lane = threadIdx.x & 63;
  for (int rr = 0; rr < LNF_RPW; ++rr) {
    const int row = ((blockIdx.x - p.blk_begin) * 4 + (threadIdx.x >> 6)) * LNF_RPW + rr;
    if (row >= p.rows) return;
    const int64_t xo = (int64_t)row * p.ldx;
    float s = 0.0f;
    for (int c = lane; c < p.d; c += 64) s += load_as_f32(p.x, p.x_dtype, xo + c);
    const float mu = wave_sum(s) / (float)p.d;
    float q = 0.0f;
    for (int c = lane; c < p.d; c += 64) {
      float v = load_as_f32(p.x, p.x_dtype, xo + c) - mu;
      q += v * v;
    }
    const float rstd = rsqrtf(wave_sum(q) / (float)p.d + p.eps);
    for (int c = lane; c < p.d; c += 64) {
      float v = (load_as_f32(p.x, p.x_dtype, xo + c) - mu) * rstd;
      store_from_f32(p.y, p.y_dtype, (int64_t)row * p.ldy + c, v * p.gamma[c] + p.beta[c]);
    }
    if (lane == 0) {
      p.mean[row] = mu;
      p.rstd[row] = rstd;
    }
  }
}
// Vector path: bf16 rows of up to 2048 columns in whole 16-byte chunks.  A wave takes LNF_RPW consecutive rows;
// a row stays in registers (NCH chunks of 8 columns per lane) for the mean, the centred second moment and the
// output, so it is read once, and the next two rows are already on their way (a ring of register sets indexed by
// constants: the row loop is unrolled).  With one row per wave all waves of a launch loaded, then all stored:
// the two halves of the traffic never overlapped.  Loads carry no branch (a lane without a chunk reads chunk 0
// and drops it, a row beyond the end re-reads the last row).
typedef __attribute__((ext_vector_type(4))) uint32_t lnf_u32x4;
template <int NCH>
__global__ __launch_bounds__(256) void k_ln_fwd_vec(const LnProb *__restrict__ probs, int n) {
  const int pi = find_prob(probs, n, blockIdx.x);
  const LnProb p = probs[pi];
  const int lane = threadIdx.x & 63;
  const int row0 = ((blockIdx.x - p.blk_begin) * 4 + (threadIdx.x >> 6)) * LNF_RPW;
  if (row0 >= p.rows) return;
  const int nchunks = p.d >> 3;
  constexpr int AHEAD = NCH <= 2 ? 2 : 1;
  lnf_u32x4 ring[AHEAD + 1][NCH];
  auto fetch = [&](lnf_u32x4 (&raw)[NCH], int row) {
    const uint16_t *xr = (const uint16_t *)p.x + (int64_t)min(row, p.rows - 1) * p.ldx;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int ch = lane + 64 * j;
      raw[j] = *(const lnf_u32x4 *)(xr + (ch < nchunks ? ch : 0) * 8);
    }
  };
#pragma unroll
  for (int u = 0; u < AHEAD; ++u) fetch(ring[u], row0 + u);
  // gamma and beta once per wave
  float4 gb[NCH][4];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int cc = (lane + 64 * j < nchunks ? lane + 64 * j : 0) * 8;
    gb[j][0] = *(const float4 *)(p.gamma + cc);
    gb[j][1] = *(const float4 *)(p.gamma + cc + 4);
    gb[j][2] = *(const float4 *)(p.beta + cc);
    gb[j][3] = *(const float4 *)(p.beta + cc + 4);
  }
  // everything asked for so far has landed before the loop starts (s_waitcnt vmcnt(0)): the compiler counts
  // loads in issue order, and gamma / beta would otherwise stay "early loads" whose wait takes in the rows in flight
  __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
  for (int rr = 0; rr < LNF_RPW; ++rr) {
    const int row = row0 + rr;
    if (row >= p.rows) break;
    if (rr + AHEAD < LNF_RPW) fetch(ring[(rr + AHEAD) % (AHEAD + 1)], row + AHEAD);
    const lnf_u32x4 (&raw)[NCH] = ring[rr % (AHEAD + 1)];
    float v[NCH][8];
    float s = 0.0f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const bool ok = lane + 64 * j < nchunks;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        v[j][2 * e] = ok ? __uint_as_float(raw[j][e] << 16) : 0.0f;
        v[j][2 * e + 1] = ok ? __uint_as_float(raw[j][e] & 0xffff0000u) : 0.0f;
        s += v[j][2 * e] + v[j][2 * e + 1];
      }
    }
    const float mu = wave_sum(s) / (float)p.d;
    float q = 0.0f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const bool ok = lane + 64 * j < nchunks;
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        const float c = ok ? v[j][e] - mu : 0.0f;
        v[j][e] = c;
        q += c * c;
      }
    }
    const float rstd = rsqrtf(wave_sum(q) / (float)p.d + p.eps);
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int ch = lane + 64 * j;
      if (ch >= nchunks) continue;
      const float4 g0 = gb[j][0], g1 = gb[j][1], b0 = gb[j][2], b1 = gb[j][3];
      const float ga[8] = {g0.x, g0.y, g0.z, g0.w, g1.x, g1.y, g1.z, g1.w};
      const float be[8] = {b0.x, b0.y, b0.z, b0.w, b1.x, b1.y, b1.z, b1.w};
      lnf_u32x4 o;
#pragma unroll
      for (int e = 0; e < 4; ++e)
        o[e] = (uint32_t)f32_to_bf16_bits(v[j][2 * e] * rstd * ga[2 * e] + be[2 * e]) |
               ((uint32_t)f32_to_bf16_bits(v[j][2 * e + 1] * rstd * ga[2 * e + 1] + be[2 * e + 1]) << 16);
      *(lnf_u32x4 *)((uint16_t *)p.y + (int64_t)row * p.ldy + ch * 8) = o;
    }
    if (lane == 0) {
      p.mean[row] = mu;
      p.rstd[row] = rstd;
    }
  }
}
bool ln_fwd_vec_supported(const LnProb &p) {
  if (p.x_dtype != DT_BF16 || p.y_dtype != DT_BF16 || (p.d & 7) || p.d > 2048) return false;
  if ((p.ldx | p.ldy) & 7) return false;
  if (((uintptr_t)p.x | (uintptr_t)p.y) & 15) return false;
  if (((uintptr_t)p.gamma | (uintptr_t)p.beta) & 15) return false;
  return true;
}
// vec: 0 = generic kernel, otherwise the number of 8-column chunks per lane (1, 2 or 4)
void launch_ln_fwd(const LnProb *probs, int n, int total_blocks, int vec, hipStream_t s) {
  if (total_blocks <= 0) return;
  if (vec == 1) hipLaunchKernelGGL(k_ln_fwd_vec<1>, dim3(total_blocks), dim3(256), 0, s, probs, n);
  else if (vec == 2) hipLaunchKernelGGL(k_ln_fwd_vec<2>, dim3(total_blocks), dim3(256), 0, s, probs, n);
  else if (vec == 4) hipLaunchKernelGGL(k_ln_fwd_vec<4>, dim3(total_blocks), dim3(256), 0, s, probs, n);
  else hipLaunchKernelGGL(k_ln_fwd, dim3(total_blocks), dim3(256), 0, s, probs, n);
}

// LayerNorm backward.  One workgroup owns 4 LN_RPW consecutive rows (LN_RPW per wave):
//   dx = rstd * (g - mean(g) - xhat * mean(g * xhat)) (+ addend), g = dy * gamma
// and, while the rows are in flight, each lane adds dy*xhat and dy of its own columns into
// per-wave LDS sums; the four waves are combined in a fixed order into partial[row_block][2][d].
// k_ln_bwd_params then folds the row blocks, again in a fixed order, into dgamma / dbeta.
constexpr int LN_RPW = 8;     // rows per wave (two: 22.6 us instead of 24.8, but four times the partial sums to fold)
int ln_bwd_rows_per_block() { return 4 * LN_RPW; }
int ln_bwd_max_d() { return 2048; }

__global__ __launch_bounds__(256) void k_ln_bwd(const LnProb *__restrict__ probs, int n) {
  extern __shared__ float part[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const LnProb p = probs[pi];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int blk = blockIdx.x - p.blk_begin;
  float *pg = part + (size_t)wave * 2 * p.d, *pb = pg + p.d;
  if (p.partial)
    for (int c = lane; c < p.d; c += 64) pg[c] = pb[c] = 0.0f;
  for (int rr = 0; rr < LN_RPW; ++rr) {
    const int row = blk * 4 * LN_RPW + wave * LN_RPW + rr;
    if (row >= p.rows) break;
    const float mu = p.mean[row], rstd = p.rstd[row];
    const int64_t xo = (int64_t)row * p.ldx, go = (int64_t)row * p.lddy;
    float s1 = 0.0f, s2 = 0.0f;
    for (int c = lane; c < p.d; c += 64) {
      float xh = (load_as_f32(p.x, p.x_dtype, xo + c) - mu) * rstd;
      float dy = load_as_f32(p.dy, p.dy_dtype, go + c);
      float g = dy * p.gamma[c];
      s1 += g;
      s2 += g * xh;
      if (p.partial) {
        pg[c] += dy * xh;
        pb[c] += dy;
      }
    }
    if (!p.y) continue;
    const float m1 = wave_sum(s1) / (float)p.d, m2 = wave_sum(s2) / (float)p.d;
    for (int c = lane; c < p.d; c += 64) {
      float xh = (load_as_f32(p.x, p.x_dtype, xo + c) - mu) * rstd;
      float g = load_as_f32(p.dy, p.dy_dtype, go + c) * p.gamma[c];
      float v = rstd * (g - m1 - xh * m2);
      if (p.addend) v += load_as_f32(p.addend, p.add_dtype, (int64_t)row * p.ldadd + c);
      store_from_f32(p.y, p.y_dtype, (int64_t)row * p.ldy + c, v);
    }
  }
  if (!p.partial) return;
  __syncthreads();
  for (int c = threadIdx.x; c < 2 * p.d; c += 256) {
    const float v = (part[c] + part[2 * p.d + c]) + (part[4 * p.d + c] + part[6 * p.d + c]);
    p.partial[(int64_t)blk * 2 * p.d + c] = v;
  }
}
// Vector variant for bf16 rows whose width is a multiple of 8: a lane owns NCH chunks of 8 columns,
// keeps the row in registers between the two passes, and carries the parameter partial sums of its
// columns in registers across the wave's rows.
typedef __attribute__((ext_vector_type(4))) uint32_t ln_u32x4;
__device__ __forceinline__ void unpack8(const ln_u32x4 &v, float (&f)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    f[2 * e] = __uint_as_float(v[e] << 16);
    f[2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
  }
}
__device__ __forceinline__ ln_u32x4 pack8f(const float (&f)[8]) {
  ln_u32x4 v;
#pragma unroll
  for (int e = 0; e < 4; ++e) v[e] = (uint32_t)f32_to_bf16_bits(f[2 * e]) | ((uint32_t)f32_to_bf16_bits(f[2 * e + 1]) << 16);
  return v;
}
template <int NCH>
__global__ __launch_bounds__(256) void k_ln_bwd_vec(const LnProb *__restrict__ probs, int n) {
  extern __shared__ float part[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const LnProb p = probs[pi];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int blk = blockIdx.x - p.blk_begin;
  const int nchunks = p.d >> 3;
  float gam[NCH][8], pg[NCH][8], pb[NCH][8];
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int ch = lane + 64 * j;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      gam[j][e] = ch < nchunks ? p.gamma[ch * 8 + e] : 0.0f;
      pg[j][e] = pb[j][e] = 0.0f;
    }
  }
  // The rows of a wave are pipelined: while row r is reduced (two wave-wide sums, each a chain of
  // shuffles) the 16-byte pieces of row r + 1 -- x, dy and the optional addend -- are already on their
  // way.  Loads carry no branch: a lane without a chunk reads chunk 0, a row beyond the end re-reads the
  // last row, an absent addend reads dy; the values are dropped.
  struct RowRaw {
    ln_u32x4 x[NCH], g[NCH], a[NCH];
    float mu, rstd;
  };
  const uint16_t *addp = p.addend ? (const uint16_t *)p.addend : (const uint16_t *)p.dy;
  const int64_t ldadd = p.addend ? p.ldadd : p.lddy;
  const int row_first = blk * 4 * LN_RPW + wave * LN_RPW;
  auto fetch_row = [&](RowRaw &r, int row) {
    const int rc = min(row, p.rows - 1);
    r.mu = p.mean[rc];
    r.rstd = p.rstd[rc];
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int ch = lane + 64 * j, cc = (ch < nchunks ? ch : 0) * 8;
      r.x[j] = *(const ln_u32x4 *)((const uint16_t *)p.x + (int64_t)rc * p.ldx + cc);
      r.g[j] = *(const ln_u32x4 *)((const uint16_t *)p.dy + (int64_t)rc * p.lddy + cc);
      r.a[j] = *(const ln_u32x4 *)(addp + (int64_t)rc * ldadd + cc);
    }
  };
  // AHEAD rows ahead: 12 KB per wave on their way while a row is reduced (one row ahead: 24.8 us, two: 19.0).  A ring of register sets indexed by
  // constants (the row loop is unrolled): copying a set whose loads are still in flight would wait for them
  constexpr int AHEAD = NCH <= 2 ? 2 : 1;      // (three ahead measured the same; rows of more than 1024 columns hold 48 registers per row in flight)
  RowRaw ring[AHEAD + 1];
#pragma unroll
  for (int u = 0; u < AHEAD; ++u) fetch_row(ring[u], row_first + u);
  // every load so far has landed before the loop starts (s_waitcnt vmcnt(0)): the compiler counts loads in issue
  // order, and gamma, loaded once up here, would otherwise stay "an early load" whose wait takes in the rows in flight
  __builtin_amdgcn_s_waitcnt(0x0F70);
#pragma unroll
  for (int rr = 0; rr < LN_RPW; ++rr) {
    const int row = row_first + rr;
    if (row >= p.rows) break;
    if (rr + AHEAD < LN_RPW) fetch_row(ring[(rr + AHEAD) % (AHEAD + 1)], row + AHEAD);
    const RowRaw &cur = ring[rr % (AHEAD + 1)];
    const float mu = cur.mu, rstd = cur.rstd;
    float xh[NCH][8], g[NCH][8];
    float s1 = 0.0f, s2 = 0.0f;
#pragma unroll
    for (int j = 0; j < NCH; ++j) {
      const int ch = lane + 64 * j;
      float xf[8], dyf[8];
      unpack8(cur.x[j], xf);
      unpack8(cur.g[j], dyf);
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (ch >= nchunks) dyf[e] = 0.0f;
        xh[j][e] = ch < nchunks ? (xf[e] - mu) * rstd : 0.0f;
        pg[j][e] += dyf[e] * xh[j][e];
        pb[j][e] += dyf[e];
        g[j][e] = dyf[e] * gam[j][e];
        s1 += g[j][e];
        s2 += g[j][e] * xh[j][e];
      }
    }
    if (p.y) {
      const float m1 = wave_sum(s1) / (float)p.d, m2 = wave_sum(s2) / (float)p.d;
#pragma unroll
      for (int j = 0; j < NCH; ++j) {
        const int ch = lane + 64 * j;
        if (ch >= nchunks) continue;
        float v[8];
#pragma unroll
        for (int e = 0; e < 8; ++e) v[e] = rstd * (g[j][e] - m1 - xh[j][e] * m2);
        if (p.addend) {
          float af[8];
          unpack8(cur.a[j], af);
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += af[e];
        }
        *(ln_u32x4 *)((uint16_t *)p.y + (int64_t)row * p.ldy + ch * 8) = pack8f(v);
      }
    }
  }
  if (!p.partial) return;
  float *mine = part + (size_t)wave * 2 * p.d;
#pragma unroll
  for (int j = 0; j < NCH; ++j) {
    const int ch = lane + 64 * j;
    if (ch >= nchunks) continue;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      mine[ch * 8 + e] = pg[j][e];
      mine[p.d + ch * 8 + e] = pb[j][e];
    }
  }
  __syncthreads();
  for (int c = threadIdx.x; c < 2 * p.d; c += 256) {
    const float v = (part[c] + part[2 * p.d + c]) + (part[4 * p.d + c] + part[6 * p.d + c]);
    p.partial[(int64_t)blk * 2 * p.d + c] = v;
  }
}

bool ln_bwd_vec_supported(const LnProb &p) {
  if (p.x_dtype != DT_BF16 || p.dy_dtype != DT_BF16 || (p.d & 7) || p.d > 2048) return false;
  if ((p.ldx | p.lddy) & 7) return false;
  if (((uintptr_t)p.x | (uintptr_t)p.dy) & 15) return false;
  if (p.y && (p.y_dtype != DT_BF16 || (p.ldy & 7) || ((uintptr_t)p.y & 15))) return false;
  if (p.addend && (p.add_dtype != DT_BF16 || (p.ldadd & 7) || ((uintptr_t)p.addend & 15))) return false;
  return true;
}

// vec: 0 = generic kernel, otherwise the number of 8-column chunks per lane (1, 2 or 4)
void launch_ln_bwd(const LnProb *probs, int n, int total_blocks, int max_d, int vec, hipStream_t s) {
  if (total_blocks <= 0) return;
  const size_t sh = (size_t)8 * max_d * sizeof(float);
  if (vec == 1) hipLaunchKernelGGL(k_ln_bwd_vec<1>, dim3(total_blocks), dim3(256), sh, s, probs, n);
  else if (vec == 2) hipLaunchKernelGGL(k_ln_bwd_vec<2>, dim3(total_blocks), dim3(256), sh, s, probs, n);
  else if (vec == 4) hipLaunchKernelGGL(k_ln_bwd_vec<4>, dim3(total_blocks), dim3(256), sh, s, probs, n);
  else hipLaunchKernelGGL(k_ln_bwd, dim3(total_blocks), dim3(256), sh, s, probs, n);
}

// dgamma[c] (+)= sum over rows of dy*xhat ; dbeta[c] (+)= sum of dy.  16 columns per workgroup, sixteen
// groups of row blocks (or of rows, when no partial sums exist) reduced through LDS in a fixed order.
__global__ __launch_bounds__(256) void k_ln_bwd_params(const LnProb *__restrict__ probs, int n, int accumulate) {
  __shared__ float red[2][LNP_GROUPS][LNP_COLS];
  const int pi = find_prob(probs, n, blockIdx.x);
  const LnProb p = probs[pi];
  const int cl = threadIdx.x % LNP_COLS, rg = threadIdx.x / LNP_COLS;
  const int c = (blockIdx.x - p.blk_begin) * LNP_COLS + cl;
  float sg = 0.0f, sb = 0.0f;
  if (c < p.d) {
    if (p.partial) {
      // four row blocks per round, all eight loads out before the first add (a loop of load-then-add
      // is one memory round trip per row block: 10 us for 64 row blocks)
      for (int rb = rg; rb < p.row_blocks; rb += 4 * LNP_GROUPS) {
        float g[4], b[4];
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const int r = min(rb + u * LNP_GROUPS, p.row_blocks - 1);
          g[u] = p.partial[(int64_t)r * 2 * p.d + c];
          b[u] = p.partial[(int64_t)r * 2 * p.d + p.d + c];
        }
#pragma unroll
        for (int u = 0; u < 4; ++u) {
          const bool ok = rb + u * LNP_GROUPS < p.row_blocks;
          sg += ok ? g[u] : 0.0f;
          sb += ok ? b[u] : 0.0f;
        }
      }
    } else {
      for (int r = rg; r < p.rows; r += LNP_GROUPS) {
        float dy = load_as_f32(p.dy, p.dy_dtype, (int64_t)r * p.lddy + c);
        float xh = (load_as_f32(p.x, p.x_dtype, (int64_t)r * p.ldx + c) - p.mean[r]) * p.rstd[r];
        sg += dy * xh;
        sb += dy;
      }
    }
  }
  red[0][rg][cl] = sg;
  red[1][rg][cl] = sb;
  __syncthreads();
  if (rg == 0 && c < p.d) {      // the groups in a fixed order
    float g = 0.0f, b = 0.0f;
#pragma unroll
    for (int q = 0; q < LNP_GROUPS; ++q) {
      g += red[0][q][cl];
      b += red[1][q][cl];
    }
    p.dgamma[c] = accumulate ? p.dgamma[c] + g : g;
    p.dbeta[c] = accumulate ? p.dbeta[c] + b : b;
  }
}
void launch_ln_bwd_params(const LnProb *probs, int n, int total_blocks, int accumulate, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_ln_bwd_params, dim3(total_blocks), dim3(256), 0, s, probs, n, accumulate);
}

// eight consecutive elements starting at element index i (a multiple of 8 from a 16-byte aligned base)
__device__ __forceinline__ void load8_as_f32(const void *base, int32_t dtype, int64_t i, float (&v)[8]) {
  if (dtype == DT_BF16) {
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
__device__ __forceinline__ void store8_from_f32(void *base, int32_t dtype, int64_t i, const float (&v)[8]) {
  if (dtype == DT_BF16) {
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

// ------------------------------------------------------------------ mean-pool
// forward: a workgroup per (sample, 64 columns): 8 lanes x 8 columns cover the 64 columns of a
// row, the 32 lane groups stride over the sequence with eight rows in flight, and are combined in a
// fixed order (128 columns, 16 groups and four rows in flight left the 16 x 8 workgroups of the transformer
// stage with eight dependent round trips each: 12.7 us for 16 MB).  backward: a thread per 8 columns of an
// output row.  Both have a vector body (bf16 or
// f32 rows of whole, aligned 16-byte chunks; the storage types are template parameters, so that no
// type test stands in front of a load) and a scalar body for everything else.
constexpr int POOL_COLS = 64, POOL_LANES = POOL_COLS / 8, POOL_GROUPS = 256 / POOL_LANES, POOL_FLIGHT = 8;
int pool_blocks(const PoolProb &p) {
  if (!p.backward) return p.batch * ((p.d + POOL_COLS - 1) / POOL_COLS);
  int64_t chunks = (int64_t)p.batch * p.seq * ((p.d + 7) / 8);
  return (int)((chunks + 255) / 256);
}
__device__ __forceinline__ bool pool_vec_ok(const PoolProb &p) {
  return (p.d & 7) == 0 && (p.ld_src & 7) == 0 && (p.ld_dst & 7) == 0 && (((uintptr_t)p.src | (uintptr_t)p.dst) & 15) == 0;
}
template <int SDT, int DDT>
__device__ __forceinline__ void pool_body(const PoolProb &p, int blk, float (*red)[POOL_COLS]) {
  if (!p.backward) {
    const int chunks = (p.d + POOL_COLS - 1) / POOL_COLS;
    const int b = blk / chunks, c0 = (blk % chunks) * POOL_COLS;
    const int l16 = threadIdx.x % POOL_LANES, grp = threadIdx.x / POOL_LANES;
    const int c = c0 + 8 * l16;
    const bool col_ok = c < p.d;
    float acc[8] = {};
    const int64_t base = (int64_t)b * p.seq * p.ld_src + (col_ok ? c : 0);
    for (int t = grp; t < p.seq; t += POOL_GROUPS * POOL_FLIGHT) {      // rows t, t + POOL_GROUPS, ... in flight
      float v[POOL_FLIGHT][8];
#pragma unroll
      for (int u = 0; u < POOL_FLIGHT; ++u)
        load8_as_f32(p.src, SDT, base + (int64_t)min(t + POOL_GROUPS * u, p.seq - 1) * p.ld_src, v[u]);
#pragma unroll
      for (int u = 0; u < POOL_FLIGHT; ++u)
        if (t + POOL_GROUPS * u < p.seq) {
#pragma unroll
          for (int e = 0; e < 8; ++e) acc[e] += v[u][e];
        }
    }
#pragma unroll
    for (int e = 0; e < 8; ++e) red[grp][8 * l16 + e] = acc[e];
    __syncthreads();
    if (threadIdx.x < POOL_COLS && c0 + (int)threadIdx.x < p.d) {
      float s = 0.0f;
#pragma unroll
      for (int g = 0; g < POOL_GROUPS; ++g) s += red[g][threadIdx.x];
      store_from_f32(p.dst, DDT, (int64_t)b * p.ld_dst + c0 + threadIdx.x, s / (float)p.seq);
    }
  } else {
    const int cpr = p.d >> 3;
    const int64_t ch = (int64_t)blk * 256 + threadIdx.x;
    if (ch >= (int64_t)p.batch * p.seq * cpr) return;
    const int r = (int)(ch / cpr), c = (int)(ch % cpr) * 8;
    float v[8];
    load8_as_f32(p.src, SDT, (int64_t)(r / p.seq) * p.ld_src + c, v);
    const float inv = 1.0f / (float)p.seq;
#pragma unroll
    for (int e = 0; e < 8; ++e) v[e] *= inv;
    store8_from_f32(p.dst, DDT, (int64_t)r * p.ld_dst + c, v);
  }
}
__device__ __forceinline__ void pool_body_scalar(const PoolProb &p, int blk, float (*red)[POOL_COLS]) {
  if (!p.backward) {
    const int chunks = (p.d + POOL_COLS - 1) / POOL_COLS;
    const int b = blk / chunks, c0 = (blk % chunks) * POOL_COLS;
    constexpr int RG = 256 / POOL_COLS;                                            // row groups
    const int cl = threadIdx.x & (POOL_COLS - 1), rg = threadIdx.x / POOL_COLS;
    const int c = c0 + cl;
    float s = 0.0f;
    if (c < p.d)
      for (int t = rg; t < p.seq; t += RG) s += load_as_f32(p.src, p.src_dtype, ((int64_t)b * p.seq + t) * p.ld_src + c);
    red[rg][cl] = s;
    __syncthreads();
    if (rg == 0 && c < p.d) {
      float total = 0.0f;
#pragma unroll
      for (int g = 0; g < RG; ++g) total += red[g][cl];
      store_from_f32(p.dst, p.dst_dtype, (int64_t)b * p.ld_dst + c, total / (float)p.seq);
    }
  } else {
    const int cpr = (p.d + 7) >> 3;
    const int64_t ch = (int64_t)blk * 256 + threadIdx.x;
    if (ch >= (int64_t)p.batch * p.seq * cpr) return;
    const int r = (int)(ch / cpr), c0 = (int)(ch % cpr) * 8;
    for (int c = c0; c < min(c0 + 8, p.d); ++c)
      store_from_f32(p.dst, p.dst_dtype, (int64_t)r * p.ld_dst + c,
                     load_as_f32(p.src, p.src_dtype, (int64_t)(r / p.seq) * p.ld_src + c) / (float)p.seq);
  }
}
__global__ __launch_bounds__(256) void k_pool(const PoolProb *__restrict__ probs, int n) {
  __shared__ float red[POOL_GROUPS][POOL_COLS];
  const int pi = find_prob(probs, n, blockIdx.x);
  const PoolProb p = probs[pi];
  const int blk = blockIdx.x - p.blk_begin;
  const bool vec = pool_vec_ok(p);
  if (vec && p.src_dtype == DT_BF16 && p.dst_dtype == DT_BF16) pool_body<DT_BF16, DT_BF16>(p, blk, red);
  else if (vec && p.src_dtype == DT_F32 && p.dst_dtype == DT_F32) pool_body<DT_F32, DT_F32>(p, blk, red);
  else pool_body_scalar(p, blk, red);
}
void launch_pool(const PoolProb *probs, int n, int total_blocks, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_pool, dim3(total_blocks), dim3(256), 0, s, probs, n);
}

// ------------------------------------------------------------------ loss heads
// kinds follow gpp_op_kind_t: 9 MSE, 10 softmax cross-entropy, 11 BCE with logits
__device__ __forceinline__ float softplus_f(float y) { return fmaxf(y, 0.0f) + log1pf(__expf(-fabsf(y))); }
__device__ __forceinline__ float sigmoid_f(float y) {
  float e = __expf(-fabsf(y));
  return y >= 0.0f ? 1.0f / (1.0f + e) : e / (1.0f + e);
}

// MSE / BCE rows can be read eight columns at a time: whole chunks, aligned rows
__device__ __forceinline__ bool loss_row_vec_ok(const LossProb &p) {
  return (p.cols & 7) == 0 && (p.ld_y & 7) == 0 && (p.ld_t & 7) == 0 && (((uintptr_t)p.y | (uintptr_t)p.target) & 15) == 0;
}

// One row of logits in a wave's registers for the softmax cross-entropy: lane l keeps columns l, l + 64, ... (NU of
// them; -inf beyond the row).  The loads are unconditional (a column beyond the row reads the last one) and all go
// out before the first value is used: a loop that loads an element, uses it and loads the next makes every pass over
// the row a chain of trips to memory, and the loss needs two passes, its gradient three.
template <int NU>
__device__ __forceinline__ void ce_row_load(const void *y, int32_t y_dtype, int64_t yo, int cols, int lane, float (&v)[NU]) {
#pragma unroll
  for (int u = 0; u < NU; ++u) v[u] = load_as_f32(y, y_dtype, yo + min(lane + 64 * u, cols - 1));
#pragma unroll
  for (int u = 0; u < NU; ++u)
    if (lane + 64 * u >= cols) v[u] = -INFINITY;
}
// row maximum and sum of exp(v - max), the same in every lane; v becomes exp(v - max)
template <int NU>
__device__ __forceinline__ void ce_row_softmax(float (&v)[NU], float &m, float &se) {
  m = -INFINITY;
#pragma unroll
  for (int u = 0; u < NU; ++u) m = fmaxf(m, v[u]);
  m = wave_max(m);
  se = 0.0f;
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    v[u] = __expf(v[u] - m);
    se += v[u];
  }
  se = wave_sum(se);
}
constexpr int CE_NU = 16;      // rows of up to 1024 classes take the register path
int loss_ce_row_limit() { return 64 * CE_NU; }
// gradient of the row's loss term with respect to its logits, scale * (softmax - one-hot), from the exponentials
// that ce_row_softmax left in v (what the backward kernel computes; written in the forward pass where the stage's
// gradient buffers are per stash slot)
template <int NU>
__device__ __forceinline__ void ce_row_grad(const LossProb &p, int64_t go, int lane, int lab, const float (&v)[NU], float se) {
  const float inv = 1.0f / se;
#pragma unroll
  for (int u = 0; u < NU; ++u) {
    const int c = lane + 64 * u;
    if (c < p.cols) store_from_f32(p.dy, p.dy_dtype, go + c, p.scale * (v[u] * inv - (c == lab ? 1.0f : 0.0f)));
  }
}
// four rows per workgroup (one wave each); every workgroup writes one partial sum, already scaled
int loss_fwd_blocks(const LossProb &p) { return (p.rows + 3) / 4; }
__global__ __launch_bounds__(256) void k_loss_fwd(const LossProb *__restrict__ probs, int n, StageFlags *flags) {
  __shared__ float red[4];
  const int pi = find_prob(probs, n, blockIdx.x);
  const LossProb p = probs[pi];
  const int blk = blockIdx.x - p.blk_begin;
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  const int r = blk * 4 + w;
  float acc = 0.0f;
  if (r < p.rows) {
    const int64_t yo = (int64_t)r * p.ld_y;
    if (p.kind == 10) {
      const int lab = ((const int32_t *)p.target)[(int64_t)r * p.ld_t];
      float m, se;
      if (p.cols <= 64 * CE_NU) {
        float v[CE_NU];
        ce_row_load<CE_NU>(p.y, p.y_dtype, yo, p.cols, lane, v);
        ce_row_softmax<CE_NU>(v, m, se);
        if (p.dy) ce_row_grad<CE_NU>(p, (int64_t)r * p.ld_dy, lane, lab, v, se);
      } else {
        m = -INFINITY;
        for (int c = lane; c < p.cols; c += 64) m = fmaxf(m, load_as_f32(p.y, p.y_dtype, yo + c));
        m = wave_max(m);
        se = 0.0f;
        for (int c = lane; c < p.cols; c += 64) se += __expf(load_as_f32(p.y, p.y_dtype, yo + c) - m);
        se = wave_sum(se);
      }
      if (lane == 0 && lab >= 0 && lab < p.cols) acc = (m + __logf(se)) - load_as_f32(p.y, p.y_dtype, yo + lab);
      if (lane == 0 && (lab < 0 || lab >= p.cols)) flags->index_error = 1;    // a label outside the classes: no loss term, reported
    } else {
      const float *t = (const float *)p.target + (int64_t)r * p.ld_t;
      if (loss_row_vec_ok(p)) {
        // eight consecutive columns per lane and step, 16-byte loads, the steps unrolled so that a
        // row's loads are in flight together
#pragma unroll 4
        for (int c = 8 * lane; c < p.cols; c += 512) {
          float y[8], tv[8];
          load8_as_f32(p.y, p.y_dtype, yo + c, y);
          load8_as_f32(t, DT_F32, c, tv);
#pragma unroll
          for (int e = 0; e < 8; ++e) {
            if (p.kind == 9) {
              const float d = y[e] - tv[e];
              acc += d * d;
            } else {
              acc += softplus_f(y[e]) - tv[e] * y[e];
            }
          }
          // the gradient with the value (stages whose gradient buffers are per stash slot ask for it)
          if (p.dy) {
            float g[8];
#pragma unroll
            for (int e = 0; e < 8; ++e) g[e] = p.kind == 9 ? 2.0f * p.scale * (y[e] - tv[e]) : p.scale * (sigmoid_f(y[e]) - tv[e]);
            const int64_t go = (int64_t)r * p.ld_dy + c;
            if ((p.ld_dy & 7) == 0 && ((uintptr_t)p.dy & 15) == 0) {
              store8_from_f32(p.dy, p.dy_dtype, go, g);
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e) store_from_f32(p.dy, p.dy_dtype, go + e, g[e]);
            }
          }
        }
      } else {
        for (int c = lane; c < p.cols; c += 64) {
          float y = load_as_f32(p.y, p.y_dtype, yo + c);
          if (p.kind == 9) {
            float d = y - t[c];
            acc += d * d;
          } else {
            acc += softplus_f(y) - t[c] * y;
          }
          if (p.dy)
            store_from_f32(p.dy, p.dy_dtype, (int64_t)r * p.ld_dy + c, p.kind == 9 ? 2.0f * p.scale * (y - t[c]) : p.scale * (sigmoid_f(y) - t[c]));
        }
      }
    }
  }
  acc = wave_sum(acc);
  if (lane == 0) red[w] = acc;
  __syncthreads();
  if (threadIdx.x == 0) p.loss[blk] = ((red[0] + red[1]) + (red[2] + red[3])) * p.scale;
}
void launch_loss_fwd(const LossProb *probs, int n, int total_blocks, StageFlags *flags, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_loss_fwd, dim3(total_blocks), dim3(256), 0, s, probs, n, flags);
}

// Small heads (all of a stage's losses together at most a few tens of thousands of elements): one
// workgroup computes every loss and their sum, so the forward pass needs one launch, not two.
// MSE / BCE: a thread per element, strided (and, where the record names a gradient buffer, the
// gradient with it); cross-entropy: a wave per row.  All sums in a fixed order.
int loss_small_limit() { return 16384; }
// element-wise losses of the one-workgroup kernel: eight elements of a thread are requested before the
// first is used and the prediction's storage type is a template parameter (one memory round trip per
// eight elements instead of one per element: 16 x 4096 elements took 110 us element by element)
template <int YDT>
__device__ __forceinline__ float loss_small_elementwise(const LossProb &p) {
  constexpr int U = 8;
  const int total_e = p.rows * p.cols;
  float acc = 0.0f;
  for (int e0 = threadIdx.x; e0 < total_e; e0 += 256 * U) {
    float y[U], t[U];
    int64_t gi[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const int e = min(e0 + 256 * u, total_e - 1);
      const int r = e / p.cols, c = e - r * p.cols;
      const int64_t yi = (int64_t)r * p.ld_y + c;
      y[u] = YDT == DT_BF16 ? bf16_bits_to_f32(((const uint16_t *)p.y)[yi]) : ((const float *)p.y)[yi];
      t[u] = ((const float *)p.target)[(int64_t)r * p.ld_t + c];
      gi[u] = (int64_t)r * p.ld_dy + c;
    }
#pragma unroll
    for (int u = 0; u < U; ++u) {
      if (e0 + 256 * u >= total_e) break;
      if (p.kind == 9) {
        const float d = y[u] - t[u];
        acc += d * d;
      } else {
        acc += softplus_f(y[u]) - t[u] * y[u];
      }
      // the gradient with the value (stages whose gradient buffers are per stash slot ask for it)
      if (p.dy)
        store_from_f32(p.dy, p.dy_dtype, gi[u], p.kind == 9 ? 2.0f * p.scale * (y[u] - t[u]) : p.scale * (sigmoid_f(y[u]) - t[u]));
    }
  }
  return acc;
}
__global__ __launch_bounds__(256) void k_loss_fwd_small(const LossProb *__restrict__ probs, int n, float *out, StageFlags *flags) {
  __shared__ float red[4];
  const int lane = threadIdx.x & 63, w = threadIdx.x >> 6;
  float total = 0.0f;
  for (int pi = 0; pi < n; ++pi) {
    const LossProb p = probs[pi];
    float acc = 0.0f;
    if (p.kind == 10) {
      for (int r = w; r < p.rows; r += 4) {
        const int64_t yo = (int64_t)r * p.ld_y;
        const int lab = ((const int32_t *)p.target)[(int64_t)r * p.ld_t];
        float m, se;
        if (p.cols <= 64 * CE_NU) {
          float v[CE_NU];
          ce_row_load<CE_NU>(p.y, p.y_dtype, yo, p.cols, lane, v);
          ce_row_softmax<CE_NU>(v, m, se);
          if (p.dy) ce_row_grad<CE_NU>(p, (int64_t)r * p.ld_dy, lane, lab, v, se);
        } else {
          m = -INFINITY;
          for (int c = lane; c < p.cols; c += 64) m = fmaxf(m, load_as_f32(p.y, p.y_dtype, yo + c));
          m = wave_max(m);
          se = 0.0f;
          for (int c = lane; c < p.cols; c += 64) se += __expf(load_as_f32(p.y, p.y_dtype, yo + c) - m);
          se = wave_sum(se);
        }
        if (lane == 0 && lab >= 0 && lab < p.cols) acc += (m + __logf(se)) - load_as_f32(p.y, p.y_dtype, yo + lab);
        if (lane == 0 && (lab < 0 || lab >= p.cols)) flags->index_error = 1;
      }
    } else {
      acc = p.y_dtype == DT_BF16 ? loss_small_elementwise<DT_BF16>(p) : loss_small_elementwise<DT_F32>(p);
    }
    acc = wave_sum(acc);
    __syncthreads();               // red is free again
    if (lane == 0) red[w] = acc;
    __syncthreads();
    total += ((red[0] + red[1]) + (red[2] + red[3])) * p.scale;
  }
  if (threadIdx.x == 0) out[0] = total;
}
void launch_loss_fwd_small(const LossProb *probs, int n, float *out, StageFlags *flags, hipStream_t s) {
  if (n <= 0 || !out) return;
  hipLaunchKernelGGL(k_loss_fwd_small, dim3(1), dim3(256), 0, s, probs, n, out, flags);
}

// One-column head (see HeadProb): per row  y = x . w + b,  the loss term and its gradient dy, and the
// gradient of x:  dx = dy w (.) act'(mask).  Workgroups of eight waves.  Workgroup 0 computes every row's
// prediction, loss term and loss gradient (a wave takes four rows at a time) and the loss sum; workgroup
// b >= 1 computes dx for rows 8 (b - 1) .. + 7, a wave per row, and for that RECOMPUTES its rows' dot
// products and gradients with the same arithmetic (same order, same roundings) instead of waiting for
// workgroup 0: a fifth of the work done twice buys a launch without any exchange between workgroups.  (One
// workgroup for everything was measured at 11 us for 64 x 1000: it is bound by the arithmetic of ONE
// compute unit.)  w sits in LDS as floats.  Every value passes through the storage type it has in the
// unfused path (y and dy are rounded before they are used), and all sums have a fixed order.
constexpr int HEAD_MAX_K = 8192, HEAD_MAX_ROWS = 256, HEAD_ROWS_IN_FLIGHT = 4, HEAD_WAVES = 8;
// Up to HEAD_MAX_ROWS rows workgroup 0 forms the loss sum itself; taller or larger heads (up to HEAD_TALL_ROWS) have no
// workgroup 0: every workgroup of eight rows also stores its rows' prediction and loss gradient and ONE partial
// loss, and the stage's loss-sum launch adds the partials in index order.
constexpr int HEAD_TALL_ROWS = 16384;
bool head_loss_supported(int64_t rows, int64_t K) { return rows >= 1 && rows <= HEAD_TALL_ROWS && K >= 8 && K <= HEAD_MAX_K && (K & 7) == 0; }
// (also when workgroup 0 alone would have to form too many dot products: 256 x 4096 took 65 us there)
bool head_loss_is_tall(int64_t rows, int64_t K) { return rows > HEAD_MAX_ROWS || rows * K > 128 * 1024; }
int head_loss_parts(int64_t rows) { return (int)((rows + HEAD_WAVES - 1) / HEAD_WAVES); }
// prediction and loss gradient of one row from its dot product, as the backward pass will read them
__device__ __forceinline__ void head_row(const HeadProb &p, float dot, float bias, float t, float &y, float &g) {
  y = wave_sum(dot) + bias;
  if (p.y_dtype == DT_BF16) y = bf16_bits_to_f32(f32_to_bf16_bits(y));
  g = p.kind == 9 ? 2.0f * p.scale * (y - t) : p.scale * (sigmoid_f(y) - t);
  if (p.dy_dtype == DT_BF16) g = bf16_bits_to_f32(f32_to_bf16_bits(g));
}
__device__ __forceinline__ float head_dot8(const ln_u32x4 &x, const float *w8) {
  float d = 0.0f;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    d += __uint_as_float(x[e] << 16) * w8[2 * e];
    d += __uint_as_float(x[e] & 0xffff0000u) * w8[2 * e + 1];
  }
  return d;
}
__global__ __launch_bounds__(64 * HEAD_WAVES) void k_head_loss(const HeadProb *__restrict__ prob, HeadOuts outs) {
  __shared__ float w_f[HEAD_MAX_K];
  __shared__ float red[HEAD_WAVES];
  const HeadProb p = prob[blockIdx.y];      // one record per micro-batch of a group launch
  float *out = outs.p[blockIdx.y];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int chunks = p.K >> 3;
  for (int c = threadIdx.x; c < chunks; c += 64 * HEAD_WAVES) {
    const ln_u32x4 v = *(const ln_u32x4 *)((const uint16_t *)p.w + 8 * c);
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      w_f[8 * c + 2 * e] = __uint_as_float(v[e] << 16);
      w_f[8 * c + 2 * e + 1] = __uint_as_float(v[e] & 0xffff0000u);
    }
  }
  const float bias = p.bias ? p.bias[0] : 0.0f;
  const bool tall = p.partials != nullptr;
  if (!tall && blockIdx.x == 0) {
    constexpr int R = HEAD_ROWS_IN_FLIGHT;
    float tv[R];
    const int first = wave * R;
#pragma unroll
    for (int q = 0; q < R; ++q) tv[q] = ((const float *)p.target)[(int64_t)min(first + q, p.rows - 1) * p.ld_t];
    __syncthreads();
    float loss_acc = 0.0f;      // lane 0 of each wave: the loss terms of the wave's rows, in row order
    for (int r0 = first; r0 < p.rows; r0 += HEAD_WAVES * R) {
      if (r0 != first) {
#pragma unroll
        for (int q = 0; q < R; ++q) tv[q] = ((const float *)p.target)[(int64_t)min(r0 + q, p.rows - 1) * p.ld_t];
      }
      float dot[R];
#pragma unroll
      for (int q = 0; q < R; ++q) dot[q] = 0.0f;
      for (int c = lane; c < chunks; c += 64) {
        ln_u32x4 xr[R];
#pragma unroll
        for (int q = 0; q < R; ++q) xr[q] = *(const ln_u32x4 *)((const uint16_t *)p.x + (int64_t)min(r0 + q, p.rows - 1) * p.ld_x + 8 * c);
#pragma unroll
        for (int q = 0; q < R; ++q) dot[q] += head_dot8(xr[q], w_f + 8 * c);
      }
#pragma unroll
      for (int q = 0; q < R; ++q) {
        float y, g;
        head_row(p, dot[q], bias, tv[q], y, g);
        const int r = r0 + q;
        if (r < p.rows && lane == 0) {
          if (p.kind == 9) {
            const float d = y - tv[q];
            loss_acc += d * d;
          } else {
            loss_acc += softplus_f(y) - tv[q] * y;
          }
          store_from_f32(p.y, p.y_dtype, (int64_t)r * p.ld_y, y);
          store_from_f32(p.dy, p.dy_dtype, (int64_t)r * p.ld_dy, g);
        }
      }
    }
    if (lane == 0) red[wave] = loss_acc;
    __syncthreads();
    if (threadIdx.x == 0) {
      float total = 0.0f;
      for (int k = 0; k < HEAD_WAVES; ++k) total += red[k];
      out[0] = total * p.scale;
    }
    return;
  }
  // ---- dx of one row per wave
  const int row = ((int)blockIdx.x - (tall ? 0 : 1)) * HEAD_WAVES + wave;
  const int rc = min(row, p.rows - 1);
  const float t = ((const float *)p.target)[(int64_t)rc * p.ld_t];
  const bool masked = p.mask != nullptr, own_mask = masked && p.mask != p.x;
  constexpr int KEEP = 4;       // chunks of the row (and of its mask source) a lane keeps: K <= 2048 needs no second read
  ln_u32x4 xk[KEEP], mk[KEEP];
#pragma unroll
  for (int j = 0; j < KEEP; ++j) {
    const int c = min(lane + 64 * j, chunks - 1);
    xk[j] = *(const ln_u32x4 *)((const uint16_t *)p.x + (int64_t)rc * p.ld_x + 8 * c);
    mk[j] = own_mask ? *(const ln_u32x4 *)((const uint16_t *)p.mask + (int64_t)rc * p.ld_mask + 8 * c) : xk[j];
  }
  __syncthreads();
  float dot = 0.0f;     // the same chunks in the same order as workgroup 0's lane
#pragma unroll
  for (int j = 0; j < KEEP; ++j)
    if (lane + 64 * j < chunks) dot += head_dot8(xk[j], w_f + 8 * (lane + 64 * j));
  for (int c = lane + 64 * KEEP; c < chunks; c += 64)
    dot += head_dot8(*(const ln_u32x4 *)((const uint16_t *)p.x + (int64_t)rc * p.ld_x + 8 * c), w_f + 8 * c);
  float y, g;
  head_row(p, dot, bias, t, y, g);
  if (tall) {      // this workgroup also owns its rows' prediction, loss gradient and loss terms
    float term = 0.0f;
    if (row < p.rows && lane == 0) {
      if (p.kind == 9) {
        const float d = y - t;
        term = d * d;
      } else {
        term = softplus_f(y) - t * y;
      }
      store_from_f32(p.y, p.y_dtype, (int64_t)row * p.ld_y, y);
      store_from_f32(p.dy, p.dy_dtype, (int64_t)row * p.ld_dy, g);
    }
    if (lane == 0) red[wave] = term;
    __syncthreads();
    if (threadIdx.x == 0) {
      float total = 0.0f;
      for (int k = 0; k < HEAD_WAVES; ++k) total += red[k];
      p.partials[blockIdx.x] = total * p.scale;
    }
  }
  if (row >= p.rows || !p.dx) return;
  auto put = [&](int c, const ln_u32x4 &m) {
    ln_u32x4 o;
#pragma unroll
    for (int e = 0; e < 4; ++e) {
      float lo = g * w_f[8 * c + 2 * e], hi = g * w_f[8 * c + 2 * e + 1];
      if (masked) {
        lo *= act_grad(__uint_as_float(m[e] << 16), p.act);
        hi *= act_grad(__uint_as_float(m[e] & 0xffff0000u), p.act);
      }
      o[e] = (uint32_t)f32_to_bf16_bits(lo) | ((uint32_t)f32_to_bf16_bits(hi) << 16);
    }
    *(ln_u32x4 *)((uint16_t *)p.dx + (int64_t)row * p.ld_dx + 8 * c) = o;
  };
#pragma unroll
  for (int j = 0; j < KEEP; ++j)
    if (lane + 64 * j < chunks) put(lane + 64 * j, mk[j]);
  for (int c = lane + 64 * KEEP; c < chunks; c += 64)
    put(c, masked ? *(const ln_u32x4 *)((const uint16_t *)p.mask + (int64_t)row * p.ld_mask + 8 * c) : ln_u32x4{0u, 0u, 0u, 0u});
}
void launch_head_loss(const HeadProb *prob, int members, int rows, int K, const HeadOuts &outs, hipStream_t s) {
  if (members <= 0 || members > HEAD_GROUP_MAX || rows <= 0) return;
  const int blocks = (head_loss_is_tall(rows, K) ? 0 : 1) + head_loss_parts(rows);
  hipLaunchKernelGGL(k_head_loss, dim3(blocks, members), dim3(64 * HEAD_WAVES), 0, s, prob, outs);
}

int loss_bwd_blocks(const LossProb &p) { return (p.rows + 3) / 4; }
// one wave per row; LossProb has no prefix field, so block ranges are passed as rows/4 per record in order
__global__ __launch_bounds__(256) void k_loss_bwd(const LossProb *__restrict__ probs, int n) {
  int blk = blockIdx.x, pi = 0;
  for (; pi < n; ++pi) {
    int nb = (probs[pi].rows + 3) / 4;
    if (blk < nb) break;
    blk -= nb;
  }
  if (pi >= n) return;
  const LossProb p = probs[pi];
  const int lane = threadIdx.x & 63;
  const int r = blk * 4 + (threadIdx.x >> 6);
  if (r >= p.rows) return;
  const int64_t yo = (int64_t)r * p.ld_y, go = (int64_t)r * p.ld_dy;
  if (p.kind == 10 && p.cols <= 64 * CE_NU) {
    const int lab = ((const int32_t *)p.target)[(int64_t)r * p.ld_t];
    float v[CE_NU], m, se;
    ce_row_load<CE_NU>(p.y, p.y_dtype, yo, p.cols, lane, v);
    ce_row_softmax<CE_NU>(v, m, se);
    ce_row_grad<CE_NU>(p, go, lane, lab, v, se);
  } else if (p.kind == 10) {
    float m = -INFINITY;
    for (int c = lane; c < p.cols; c += 64) m = fmaxf(m, load_as_f32(p.y, p.y_dtype, yo + c));
    m = wave_max(m);
    float se = 0.0f;
    for (int c = lane; c < p.cols; c += 64) se += __expf(load_as_f32(p.y, p.y_dtype, yo + c) - m);
    const float inv = 1.0f / wave_sum(se);
    const int lab = ((const int32_t *)p.target)[(int64_t)r * p.ld_t];
    for (int c = lane; c < p.cols; c += 64) {
      float pr = __expf(load_as_f32(p.y, p.y_dtype, yo + c) - m) * inv;
      store_from_f32(p.dy, p.dy_dtype, go + c, p.scale * (pr - (c == lab ? 1.0f : 0.0f)));
    }
  } else {
    const float *t = (const float *)p.target + (int64_t)r * p.ld_t;
    if (loss_row_vec_ok(p) && (p.ld_dy & 7) == 0 && ((uintptr_t)p.dy & 15) == 0) {
#pragma unroll 4
      for (int c = 8 * lane; c < p.cols; c += 512) {
        float y[8], tv[8], g[8];
        load8_as_f32(p.y, p.y_dtype, yo + c, y);
        load8_as_f32(t, DT_F32, c, tv);
#pragma unroll
        for (int e = 0; e < 8; ++e) g[e] = p.kind == 9 ? 2.0f * p.scale * (y[e] - tv[e]) : p.scale * (sigmoid_f(y[e]) - tv[e]);
        store8_from_f32(p.dy, p.dy_dtype, go + c, g);
      }
    } else {
      for (int c = lane; c < p.cols; c += 64) {
        float y = load_as_f32(p.y, p.y_dtype, yo + c);
        float g = p.kind == 9 ? 2.0f * p.scale * (y - t[c]) : p.scale * (sigmoid_f(y) - t[c]);
        store_from_f32(p.dy, p.dy_dtype, go + c, g);
      }
    }
  }
}
void launch_loss_bwd(const LossProb *probs, int n, int total_blocks, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_loss_bwd, dim3(total_blocks), dim3(256), 0, s, probs, n);
}

// one wave: lane-strided sums, then a butterfly; the order is fixed, so the result is reproducible
__global__ void k_loss_sum(const float *losses, int n, float *out) {
  float s = 0.0f;
  for (int i = threadIdx.x; i < n; i += 64) s += losses[i];
  s = wave_sum(s);
  if (threadIdx.x == 0) out[0] = s;
}
void launch_loss_sum(const float *losses, int n, float *out, hipStream_t s) {
  hipLaunchKernelGGL(k_loss_sum, dim3(1), dim3(64), 0, s, losses, n, out);
}

}  // namespace gpp
