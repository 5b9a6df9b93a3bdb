// Device-side body of the backward-weight GEMM for small weight matrices and many rows (see
// gemm_dw_ksplit.hip); a function of (record, tile index, LDS block) so that the stand-alone kernel
// and the merged backward launch of a level can both run it.
#pragma once
#include "gemm_tile_body.h"

namespace gpp {

constexpr int KS_T = 64;          // tile edge and rows per step
constexpr int KS_ST = KS_T + 8;   // LDS row stride (elements): 144 bytes, the four rows a 16-lane block of the
                                  // transposing read touches fall on disjoint banks
constexpr int KS_NW = 8;

// transposing read of a [64 rows m][KS_ST] tile: operand fragment for output rows/columns col0 .. col0 + 31,
// contraction rows k0 .. k0 + 15
__device__ __forceinline__ bf16x8 ks_frag(const uint16_t *lds, int col0, int k0) {
  const int l = threadIdx.x & 63;
  const int blk = l >> 4, q = l & 15;
  const uint16_t *p = lds + (k0 + 8 * (blk >> 1) + (q >> 2)) * KS_ST + col0 + 16 * (blk & 1) + 4 * (q & 3);
  typedef __attribute__((address_space(3))) s16x4 lds_v4;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)p);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p + 4 * KS_ST));
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

struct KsStep {
  u32x4 a[8], b[8];   // 64 rows x 64 columns of each operand: eight lanes per 128-byte row
};

constexpr int KS_WAVE_ELEMS = 2 * KS_T * KS_ST;
constexpr int KS_RED_FLOATS = KS_NW * KS_T * KS_T;   // after the k-loop: every wave's partial tile
constexpr int KS_MAIN_BYTES = KS_RED_FLOATS * 4 > KS_NW * KS_WAVE_ELEMS * 2 ? KS_RED_FLOATS * 4 : KS_NW * KS_WAVE_ELEMS * 2;
constexpr int KS_LDS_BYTES = KS_MAIN_BYTES + KS_NW * KS_T * 4;   // + the waves' bias-gradient partials

// `local`: index of the tile inside the record; `lds_raw`: KS_LDS_BYTES bytes, 16-byte aligned; 512 threads
__device__ __forceinline__ void gemm_dw_ksplit_body(const GemmProb &p, int local, unsigned char *lds_raw, int accumulate_dw) {
  constexpr int WAVE_ELEMS = KS_WAVE_ELEMS;
  float *red = (float *)lds_raw;
  float (*bias_part)[KS_T] = (float (*)[KS_T])(lds_raw + KS_MAIN_BYTES);
  const int tiles_m = cdiv(p.M, KS_T);
  const int m0 = (local % tiles_m) * KS_T, n0 = (local / tiles_m) * KS_T;   // rows (out features) / columns (in features) of dW
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, h = lane >> 5;
  // A = dZ [K x M], B = X [K x N]: the contraction index is the row of both
  const __amdgpu_buffer_rsrc_t rs_a = matrix_rsrc(p.A, p.K, p.lda, p.M);
  const __amdgpu_buffer_rsrc_t rs_b = matrix_rsrc(p.B, p.K, p.ldb, p.N);
  uint16_t *lds_a = (uint16_t *)lds_raw + wave * WAVE_ELEMS;
  uint16_t *lds_b = lds_a + KS_T * KS_ST;

  // old gradient values of this thread's epilogue elements: row tid / 8, eight columns from (tid % 8) * 8
  const int er = threadIdx.x >> 3, ec = (threadIdx.x & 7) * 8;
  float c_old[8];
  {
    const float *c = (const float *)p.C + (int64_t)(m0 + er) * p.ldc + n0 + ec;
#pragma unroll
    for (int e = 0; e < 8; ++e) c_old[e] = (accumulate_dw && m0 + er < p.M && n0 + ec + e < p.N) ? c[e] : 0.0f;
  }

  f32x16 acc[2][2];
#pragma unroll
  for (int i = 0; i < 2; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  const int steps = cdiv(p.K, KS_T), per = cdiv(steps, KS_NW);
  const int s_lo = wave * per, s_hi = min(steps, s_lo + per);
  const int crow = lane >> 3, ccol = (lane & 7) * 8;
  const bool do_bias = p.bias != nullptr && n0 == 0;
  float bsum = 0.0f;

  auto load = [&](KsStep &f, int s) {
    const int k0 = KS_T * s;
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      f.a[q] = chunk_load(rs_a, p.lda, k0 + 8 * q + crow, m0 + ccol, p.K, p.M);
      f.b[q] = chunk_load(rs_b, p.ldb, k0 + 8 * q + crow, n0 + ccol, p.K, p.N);
    }
  };
  auto stage = [&](const KsStep &f) {
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      *(u32x4 *)(lds_a + (8 * q + crow) * KS_ST + ccol) = f.a[q];
      *(u32x4 *)(lds_b + (8 * q + crow) * KS_ST + ccol) = f.b[q];
    }
  };
  auto multiply = [&]() {
#pragma unroll
    for (int c = 0; c < 4; ++c) {   // four 16-row chunks of the step
      bf16x8 a[2], b[2];
#pragma unroll
      for (int i = 0; i < 2; ++i) a[i] = ks_frag(lds_a, 32 * i, 16 * c);
#pragma unroll
      for (int j = 0; j < 2; ++j) b[j] = ks_frag(lds_b, 32 * j, 16 * c);
#pragma unroll
      for (int i = 0; i < 2; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
    if (do_bias) {   // lane = output feature of the tile: its column of the staged dZ tile, rows in order
#pragma unroll 8
      for (int m = 0; m < KS_T; ++m) bsum += bf16_bits_to_f32(lds_a[m * KS_ST + lane]);
    }
  };

  KsStep f[2];
  if (s_lo < s_hi) load(f[0], s_lo);
  if (s_lo + 1 < s_hi) load(f[1], s_lo + 1);
  for (int s = s_lo; s < s_hi; s += 2) {
#pragma unroll
    for (int u = 0; u < 2; ++u) {
      if (s + u >= s_hi) break;
      stage(f[u]);
      if (s + u + 2 < s_hi) load(f[u], s + u + 2);
      multiply();
    }
  }

  // ---- the waves' partial tiles meet in LDS behind one barrier; the epilogue's threads add them, and the bias
  // partials, in wave order (a fixed order; a tree of hand-overs between the waves cost seven barriers)
  bias_part[wave][lane] = bsum;
  __syncthreads();                 // the waves' private operand tiles are dead from here on
  {
    float *buf = red + wave * KS_T * KS_T;
#pragma unroll
    for (int i = 0; i < 2; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) buf[(32 * i + 8 * (q >> 2) + 4 * h + (q & 3)) * KS_T + 32 * j + r] = acc[i][j][q];
  }
  __syncthreads();

  if (do_bias && threadIdx.x < KS_T && m0 + (int)threadIdx.x < p.M) {
    float total = 0.0f;
#pragma unroll
    for (int w = 0; w < KS_NW; ++w) total += bias_part[w][threadIdx.x];
    GPP_G float *db = (GPP_G float *)p.bias + m0 + threadIdx.x;
    *db = accumulate_dw ? *db + total : total;
  }
  if (m0 + er < p.M) {
    float *c = (float *)p.C + (int64_t)(m0 + er) * p.ldc + n0 + ec;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      float v = red[er * KS_T + ec + e];
#pragma unroll
      for (int w = 1; w < KS_NW; ++w) v += red[w * KS_T * KS_T + er * KS_T + ec + e];
      if (n0 + ec + e < p.N) c[e] = c_old[e] + v;
    }
  }
}


}  // namespace gpp
