// Branch-grouped bf16 GEMM for few rows (a micro-batch of at most 256 rows):
// forward  C[m,n] = sum_k X[m,k] W[n,k]  and backward-data  C[m,k] = sum_n dZ[m,n] W[n,k].
//
// With so few rows the work is streaming the weights once, and there are too
// few output tiles to fill the chip.  Parallelism therefore comes from the
// contraction: a workgroup owns all rows and 64 output columns, and its
// waves (eight, or four for more than 64 rows) each take a contiguous slice of K and run WITHOUT workgroup barriers
// (a barrier per k-step couples the waves to the slowest memory access and was
// measured at ~0.6 us per 32-wide step).  Each wave fetches its own 64-wide
// k-steps with fully coalesced 16-byte loads (eight lanes per 128-byte row),
// keeps several steps in flight in registers, stages them in a wave-private LDS tile
// and reads MFMA operands from there; W in the backward-data form is read
// with the transposing LDS read.  The partial accumulators are added in a
// fixed tree order through LDS, then all waves share the epilogue.
#include "device_utils.h"

namespace gpp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int SK_BN = 64;             // output columns per workgroup
constexpr int SK_ST = SK_BN + 8;      // LDS row stride of a k-contiguous 64-wide tile (elements)
constexpr int SK_ST_TR = SK_BN + 32;  // row stride of the contraction-row W tile read with the transposing read

// 32-row tiles per workgroup (1 or 2); 0 when the problem has too many rows for this kernel.
// More than 64 rows are covered by several workgroups per column block, which re-read W from L2.
int gemm_skinny_row_tiles(int M) { return M <= 32 ? 1 : (M <= 256 ? 2 : 0); }
int gemm_skinny_blocks(int M, int N, int row_tiles) {
  return ((N + SK_BN - 1) / SK_BN) * ((M + 32 * row_tiles - 1) / (32 * row_tiles));
}

// 8 consecutive elements of one row; zero outside [0,row_lim) x [0,col_lim), ragged tail cleared
__device__ __forceinline__ u32x4 load8(const uint16_t *__restrict__ base, int64_t ld, int row, int row_lim, int col, int col_lim) {
  u32x4 v = {0u, 0u, 0u, 0u};
  if (row < row_lim && col < col_lim) {
    v = *(const u32x4 *)(base + (int64_t)row * ld + col);
    if (col + 8 > col_lim) {
      const int keep = col_lim - col;
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        if (2 * e >= keep) v[e] = 0u;
        else if (2 * e + 1 >= keep) v[e] &= 0xffffu;
      }
    }
  }
  return v;
}

// one 64-wide k-step of a wave, as fetched from memory: BM x 64 of A and 64 x 64 of B in 16-byte
// chunks, eight lanes per 128-byte row, so every load instruction covers whole cache lines
template <int TI>
struct SkStep {
  u32x4 a[4 * TI];
  u32x4 b[8];
};

// NW waves per workgroup split K: 8 when the private tiles of 8 waves fit in LDS (up to 64 rows), else 4
template <int TI>
struct SkWaves {
  static constexpr int value = TI <= 2 ? 8 : 4;
};

template <int FORM, int TI>
__global__ __launch_bounds__(64 * SkWaves<TI>::value) void k_gemm_skinny(const GemmProb *__restrict__ probs, int n) {
  constexpr int NW = SkWaves<TI>::value;
  constexpr int BM = 32 * TI;
  constexpr int RED_FLOATS = (NW / 2) * BM * SK_BN;
  // row stride of the B tile: the conflict-free stride of the transposing read when the waves' tiles
  // still fit in the 160 KB of LDS, else the compact one
  constexpr int SB = (FORM == FORM_DX && NW * (BM * SK_ST + 64 * SK_ST_TR) * 2 <= 160 * 1024) ? SK_ST_TR : SK_ST;
  constexpr int WAVE_ELEMS = BM * SK_ST + 64 * SB;         // a wave's private A and B tiles
  constexpr int LDS_BYTES = RED_FLOATS * 4 > NW * WAVE_ELEMS * 2 ? RED_FLOATS * 4 : NW * WAVE_ELEMS * 2;
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[LDS_BYTES];
  float *red = (float *)lds_raw;           // after the k-loop: two BM x 64 fp32 buffers

  const int pi = find_prob(probs, n, blockIdx.x);
  const GemmProb p = probs[pi];
  const int m_blocks = (p.M + BM - 1) / BM;                      // row blocks of one column block are neighbours
  const int n0 = ((blockIdx.x - p.blk_begin) / m_blocks) * SK_BN;
  const int m0 = ((blockIdx.x - p.blk_begin) % m_blocks) * BM;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, h = lane >> 5;
  const uint16_t *A = (const uint16_t *)p.A;
  const uint16_t *B = (const uint16_t *)p.B;
  uint16_t *lds_a = (uint16_t *)lds_raw + wave * WAVE_ELEMS;   // [BM][SK_ST]
  uint16_t *lds_b = lds_a + BM * SK_ST;                        // [64][SK_ST]

  f32x16 acc[TI][2];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < 2; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  const int steps = (p.K + 63) / 64, per = (steps + NW - 1) / NW;
  const int s_lo = wave * per, s_hi = min(steps, s_lo + per);
  const int crow = lane >> 3, ccol = (lane & 7) * 8;     // this lane's chunk inside an 8-row slab

  auto load = [&](SkStep<TI> &f, int s) {
    const int k0 = 64 * s;
#pragma unroll
    for (int q = 0; q < 4 * TI; ++q) f.a[q] = load8(A, p.lda, m0 + 8 * q + crow, p.M, k0 + ccol, p.K);
#pragma unroll
    for (int q = 0; q < 8; ++q) {
      if (FORM == FORM_FWD) f.b[q] = load8(B, p.ldb, n0 + 8 * q + crow, p.N, k0 + ccol, p.K);   // W[n][k]
      else f.b[q] = load8(B, p.ldb, k0 + 8 * q + crow, p.K, n0 + ccol, p.N);                    // W[k][n]
    }
  };
  auto stage = [&](const SkStep<TI> &f) {
#pragma unroll
    for (int q = 0; q < 4 * TI; ++q) *(u32x4 *)(lds_a + (8 * q + crow) * SK_ST + ccol) = f.a[q];
#pragma unroll
    for (int q = 0; q < 8; ++q) *(u32x4 *)(lds_b + (8 * q + crow) * SB + ccol) = f.b[q];
  };
  auto multiply = [&]() {
    const int blk = lane >> 4, q16 = lane & 15;
    typedef __attribute__((address_space(3))) s16x4 lds_v4;
#pragma unroll
    for (int c = 0; c < 4; ++c) {            // four 16-wide chunks of the step
      bf16x8 a[TI], b[2];
#pragma unroll
      for (int i = 0; i < TI; ++i) a[i] = *(const bf16x8 *)(lds_a + (32 * i + r) * SK_ST + 16 * c + 8 * h);
#pragma unroll
      for (int j = 0; j < 2; ++j) {
        if (FORM == FORM_FWD) {
          b[j] = *(const bf16x8 *)(lds_b + (32 * j + r) * SK_ST + 16 * c + 8 * h);
        } else {
          // transposing read: in each block of 16 lanes, lane q addresses row (q / 4), columns 4 (q % 4)..+3
          const uint16_t *ptr = lds_b + (16 * c + 8 * (blk >> 1) + (q16 >> 2)) * SB + 32 * j + 16 * (blk & 1) + 4 * (q16 & 3);
          s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)ptr);
          s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(ptr + 4 * SB));
          b[j] = __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
        }
      }
#pragma unroll
      for (int i = 0; i < TI; ++i)
#pragma unroll
        for (int j = 0; j < 2; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  // NS register sets rotate: while one step is multiplied, the next NS-1 are on their way from memory
  constexpr int NS = NW == 8 ? 2 : 3;   // bounded by the register file: 256 VGPRs per lane at 8 waves
  SkStep<TI> f[NS];
#pragma unroll
  for (int u = 0; u < NS; ++u)
    if (s_lo + u < s_hi) load(f[u], s_lo + u);
  for (int s = s_lo; s < s_hi; s += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      if (s + u >= s_hi) break;
      stage(f[u]);
      if (s + u + NS < s_hi) load(f[u], s + u + NS);
      multiply();
    }
  }

  // ---- add the waves' partial tiles through LDS
  auto put = [&](float *buf) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) buf[(32 * i + 8 * (q >> 2) + 4 * h + (q & 3)) * SK_BN + 32 * j + r] = acc[i][j][q];
  };
  auto add = [&](const float *buf) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < 2; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) acc[i][j][q] += buf[(32 * i + 8 * (q >> 2) + 4 * h + (q & 3)) * SK_BN + 32 * j + r];
  };
  // binary tree with a fixed shape: in every round the upper half of the live waves hands its tile
  // to the lower half; the final sum ends up in buffer 0
  __syncthreads();                 // the waves' private operand tiles are dead from here on
#pragma unroll
  for (int live = NW; live > 1; live >>= 1) {
    const int half = live >> 1;
    if (wave >= half && wave < live) put(red + (wave - half) * BM * SK_BN);
    __syncthreads();
    if (wave < half) add(red + wave * BM * SK_BN);
    __syncthreads();
  }
  if (wave == 0) put(red);
  __syncthreads();
  const float *r1 = red;

  // ---- epilogue, all waves: thread t owns 8 consecutive columns of rows t/8, t/8 + 8 NW, ...
  const int cg = (threadIdx.x & 7) * 8;
  for (int lr = threadIdx.x >> 3; lr < BM; lr += 8 * NW) {
    const int row = m0 + lr;
    if (row >= p.M) break;
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int col = n0 + cg + e;
      if (col >= p.N) break;
      float v = r1[lr * SK_BN + cg + e];
      const int64_t ci = (int64_t)row * p.ldc + col;
      if (FORM == FORM_FWD) {
        if (p.bias) v += p.bias[col];
        if (p.aux) store_from_f32(p.aux, p.aux_dtype, (int64_t)row * p.ldaux + col, v);
        v = act_apply(v, p.act);
        if (p.res) v += load_as_f32(p.res, p.res_dtype, (int64_t)row * p.ldres + col);
      } else {
        if (p.res) v += load_as_f32(p.res, p.res_dtype, (int64_t)row * p.ldres + col);
        if (p.act != ACT_NONE) v *= act_grad(load_as_f32(p.aux, p.aux_dtype, (int64_t)row * p.ldaux + col), p.act);
      }
      store_from_f32(p.C, p.c_dtype, ci, v);
    }
  }
}

template <int FORM>
static void launch_rows(const GemmProb *probs, int n, int blocks, int row_tiles, hipStream_t s) {
  if (row_tiles == 1) hipLaunchKernelGGL((k_gemm_skinny<FORM, 1>), dim3(blocks), dim3(64 * SkWaves<1>::value), 0, s, probs, n);
  else hipLaunchKernelGGL((k_gemm_skinny<FORM, 2>), dim3(blocks), dim3(64 * SkWaves<2>::value), 0, s, probs, n);
}
void launch_gemm_skinny(const GemmProb *probs, int n, int total_blocks, int form, int row_tiles, hipStream_t s) {
  if (total_blocks <= 0) return;
  if (form == FORM_FWD) launch_rows<FORM_FWD>(probs, n, total_blocks, row_tiles, s);
  else launch_rows<FORM_DX>(probs, n, total_blocks, row_tiles, s);
}

}  // namespace gpp
