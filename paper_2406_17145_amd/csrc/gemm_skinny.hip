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
// with the transposing LDS read.  The partial accumulators meet in LDS and are
// added in wave order by the threads of the epilogue, which all waves share.
//
// The backward pass of a level runs both consumers of dZ in ONE launch: workgroups of the first
// records compute dX with the few-row body, the rest compute dW (+ db) with the tile body, two
// 256-thread teams per workgroup on neighbouring tiles.
#include "gemm_dw_ksplit_body.h"

namespace gpp {

constexpr int SK_KS = 64;             // contraction elements per k-step of a wave
constexpr int SK_ST = SK_KS + 8;      // LDS row stride of a k-contiguous 64-wide tile (elements)

// 32-row tiles per workgroup (1 or 2); 0 when the problem has too many rows for this kernel.
// More than 64 rows are covered by several workgroups per column block, which re-read W from L2.
int gemm_skinny_row_tiles(int M) { return M <= 32 ? 1 : (M <= 256 ? 2 : 0); }
// 32-column tiles per workgroup: 2 (64 output columns) unless that leaves most of the chip idle;
// `blocks64` is the launch's workgroup count at 64 columns
int gemm_skinny_col_tiles(int blocks64) { return blocks64 >= 128 ? 2 : 1; }
int gemm_skinny_blocks(int M, int N, int row_tiles, int col_tiles) {
  return ((N + 32 * col_tiles - 1) / (32 * col_tiles)) * ((M + 32 * row_tiles - 1) / (32 * row_tiles));
}

// one 64-wide k-step of a wave, as fetched from memory: BM x 64 of A and the W tile (BN x 64 forward,
// 64 x BN backward-data) in 16-byte chunks of whole rows, so every load instruction covers whole
// 128-byte (64-byte for a 32-wide backward tile) row segments
template <int TI, int TJ>
struct SkStep {
  u32x4 a[4 * TI];
  u32x4 b[4 * TJ];
};

// NW waves per workgroup split K: 8 when the private tiles of 8 waves fit in LDS (up to 64 rows), else 4
template <int TI>
struct SkWaves {
  static constexpr int value = TI <= 2 ? 8 : 4;
};

// LDS bytes of the few-row body
template <int FORM, int TI, int TJ, int NW_ = SkWaves<TI>::value>
struct SkLds {
  static constexpr int NW = NW_;
  static constexpr int BM = 32 * TI, BN = 32 * TJ;
  static constexpr int RED_FLOATS = NW * BM * BN;      // after the k-loop: every wave's partial tile
  // W tile: forward [BN][64 + 8]; backward-data [64][BN + pad], read with the transposing read.  A
  // 16-lane block of that read touches 32 bytes in each of four consecutive rows, and the neighbouring
  // block the next 32 bytes of the same rows, so the row stride should spread four rows over the 64
  // banks (256 bytes): 64 bytes for 32-wide rows (no padding: four rows are exactly the 64 banks, and the
  // staging stores are contiguous), 192 for 64-wide ones (only when the waves' tiles still fit in the
  // 160 KB of LDS, else 144)
  static constexpr int SB = FORM == FORM_FWD ? SK_ST
                            : BN == 32       ? BN
                                             : (NW * (BM * SK_ST + SK_KS * (BN + 32)) * 2 <= 160 * 1024 ? BN + 32 : BN + 8);
  static constexpr int B_ROWS = FORM == FORM_FWD ? BN : SK_KS;
  static constexpr int WAVE_ELEMS = BM * SK_ST + B_ROWS * SB;     // a wave's private A and B tiles
  static constexpr int BYTES = RED_FLOATS * 4 > NW * WAVE_ELEMS * 2 ? RED_FLOATS * 4 : NW * WAVE_ELEMS * 2;
};

// `local`: index of this workgroup inside the record.  Hardware deals consecutive workgroup ids
// round-robin over the 8 XCDs (one L2 each): the column blocks of a record are spread over all of them
// (a wide problem's weights then stream through every L2 and memory channel), while the row blocks
// of ONE column block, which read the same slice of W, get ids 8 apart and so meet in one L2.
// A group launch covers the same problems for several micro-batches ("members"): their operands and results
// sit at the same offsets of stash slots `stride` bytes apart, and a member's per-call pointers `ext_stride`
// entries behind the previous member's.  The members take the place of further row blocks of a column block:
// their workgroups get ids 8 apart like the row blocks of one micro-batch, so the weight tile they all read
// is fetched into one L2 once.
struct SkGroup {
  int32_t members, ext_stride;
  int64_t stride;
};
template <int FORM, int TI, int TJ, int NW_ = SkWaves<TI>::value>
__device__ __forceinline__ void gemm_skinny_body(const GemmProb &pin, int local, unsigned char *lds_raw, const ExtPtrs &ext,
                                                 const SkGroup &group) {
  typedef SkLds<FORM, TI, TJ, NW_> L;
  constexpr int NW = L::NW, BM = L::BM, BN = L::BN, SB = L::SB, WAVE_ELEMS = L::WAVE_ELEMS;
  float *red = (float *)lds_raw;           // after the k-loop: NW BM x BN fp32 buffers, one per wave

  const int m_blocks1 = (pin.M + BM - 1) / BM, m_blocks = m_blocks1 * group.members, n_blocks = (pin.N + BN - 1) / BN;
  int cb, rb;                      // column block, row block
  {
    const int grp = local / (8 * m_blocks), r = local - grp * 8 * m_blocks;
    const int cols_here = min(8, n_blocks - 8 * grp);            // the last group may hold fewer than 8 column blocks
    cb = 8 * grp + r % cols_here;
    rb = r / cols_here;
  }
  GemmProb p = pin;
  if (group.members > 1) {         // this workgroup's member: everything that lives in a stash slot moves with it
    const int member = rb / m_blocks1;
    rb -= member * m_blocks1;
    const int64_t off = (int64_t)member * group.stride;
    p.A = (const GPP_G char *)p.A + off;
    if (p.C) p.C = (GPP_G char *)p.C + off;
    if (p.aux) p.aux = (GPP_G char *)p.aux + off;
    if (p.res) p.res = (const GPP_G char *)p.res + off;
    if (p.c_ext > 0) p.c_ext += member * group.ext_stride;
  }
  void *Cout = result_ptr(p, ext);
  const int n0 = cb * BN;
  const int m0 = rb * BM;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int r = lane & 31, h = lane >> 5;
  // operand descriptors: A = X or dZ [M x K]; B = W, [N x K] forward, [K x N] backward-data
  const __amdgpu_buffer_rsrc_t rs_a = matrix_rsrc(p.A, p.M, p.lda, p.K);
  const __amdgpu_buffer_rsrc_t rs_b = matrix_rsrc(p.B, FORM == FORM_FWD ? p.N : p.K, p.ldb, FORM == FORM_FWD ? p.K : p.N);
  const bool ragged_k = (p.K & 7) != 0;                        // forward: both operands end inside a chunk; backward-data: A
  uint16_t *lds_a = (uint16_t *)lds_raw + wave * WAVE_ELEMS;   // [BM][SK_ST]
  uint16_t *lds_b = lds_a + BM * SK_ST;                        // [B_ROWS][SB]

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int q = 0; q < 16; ++q) acc[i][j][q] = 0.0f;

  const int steps = (p.K + SK_KS - 1) / SK_KS, per = (steps + NW - 1) / NW;
  const int s_lo = wave * per, s_hi = min(steps, s_lo + per);
  const int crow = lane >> 3, ccol = (lane & 7) * 8;     // this lane's chunk inside an 8-row slab of 64-wide rows
  // backward-data W tile rows are BN wide: BN / 8 chunks per row, 512 / BN rows per load instruction
  constexpr int DX_CPR = BN / 8, DX_RPI = 64 / DX_CPR;
  const int drow = lane / DX_CPR, dcol = (lane % DX_CPR) * 8;

  auto load = [&](SkStep<TI, TJ> &f, int s) {
    const int k0 = SK_KS * s;
#pragma unroll
    for (int q = 0; q < 4 * TI; ++q) f.a[q] = chunk_load(rs_a, p.lda, m0 + 8 * q + crow, k0 + ccol, p.M, p.K);
#pragma unroll
    for (int q = 0; q < 4 * TJ; ++q) {
      if (FORM == FORM_FWD) f.b[q] = chunk_load(rs_b, p.ldb, n0 + 8 * q + crow, k0 + ccol, p.N, p.K);          // W[n][k]
      else f.b[q] = chunk_load(rs_b, p.ldb, k0 + DX_RPI * q + drow, n0 + dcol, p.K, p.N);                      // W[k][n]
    }
    if (ragged_k) {   // the contraction ends inside a chunk: clear what lies beyond it (row padding)
#pragma unroll
      for (int q = 0; q < 4 * TI; ++q) f.a[q] = chunk_clear_tail(f.a[q], k0 + ccol, p.K);
      if (FORM == FORM_FWD) {
#pragma unroll
        for (int q = 0; q < 4 * TJ; ++q) f.b[q] = chunk_clear_tail(f.b[q], k0 + ccol, p.K);
      }
    }
  };
  auto stage = [&](const SkStep<TI, TJ> &f) {
#pragma unroll
    for (int q = 0; q < 4 * TI; ++q) *(u32x4 *)(lds_a + (8 * q + crow) * SK_ST + ccol) = f.a[q];
#pragma unroll
    for (int q = 0; q < 4 * TJ; ++q) {
      if (FORM == FORM_FWD) *(u32x4 *)(lds_b + (8 * q + crow) * SB + ccol) = f.b[q];
      else *(u32x4 *)(lds_b + (DX_RPI * q + drow) * SB + dcol) = f.b[q];
    }
  };
  auto multiply = [&]() {
    const int blk = lane >> 4, q16 = lane & 15;
    typedef __attribute__((address_space(3))) s16x4 lds_v4;
#pragma unroll
    for (int c = 0; c < 4; ++c) {            // four 16-wide chunks of the step
      bf16x8 a[TI], b[TJ];
#pragma unroll
      for (int i = 0; i < TI; ++i) a[i] = *(const bf16x8 *)(lds_a + (32 * i + r) * SK_ST + 16 * c + 8 * h);
#pragma unroll
      for (int j = 0; j < TJ; ++j) {
        if (FORM == FORM_FWD) {
          b[j] = *(const bf16x8 *)(lds_b + (32 * j + r) * SB + 16 * c + 8 * h);
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
        for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  // ---- what the epilogue reads from memory besides the product (residual / gradient addend, mask source
  // or stashed derivative) is requested HERE, before the k-loop: a thread owns one 8-column piece of one
  // row when the workgroup's threads cover the tile in one pass, and a load issued only after the
  // reduction would add a whole memory round trip to a kernel that lasts a few of them.
  constexpr int TPR = BN / 8, ROWS_PER_PASS = 64 * NW / TPR;
  constexpr bool ONE_PASS = ROWS_PER_PASS >= BM;
  const int cg = (threadIdx.x % TPR) * 8;
  // Fast path: bf16 result (and bf16 residual / mask source / stash where present) in whole, aligned
  // 16-byte chunks.  The storage types are known here, so no type test stands between the loads.
  const bool chunked = Cout != nullptr && p.c_dtype == DT_BF16 && (p.N & 7) == 0 && (p.ldc & 7) == 0 && ((uintptr_t)Cout & 15) == 0 &&
                       (!p.res || (p.res_dtype == DT_BF16 && (p.ldres & 7) == 0 && ((uintptr_t)p.res & 15) == 0)) &&
                       (!p.aux || (p.aux_dtype == DT_BF16 && (p.ldaux & 7) == 0 && ((uintptr_t)p.aux & 15) == 0)) &&
                       (FORM == FORM_DX || !p.bias || ((uintptr_t)p.bias & 15) == 0);
  const bool use_aux_in = FORM == FORM_DX && p.act != ACT_NONE;
  u32x4 pre_res = {0u, 0u, 0u, 0u}, pre_aux = {0u, 0u, 0u, 0u};
  float pre_bias[8] = {};
  if (ONE_PASS && chunked) {    // uniform: nothing is outstanding yet, so the branch costs no wait
    // clamped to the tile's valid part: a thread without a piece reads a valid one and drops it
    const int row = min(m0 + (int)threadIdx.x / TPR, p.M - 1), col = min(n0 + cg, p.N - 8);
    if (FORM == FORM_FWD && p.bias) {
      const float4 b0 = *(const float4 *)(p.bias + col), b1 = *(const float4 *)(p.bias + col + 4);
      pre_bias[0] = b0.x; pre_bias[1] = b0.y; pre_bias[2] = b0.z; pre_bias[3] = b0.w;
      pre_bias[4] = b1.x; pre_bias[5] = b1.y; pre_bias[6] = b1.z; pre_bias[7] = b1.w;
    }
    // an absent operand is read from the result buffer instead (valid memory, value unused): no
    // branch stands between these loads and the loads of the k-loop behind them
    const uint16_t *resp = p.res ? (const uint16_t *)p.res : (const uint16_t *)Cout;
    const uint16_t *auxp = use_aux_in ? (const uint16_t *)p.aux : (const uint16_t *)Cout;
    const int64_t ldr = p.res ? p.ldres : p.ldc, lda = use_aux_in ? p.ldaux : p.ldc;
    pre_res = *(const u32x4 *)(resp + (int64_t)row * ldr + col);
    pre_aux = *(const u32x4 *)(auxp + (int64_t)row * lda + col);
  }

  // NS register sets rotate: while one step is multiplied, the next NS-1 are on their way from memory
  // (bounded by the register file: 256 VGPRs per lane at 8 waves)
  // (four-wave workgroups share a compute unit with others: the 64 x 32 and 32 x 64 tiles keep two sets, 188
  // registers per lane; three sets measured 2 % slower in the step, four sets 30 %)
  constexpr int NS = NW == 8 ? (TI + TJ <= 3 ? 3 : 2) : (TI + TJ <= 2 ? 4 : (TI + TJ == 3 ? 2 : 3));
  SkStep<TI, TJ> f[NS];
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

  // ---- the waves' partial tiles meet in LDS: every wave stores its own, one barrier, and whoever needs an element
  // of the result adds the NW partials in wave order (a fixed order: the result does not depend on timing).  A
  // tree of hand-overs between waves took three rounds of store, barrier, add, barrier plus a last store: seven
  // barriers and four LDS round trips in a kernel that lasts a few microseconds.
  __syncthreads();                 // the waves' private operand tiles are dead from here on
  {
    float *buf = red + wave * BM * BN;
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int q = 0; q < 16; ++q) buf[(32 * i + 8 * (q >> 2) + 4 * h + (q & 3)) * BN + 32 * j + r] = acc[i][j][q];
  }
  __syncthreads();
  // eight consecutive elements of row lr of the tile, from column c on
  auto summed8 = [&](int lr, int c, float (&v)[8]) {
    float4 a[NW], b[NW];
#pragma unroll
    for (int w8 = 0; w8 < NW; ++w8) {
      a[w8] = *(const float4 *)(red + w8 * BM * BN + lr * BN + c);
      b[w8] = *(const float4 *)(red + w8 * BM * BN + lr * BN + c + 4);
    }
    v[0] = a[0].x; v[1] = a[0].y; v[2] = a[0].z; v[3] = a[0].w; v[4] = b[0].x; v[5] = b[0].y; v[6] = b[0].z; v[7] = b[0].w;
#pragma unroll
    for (int w8 = 1; w8 < NW; ++w8) {
      v[0] += a[w8].x; v[1] += a[w8].y; v[2] += a[w8].z; v[3] += a[w8].w;
      v[4] += b[w8].x; v[5] += b[w8].y; v[6] += b[w8].z; v[7] += b[w8].w;
    }
  };
  if (Cout == nullptr) return;     // the caller does not want this result (all barriers are behind us)

  // ---- epilogue, all waves: thread t owns 8 consecutive columns; BN / 8 threads per row
  if (chunked) {
    const int col = n0 + cg;
    if (col >= p.N) return;
    float bias[8] = {};
    if (ONE_PASS) {
#pragma unroll
      for (int e = 0; e < 8; ++e) bias[e] = pre_bias[e];
    } else if (FORM == FORM_FWD && p.bias) {
      const float4 b0 = *(const float4 *)(p.bias + col), b1 = *(const float4 *)(p.bias + col + 4);
      bias[0] = b0.x; bias[1] = b0.y; bias[2] = b0.z; bias[3] = b0.w;
      bias[4] = b1.x; bias[5] = b1.y; bias[6] = b1.z; bias[7] = b1.w;
    }
    // (several passes over the tile) an absent operand is read from the result buffer instead (valid memory, value unused): the two
    // loads of a row then carry no branch
    const uint16_t *resp = p.res ? (const uint16_t *)p.res : (const uint16_t *)Cout;
    const uint16_t *auxp = use_aux_in ? (const uint16_t *)p.aux : (const uint16_t *)Cout;
    const int64_t ldr = p.res ? p.ldres : p.ldc, lda = use_aux_in ? p.ldaux : p.ldc;
    for (int lr = threadIdx.x / TPR; lr < BM; lr += ROWS_PER_PASS) {
      const int row = m0 + lr;
      if (row >= p.M) break;
      u32x4 res_raw = pre_res, aux_raw = pre_aux;
      if (!ONE_PASS) {
        res_raw = *(const u32x4 *)(resp + (int64_t)row * ldr + col);
        aux_raw = *(const u32x4 *)(auxp + (int64_t)row * lda + col);
      }
      float v[8], rs[8], ax[8];
      summed8(lr, cg, v);
#pragma unroll
      for (int e = 0; e < 4; ++e) {
        rs[2 * e] = __uint_as_float(res_raw[e] << 16);
        rs[2 * e + 1] = __uint_as_float(res_raw[e] & 0xffff0000u);
        ax[2 * e] = __uint_as_float(aux_raw[e] << 16);
        ax[2 * e + 1] = __uint_as_float(aux_raw[e] & 0xffff0000u);
      }
      float stash[8];
#pragma unroll
      for (int e = 0; e < 8; ++e) {
        if (FORM == FORM_FWD) {
          v[e] += bias[e];
          stash[e] = act_stash(v[e], p.act);
          v[e] = act_apply(v[e], p.act);
          if (p.res) v[e] += rs[e];
        } else {
          if (p.res) v[e] += rs[e];
          if (use_aux_in) v[e] *= act_grad(ax[e], p.act);
        }
      }
      u32x4 out;
#pragma unroll
      for (int e = 0; e < 4; ++e) out[e] = (uint32_t)f32_to_bf16_bits(v[2 * e]) | ((uint32_t)f32_to_bf16_bits(v[2 * e + 1]) << 16);
      *(u32x4 *)((uint16_t *)Cout + (int64_t)row * p.ldc + col) = out;
      if (FORM == FORM_FWD && p.aux) {
#pragma unroll
        for (int e = 0; e < 4; ++e) out[e] = (uint32_t)f32_to_bf16_bits(stash[2 * e]) | ((uint32_t)f32_to_bf16_bits(stash[2 * e + 1]) << 16);
        *(u32x4 *)((uint16_t *)p.aux + (int64_t)row * p.ldaux + col) = out;
      }
    }
    return;
  }
  for (int lr = threadIdx.x / TPR; lr < BM; lr += ROWS_PER_PASS) {
    const int row = m0 + lr;
    if (row >= p.M) break;
    float v8[8];
    summed8(lr, cg, v8);
#pragma unroll
    for (int e = 0; e < 8; ++e) {
      const int col = n0 + cg + e;
      if (col >= p.N) break;
      float v = v8[e];
      const int64_t ci = (int64_t)row * p.ldc + col;
      if (FORM == FORM_FWD) {
        if (p.bias) v += p.bias[col];
        if (p.aux) store_from_f32(p.aux, p.aux_dtype, (int64_t)row * p.ldaux + col, act_stash(v, p.act));
        v = act_apply(v, p.act);
        if (p.res) v += load_as_f32(p.res, p.res_dtype, (int64_t)row * p.ldres + col);
      } else {
        if (p.res) v += load_as_f32(p.res, p.res_dtype, (int64_t)row * p.ldres + col);
        if (p.act != ACT_NONE) v *= act_grad(load_as_f32(p.aux, p.aux_dtype, (int64_t)row * p.ldaux + col), p.act);
      }
      store_from_f32(Cout, p.c_dtype, ci, v);
    }
  }
}

template <int FORM, int TI, int TJ, int NW = SkWaves<TI>::value>
__global__ __launch_bounds__(64 * NW) void k_gemm_skinny(const GemmProb *__restrict__ probs, int n, ExtPtrs ext, SkGroup group) {
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[SkLds<FORM, TI, TJ, NW>::BYTES];
  // every record's workgroup range is `members` times the one in its table
  int lo = 0, hi = n - 1;
  while (lo < hi) {
    const int mid = (lo + hi + 1) >> 1;
    if (probs[mid].blk_begin * group.members <= (int)blockIdx.x)
      lo = mid;
    else
      hi = mid - 1;
  }
  const GemmProb p = probs[lo];
  gemm_skinny_body<FORM, TI, TJ, NW>(p, blockIdx.x - p.blk_begin * group.members, lds_raw, ext, group);
}

// backward of one level in one launch: records with form DX run the few-row body; records with
// form DW either the 128 x 128 tile body, two teams per workgroup on tiles 2 * local and 2 * local + 1
// (few rows to contract over), or, marked by split_k == BWD_DW_KSPLIT, the 64 x 64 tile body whose
// waves split a long contraction (many rows)
constexpr int BWD_DW_TILE = 128;
constexpr int BWD_DW_KSPLIT = -64;
int gemm_bwd_merged_ksplit_mark() { return BWD_DW_KSPLIT; }
template <int TI, int TJ>
__global__ __launch_bounds__(512) void k_gemm_bwd_merged(const GemmProb *__restrict__ probs, int n, int accumulate_dw,
                                                         ExtPtrs ext) {
  static_assert(SkWaves<TI>::value == 8, "the merged launch uses 512-thread workgroups");
  typedef TileLds<FORM_DW, BWD_DW_TILE, BWD_DW_TILE> DwLds;
  typedef SkLds<FORM_DX, TI, TJ> DxLds;
  constexpr int BYTES0 = DxLds::BYTES > 4 * DwLds::ELEMS ? DxLds::BYTES : 4 * DwLds::ELEMS;
  constexpr int BYTES = BYTES0 > KS_LDS_BYTES ? BYTES0 : KS_LDS_BYTES;
  static_assert(BYTES <= 160 * 1024, "the merged launch's bodies do not fit the LDS");
  __shared__ __attribute__((aligned(16))) unsigned char lds_raw[BYTES];
  const int pi = find_prob(probs, n, blockIdx.x);
  const GemmProb p = probs[pi];
  const int local = blockIdx.x - p.blk_begin;
  if (p.form == FORM_DX) {
    gemm_skinny_body<FORM_DX, TI, TJ>(p, local, lds_raw, ext, SkGroup{1, 0, 0});
  } else if (p.split_k == BWD_DW_KSPLIT) {
    gemm_dw_ksplit_body(p, local, lds_raw, accumulate_dw);
  } else {
    const int team = threadIdx.x >> 8;
    // few rows to contract over: two k-steps in flight are enough and keep the kernel free of spills
    gemm_tile_body<FORM_DW, BWD_DW_TILE, BWD_DW_TILE, false, 2, true>(p, 2 * local + team, threadIdx.x & 255,
                                                             (uint16_t *)lds_raw + team * DwLds::ELEMS, accumulate_dw, ext);
  }
}
int gemm_bwd_merged_dw_tile() { return BWD_DW_TILE; }
// workgroups of one backward-weight record in the merged launch
int gemm_bwd_merged_dw_blocks(int M, int N) {
  const int tiles = cdiv(M, BWD_DW_TILE) * cdiv(N, BWD_DW_TILE);
  return (tiles + 1) / 2;
}

template <int FORM>
static void launch_rows(const GemmProb *probs, int n, int blocks, int row_tiles, int col_tiles, int waves, const ExtPtrs &ext,
                        const SkGroup &group, hipStream_t s) {
  if (waves == 4) {   // workgroups sized to share a compute unit with those of concurrent launches
    const dim3 g4(blocks), b4(256);
    if (row_tiles == 1 && col_tiles == 1) hipLaunchKernelGGL((k_gemm_skinny<FORM, 1, 1, 4>), g4, b4, 0, s, probs, n, ext, group);
    else if (row_tiles == 1) hipLaunchKernelGGL((k_gemm_skinny<FORM, 1, 2, 4>), g4, b4, 0, s, probs, n, ext, group);
    else if (col_tiles == 1) hipLaunchKernelGGL((k_gemm_skinny<FORM, 2, 1, 4>), g4, b4, 0, s, probs, n, ext, group);
    else hipLaunchKernelGGL((k_gemm_skinny<FORM, 2, 2, 4>), g4, b4, 0, s, probs, n, ext, group);
    return;
  }
  const dim3 g(blocks), b(512);
  if (row_tiles == 1 && col_tiles == 1) hipLaunchKernelGGL((k_gemm_skinny<FORM, 1, 1>), g, b, 0, s, probs, n, ext, group);
  else if (row_tiles == 1) hipLaunchKernelGGL((k_gemm_skinny<FORM, 1, 2>), g, b, 0, s, probs, n, ext, group);
  else if (col_tiles == 1) hipLaunchKernelGGL((k_gemm_skinny<FORM, 2, 1>), g, b, 0, s, probs, n, ext, group);
  else hipLaunchKernelGGL((k_gemm_skinny<FORM, 2, 2>), g, b, 0, s, probs, n, ext, group);
}
void launch_gemm_skinny(const GemmProb *probs, int n, int total_blocks, int form, int row_tiles, int col_tiles, int waves,
                        const ExtPtrs &ext, hipStream_t s, int members, int64_t member_stride_bytes, int member_ext_stride) {
  if (total_blocks <= 0 || members <= 0) return;
  const SkGroup group{members, member_ext_stride, member_stride_bytes};
  if (form == FORM_FWD) launch_rows<FORM_FWD>(probs, n, total_blocks * members, row_tiles, col_tiles, waves, ext, group, s);
  else launch_rows<FORM_DX>(probs, n, total_blocks * members, row_tiles, col_tiles, waves, ext, group, s);
}
void launch_gemm_bwd_merged(const GemmProb *probs, int n, int total_blocks, int row_tiles, int col_tiles, int accumulate_dw,
                            const ExtPtrs &ext, hipStream_t s) {
  if (total_blocks <= 0) return;
  const dim3 g(total_blocks), b(512);
  if (row_tiles == 1 && col_tiles == 1) hipLaunchKernelGGL((k_gemm_bwd_merged<1, 1>), g, b, 0, s, probs, n, accumulate_dw, ext);
  else if (row_tiles == 1) hipLaunchKernelGGL((k_gemm_bwd_merged<1, 2>), g, b, 0, s, probs, n, accumulate_dw, ext);
  else if (col_tiles == 1) hipLaunchKernelGGL((k_gemm_bwd_merged<2, 1>), g, b, 0, s, probs, n, accumulate_dw, ext);
  else hipLaunchKernelGGL((k_gemm_bwd_merged<2, 2>), g, b, 0, s, probs, n, accumulate_dw, ext);
}

}  // namespace gpp
