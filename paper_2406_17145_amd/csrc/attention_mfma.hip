// Multi-head softmax attention on the CDNA4 matrix cores (bf16 in, fp32
// accumulate, head dimension 64), forward and backward, grouped over all
// transformer branches of a level.  Flash-style: scores are never written to
// memory; the forward keeps the row log-sum-exp, the backward recomputes the
// probabilities from it.
//
// Orientation.  v_mfma_f32_32x32x16 leaves lane l with column (l % 32) of the
// result and 16 of its rows.  Every kernel arranges its score product so that
// the softmax row (a query) is a lane's column wherever a row reduction is
// needed, and so that the probabilities a lane holds are, without any
// cross-lane traffic, the operand of the next product: the 8 contraction slots
// a lane feeds into one MFMA are accumulator registers 8c .. 8c+7, i.e. score
// rows 16c + {0..3, 8..11} + 4*(l / 32); the other operand is fetched from LDS
// with the transposing read at exactly those rows (tr_frag).  Summation order
// inside a product does not matter, so both operands only have to agree.
//
//   forward      S^T = K Q^T            O^T  += V^T P^T
//   backward dQ  S^T = K Q^T, dP^T = V dO^T,  dQ^T += K^T dS^T
//   backward dKV S   = Q K^T, dP   = dO V^T,  dV += P^T dO,  dK += dS^T Q
// No atomics: dQ and dK/dV come from two kernels that each own their outputs.
#include "device_utils.h"

namespace gpp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int DH = 64;            // head dimension of the MFMA path
constexpr int LDS_ST = DH + 8;    // LDS row stride (elements) of tiles read along their rows: 144-byte rows put sixteen
                                  // consecutive rows' 16-byte pieces into sixteen different groups of four banks
constexpr int LDS_TR = DH + 32;   // row stride of tiles read with the transposing read: that read serves 32 lanes per
                                  // cycle, 64 bytes in each of four consecutive rows; 192-byte rows put the four rows into
                                  // the four quarters of the 64 banks (with 144-byte rows two of them shared banks:
                                  // 0.7 conflicts per LDS cycle).  No stride serves both reads, so a tile that is read
                                  // both ways is kept twice
constexpr int QT = 128;           // rows (queries or keys) owned by a workgroup: 4 waves x 32
constexpr int KT = 32;            // rows of the streamed tile

int attn_mfma_blocks(int batch, int heads, int seq) { return batch * heads * ((seq + QT - 1) / QT); }

bool attn_mfma_supported(const AttnProb &p) {
  if (p.dh != DH || p.dtype != DT_BF16 || p.out_dtype != DT_BF16) return false;
  if ((p.ld_qkv | p.ld_out | p.ld_dout | p.ld_o) & 7) return false;
  if (((uintptr_t)p.qkv | (uintptr_t)p.out | (uintptr_t)p.dout | (uintptr_t)p.o) & 15) return false;
  return true;
}

// Consecutive workgroup ids go round-robin over the 8 XCDs (one L2 each).  The workgroups of one (sample, head) read the
// same K and V (the same Q and dO in the dK/dV kernel): numbered one after the other they would land on four or more
// different XCDs and fetch those rows into as many L2s.  Each XCD takes a contiguous run of the numbering instead.
__device__ __forceinline__ int xcd_contiguous_block() {
  const int total = gridDim.x, bid = blockIdx.x;
  const int xcd = bid & 7, idx = bid >> 3, per = total >> 3, rem = total & 7;
  return xcd * per + min(xcd, rem) + idx;
}

struct Where {
  int b, h, r0;  // sample, head, first row of this workgroup's 128-row block
};
__device__ __forceinline__ Where where(const AttnProb &p, int blk) {
  const int nb = (p.seq + QT - 1) / QT;
  const int bh = blk / nb;
  Where w;
  w.b = bh / p.heads;
  w.h = bh % p.heads;
  w.r0 = (blk % nb) * QT;
  return w;
}

// 16-byte chunk of row `row`.  No branch around the load (a wave waits for its earlier loads at a
// branch): a row outside the sequence reads the last row instead.  Such rows only ever meet
// probabilities that the tail mask has set to zero, or belong to queries / keys whose results are
// not stored, so finite stand-in values are all that is needed.
__device__ __forceinline__ u32x4 row_chunk(const void *base, int64_t ld, int64_t first_row, int row, int seq, int col) {
  return *(const u32x4 *)((const uint16_t *)base + (first_row + min(row, seq - 1)) * ld + col);
}
// the four 8-element slices of a lane's own row that one MFMA operand chain over DH = 64 needs
struct RowFrags {
  bf16x8 f[4];
};
__device__ __forceinline__ RowFrags load_row_frags(const void *base, int64_t ld, int64_t first_row, int row, int seq, int col0) {
  const int h = (threadIdx.x & 63) >> 5;
  RowFrags r;
#pragma unroll
  for (int s = 0; s < 4; ++s) r.f[s] = __builtin_bit_cast(bf16x8, row_chunk(base, ld, first_row, row, seq, col0 + 16 * s + 8 * h));
  return r;
}
// k-contiguous operand from an LDS tile [rows][LDS_ST]: lane takes row (l % 32), columns 16 s + 8 (l / 32) ..
__device__ __forceinline__ bf16x8 row_frag(const uint16_t *lds, int s) {
  const int l = threadIdx.x & 63;
  return *(const bf16x8 *)(lds + (l & 31) * LDS_ST + 16 * s + 8 * (l >> 5));
}
// transposed operand from an LDS tile [rows][LDS_TR]: lane takes column col0 + (l % 32) and rows
// 16 c + 4 (l / 32) + {0..3} and + 8 (matching accumulator registers 8c .. 8c+7 of a score tile)
__device__ __forceinline__ bf16x8 tr_frag(const uint16_t *lds, int col0, int c) {
  const int l = threadIdx.x & 63;
  const int blk = l >> 4, q = l & 15;
  const uint16_t *p = lds + (16 * c + 4 * (blk >> 1) + (q >> 2)) * LDS_TR + col0 + 16 * (blk & 1) + 4 * (q & 3);
  typedef __attribute__((address_space(3))) s16x4 lds_v4;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)p);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p + 8 * LDS_TR));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}
__device__ __forceinline__ bf16x8 pack8(const f32x16 &v, int c) {
  bf16x8 r;
#pragma unroll
  for (int e = 0; e < 8; ++e) r[e] = (bf16_t)v[8 * c + e];
  return r;
}
__device__ __forceinline__ f32x16 zero16() {
  f32x16 z;
#pragma unroll
  for (int r = 0; r < 16; ++r) z[r] = 0.0f;
  return z;
}
// row index inside a 32-row score tile held by accumulator register r of this lane
__device__ __forceinline__ int acc_row(int r) { return 8 * (r >> 2) + 4 * ((threadIdx.x & 63) >> 5) + (r & 3); }

// Before a loop that keeps loads of the next tile in flight: wait for every load issued so far (s_waitcnt vmcnt(0),
// the other counters left alone).  The compiler counts loads in issue order; fragments loaded once in front of
// the loop would otherwise be "the n-th last load" for it in every iteration, and its wait for them would take
// in the loads of the next tile, which were meant to fly under the whole step.
__device__ __forceinline__ void loads_landed() { __builtin_amdgcn_s_waitcnt(0x0F70); }

// two streamed 32 x 64 tiles (one 16-byte chunk per thread each)
struct Stream2 {
  u32x4 a, b;
};
// one 16-byte chunk per thread into a tile with row stride ST
template <int ST>
__device__ __forceinline__ void chunk_store(const u32x4 &v, uint16_t *tile) {
  const int c = threadIdx.x;
  *(u32x4 *)(tile + (c >> 3) * ST + (c & 7) * 8) = v;
}

// writes a wave's transposed 64 x 32 accumulator pair (rows = dh, lane column = its row of the block)
// through LDS to out[row][dh] with coalesced rows
__device__ __forceinline__ void store_transposed(uint16_t *stage, const f32x16 (&acc)[2], float mul, void *out, int64_t ld,
                                                 int64_t first_row, int r0, int seq, int col0) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
#pragma unroll
  for (int d = 0; d < 2; ++d)
#pragma unroll
    for (int r = 0; r < 16; ++r)
      stage[(wave * 32 + (lane & 31)) * LDS_ST + 32 * d + acc_row(r)] = f32_to_bf16_bits(acc[d][r] * mul);
  __syncthreads();
  for (int c = threadIdx.x; c < QT * (DH / 8); c += 256) {
    const int row = c >> 3, cc = (c & 7) * 8;
    if (r0 + row < seq)
      *(u32x4 *)((uint16_t *)out + (first_row + r0 + row) * ld + col0 + cc) = *(const u32x4 *)(stage + row * LDS_ST + cc);
  }
}

// ======================================================================= forward
__global__ __launch_bounds__(256, 4) void k_attn_fwd_mfma(const AttnProb *__restrict__ probs, int n) {
  // one array: the streamed tiles, and over them (they are dead after the loop, which ends with a barrier) the
  // block through which the result is written.  21 KB and at most 128 registers: four workgroups per compute unit
  constexpr int TILES = 2 * KT * LDS_ST + 2 * KT * LDS_TR;
  static_assert(TILES >= QT * LDS_ST, "the output block fits over the tiles");
  __shared__ __attribute__((aligned(16))) uint16_t lds[TILES];
  uint16_t(*lds_k)[KT * LDS_ST] = (uint16_t(*)[KT * LDS_ST])lds;
  uint16_t(*lds_v)[KT * LDS_TR] = (uint16_t(*)[KT * LDS_TR])(lds + 2 * KT * LDS_ST);
  uint16_t *stage = lds;
  const int bid = xcd_contiguous_block();
  const int pi = find_prob(probs, n, bid);
  const AttnProb p = probs[pi];
  const Where w = where(p, bid - p.blk_begin);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d = p.heads * DH;
  const int64_t first = (int64_t)w.b * p.seq;
  const int qcol = w.h * DH, kcol = d + w.h * DH, vcol = 2 * d + w.h * DH;
  const int my_q = w.r0 + wave * 32 + (lane & 31);
  const float scale2 = rsqrtf((float)DH) * 1.4426950408889634f;   // 1/sqrt(dh) * log2(e)

  const RowFrags qf = load_row_frags(p.qkv, p.ld_qkv, first, my_q, p.seq, qcol);
  f32x16 o[2] = {zero16(), zero16()};
  float m = -1e30f, lsum = 0.0f;

  const int nt = (p.seq + KT - 1) / KT;
  auto fetch = [&](int t) {
    Stream2 s;
    const int row = t * KT + (threadIdx.x >> 3), cc = (threadIdx.x & 7) * 8;
    s.a = row_chunk(p.qkv, p.ld_qkv, first, row, p.seq, kcol + cc);
    s.b = row_chunk(p.qkv, p.ld_qkv, first, row, p.seq, vcol + cc);
    return s;
  };
  Stream2 nxt = fetch(0);
  chunk_store<LDS_ST>(nxt.a, lds_k[0]);
  chunk_store<LDS_TR>(nxt.b, lds_v[0]);
  __syncthreads();
  loads_landed();
  for (int t = 0; t < nt; ++t) {
    const int cur = t & 1;
    if (t + 1 < nt) nxt = fetch(t + 1);
    f32x16 st = zero16();
#pragma unroll
    for (int s = 0; s < 4; ++s) st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(lds_k[cur], s), qf.f[s], st, 0, 0, 0);
    // softmax in base 2 (one multiply folds the 1/sqrt(dh) scale and log2 e; v_exp_f32 is 2^x); only the
    // last tile of a ragged sequence needs the key mask; the running output is rescaled only when
    // some lane's running maximum moved
    if (t == nt - 1 && (p.seq % KT)) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (t * KT + acc_row(r) >= p.seq) st[r] = -1e30f;
    }
    float mx = -1e30f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      st[r] *= scale2;
      mx = fmaxf(mx, st[r]);
    }
    mx = fmaxf(mx, __shfl_xor(mx, 32, 64));
    const float m_new = fmaxf(m, mx);
    const float alpha = __builtin_amdgcn_exp2f(m - m_new);
    float ps = 0.0f;
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      st[r] = __builtin_amdgcn_exp2f(st[r] - m_new);
      ps += st[r];
    }
    lsum = lsum * alpha + ps;
    if (__ballot(m_new != m) != 0ull) {
#pragma unroll
      for (int dd = 0; dd < 2; ++dd)
#pragma unroll
        for (int r = 0; r < 16; ++r) o[dd][r] *= alpha;
    }
    m = m_new;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const bf16x8 pf = pack8(st, c);
#pragma unroll
      for (int dd = 0; dd < 2; ++dd) o[dd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(lds_v[cur], 32 * dd, c), pf, o[dd], 0, 0, 0);
    }
    if (t + 1 < nt) {
      chunk_store<LDS_ST>(nxt.a, lds_k[cur ^ 1]);
      chunk_store<LDS_TR>(nxt.b, lds_v[cur ^ 1]);
    }
    __syncthreads();
  }
  lsum += __shfl_xor(lsum, 32, 64);
  if (lane < 32 && my_q < p.seq) p.lse[((int64_t)w.b * p.heads + w.h) * p.seq + my_q] = m * 0.6931471805599453f + __logf(lsum);
  store_transposed(stage, o, 1.0f / lsum, p.out, p.ld_out, first, w.r0, p.seq, w.h * DH);
}

// ======================================================================= backward: dQ (and delta)
__global__ __launch_bounds__(256, 4) void k_attn_bwd_dq_mfma(const AttnProb *__restrict__ probs, int n) {
  // K read along its rows (scores), K read transposed (dQ), V; the output block lies over them as in the forward
  constexpr int TILES = 4 * KT * LDS_ST + 2 * KT * LDS_TR;
  static_assert(TILES >= QT * LDS_ST, "the output block fits over the tiles");
  __shared__ __attribute__((aligned(16))) uint16_t lds[TILES];
  uint16_t(*lds_k)[KT * LDS_ST] = (uint16_t(*)[KT * LDS_ST])lds;
  uint16_t(*lds_v)[KT * LDS_ST] = (uint16_t(*)[KT * LDS_ST])(lds + 2 * KT * LDS_ST);
  uint16_t(*lds_kt)[KT * LDS_TR] = (uint16_t(*)[KT * LDS_TR])(lds + 4 * KT * LDS_ST);
  uint16_t *stage = lds;
  const int bid = xcd_contiguous_block();
  const int pi = find_prob(probs, n, bid);
  const AttnProb p = probs[pi];
  const Where w = where(p, bid - p.blk_begin);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d = p.heads * DH;
  const int64_t first = (int64_t)w.b * p.seq;
  const int qcol = w.h * DH, kcol = d + w.h * DH, vcol = 2 * d + w.h * DH;
  const int my_q = w.r0 + wave * 32 + (lane & 31);
  const float scale = rsqrtf((float)DH);
  const int64_t stat = ((int64_t)w.b * p.heads + w.h) * p.seq + my_q;

  const RowFrags qf = load_row_frags(p.qkv, p.ld_qkv, first, my_q, p.seq, qcol);
  const RowFrags gf = load_row_frags(p.dout, p.ld_dout, first, my_q, p.seq, w.h * DH);
  float delta;
  {  // delta = rowsum(dO * O); a lane holds half of its row, its partner (lane ^ 32) the other half
    const RowFrags of = load_row_frags(p.o, p.ld_o, first, my_q, p.seq, w.h * DH);
    float s = 0.0f;
#pragma unroll
    for (int k = 0; k < 4; ++k)
#pragma unroll
      for (int e = 0; e < 8; ++e) s += (float)gf.f[k][e] * (float)of.f[k][e];
    delta = s + __shfl_xor(s, 32, 64);
    if (lane < 32 && my_q < p.seq) p.delta[stat] = delta;
  }
  const float scale2 = scale * 1.4426950408889634f;                              // 1/sqrt(dh) * log2(e)
  const float lse2 = (my_q < p.seq ? p.lse[stat] : 0.0f) * 1.4426950408889634f;   // log-sum-exp in base 2
  f32x16 dq[2] = {zero16(), zero16()};

  const int nt = (p.seq + KT - 1) / KT;
  auto fetch = [&](int t) {
    Stream2 s;
    const int row = t * KT + (threadIdx.x >> 3), cc = (threadIdx.x & 7) * 8;
    s.a = row_chunk(p.qkv, p.ld_qkv, first, row, p.seq, kcol + cc);
    s.b = row_chunk(p.qkv, p.ld_qkv, first, row, p.seq, vcol + cc);
    return s;
  };
  Stream2 nxt = fetch(0);
  auto put = [&](const Stream2 &x, int buf) {
    chunk_store<LDS_ST>(x.a, lds_k[buf]);
    chunk_store<LDS_TR>(x.a, lds_kt[buf]);
    chunk_store<LDS_ST>(x.b, lds_v[buf]);
  };
  put(nxt, 0);
  __syncthreads();
  loads_landed();
  for (int t = 0; t < nt; ++t) {
    const int cur = t & 1;
    if (t + 1 < nt) nxt = fetch(t + 1);
    f32x16 st = zero16(), dp = zero16();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(lds_k[cur], s), qf.f[s], st, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(lds_v[cur], s), gf.f[s], dp, 0, 0, 0);
    }
#pragma unroll
    for (int r = 0; r < 16; ++r) st[r] = __builtin_amdgcn_exp2f(st[r] * scale2 - lse2) * (dp[r] - delta);
    if (t == nt - 1 && (p.seq % KT)) {   // keys beyond a ragged sequence
      asm volatile("");                  // keeps this a branch (as selects it costs an instruction per element in every step)
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (t * KT + acc_row(r) >= p.seq) st[r] = 0.0f;
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const bf16x8 sf = pack8(st, c);
#pragma unroll
      for (int dd = 0; dd < 2; ++dd) dq[dd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(tr_frag(lds_kt[cur], 32 * dd, c), sf, dq[dd], 0, 0, 0);
    }
    if (t + 1 < nt) put(nxt, cur ^ 1);
    __syncthreads();
  }
  store_transposed(stage, dq, scale, p.out, p.ld_out, first, w.r0, p.seq, w.h * DH);
}

// ======================================================================= backward: dK, dV
// 220 registers per lane leave two waves per SIMD, too few to hide one wave's chain (LDS reads -> score products ->
// exponentials -> gradient products) behind another's.  The loop is therefore software-pipelined inside the wave:
// the score products of query tile t + 1 are issued BEFORE the exponentials of tile t and run on the matrix pipe
// under them; the gradient products of tile t run under the next iteration's loads and exponentials.  Tile t + 1 is
// read while tile t is still needed and tile t + 2 is being written: three LDS buffers.  Loads and LDS writes past
// the last tile are not skipped but clamped to the last query row (finite values in a buffer nobody reads, products
// nobody uses): the loop body has no branches, so every wait in it is for exactly the loads it needs.
__global__ __launch_bounds__(256, 2) void k_attn_bwd_dkv_mfma(const AttnProb *__restrict__ probs, int n) {
  constexpr int NB = 3;
  __shared__ __attribute__((aligned(16))) uint16_t lds_q[NB][KT * LDS_ST], lds_g[NB][KT * LDS_ST];     // read along rows
  __shared__ __attribute__((aligned(16))) uint16_t lds_qt[NB][KT * LDS_TR], lds_gt[NB][KT * LDS_TR];   // read transposed
  __shared__ float lds_lse[NB][KT], lds_delta[NB][KT];
  const int bid = xcd_contiguous_block();
  const int pi = find_prob(probs, n, bid);
  const AttnProb p = probs[pi];
  const Where w = where(p, bid - p.blk_begin);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int d = p.heads * DH;
  const int64_t first = (int64_t)w.b * p.seq;
  const int qcol = w.h * DH, kcol = d + w.h * DH, vcol = 2 * d + w.h * DH;
  const int my_k = w.r0 + wave * 32 + (lane & 31);
  const float scale = rsqrtf((float)DH), scale2 = scale * 1.4426950408889634f;
  const int64_t stat0 = ((int64_t)w.b * p.heads + w.h) * p.seq;

  const RowFrags kf = load_row_frags(p.qkv, p.ld_qkv, first, my_k, p.seq, kcol);
  const RowFrags vf = load_row_frags(p.qkv, p.ld_qkv, first, my_k, p.seq, vcol);
  f32x16 dk[2] = {zero16(), zero16()}, dv[2] = {zero16(), zero16()};

  const int nt = (p.seq + KT - 1) / KT;
  float n_lse = 0.0f, n_delta = 0.0f;
  auto fetch = [&](int t) {   // (rows beyond the sequence: the last row, see row_chunk)
    Stream2 s;
    const int row = t * KT + (threadIdx.x >> 3), cc = (threadIdx.x & 7) * 8;
    s.a = row_chunk(p.qkv, p.ld_qkv, first, row, p.seq, qcol + cc);
    s.b = row_chunk(p.dout, p.ld_dout, first, row, p.seq, w.h * DH + cc);
    // (the statistics: plain loads whose values are first touched in put(), so that nothing waits for them here)
    const int q = min(t * KT + (int)(threadIdx.x & (KT - 1)), p.seq - 1);
    n_lse = p.lse[stat0 + q];
    n_delta = p.delta[stat0 + q];
    return s;
  };
  auto put = [&](const Stream2 &s, int buf) {
    chunk_store<LDS_ST>(s.a, lds_q[buf]);
    chunk_store<LDS_TR>(s.a, lds_qt[buf]);
    chunk_store<LDS_ST>(s.b, lds_g[buf]);
    chunk_store<LDS_TR>(s.b, lds_gt[buf]);
    if (threadIdx.x < KT) {
      lds_lse[buf][threadIdx.x] = n_lse * 1.4426950408889634f;   // base 2
      lds_delta[buf][threadIdx.x] = n_delta;
    }
  };
  // S = Q K^T and dP = dO V^T of the tile in `buf`: rows = queries of the tile, lane column = this lane's key
  auto scores = [&](int buf, f32x16 &st, f32x16 &dp) {
    st = zero16();
    dp = zero16();
#pragma unroll
    for (int s = 0; s < 4; ++s) {
      st = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(lds_q[buf], s), kf.f[s], st, 0, 0, 0);
      dp = __builtin_amdgcn_mfma_f32_32x32x16_bf16(row_frag(lds_g[buf], s), vf.f[s], dp, 0, 0, 0);
    }
  };
  // probabilities and score gradients of tile t (in `buf`) from its products, then dV += P^T dO, dK += dS^T Q
  auto gradients = [&](int t, int buf, f32x16 &st, f32x16 &dp) {
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      const int qi = acc_row(r);
      st[r] = __builtin_amdgcn_exp2f(st[r] * scale2 - lds_lse[buf][qi]);
      dp[r] = st[r] * (dp[r] - lds_delta[buf][qi]);
    }
    if (t == nt - 1 && (p.seq % KT)) {   // queries beyond a ragged sequence (uniform, last tile only)
      asm volatile("");                  // keeps this a branch: as selects it costs three instructions per element in EVERY step
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (t * KT + acc_row(r) >= p.seq) st[r] = dp[r] = 0.0f;
    }
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const bf16x8 pf = pack8(st, c), sf = pack8(dp, c);
#pragma unroll
      for (int dd = 0; dd < 2; ++dd) {
        dv[dd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(pf, tr_frag(lds_gt[buf], 32 * dd, c), dv[dd], 0, 0, 0);
        dk[dd] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(sf, tr_frag(lds_qt[buf], 32 * dd, c), dk[dd], 0, 0, 0);
      }
    }
  };
  // one step: tile t's products are in (st, dp); tile t + 1's go to (st_n, dp_n); tile t + 2 comes in
  auto step = [&](int t, int b_cur, int b_nxt, int b_in, f32x16 &st, f32x16 &dp, f32x16 &st_n, f32x16 &dp_n) {
    const Stream2 in = fetch(t + 2);
    scores(b_nxt, st_n, dp_n);
    __builtin_amdgcn_sched_barrier(0);     // the score products go out before the exponentials, not after them
    gradients(t, b_cur, st, dp);
    put(in, b_in);                         // over tile t - 1, which every wave left at the last barrier
    __syncthreads();
  };

  put(fetch(0), 0);
  put(fetch(1), 1);
  __syncthreads();
  loads_landed();
  f32x16 st_a, dp_a, st_b, dp_b;
  scores(0, st_a, dp_a);
  int b0 = 0, b1 = 1, b2 = 2;              // buffers of tiles t, t + 1, t + 2
  int t = 0;
  for (; t + 1 < nt; t += 2) {
    step(t, b0, b1, b2, st_a, dp_a, st_b, dp_b);
    step(t + 1, b1, b2, b0, st_b, dp_b, st_a, dp_a);
    const int o0 = b0;
    b0 = b2;
    b2 = b1;
    b1 = o0;
  }
  if (t < nt) step(t, b0, b1, b2, st_a, dp_a, st_b, dp_b);
  // dk/dv: rows = this wave's keys (accumulator rows), lane column = dh.  Stored straight from the registers that is
  // 64 two-byte stores per lane; instead each wave turns its two 32 x 64 blocks in LDS (the transposed-read tiles are
  // dead after the loop's last barrier; a wave's 32 rows of stride LDS_ST take a quarter of one array) and writes
  // whole 16-byte pieces of rows.
  static_assert(sizeof(lds_qt) >= 4 * 32 * LDS_ST * sizeof(uint16_t), "a block per wave fits the dead tiles");
  uint16_t *blk_k = &lds_qt[0][0] + wave * 32 * LDS_ST, *blk_v = &lds_gt[0][0] + wave * 32 * LDS_ST;
#pragma unroll
  for (int dd = 0; dd < 2; ++dd)
#pragma unroll
    for (int r = 0; r < 16; ++r) {
      blk_k[acc_row(r) * LDS_ST + 32 * dd + (lane & 31)] = f32_to_bf16_bits(dk[dd][r] * scale);
      blk_v[acc_row(r) * LDS_ST + 32 * dd + (lane & 31)] = f32_to_bf16_bits(dv[dd][r]);
    }
  GPP_G uint16_t *out = (GPP_G uint16_t *)p.out;
#pragma unroll
  for (int c = lane; c < 32 * (DH / 8); c += 64) {
    const int row = c >> 3, cc = (c & 7) * 8, key = w.r0 + wave * 32 + row;
    if (key >= p.seq) continue;
    const int64_t ro = (first + key) * p.ld_out + w.h * DH + cc;
    *(GPP_G u32x4 *)(out + ro + d) = *(const u32x4 *)(blk_k + row * LDS_ST + cc);
    *(GPP_G u32x4 *)(out + ro + 2 * d) = *(const u32x4 *)(blk_v + row * LDS_ST + cc);
  }
}

void launch_attn_fwd_mfma(const AttnProb *probs, int n, int total_blocks, hipStream_t s) {
  if (total_blocks > 0) hipLaunchKernelGGL(k_attn_fwd_mfma, dim3(total_blocks), dim3(256), 0, s, probs, n);
}
void launch_attn_bwd_dq_mfma(const AttnProb *probs, int n, int total_blocks, hipStream_t s) {
  if (total_blocks > 0) hipLaunchKernelGGL(k_attn_bwd_dq_mfma, dim3(total_blocks), dim3(256), 0, s, probs, n);
}
void launch_attn_bwd_dkv_mfma(const AttnProb *probs, int n, int total_blocks, hipStream_t s) {
  if (total_blocks > 0) hipLaunchKernelGGL(k_attn_bwd_dkv_mfma, dim3(total_blocks), dim3(256), 0, s, probs, n);
}

}  // namespace gpp
