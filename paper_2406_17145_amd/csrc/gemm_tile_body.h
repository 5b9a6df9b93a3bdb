// Device-side body of the tiled bf16 MFMA GEMM (v_mfma_f32_32x32x16_bf16, fp32
// accumulation, LDS-staged tiles, register ring of k-steps in flight).  It is a
// function of (record, tile index, thread index in a 256-thread team, LDS block)
// so that one kernel can run it stand-alone and another can run two teams side
// by side in a 512-thread workgroup next to other roles.
//
// Three forms share the body.  What differs is which dimension of an operand is
// contiguous in memory:
//   FWD  C[m,n] = sum_k X[m,k] W[n,k]      A k-contiguous,  B k-contiguous
//   DX   C[m,k] = sum_n dZ[m,n] W[n,k]     A k-contiguous,  B row = contraction index
//   DW   C[n,k] += sum_m dZ[m,n] X[m,k]    A and B: row = contraction index
// Operands whose rows run along the contraction index are stored in LDS as they
// are in memory and fetched with the transposing LDS read (ds_read_b64_tr_b16),
// which hands each lane four consecutive contraction steps of its own
// row/column, exactly what the MFMA operand layout wants.
#pragma once
#include "device_utils.h"

namespace gpp {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) short s16x4;
typedef __attribute__((ext_vector_type(8))) short s16x8;
typedef __attribute__((ext_vector_type(16))) float f32x16;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int BK = 32;        // contraction elements per k-step
constexpr int PAD = 8;        // LDS row padding (elements) of k-contiguous tiles: 80-byte rows, conflict-free b128 reads
constexpr int PAD_TR = 32;    // padding of contraction-row tiles: the four rows a 16-lane block of the transposing
                              // read touches then start 16 banks apart (measured: halves LDS bank-conflict cycles)

__host__ __device__ constexpr int cdiv(int a, int b) { return (a + b - 1) / b; }

// the caller's buffer when the record's result goes straight to a per-call pointer
__device__ __forceinline__ void *result_ptr(const GemmProb &p, const ExtPtrs &ext) {
  return p.c_ext > 0 ? ext.p[p.c_ext - 1] : p.C;
}

// ---- global -> register tile fetch -------------------------------------------
// A tile is ROWS x COLS elements, COLS contiguous in memory; each thread of the
// 256-thread team owns 16-byte chunks (8 elements).  Out-of-range rows / columns read as zero.
template <int ROWS, int COLS>
struct TileRegs {
  static constexpr int CHUNKS = ROWS * COLS / 8;
  static constexpr int PER_THREAD = (CHUNKS + 255) / 256;
  u32x4 v[PER_THREAD];
};

// ---- branch-free 16-byte operand loads -------------------------------------------------
// Operands are read through buffer descriptors: an offset beyond the descriptor's size returns zeros,
// so rows and chunks outside the matrix need no branch (a branch around a load makes the compiler
// wait for earlier loads in between, which exposes the memory latency once per load).
constexpr uint32_t OOB_OFFSET = 0xfffffff0u;   // beyond any descriptor's size

// bytes from the first to the last valid element of a [rows x width] bf16 matrix with row stride ld
// (it may be a column slice of a wider buffer); the descriptor holds 32 bits
__device__ __forceinline__ uint32_t matrix_bytes(int rows, int64_t ld, int width) {
  const int64_t b = ((int64_t)(rows - 1) * ld + ((width + 7) & ~7)) * 2;   // whole 16-byte chunks (ld is a multiple of 8)
  return (uint32_t)(b < 0xffffff00ll ? b : 0xffffff00ll);
}
__device__ __forceinline__ __amdgpu_buffer_rsrc_t matrix_rsrc(const void *base, int rows, int64_t ld, int width) {
  return __builtin_amdgcn_make_buffer_rsrc((void *)base, 0, matrix_bytes(rows, ld, width), 0x00020000);
}
// 8 consecutive elements of row r starting at column c; zero when r >= row_lim or c >= col_lim
__device__ __forceinline__ u32x4 chunk_load(__amdgpu_buffer_rsrc_t rs, int64_t ld, int r, int c, int row_lim, int col_lim) {
  const uint32_t oob = (uint32_t)-(int32_t)((r >= row_lim) | (c >= col_lim)) & OOB_OFFSET;
  return __builtin_amdgcn_raw_buffer_load_b128(rs, (uint32_t)(((int64_t)r * ld + c) * 2) | oob, 0, 0);
}
// clears the elements at columns >= col_lim of a chunk that starts at column c (only matrices whose
// width is not a multiple of 8 need it: the rest of such a chunk is row padding)
__device__ __forceinline__ u32x4 chunk_clear_tail(u32x4 v, int c, int col_lim) {
  const int keep = col_lim - c;
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    const uint32_t lo = 2 * e < keep ? 0x0000ffffu : 0u, hi = 2 * e + 1 < keep ? 0xffff0000u : 0u;
    v[e] &= lo | hi;
  }
  return v;
}

// ---- global -> register tile fetch -------------------------------------------
// (rows [row0, ..) x columns [col0, ..) of the operand behind `rs`; `ragged`: col_lim is not a multiple of 8)
template <int ROWS, int COLS>
__device__ __forceinline__ void tile_fetch(TileRegs<ROWS, COLS> &t, __amdgpu_buffer_rsrc_t rs, int64_t ld, int row0, int col0,
                                           int row_lim, int col_lim, bool ragged, int tid) {
  constexpr int CPR = COLS / 8;  // chunks per row
#pragma unroll
  for (int q = 0; q < TileRegs<ROWS, COLS>::PER_THREAD; ++q) {
    const int c = tid + 256 * q;
    const int r = row0 + c / CPR, cc = col0 + (c % CPR) * 8;
    // a thread without a chunk in a partial last round reads out of range
    const bool mine = TileRegs<ROWS, COLS>::CHUNKS % 256 == 0 || c < TileRegs<ROWS, COLS>::CHUNKS;
    t.v[q] = chunk_load(rs, ld, r, cc, mine ? row_lim : 0, col_lim);
  }
  if (ragged) {
#pragma unroll
    for (int q = 0; q < TileRegs<ROWS, COLS>::PER_THREAD; ++q) {
      const int c = tid + 256 * q;
      t.v[q] = chunk_clear_tail(t.v[q], col0 + (c % CPR) * 8, col_lim);
    }
  }
}

template <int ROWS, int COLS>
__device__ __forceinline__ void tile_store_lds(const TileRegs<ROWS, COLS> &t, uint16_t *lds, int tid) {
  constexpr int CPR = COLS / 8;
  constexpr int STRIDE = COLS + (COLS == BK ? PAD : PAD_TR);
#pragma unroll
  for (int q = 0; q < TileRegs<ROWS, COLS>::PER_THREAD; ++q) {
    const int c = tid + 256 * q;
    if (TileRegs<ROWS, COLS>::CHUNKS % 256 == 0 || c < TileRegs<ROWS, COLS>::CHUNKS)
      *(u32x4 *)(lds + (c / CPR) * STRIDE + (c % CPR) * 8) = t.v[q];
  }
}

// ---- LDS -> MFMA operand ---------------------------------------------------------
// k-contiguous tile [rows][BK + PAD]: lane l takes row (l % 32), 8 k-values at 8 * (l / 32)
__device__ __forceinline__ bf16x8 frag_kmajor(const uint16_t *lds, int row0, int k0) {
  const int l = threadIdx.x & 63;
  return *(const bf16x8 *)(lds + (row0 + (l & 31)) * (BK + PAD) + k0 + 8 * (l >> 5));
}
// contraction-row tile [BK][cols + PAD_TR]: transposing read.  In each block of 16 lanes, lane q
// addresses row (q / 4) at columns 4 * (q % 4) .. +3 and receives rows 0..3 of column q.
template <int COLS>
__device__ __forceinline__ bf16x8 frag_tr(const uint16_t *lds, int col0, int k0) {
  const int l = threadIdx.x & 63;
  const int blk = l >> 4, q = l & 15;
  const uint16_t *p = lds + (k0 + 8 * (blk >> 1) + (q >> 2)) * (COLS + PAD_TR) + col0 + 16 * (blk & 1) + 4 * (q & 3);
  typedef __attribute__((address_space(3))) s16x4 lds_v4;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)p);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p + 4 * (COLS + PAD_TR)));
  s16x8 v = __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7);
  return __builtin_bit_cast(bf16x8, v);
}

// Split-K partial sums cross workgroups (and XCDs, whose L2 caches are not coherent with each other
// inside a kernel).  They are written and read with device-scope relaxed atomics, which go through
// to memory instead of staying in the writer's L2, so no cache-wide write-back or invalidate is
// needed: ordering comes from waiting for the stores' acknowledgements before the ticket is taken.
__device__ __forceinline__ void put_partial(float *p, float v) {
  __hip_atomic_store(p, v, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
__device__ __forceinline__ float get_partial(const float *p) {
  return __hip_atomic_load(p, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
}
// After a workgroup's put_partial stores and before one of its threads takes the tile's ticket: every wave waits
// until its own stores have been acknowledged (s_waitcnt vmcnt(0); stores count there), then the workgroup meets.
// A workgroup-scope release fence alone compiles to no wait for stores: it orders them for the waves of this
// compute unit only, and the ticket could overtake partial tiles that are still on their way to memory, where
// the last workgroup, on another compute unit, reads them.
__device__ __forceinline__ void partials_published() {
  __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
  __builtin_amdgcn_s_waitcnt(0x0F70);
  __syncthreads();
}

// ---- epilogue of one 32 x 32 accumulator tile, in two phases -----------------------------
// Register r of the tile holds row row0 + 8 * (r / 4) + r % 4 (row0 already includes this lane's
// 4 * (lane / 32)) of column `col`.  Everything that does not depend on r (which optional operands
// exist, the activation, the storage types, the 64-bit base addresses) is decided once per tile, so
// the sixteen elements cost a handful of instructions each.  CHECK = false: the tile is known to lie
// inside the matrix.
// Phase 1 (epi_fetch) issues the loads a tile's epilogue needs -- residual / gradient addend, the
// stashed activation derivative, the old gradient of a backward-weight tile -- and phase 2
// (epi_finish) consumes them, so a caller can fetch tile t + 1 before it finishes tile t and the
// memory latency is paid once per workgroup, not once per tile.
struct EpiIn {
  f32x16 a;   // DX: stashed derivative / mask source; DW: old gradient values
  f32x16 r;   // FWD: residual addend; DX: gradient addend
};
__device__ __forceinline__ float elem_load(const void *base, int32_t dtype, int64_t at) {
  return dtype == DT_BF16 ? bf16_bits_to_f32(((const uint16_t *)base)[at]) : ((const float *)base)[at];
}
__device__ __forceinline__ int epi_row(int r) { return 8 * (r >> 2) + (r & 3); }

template <int FORM, bool CHECK>
__device__ __forceinline__ void epi_fetch(const GemmProb &p, const void *Cout, int row0, int col, int accumulate_dw, EpiIn &in) {
  const bool col_ok = !CHECK || col < p.N;
  if (FORM != FORM_DW && p.res) {
    const int64_t base = (int64_t)row0 * p.ldres + col;
    const int ld = (int)p.ldres;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      in.r[r] = (col_ok && (!CHECK || row0 + epi_row(r) < p.M)) ? elem_load(p.res, p.res_dtype, base + epi_row(r) * ld) : 0.0f;
  }
  if (FORM == FORM_DX && p.act != ACT_NONE) {
    const int64_t base = (int64_t)row0 * p.ldaux + col;
    const int ld = (int)p.ldaux;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      in.a[r] = (col_ok && (!CHECK || row0 + epi_row(r) < p.M)) ? elem_load(p.aux, p.aux_dtype, base + epi_row(r) * ld) : 0.0f;
  }
  if (FORM == FORM_DW && accumulate_dw) {
    const float *c = (const float *)Cout + (int64_t)row0 * p.ldc + col;
    const int ld = (int)p.ldc;
#pragma unroll
    for (int r = 0; r < 16; ++r) in.a[r] = (col_ok && (!CHECK || row0 + epi_row(r) < p.M)) ? c[epi_row(r) * ld] : 0.0f;
  }
}

template <int FORM, bool CHECK>
__device__ __forceinline__ void epi_finish(const GemmProb &p, void *Cout, const f32x16 &acc, int row0, int col,
                                           int accumulate_dw, const EpiIn &in) {
  if (CHECK && col >= p.N) return;
  float v[16];
  bool ok[16];
  int ro[16];   // row offsets from row0
#pragma unroll
  for (int r = 0; r < 16; ++r) {
    v[r] = acc[r];
    ro[r] = epi_row(r);
    ok[r] = !CHECK || row0 + ro[r] < p.M;
  }
  const int64_t cbase = (int64_t)row0 * p.ldc + col;
  const int ldc = (int)p.ldc;
  if (FORM == FORM_FWD) {
    if (p.bias) {
      const float b = p.bias[col];
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] += b;
    }
    if (p.act == ACT_RELU) {
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = v[r] > 0.0f ? v[r] : 0.0f;
    } else if (p.act == ACT_GELU) {
      float d[16];   // derivative at the pre-activation: what the backward pass multiplies by
#pragma unroll
      for (int r = 0; r < 16; ++r) gelu_both(v[r], v[r], d[r]);
      if (p.aux) {
        const int64_t abase = (int64_t)row0 * p.ldaux + col;
        const int lda = (int)p.ldaux;
        if (p.aux_dtype == DT_BF16) {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (ok[r]) ((uint16_t *)p.aux)[abase + ro[r] * lda] = f32_to_bf16_bits(d[r]);
        } else {
#pragma unroll
          for (int r = 0; r < 16; ++r)
            if (ok[r]) ((float *)p.aux)[abase + ro[r] * lda] = d[r];
        }
      }
    }
  }
  if (FORM != FORM_DW && p.res) {   // forward: residual addend; backward-data: gradient addend
#pragma unroll
    for (int r = 0; r < 16; ++r) v[r] += in.r[r];
  }
  if (FORM == FORM_DX && p.act != ACT_NONE) {
    if (p.act == ACT_RELU) {
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] = in.a[r] > 0.0f ? v[r] : 0.0f;
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r) v[r] *= in.a[r];   // stashed derivative
    }
  }
  if (FORM == FORM_DW) {
    float *c = (float *)Cout + cbase;
    if (accumulate_dw) {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (ok[r]) c[ro[r] * ldc] = in.a[r] + v[r];
    } else {
#pragma unroll
      for (int r = 0; r < 16; ++r)
        if (ok[r]) c[ro[r] * ldc] = v[r];
    }
  } else if (p.c_dtype == DT_BF16) {
    uint16_t *c = (uint16_t *)Cout + cbase;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (ok[r]) c[ro[r] * ldc] = f32_to_bf16_bits(v[r]);
  } else {
    float *c = (float *)Cout + cbase;
#pragma unroll
    for (int r = 0; r < 16; ++r)
      if (ok[r]) c[ro[r] * ldc] = v[r];
  }
}

// all TI x TJ accumulator tiles of a wave (wave tile origin wr0 x wc0), the fetch of tile t + 1
// issued before tile t is finished
template <int FORM, bool CHECK, int TI, int TJ>
__device__ __forceinline__ void epilogue_wave(const GemmProb &p, void *Cout, const f32x16 (&acc)[TI][TJ], int wr0, int wc0,
                                              int lane, int accumulate_dw) {
  EpiIn in[2];
  auto origin = [&](int t, int &row0, int &col) {
    row0 = wr0 + 32 * (t / TJ) + 4 * (lane >> 5);
    col = wc0 + 32 * (t % TJ) + (lane & 31);
  };
  int row0, col;
  origin(0, row0, col);
  epi_fetch<FORM, CHECK>(p, Cout, row0, col, accumulate_dw, in[0]);
#pragma unroll
  for (int t = 0; t < TI * TJ; ++t) {
    if (t + 1 < TI * TJ) {
      origin(t + 1, row0, col);
      epi_fetch<FORM, CHECK>(p, Cout, row0, col, accumulate_dw, in[(t + 1) & 1]);
    }
    origin(t, row0, col);
    epi_finish<FORM, CHECK>(p, Cout, acc[t / TJ][t % TJ], row0, col, accumulate_dw, in[t & 1]);
  }
}

// ---- epilogue through LDS: whole rows instead of accumulator columns ------------------------
// The accumulator layout gives a lane ONE column and sixteen rows of a 32 x 32 tile, so an epilogue
// that works on it touches memory in 2-byte (bf16) pieces, sixteen rows apart.  Here a wave passes
// its tile through a private LDS block, 32 rows x (32 TJ) columns at a time, and reads it back row-wise:
// a lane then owns 8 consecutive columns of a row, every optional operand (residual / gradient
// addend, stashed derivative or mask source, old gradient) is one or two 16-byte loads, the result
// one 16-byte store (two for fp32), and the loads of a 32-row block are all requested before the
// first is used.  For tiles that lie inside the matrix, with 16-byte aligned rows everywhere.
constexpr int EPI_LDS_PAD = 4;   // floats: keeps rows 16-byte aligned and spreads them over the banks
template <int TJ>
constexpr int epi_lds_floats() { return 32 * (32 * TJ + EPI_LDS_PAD); }

__device__ __forceinline__ bool epi_lds_ok(const GemmProb &p, const void *Cout, int form) {
  if ((p.ldc & 7) || ((uintptr_t)Cout & 15)) return false;
  if (form == FORM_DW) return true;                       // fp32 result, no optional operands
  if (p.c_dtype != DT_BF16) return false;
  if (p.res && (p.res_dtype != DT_BF16 || (p.ldres & 7) || ((uintptr_t)p.res & 15))) return false;
  if (p.aux && (p.aux_dtype != DT_BF16 || (p.ldaux & 7) || ((uintptr_t)p.aux & 15))) return false;
  if (form == FORM_FWD && p.bias && ((uintptr_t)p.bias & 15)) return false;
  return true;
}
__device__ __forceinline__ void unpack_bf16x8(const u32x4 &u, float (&v)[8]) {
#pragma unroll
  for (int e = 0; e < 4; ++e) {
    v[2 * e] = __uint_as_float(u[e] << 16);
    v[2 * e + 1] = __uint_as_float(u[e] & 0xffff0000u);
  }
}
__device__ __forceinline__ u32x4 pack_bf16x8(const float (&v)[8]) {
  u32x4 u;
#pragma unroll
  for (int e = 0; e < 4; ++e) u[e] = (uint32_t)f32_to_bf16_bits(v[2 * e]) | ((uint32_t)f32_to_bf16_bits(v[2 * e + 1]) << 16);
  return u;
}

template <int FORM, int TI, int TJ>
__device__ __forceinline__ void epilogue_wave_lds(const GemmProb &p, void *Cout, const f32x16 (&acc)[TI][TJ], int wr0, int wc0,
                                                  int lane, int accumulate_dw, float *stage) {
  constexpr int COLS = 32 * TJ, ST = COLS + EPI_LDS_PAD;
  constexpr int LPR = COLS / 8, RPI = 64 / LPR, ITS = 32 / RPI;   // lanes per row, rows per step, steps per block
  const int rl = lane / LPR, c8 = (lane % LPR) * 8;
  const int col = wc0 + c8;
  float bias[8] = {};
  if (FORM == FORM_FWD && p.bias) {
    const float4 b0 = *(const float4 *)(p.bias + col), b1 = *(const float4 *)(p.bias + col + 4);
    bias[0] = b0.x; bias[1] = b0.y; bias[2] = b0.z; bias[3] = b0.w;
    bias[4] = b1.x; bias[5] = b1.y; bias[6] = b1.z; bias[7] = b1.w;
  }
  const bool use_res = FORM != FORM_DW && p.res != nullptr;
  const bool aux_in = FORM == FORM_DX && p.act != ACT_NONE;          // stashed derivative / mask source is read
  const bool aux_out = FORM == FORM_FWD && p.act == ACT_GELU && p.aux != nullptr;   // derivative is stashed
  // an absent bf16 operand is read from the result buffer instead (valid memory, value unused), so
  // that the loads of a block carry no branch
  // (with a row stride of zero: every row reads the same few lines of the result's first row, which stay in the
  // cache -- the loads cost no memory traffic)
  const uint16_t *resp = use_res ? (const uint16_t *)p.res : (const uint16_t *)Cout;
  const uint16_t *auxp = aux_in ? (const uint16_t *)p.aux : (const uint16_t *)Cout;
  const int64_t ldr = use_res ? p.ldres : 0, lda = aux_in ? p.ldaux : 0;
#pragma unroll
  for (int i = 0; i < TI; ++i) {
    // accumulators of the 32-row block -> LDS, in their own layout (a half-wave writes 32 consecutive floats)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) stage[(epi_row(r) + 4 * (lane >> 5)) * ST + 32 * j + (lane & 31)] = acc[i][j][r];
    __builtin_amdgcn_wave_barrier();
    const int row0 = wr0 + 32 * i + rl;
    if (FORM == FORM_DW) {
      float4 old[ITS][2];
      float *c = (float *)Cout + (int64_t)row0 * p.ldc + col;
      if (accumulate_dw) {
#pragma unroll
        for (int t = 0; t < ITS; ++t) {
          old[t][0] = *(const float4 *)(c + (int64_t)t * RPI * p.ldc);
          old[t][1] = *(const float4 *)(c + (int64_t)t * RPI * p.ldc + 4);
        }
      }
#pragma unroll
      for (int t = 0; t < ITS; ++t) {
        float4 v0 = *(const float4 *)(stage + (rl + RPI * t) * ST + c8), v1 = *(const float4 *)(stage + (rl + RPI * t) * ST + c8 + 4);
        if (accumulate_dw) {
          v0 = make_float4(old[t][0].x + v0.x, old[t][0].y + v0.y, old[t][0].z + v0.z, old[t][0].w + v0.w);
          v1 = make_float4(old[t][1].x + v1.x, old[t][1].y + v1.y, old[t][1].z + v1.z, old[t][1].w + v1.w);
        }
        *(float4 *)(c + (int64_t)t * RPI * p.ldc) = v0;
        *(float4 *)(c + (int64_t)t * RPI * p.ldc + 4) = v1;
      }
    } else {
      u32x4 res_raw[ITS], aux_raw[ITS];
#pragma unroll
      for (int t = 0; t < ITS; ++t) {
        res_raw[t] = *(const u32x4 *)(resp + (int64_t)(row0 + RPI * t) * ldr + col);
        aux_raw[t] = *(const u32x4 *)(auxp + (int64_t)(row0 + RPI * t) * lda + col);
      }
#pragma unroll
      for (int t = 0; t < ITS; ++t) {
        float v[8], rs[8], ax[8], d[8];
        {
          const float4 a = *(const float4 *)(stage + (rl + RPI * t) * ST + c8), b = *(const float4 *)(stage + (rl + RPI * t) * ST + c8 + 4);
          v[0] = a.x; v[1] = a.y; v[2] = a.z; v[3] = a.w; v[4] = b.x; v[5] = b.y; v[6] = b.z; v[7] = b.w;
        }
        unpack_bf16x8(res_raw[t], rs);
        unpack_bf16x8(aux_raw[t], ax);
        if (FORM == FORM_FWD) {
#pragma unroll
          for (int e = 0; e < 8; ++e) v[e] += bias[e];
          if (p.act == ACT_RELU) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] = v[e] > 0.0f ? v[e] : 0.0f;
          } else if (p.act == ACT_GELU) {
#pragma unroll
            for (int e = 0; e < 8; ++e) gelu_both(v[e], v[e], d[e]);
            if (aux_out) *(u32x4 *)((uint16_t *)p.aux + (int64_t)(row0 + RPI * t) * p.ldaux + col) = pack_bf16x8(d);
          }
          if (use_res) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += rs[e];
          }
        } else {
          if (use_res) {
#pragma unroll
            for (int e = 0; e < 8; ++e) v[e] += rs[e];
          }
          if (aux_in) {
            if (p.act == ACT_RELU) {
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] = ax[e] > 0.0f ? v[e] : 0.0f;
            } else {
#pragma unroll
              for (int e = 0; e < 8; ++e) v[e] *= ax[e];
            }
          }
        }
        *(u32x4 *)((uint16_t *)Cout + (int64_t)(row0 + RPI * t) * p.ldc + col) = pack_bf16x8(v);
      }
    }
    __builtin_amdgcn_wave_barrier();   // the block is free again
  }
}

// LDS elements (uint16) one 256-thread team needs: both operands, double buffered
template <int FORM, int BM, int BN>
struct TileLds {
  static constexpr bool A_TR = FORM == FORM_DW;
  static constexpr bool B_TR = FORM != FORM_FWD;
  static constexpr int A_ELEMS = A_TR ? BK * (BM + PAD_TR) : BM * (BK + PAD);
  static constexpr int B_ELEMS = B_TR ? BK * (BN + PAD_TR) : BN * (BK + PAD);
  static constexpr int ELEMS = 2 * (A_ELEMS + B_ELEMS);
};

// ---- the body -----------------------------------------------------------------------
// `local`  index of this team's unit of work inside the record: tile * split_k + split
// `tid`    thread index inside the 256-thread team (0..255)
// `lds`    TileLds<FORM,BM,BN>::ELEMS elements, private to the team
// Every team of a workgroup must call with records of the same K range: the body synchronises with
// workgroup barriers.  A `local` beyond the record's tiles computes on zeros and stores nothing.
// SPLIT = false ignores the record's split_k (taken as 1).  RING = k-steps kept in flight in
// registers (even; 0 picks the default for the tile size).  EARLY_OLD (backward-weight): request the
// old gradient tile before the k-loop instead of in the epilogue -- worth its registers when the
// contraction is short and the tile's time is mostly that round trip.
template <int FORM, int BM, int BN, bool SPLIT, int RING = 0, bool EARLY_OLD = false>
__device__ __forceinline__ void gemm_tile_body(const GemmProb &p, int local, int tid, uint16_t *lds, int accumulate_dw,
                                               const ExtPtrs &ext) {
  constexpr bool A_TR = TileLds<FORM, BM, BN>::A_TR;     // A rows run along the contraction index
  constexpr bool B_TR = TileLds<FORM, BM, BN>::B_TR;
  constexpr int WM = BM / 2, WN = BN / 2;                 // 2 x 2 waves
  constexpr int TI = WM / 32, TJ = WN / 32;               // 32x32 MFMA tiles per wave
  constexpr int A_ELEMS = TileLds<FORM, BM, BN>::A_ELEMS;
  constexpr int B_ELEMS = TileLds<FORM, BM, BN>::B_ELEMS;
  uint16_t *lds_a[2] = {lds, lds + A_ELEMS};
  uint16_t *lds_b[2] = {lds + 2 * A_ELEMS, lds + 2 * A_ELEMS + B_ELEMS};

  // split-K: `split` teams with consecutive ids share one output tile, each sums a slice of K
  const int S = SPLIT ? p.split_k : 1, split = local % S;
  const int tile = local / S;
  const int kslice = cdiv(cdiv(p.K, BK), S) * BK;
  const int k_begin = split * kslice, k_end = min(p.K, k_begin + kslice);
  const int tiles_m = cdiv(p.M, BM);
  const int m0 = (tile % tiles_m) * BM, n0 = (tile / tiles_m) * BN;   // consecutive tiles share the B panel
  const int wave = tid >> 6, lane = tid & 63;
  const int wi0 = (wave >> 1) * WM, wj0 = (wave & 1) * WN;
  // operand descriptors: FWD A = X [M x K], B = W [N x K]; DX A = dZ [M x K], B = W [K x N];
  // DW A = dZ [K x M], B = X [K x N]  (K = contraction length)
  const __amdgpu_buffer_rsrc_t rs_a = matrix_rsrc(p.A, A_TR ? p.K : p.M, p.lda, A_TR ? p.M : p.K);
  const __amdgpu_buffer_rsrc_t rs_b = matrix_rsrc(p.B, B_TR ? p.K : p.N, p.ldb, B_TR ? p.N : p.K);
  const bool ragged_a = ((A_TR ? p.M : p.K) & 7) != 0, ragged_b = ((B_TR ? p.N : p.K) & 7) != 0;
  void *Cout = FORM == FORM_DW ? p.C : result_ptr(p, ext);

  f32x16 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  const bool early_old = EARLY_OLD && FORM == FORM_DW && accumulate_dw && Cout != nullptr;
  f32x16 c_old[TI][TJ];
  if (EARLY_OLD && early_old) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) {
        const int col = n0 + wj0 + 32 * j + (lane & 31);
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          const int row = m0 + wi0 + 32 * i + 4 * (lane >> 5) + epi_row(r);
          c_old[i][j][r] = (row < p.M && col < p.N) ? ((const float *)Cout)[(int64_t)row * p.ldc + col] : 0.0f;
        }
      }
  }
  typedef TileRegs<A_TR ? BK : BM, A_TR ? BM : BK> RegsA;
  typedef TileRegs<B_TR ? BK : BN, B_TR ? BN : BK> RegsB;
  // NS k-steps are kept in flight in registers: the tile consumed at step kt was requested NS-1
  // steps earlier, so the k-loop runs at the rate of its own work, not of the memory latency
  constexpr int NS = RING > 0 ? RING : (BM * BN >= 128 * 128 ? 4 : 8);
  static_assert(NS % 2 == 0, "the LDS double buffer alternates with the ring slot");
  RegsA ra[NS];
  RegsB rb[NS];
  auto fetch = [&](RegsA &xa, RegsB &xb, int k0) {
    if (A_TR) tile_fetch<A_TR ? BK : BM, A_TR ? BM : BK>(xa, rs_a, p.lda, k0, m0, k_end, p.M, ragged_a, tid);
    else      tile_fetch<A_TR ? BK : BM, A_TR ? BM : BK>(xa, rs_a, p.lda, m0, k0, p.M, k_end, ragged_a, tid);
    if (B_TR) tile_fetch<B_TR ? BK : BN, B_TR ? BN : BK>(xb, rs_b, p.ldb, k0, n0, k_end, p.N, ragged_b, tid);
    else      tile_fetch<B_TR ? BK : BN, B_TR ? BN : BK>(xb, rs_b, p.ldb, n0, k0, p.N, k_end, ragged_b, tid);
  };
  // backward-weight tiles of the first column block also sum the rows of dZ^T they stream: the bias
  // gradient db[n] = sum_m dZ[m,n] comes out of the same launch
  constexpr int BGROUPS = 256 / BM, BROWS = BK / BGROUPS;
  const bool do_bias = FORM == FORM_DW && p.bias != nullptr && n0 == 0 && m0 < p.M;
  float bsum = 0.0f;
  const int nk = max(0, cdiv(k_end - k_begin, BK));
#pragma unroll
  for (int u = 0; u < NS; ++u)
    if (u < nk || u == 0) fetch(ra[u], rb[u], k_begin + u * BK);
  tile_store_lds<A_TR ? BK : BM, A_TR ? BM : BK>(ra[0], lds_a[0], tid);
  tile_store_lds<B_TR ? BK : BN, B_TR ? BN : BK>(rb[0], lds_b[0], tid);
  __syncthreads();
  for (int kt0 = 0; kt0 < nk; kt0 += NS) {
#pragma unroll
    for (int u = 0; u < NS; ++u) {
      const int kt = kt0 + u;
      if (kt >= nk) break;
      const int cur = u & 1;   // NS is even, so the LDS buffer of step kt is kt & 1 = u & 1
      // slot u held tile kt, already copied to LDS: reuse it for tile kt + NS
      if (kt + NS < nk) fetch(ra[u], rb[u], k_begin + (kt + NS) * BK);
#pragma unroll
      for (int kc = 0; kc < BK; kc += 16) {
        bf16x8 a[TI], b[TJ];
#pragma unroll
        for (int i = 0; i < TI; ++i)
          a[i] = A_TR ? frag_tr<BM>(lds_a[cur], wi0 + 32 * i, kc) : frag_kmajor(lds_a[cur], wi0 + 32 * i, kc);
#pragma unroll
        for (int j = 0; j < TJ; ++j)
          b[j] = B_TR ? frag_tr<BN>(lds_b[cur], wj0 + 32 * j, kc) : frag_kmajor(lds_b[cur], wj0 + 32 * j, kc);
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
          for (int j = 0; j < TJ; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
      }
      if (FORM == FORM_DW && do_bias) {
        const uint16_t *la = lds_a[cur] + (tid / BM) * BROWS * (BM + PAD_TR) + (tid % BM);
#pragma unroll
        for (int rr = 0; rr < BROWS; ++rr) bsum += bf16_bits_to_f32(la[rr * (BM + PAD_TR)]);
      }
      if (kt + 1 < nk) {
        tile_store_lds<A_TR ? BK : BM, A_TR ? BM : BK>(ra[(u + 1) % NS], lds_a[cur ^ 1], tid);
        tile_store_lds<B_TR ? BK : BN, B_TR ? BN : BK>(rb[(u + 1) % NS], lds_b[cur ^ 1], tid);
      }
      __syncthreads();
    }
  }

  float bias_total = 0.0f;            // threads < BM: this split's column sum of the dZ^T tile
  if (FORM == FORM_DW) {              // fold the row groups in a fixed order (the k-loop ended with a barrier)
    float *red = (float *)lds_b[0];
    if (do_bias) red[tid] = bsum;
    __syncthreads();                  // unconditional: every team of the workgroup passes here
    if (do_bias && tid < BM) {
#pragma unroll
      for (int g = 0; g < BGROUPS; ++g) bias_total += red[g * BM + tid];
    }
  }

  if (SPLIT && S > 1) {
    // Deterministic split-K: every split stores its fp32 partial tile; the split that arrives last
    // (arrival counter, no waiting) adds all partials in split order and runs the epilogue.
    constexpr int PSTRIDE = BM * BN + BM;
    float *mine = p.partial + ((int64_t)tile * S + split) * PSTRIDE;
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) put_partial(mine + ((i * TJ + j) * 16 + r) * 256 + tid, acc[i][j][r]);
    if (FORM == FORM_DW && tid < BM) put_partial(mine + BM * BN + tid, bias_total);
    // the partial stores go through to memory; once every wave's stores have been acknowledged and
    // the workgroup has met, one thread takes a ticket
    partials_published();
    int *ticket = (int *)lds_a[0];
    if (tid == 0) *ticket = __hip_atomic_fetch_add(&p.counters[tile], 1, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    __syncthreads();
    if (*ticket != S - 1) return;
    if (tid == 0) __hip_atomic_store(&p.counters[tile], 0, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);  // next launch
    const float *all = p.partial + (int64_t)tile * S * PSTRIDE;
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j)
#pragma unroll
        for (int r = 0; r < 16; ++r) {
          float v = 0.0f;
          for (int q = 0; q < S; ++q) v += get_partial(all + (int64_t)q * PSTRIDE + ((i * TJ + j) * 16 + r) * 256 + tid);
          acc[i][j][r] = v;
        }
    if (FORM == FORM_DW && tid < BM) {
      bias_total = 0.0f;
      for (int q = 0; q < S; ++q) bias_total += get_partial(all + (int64_t)q * PSTRIDE + BM * BN + tid);
    }
  }
  if (FORM == FORM_DW && do_bias && tid < BM && m0 + tid < p.M) {
    GPP_G float *db = (GPP_G float *)p.bias + m0 + tid;
    *db = accumulate_dw ? *db + bias_total : bias_total;
  }
  if (Cout == nullptr) return;   // the caller does not want this result (all barriers are behind us)

  // ---- epilogue; tiles inside the matrix skip the bounds checks
  if (EARLY_OLD && early_old) {
#pragma unroll
    for (int i = 0; i < TI; ++i)
#pragma unroll
      for (int j = 0; j < TJ; ++j) {
        EpiIn in;
        in.a = c_old[i][j];
        epi_finish<FORM, true>(p, Cout, acc[i][j], m0 + wi0 + 32 * i + 4 * (lane >> 5), n0 + wj0 + 32 * j + (lane & 31), 1, in);
      }
    return;
  }
  if (m0 + BM <= p.M && n0 + BN <= p.N) epilogue_wave<FORM, false, TI, TJ>(p, Cout, acc, m0 + wi0, n0 + wj0, lane, accumulate_dw);
  else epilogue_wave<FORM, true, TI, TJ>(p, Cout, acc, m0 + wi0, n0 + wj0, lane, accumulate_dw);
}

}  // namespace gpp
