// Branch-grouped bf16 GEMM for problems with many rows AND many columns (the transformer and MLP
// stacks at full micro-batch), on v_mfma_f32_32x32x16_bf16 with fp32 accumulation.  Two kernels:
//
// k_gemm_big   eight waves (512 threads) share a 256 x 256 (or 128 x 256) output tile as a 2 x 4 grid
//              of wave tiles of 128 x 64 (64 x 64) elements.  Per 16-wide contraction chunk a wave reads
//              6 KB (4 KB) of operand fragments from LDS for 8 (4) MFMAs.  One workgroup per compute
//              unit (the double-buffered tiles fill the LDS), so prologue and epilogue of a tile are
//              exposed: best when the launch has a whole number of tiles per compute unit.
// k_gemm_mid   four waves (256 threads), 128 x 128 tile, ONE LDS buffer (37 KB) and a register
//              budget of three waves per SIMD, so three workgroups share a compute unit and one
//              workgroup's loads, barriers and epilogue hide behind the others' MFMAs.  Best when the
//              large tiles would leave compute units idle (few tiles) or quantise badly.
//
// A k-step is 64 contraction elements, so a k-contiguous operand row contributes one whole 128-byte
// cache line per step.  Operands come from memory through buffer loads (out-of-range rows read as
// zero without a branch; a chunk beyond the contraction length is steered out of range).  Two kinds of loop:
// staged (operands wait in registers and are stored to padded LDS tiles) and direct (copied straight into
// swizzled LDS tiles, with the LDS reads software-pipelined under the MFMAs).  The three forms and the two
// LDS layouts (k-contiguous rows read with b128, contraction-major rows read with the transposing read) are
// those of the smaller tile kernel.
#include "gemm_tile_body.h"

namespace gpp {

constexpr int GB_BK = 64;           // contraction elements per k-step
constexpr int GB_KST = GB_BK + 8;   // LDS row stride of k-contiguous tiles: 144-byte rows, conflict-free b128 reads

// tile geometry: WGM x WGN waves, each WTM x WTN MFMA tiles of 32 x 32; LDS buffers (1 or 2)
// DIRECT: the operand tiles go from memory straight into LDS (buffer loads with the LDS destination,
// no staging registers), unpadded and XOR-swizzled instead of padded (see the direct loaders below).
template <int FORM, int WGM, int WGN, int WTM, int WTN, int BUFS, bool DIRECT = false>
struct BigCfg {
  static constexpr int NW = WGM * WGN, THREADS = 64 * NW;
  static constexpr int BM = 32 * WTM * WGM, BN = 32 * WTN * WGN;
  static constexpr bool A_TR = FORM == FORM_DW, B_TR = FORM != FORM_FWD;
  static constexpr int A_ELEMS = DIRECT ? GB_BK * BM : (A_TR ? GB_BK * (BM + PAD_TR) : BM * GB_KST);
  static constexpr int B_ELEMS = DIRECT ? GB_BK * BN : (B_TR ? GB_BK * (BN + PAD_TR) : BN * GB_KST);
  static constexpr int LDS_ELEMS = BUFS * (A_ELEMS + B_ELEMS);
  static_assert(LDS_ELEMS * 2 <= 160 * 1024, "tile does not fit the LDS");
};

// one k-step of one operand in registers: EXT rows/columns of the tile, 16-byte chunks, THREADS threads
template <int EXT, int THREADS>
struct BigRegs {
  static constexpr int PER_THREAD = EXT * GB_BK / 8 / THREADS;
  u32x4 v[PER_THREAD];
};

// k-contiguous operand: tile rows [r0, r0 + EXT) x k [k0, k0 + 64); eight lanes read one 128-byte row
// segment.  Rows beyond the buffer read zero, chunks at k >= k_lim are steered out of range (k_lim
// is a multiple of 8).
template <int EXT, int THREADS>
__device__ __forceinline__ void big_fetch_kmajor(BigRegs<EXT, THREADS> &t, __amdgpu_buffer_rsrc_t rs, int64_t ld, int r0, int k0,
                                                 int k_lim, int tid) {
#pragma unroll
  for (int q = 0; q < BigRegs<EXT, THREADS>::PER_THREAD; ++q) {
    const int row = r0 + (tid >> 3) + (THREADS / 8) * q, k = k0 + (tid & 7) * 8;
    // branch-free (a branch here makes the compiler wait for earlier loads between the loads)
    const uint32_t oob = (uint32_t)-(int32_t)(k >= k_lim) & OOB_OFFSET;
    const uint32_t off = (uint32_t)(((int64_t)row * ld + k) * 2) | oob;
    t.v[q] = __builtin_amdgcn_raw_buffer_load_b128(rs, off, 0, 0);
  }
}
template <int EXT, int THREADS>
__device__ __forceinline__ void big_store_kmajor(const BigRegs<EXT, THREADS> &t, uint16_t *lds, int tid) {
#pragma unroll
  for (int q = 0; q < BigRegs<EXT, THREADS>::PER_THREAD; ++q)
    *(u32x4 *)(lds + ((tid >> 3) + (THREADS / 8) * q) * GB_KST + (tid & 7) * 8) = t.v[q];
}
// contraction-major operand: rows k [k0, k0 + 64) x columns [c0, c0 + EXT); rows beyond the buffer
// (k >= contraction length) read zero; columns beyond the matrix only feed outputs that are never stored
template <int EXT, int THREADS>
__device__ __forceinline__ void big_fetch_tr(BigRegs<EXT, THREADS> &t, __amdgpu_buffer_rsrc_t rs, int64_t ld, int k0, int c0,
                                             int tid) {
  constexpr int CPR = EXT / 8, RPP = THREADS / CPR;   // chunks per row, rows per pass
#pragma unroll
  for (int q = 0; q < BigRegs<EXT, THREADS>::PER_THREAD; ++q) {
    const int row = k0 + tid / CPR + RPP * q, col = c0 + (tid % CPR) * 8;
    t.v[q] = __builtin_amdgcn_raw_buffer_load_b128(rs, (uint32_t)(((int64_t)row * ld + col) * 2), 0, 0);
  }
}
template <int EXT, int THREADS>
__device__ __forceinline__ void big_store_tr(const BigRegs<EXT, THREADS> &t, uint16_t *lds, int tid) {
  constexpr int CPR = EXT / 8, RPP = THREADS / CPR;
#pragma unroll
  for (int q = 0; q < BigRegs<EXT, THREADS>::PER_THREAD; ++q)
    *(u32x4 *)(lds + (tid / CPR + RPP * q) * (EXT + PAD_TR) + (tid % CPR) * 8) = t.v[q];
}

// LDS -> MFMA operand.  k-contiguous tile [rows][64 + 8]: lane l takes row (l % 32), 8 k-values at 8 * (l / 32)
__device__ __forceinline__ bf16x8 big_frag_kmajor(const uint16_t *lds, int row0, int k0) {
  const int l = threadIdx.x & 63;
  return *(const bf16x8 *)(lds + (row0 + (l & 31)) * GB_KST + k0 + 8 * (l >> 5));
}

// ---- direct loads: memory -> LDS without passing through registers.  One load instruction of a wave
// fills 1 KB of consecutive LDS (lane l writes 16 bytes at 16 l behind the wave-uniform destination), so
// the layout of a tile in LDS is the order of its 16-byte chunks, and the padding that keeps the operand
// reads free of bank conflicts in the staged path is replaced by a swizzle: WHICH chunk of memory a lane
// loads.  The asynchronous copy runs while the previous k-step is multiplied; nothing waits in registers.
typedef __attribute__((address_space(3))) void lds_void_t;
// The LDS moves 256 bytes per cycle (64 banks of 4 bytes), so what must not collide is:
// k-contiguous operand, tile [EXT][64]: 128-byte rows, two per bank line; a 16-byte operand read serves 16
// lanes per cycle, the same chunk column of 16 consecutive rows.  Chunk c of row r sits at chunk position
// c ^ ((r / 2) % 8): the two rows of a bank line keep their halves, the eight row pairs take eight positions
template <int EXT, int THREADS>
__device__ __forceinline__ void big_direct_kmajor(__amdgpu_buffer_rsrc_t rs, int64_t ld, int r0, int k0, int k_lim,
                                                  uint16_t *tile, int tid) {
  constexpr int NW = THREADS / 64, ROWS_PER_WAVE = EXT / NW, INSTR = ROWS_PER_WAVE / 8;
  static_assert(EXT % (8 * NW) == 0, "a wave loads whole groups of eight rows");
  const int wave = tid >> 6, l = tid & 63;
#pragma unroll
  for (int q = 0; q < INSTR; ++q) {
    const int row = wave * ROWS_PER_WAVE + 8 * q + (l >> 3);
    const int k = k0 + (((l & 7) ^ ((row >> 1) & 7)) << 3);
    const uint32_t oob = (uint32_t)-(int32_t)(k >= k_lim) & OOB_OFFSET;
    const uint32_t off = (uint32_t)(((int64_t)(r0 + row) * ld + k) * 2) | oob;
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t *)(tile + (wave * ROWS_PER_WAVE + 8 * q) * GB_BK), 16, off, 0, 0, 0);
  }
}
__device__ __forceinline__ bf16x8 big_direct_frag_kmajor(const uint16_t *tile, int row0, int k0) {
  const int l = threadIdx.x & 63;
  const int row = row0 + (l & 31), c = (k0 >> 3) + (l >> 5);
  return *(const bf16x8 *)(tile + row * GB_BK + ((c ^ ((row >> 1) & 7)) << 3));
}
// contraction-major operand, tile [64][EXT]: rows of EXT elements (a multiple of 256 bytes).  The transposing
// 8-byte read serves 32 lanes per cycle: 64 bytes in each of four consecutive rows.  Chunk c of row k sits at
// chunk position c ^ (4 (k % 4)), which spreads the four rows over the four 64-byte quarters of a bank line
template <int EXT, int THREADS>
__device__ __forceinline__ void big_direct_tr(__amdgpu_buffer_rsrc_t rs, int64_t ld, int k0, int c0, uint16_t *tile, int tid) {
  constexpr int CPR = EXT / 8;                         // chunks per row
  constexpr int NW = THREADS / 64, INSTR = GB_BK * CPR / 64 / NW;
  static_assert((GB_BK * CPR) % (64 * NW) == 0, "whole load instructions per wave");
  const int wave = tid >> 6, l = tid & 63;
#pragma unroll
  for (int q = 0; q < INSTR; ++q) {
    const int first = (wave * INSTR + q) * 64;         // first chunk (in LDS order) of this instruction
    const int row = (first + l) / CPR, pos = (first + l) % CPR;
    const int col = c0 + ((pos ^ ((row & 3) << 2)) << 3);
    // the whole address in the vector offset: the descriptor's range check (rows at or beyond the contraction
    // length read zero) does not cover a scalar offset
    __builtin_amdgcn_raw_ptr_buffer_load_lds(rs, (lds_void_t *)(tile + first * 8), 16,
                                             (uint32_t)(((int64_t)(k0 + row) * ld + col) * 2), 0, 0, 0);
  }
}
template <int COLS>
__device__ __forceinline__ bf16x8 big_direct_frag_tr(const uint16_t *tile, int col0, int k0) {
  const int l = threadIdx.x & 63;
  const int blk = l >> 4, q = l & 15;
  const int row = k0 + 8 * (blk >> 1) + (q >> 2), col = col0 + 16 * (blk & 1) + 4 * (q & 3);
  const uint16_t *p = tile + row * COLS + ((((col >> 3) ^ ((row & 3) << 2)) << 3) | (col & 7));
  typedef __attribute__((address_space(3))) s16x4 lds_v4;
  s16x4 lo = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)p);
  s16x4 hi = __builtin_amdgcn_ds_read_tr16_b64_v4i16((lds_v4 *)(p + 4 * COLS));     // row + 4: same swizzle
  return __builtin_bit_cast(bf16x8, __builtin_shufflevector(lo, hi, 0, 1, 2, 3, 4, 5, 6, 7));
}

// End of a k-step of the direct path: wait until at most VM of this wave's copy instructions are outstanding
// (they land in issue order, so the older k-steps are in LDS) and until its LDS reads have returned, then the
// workgroup barrier.  Written out instead of __syncthreads(): the fence in front of that barrier waits for ALL
// outstanding copies, which would keep only one k-step in flight whatever the number of LDS buffers.  The
// "memory" clobber keeps the compiler from moving LDS accesses across it.
template <int VM>
__device__ __forceinline__ void copies_landed_barrier() {
  asm volatile("s_waitcnt vmcnt(%0) lgkmcnt(0)\n\ts_barrier" ::"n"(VM) : "memory");
}

// Order for the scheduler: one LDS read behind each of the next MF MFMAs (the last MFMA takes the reads left over)
template <int MF, int READS, int Q = 0>
__device__ __forceinline__ void big_mix() {
  if constexpr (Q < MF) {
    __builtin_amdgcn_sched_group_barrier(0x008, 1, 0);
    if constexpr (Q < READS) __builtin_amdgcn_sched_group_barrier(0x100, (Q + 1 == MF && READS > MF) ? READS - MF + 1 : 1, 0);
    big_mix<MF, READS, Q + 1>();
  }
}

// what every tile kernel of this file does first: XCD-aware spreading (consecutive workgroup ids go
// round-robin over the 8 XCDs; give each XCD one contiguous range of tiles instead, so that
// neighbours share operand panels in one L2), then (record, tile) from the records' prefix sums
struct BigTile {
  int pi, m0, n0;
};
// GM > 0: the tiles of a record are numbered in bands of GM tile rows, column by column inside a band, so that
// the tiles in flight on an XCD form a block that is about as wide as it is high (fewest distinct operand panels
// per tile); GM = 0: whole columns of tiles one after the other.
template <int BM, int BN, int GM = 0>
__device__ __forceinline__ BigTile big_locate(const GemmProb *__restrict__ probs, int n, int total_blocks) {
  int bid = blockIdx.x;
  {
    const int xcd = bid & 7, idx = bid >> 3, per = total_blocks >> 3, rem = total_blocks & 7;
    bid = xcd * per + min(xcd, rem) + idx;
  }
  BigTile t;
  t.pi = find_prob(probs, n, bid);
  const int tile = bid - probs[t.pi].blk_begin;
  const int tiles_m = cdiv(probs[t.pi].M, BM);
  if constexpr (GM > 0) {
    const int tiles_n = cdiv(probs[t.pi].N, BN), band = tile / (GM * tiles_n), first = band * GM;
    const int rows = min(GM, tiles_m - first), in_band = tile - band * GM * tiles_n;
    t.m0 = (first + in_band % rows) * BM;
    t.n0 = (in_band / rows) * BN;
    return t;
  }
  t.m0 = (tile % tiles_m) * BM;          // consecutive tiles share the B panel
  t.n0 = (tile / tiles_m) * BN;
  return t;
}

// k-loop + bias gradient + epilogue of one output tile.  BUFS = 2: LDS double buffer and a ring of NS
// k-steps in registers (one barrier per step).  BUFS = 1: one LDS buffer, the next k-step waits in
// registers while the current one is multiplied (two barriers per step; other workgroups on the
// compute unit fill the gaps).
//
// GROUP (backward-weight only): the contraction runs over the rows of SEVERAL stash slots, one after
// the other -- the weight gradient of a group of backward passes in one pass over the accumulator.
// Both operands live in the slots at the same offsets: slot g of the group is `grp.stride` bytes times
// its slot number behind slot 0, whose addresses the record holds.
template <int FORM, int WGM, int WGN, int WTM, int WTN, int BUFS, int NS, bool GROUP = false, int PIPE = 0>
__device__ __forceinline__ void big_tile_body(const GemmProb &p, int m0, int n0, uint16_t *lds, int accumulate_dw,
                                              const ExtPtrs &ext, const SlotGroup grp = SlotGroup()) {
  static_assert(!GROUP || FORM == FORM_DW, "only the weight gradient contracts over a group of slots");
  constexpr bool DIRECT = PIPE != 0;     // operands copied straight into LDS, software-pipelined loop 1 or 2 (below)
  static_assert(!DIRECT || BUFS >= 2, "direct loads fill the other LDS buffers while one is multiplied");
  typedef BigCfg<FORM, WGM, WGN, WTM, WTN, BUFS, DIRECT> C;
  constexpr int BM = C::BM, BN = C::BN, THREADS = C::THREADS;
  constexpr bool A_TR = C::A_TR, B_TR = C::B_TR;
  static_assert(BUFS == 1 || NS % 2 == 0, "the LDS double buffer alternates with the ring slot");
  static_assert(DIRECT || BUFS <= 2, "the staged path has one or two LDS buffers");
  uint16_t *lds_a[2] = {lds, lds + (BUFS > 1 ? 1 : 0) * C::A_ELEMS};
  uint16_t *lds_b[2] = {lds + BUFS * C::A_ELEMS, lds + BUFS * C::A_ELEMS + (BUFS > 1 ? 1 : 0) * C::B_ELEMS};
  const int tid = threadIdx.x, wave = tid >> 6, lane = tid & 63;
  const int wi0 = (wave / WGN) * (32 * WTM), wj0 = (wave % WGN) * (32 * WTN);

  // operand buffers: rows beyond the matrix read as zero
  //   FWD: A = X [M x K],  B = W [N x K]      DX: A = dZ [M x K],  B = W [K x N]
  //   DW:  A = dZ [K x M], B = X [K x N]      (K = contraction length in every form)
  const __amdgpu_buffer_rsrc_t rs_a = matrix_rsrc(p.A, A_TR ? p.K : p.M, p.lda, A_TR ? p.M : p.K);
  const __amdgpu_buffer_rsrc_t rs_b = matrix_rsrc(p.B, B_TR ? p.K : p.N, p.ldb, B_TR ? p.N : p.K);

  f32x16 acc[WTM][WTN];
#pragma unroll
  for (int i = 0; i < WTM; ++i)
#pragma unroll
    for (int j = 0; j < WTN; ++j)
#pragma unroll
      for (int r = 0; r < 16; ++r) acc[i][j][r] = 0.0f;

  typedef BigRegs<BM, THREADS> RegsA;
  typedef BigRegs<BN, THREADS> RegsB;
  RegsA ra[DIRECT ? 1 : NS];       // unused (and removed by the compiler) with direct loads
  RegsB rb[DIRECT ? 1 : NS];
  const int nk_slot = cdiv(p.K, GB_BK);              // k-steps of one slot (of the whole contraction without a group)
  const int nk = GROUP ? nk_slot * grp.n : nk_slot;
  // k-step `kt` of the tile: without a group, contraction elements [64 kt, 64 kt + 64)
  auto fetch = [&](RegsA &xa, RegsB &xb, int kt) {
    if (GROUP) {
      const int g = kt / nk_slot, k0 = (kt - g * nk_slot) * GB_BK;    // wave-uniform
      int slot = grp.first + g;
      slot = slot >= grp.total ? slot - grp.total : slot;
      const int64_t off = (int64_t)slot * grp.stride;
      const __amdgpu_buffer_rsrc_t ga = matrix_rsrc((const char *)p.A + off, p.K, p.lda, p.M);
      const __amdgpu_buffer_rsrc_t gb = matrix_rsrc((const char *)p.B + off, p.K, p.ldb, p.N);
      big_fetch_tr<BM, THREADS>(xa, ga, p.lda, k0, m0, tid);
      big_fetch_tr<BN, THREADS>(xb, gb, p.ldb, k0, n0, tid);
      return;
    }
    const int k0 = kt * GB_BK;
    if (A_TR) big_fetch_tr<BM, THREADS>(xa, rs_a, p.lda, k0, m0, tid);
    else      big_fetch_kmajor<BM, THREADS>(xa, rs_a, p.lda, m0, k0, p.K, tid);
    if (B_TR) big_fetch_tr<BN, THREADS>(xb, rs_b, p.ldb, k0, n0, tid);
    else      big_fetch_kmajor<BN, THREADS>(xb, rs_b, p.ldb, n0, k0, p.K, tid);
  };
  // LDS buffers of the direct path as offsets from the array itself: a pointer picked out of a small array
  // of pointers loses its address space, and the operand reads then turn into generic (flat) loads
  auto da = [&](int b) { return lds + b * C::A_ELEMS; };
  auto db = [&](int b) { return lds + BUFS * C::A_ELEMS + b * C::B_ELEMS; };
  // the same k-step straight into LDS buffer `buf` (a k-step beyond the contraction copies zeros: its rows or
  // chunks lie outside the buffer range)
  auto fetch_direct = [&](int kt, int buf) {
    const int k0 = kt * GB_BK;
    if (A_TR) big_direct_tr<BM, THREADS>(rs_a, p.lda, k0, m0, da(buf), tid);
    else      big_direct_kmajor<BM, THREADS>(rs_a, p.lda, m0, k0, p.K, da(buf), tid);
    if (B_TR) big_direct_tr<BN, THREADS>(rs_b, p.ldb, k0, n0, db(buf), tid);
    else      big_direct_kmajor<BN, THREADS>(rs_b, p.ldb, n0, k0, p.K, db(buf), tid);
  };
  auto to_lds = [&](const RegsA &xa, const RegsB &xb, int buf) {
    if (A_TR) big_store_tr<BM, THREADS>(xa, lds_a[buf], tid);
    else      big_store_kmajor<BM, THREADS>(xa, lds_a[buf], tid);
    if (B_TR) big_store_tr<BN, THREADS>(xb, lds_b[buf], tid);
    else      big_store_kmajor<BN, THREADS>(xb, lds_b[buf], tid);
  };
  auto multiply = [&](int buf) {       // staged loops
#pragma unroll
    for (int kc = 0; kc < GB_BK; kc += 16) {
      bf16x8 a[WTM], b[WTN];
#pragma unroll
      for (int i = 0; i < WTM; ++i) a[i] = A_TR ? frag_tr<BM>(lds_a[buf], wi0 + 32 * i, kc) : big_frag_kmajor(lds_a[buf], wi0 + 32 * i, kc);
#pragma unroll
      for (int j = 0; j < WTN; ++j) b[j] = B_TR ? frag_tr<BN>(lds_b[buf], wj0 + 32 * j, kc) : big_frag_kmajor(lds_b[buf], wj0 + 32 * j, kc);
#pragma unroll
      for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(a[i], b[j], acc[i][j], 0, 0, 0);
    }
  };

  // backward-weight tiles of the first column block also sum the rows of dZ^T they stream: the bias
  // gradient db[n] = sum_m dZ[m,n] comes out of the same launch
  constexpr int BGROUPS = THREADS / BM, BROWS = GB_BK / BGROUPS;
  const bool do_bias = FORM == FORM_DW && p.bias != nullptr && n0 == 0;
  float bsum = 0.0f;
  auto bias_rows = [&](int buf) {
    if (FORM == FORM_DW && do_bias) {
      const uint16_t *la = lds_a[buf] + (tid / BM) * BROWS * (BM + PAD_TR) + (tid % BM);
#pragma unroll
      for (int rr = 0; rr < BROWS; ++rr) bsum += bf16_bits_to_f32(la[rr * (BM + PAD_TR)]);
    }
  };
  static_assert(!DIRECT || (FORM != FORM_DW && !GROUP), "backward-weight stages its operands through registers");

  if constexpr (PIPE == 1) {
    // Software-pipelined form: the operand fragments of 16-wide chunk c + 1 are read from LDS while the MFMAs
    // of chunk c run (two register sets), also across the k-step boundary.  One barrier per k-step, in front of
    // its LAST chunk: by then every wave has all fragments of the k-step in registers, so the buffer is free
    // and is refilled at once with k-step kt + BUFS; behind the barrier the first fragments of k-step kt + 1
    // (landed: at most BUFS - 2 later k-steps are outstanding) are read under the last chunk's MFMAs.
    constexpr int LPF = (A_TR ? GB_BK * (BM / 8) / 64 / C::NW : BM / C::NW / 8) + (B_TR ? GB_BK * (BN / 8) / 64 / C::NW : BN / C::NW / 8);
    bf16x8 fa[2][WTM], fb[2][WTN];
    // read in the order of first use: the MFMAs run a-major, so the first of them needs every b and a[0]
    auto frags = [&](int set, int buf, int kc) {
#pragma unroll
      for (int j = 0; j < WTN; ++j)
        fb[set][j] = B_TR ? big_direct_frag_tr<BN>(db(buf), wj0 + 32 * j, kc) : big_direct_frag_kmajor(db(buf), wj0 + 32 * j, kc);
#pragma unroll
      for (int i = 0; i < WTM; ++i)
        fa[set][i] = A_TR ? big_direct_frag_tr<BM>(da(buf), wi0 + 32 * i, kc) : big_direct_frag_kmajor(da(buf), wi0 + 32 * i, kc);
    };
    auto mfmas = [&](int set) {
#pragma unroll
      for (int i = 0; i < WTM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j) acc[i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[set][j], acc[i][j], 0, 0, 0);
    };
    constexpr int READS = (A_TR ? 2 : 1) * WTM + (B_TR ? 2 : 1) * WTN, MFMAS = WTM * WTN;
    static_assert((BUFS - 1) * LPF < 64, "vmcnt is a 6-bit counter");
    auto interleave = [&]() { big_mix<MFMAS, READS>(); };
    // No branch inside the loop (a branch would end the scheduling region and the interleaving with it): k-steps
    // beyond the contraction are copied like the others -- their rows lie outside the operand's buffer range and
    // read zero -- into buffers nobody multiplies any more, and the fragments read for a k-step that does not
    // exist are dropped.  The number of outstanding copies is then the same in every iteration.
    // L2 prefetch PD k-steps ahead of the copies, issued BEHIND the copies of its iteration: the loads of a wave
    // complete in order, so a wait for copies never includes the prefetch issued after them, only the one of the
    // iteration before, which has had a whole k-step more
#pragma unroll
    for (int u = 0; u < BUFS; ++u) fetch_direct(u, u);
    copies_landed_barrier<(BUFS - 1) * LPF>();
    frags(0, 0, 0);
    int cur = 0;
    for (int kt = 0; kt < nk; ++kt) {
      const int nxt = cur + 1 == BUFS ? 0 : cur + 1;
      frags(1, cur, 16); mfmas(0); interleave();
      frags(0, cur, 32); mfmas(1); interleave();
      frags(1, cur, 48); mfmas(0); interleave();
      copies_landed_barrier<(BUFS - 2) * LPF>();
      fetch_direct(kt + BUFS, cur);
      frags(0, nxt, 0); mfmas(1); interleave();
      cur = nxt;
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the copies of the k-steps beyond the end
    __syncthreads();      // the epilogue reuses the operand LDS
  } else if constexpr (PIPE == 2) {
    // As above, and the copies of a k-step are issued in TWO batches so that the copy path never runs empty (with
    // one batch per k-step and two buffers, a batch can only be issued when the batch before it has landed: one
    // memory round trip per k-step in which nothing moves).  A wave multiplies the TOP half of its rows for all
    // four 16-wide chunks first (keeping the b fragments of the four chunks), then the BOTTOM half: after the
    // first phase the b tile and the top halves of the a tile are free and are refilled with k-step kt + 2 (batch
    // 1) while the second phase runs; after the second phase the bottom halves follow (batch 2).  Every batch has
    // one and a half k-steps to land, and two batches are in flight at any time.  Each accumulator still adds
    // its chunks in the order 0..3, so the result is the same as in the other loops, bit by bit.
    static_assert(!A_TR && BUFS == 2 && WTM % 2 == 0, "rows of a k-contiguous A split into halves");
    constexpr int HM = WTM / 2, RB = 16 * WTM;                    // MFMA row tiles and rows of a half of a wave's rows
    constexpr int A_HALF = BM / 2 / 8 / C::NW;                    // copy instructions per wave and half of the a tile
    static_assert(A_HALF * C::NW * 8 * 2 == BM, "whole copy instructions");
    constexpr int B_ALL = B_TR ? GB_BK * (BN / 8) / 64 / C::NW : BN / C::NW / 8;
    constexpr int N1 = A_HALF + B_ALL, N2 = A_HALF;
    static_assert(2 * (N1 + N2) < 64, "vmcnt is a 6-bit counter");
    auto copy_a = [&](int kt, int buf, int h) {                   // rows [h RB, h RB + RB) of every wave row block
      const int k0 = kt * GB_BK;
#pragma unroll
      for (int q = 0; q < A_HALF; ++q) {
        const int idx = q * C::NW + wave, wr = idx / (RB / 8), sub = idx % (RB / 8);
        const int base = wr * 32 * WTM + h * RB + sub * 8, row = base + (lane >> 3);
        const int k = k0 + (((lane & 7) ^ ((row >> 1) & 7)) << 3);
        const uint32_t oob = (uint32_t)-(int32_t)(k >= p.K) & OOB_OFFSET;
        __builtin_amdgcn_raw_ptr_buffer_load_lds(rs_a, (lds_void_t *)(da(buf) + base * GB_BK), 16,
                                                 (uint32_t)(((int64_t)(m0 + row) * p.lda + k) * 2) | oob, 0, 0, 0);
      }
    };
    auto copy_b = [&](int kt, int buf) {
      if (B_TR) big_direct_tr<BN, THREADS>(rs_b, p.ldb, kt * GB_BK, n0, db(buf), tid);
      else big_direct_kmajor<BN, THREADS>(rs_b, p.ldb, n0, kt * GB_BK, p.K, db(buf), tid);
    };
    bf16x8 fa[2][HM], fb[4][WTN];
    auto read_b = [&](int buf, int c) {
#pragma unroll
      for (int j = 0; j < WTN; ++j)
        fb[c][j] = B_TR ? big_direct_frag_tr<BN>(db(buf), wj0 + 32 * j, 16 * c) : big_direct_frag_kmajor(db(buf), wj0 + 32 * j, 16 * c);
    };
    auto read_a = [&](int set, int buf, int h, int c) {
#pragma unroll
      for (int i = 0; i < HM; ++i) fa[set][i] = big_direct_frag_kmajor(da(buf), wi0 + 32 * (h * HM + i), 16 * c);
    };
    auto mf = [&](int set, int h, int c) {
#pragma unroll
      for (int i = 0; i < HM; ++i)
#pragma unroll
        for (int j = 0; j < WTN; ++j)
          acc[h * HM + i][j] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(fa[set][i], fb[c][j], acc[h * HM + i][j], 0, 0, 0);
    };
    constexpr int MF = HM * WTN, R1 = (B_TR ? 2 : 1) * WTN + HM, R2 = HM;
    copy_a(0, 0, 0); copy_b(0, 0); copy_a(0, 0, 1);
    copy_a(1, 1, 0); copy_b(1, 1); copy_a(1, 1, 1);
    copies_landed_barrier<N2 + N1 + N2>();
    read_b(0, 0); read_a(0, 0, 0, 0);
    for (int kt = 0; kt < nk; ++kt) {
      const int cur = kt & 1, nxt = cur ^ 1;
      read_b(cur, 1); read_a(1, cur, 0, 1); mf(0, 0, 0); big_mix<MF, R1>();
      read_b(cur, 2); read_a(0, cur, 0, 2); mf(1, 0, 1); big_mix<MF, R1>();
      read_b(cur, 3); read_a(1, cur, 0, 3); mf(0, 0, 2); big_mix<MF, R1>();
      copies_landed_barrier<N1 + N2>();        // the bottom halves of this k-step have landed; top halves and b are free
      copy_a(kt + 2, cur, 0); copy_b(kt + 2, cur);
      read_a(0, cur, 1, 0); mf(1, 0, 3);
      __builtin_amdgcn_sched_group_barrier(0x010, N1, 0);      // the copies first: they have the longest way
      big_mix<MF, R2>();
      read_a(1, cur, 1, 1); mf(0, 1, 0); big_mix<MF, R2>();
      read_a(0, cur, 1, 2); mf(1, 1, 1); big_mix<MF, R2>();
      read_a(1, cur, 1, 3); mf(0, 1, 2); big_mix<MF, R2>();
      copies_landed_barrier<N1 + N2>();        // top halves and b of the next k-step have landed; bottom halves are free
      copy_a(kt + 2, cur, 1);
      read_b(nxt, 0); read_a(0, nxt, 0, 0); mf(1, 1, 3);
      __builtin_amdgcn_sched_group_barrier(0x010, N2, 0);
      big_mix<MF, R1>();
    }
    asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // the copies of the k-steps beyond the end
    __syncthreads();      // the epilogue reuses the operand LDS
  } else if (BUFS == 2) {
#pragma unroll
    for (int u = 0; u < NS - 1; ++u)
      if (u < nk) fetch(ra[u], rb[u], u);
    to_lds(ra[0], rb[0], 0);
    __syncthreads();
    for (int kt0 = 0; kt0 < nk; kt0 += NS) {
#pragma unroll
      for (int u = 0; u < NS; ++u) {
        const int kt = kt0 + u;
        if (kt >= nk) break;
        const int cur = u & 1;   // NS is even: the LDS buffer of step kt is kt & 1 = u & 1
        // ring slot (u + NS - 1) % NS was copied to LDS one step ago: refill it with step kt + NS - 1
        if (kt + NS - 1 < nk) fetch(ra[(u + NS - 1) % NS], rb[(u + NS - 1) % NS], kt + NS - 1);
        multiply(cur);
        bias_rows(cur);
        if (kt + 1 < nk) to_lds(ra[(u + 1) % NS], rb[(u + 1) % NS], cur ^ 1);
        __syncthreads();
      }
    }
  } else {
    fetch(ra[0], rb[0], 0);
    for (int kt = 0; kt < nk; ++kt) {
      to_lds(ra[0], rb[0], 0);
      __syncthreads();
      if (kt + 1 < nk) fetch(ra[0], rb[0], kt + 1);
      multiply(0);
      bias_rows(0);
      __syncthreads();
    }
  }

  if (FORM == FORM_DW && do_bias) {   // fold the row groups in a fixed order (the k-loop ended with a barrier)
    float *red = (float *)lds;
    red[tid] = bsum;
    __syncthreads();
    if (tid < BM && m0 + tid < p.M) {
      float total = 0.0f;
#pragma unroll
      for (int g = 0; g < BGROUPS; ++g) total += red[g * BM + tid];
      GPP_G float *db = (GPP_G float *)p.bias + m0 + tid;
      *db = accumulate_dw ? *db + total : total;
    }
  }

  void *Cout = FORM == FORM_DW ? p.C : result_ptr(p, ext);
  if (Cout == nullptr) return;
  // ---- epilogue.  Tiles inside the matrix whose rows are 16-byte aligned go through LDS and touch
  // memory in whole 16-byte pieces of rows (each wave has a private block; the operand tiles are dead:
  // the k-loop and the bias sums ended with a barrier); the rest keeps the accumulator layout.
  static_assert(C::NW * epi_lds_floats<WTN>() * 4 <= C::LDS_ELEMS * 2, "epilogue blocks do not fit the operand LDS");
  if (m0 + BM <= p.M && n0 + BN <= p.N) {
    // (also for a plain bias / cast epilogue: rows in 16-byte pieces beat the accumulator layout's 2-byte pieces
    // sixteen rows apart -- 4 x [2048 x 4096 x 1024] forward 78 -> 75.5 us, a one-k-step launch of the same output
    // 29 -> 26 us.  While the stores were flat instructions, which count on the LDS wait counter as well, it
    // was the other way round: 87 against 95 us)
    if (epi_lds_ok(p, Cout, FORM)) {
      if (FORM == FORM_DW && do_bias) __syncthreads();   // the bias sums were read from LDS after the last barrier
      epilogue_wave_lds<FORM, WTM, WTN>(p, Cout, acc, m0 + wi0, n0 + wj0, lane, accumulate_dw,
                                        (float *)lds + wave * epi_lds_floats<WTN>());
    } else {
      epilogue_wave<FORM, false, WTM, WTN>(p, Cout, acc, m0 + wi0, n0 + wj0, lane, accumulate_dw);
    }
  } else {
    epilogue_wave<FORM, true, WTM, WTN>(p, Cout, acc, m0 + wi0, n0 + wj0, lane, accumulate_dw);
  }
}

template <int FORM, int WTM, int WTN, int NS, int PIPE, int BUFS = 2>
__global__ __launch_bounds__(512) void k_gemm_big(const GemmProb *__restrict__ probs, int n, int total_blocks,
                                                  int accumulate_dw, ExtPtrs ext) {
  typedef BigCfg<FORM, 2, 4, WTM, WTN, BUFS, PIPE != 0> C;
  __shared__ __attribute__((aligned(16))) uint16_t lds[C::LDS_ELEMS];
  const BigTile t = big_locate<C::BM, C::BN>(probs, n, total_blocks);
  const GemmProb p = probs[t.pi];
  big_tile_body<FORM, 2, 4, WTM, WTN, BUFS, NS, false, PIPE>(p, t.m0, t.n0, lds, accumulate_dw, ext);
}

// 128 x 128 tile, 2 x 2 waves of 64 x 64, one LDS buffer, three waves per SIMD
template <int FORM>
__global__ __launch_bounds__(256, 3) void k_gemm_mid(const GemmProb *__restrict__ probs, int n, int total_blocks,
                                                     int accumulate_dw, ExtPtrs ext) {
  typedef BigCfg<FORM, 2, 2, 2, 2, 1> C;
  __shared__ __attribute__((aligned(16))) uint16_t lds[C::LDS_ELEMS];
  const BigTile t = big_locate<C::BM, C::BN>(probs, n, total_blocks);
  const GemmProb p = probs[t.pi];
  big_tile_body<FORM, 2, 2, 2, 2, 1, 1>(p, t.m0, t.n0, lds, accumulate_dw, ext);
}

// backward-weight over a group of stash slots (see big_tile_body)
template <int WTM, int WTN, int NS>
__global__ __launch_bounds__(512) void k_gemm_big_dw_group(const GemmProb *__restrict__ probs, int n, int total_blocks,
                                                           int accumulate_dw, SlotGroup grp) {
  typedef BigCfg<FORM_DW, 2, 4, WTM, WTN, 2> C;
  __shared__ __attribute__((aligned(16))) uint16_t lds[C::LDS_ELEMS];
  // (bands of four tile rows: one workgroup per compute unit, 32 tiles in flight per XCD as a 4 x 8 block; seven
  // [4096 x 4096] gradients over 2048 rows: 3226 -> 2684 us)
  const BigTile t = big_locate<C::BM, C::BN, 4>(probs, n, total_blocks);
  const GemmProb p = probs[t.pi];
  ExtPtrs none;
  big_tile_body<FORM_DW, 2, 4, WTM, WTN, 2, NS, true>(p, t.m0, t.n0, lds, accumulate_dw, none, grp);
}
// Tile order of the grouped weight gradient: bands of eight tile rows.  Its launch holds thousands of 128 x 128 tiles,
// 128 of them in flight per XCD; numbered column by column these are 32 rows x 4 columns of a [4096 x 1024] gradient
// (36 operand panels of 512 KB through a 4 MB L2), in bands 8 x 16 (24 panels).  Measured on the transformer stage's
// launch of all layers: 497-505 -> 483 us (bands of 4: 497, of 16: 487 scaled to the same box).
constexpr int DW_BAND = 8;
// (four workgroups per compute unit: 40 KB of LDS and 128 registers each; with three the transformer stage's launch
// is 6 % slower)
__global__ __launch_bounds__(256, 4) void k_gemm_mid_dw_group(const GemmProb *__restrict__ probs, int n, int total_blocks,
                                                              int accumulate_dw, SlotGroup grp) {
  typedef BigCfg<FORM_DW, 2, 2, 2, 2, 1> C;
  __shared__ __attribute__((aligned(16))) uint16_t lds[C::LDS_ELEMS];
  const BigTile t = big_locate<C::BM, C::BN, DW_BAND>(probs, n, total_blocks);
  const GemmProb p = probs[t.pi];
  ExtPtrs none;
  big_tile_body<FORM_DW, 2, 2, 2, 2, 1, 1, true>(p, t.m0, t.n0, lds, accumulate_dw, none, grp);
}

// ---- host side -------------------------------------------------------------------------
// The kernels take a problem when the chunks of its k-contiguous operands are whole (contraction
// length a multiple of 8) and the matrices fit the 32-bit buffer offsets.
// Direct loads move whole, aligned 16-byte chunks: rows and base pointers of both operands must be 16-byte
// aligned (the planner pads leading dimensions to 64 elements, so only unusual callers fail this).
bool gemm_big_direct_ok(const GemmProb &p) {
  return (p.lda & 7) == 0 && (p.ldb & 7) == 0 && ((uintptr_t)p.A & 15) == 0 && ((uintptr_t)p.B & 15) == 0;
}
bool gemm_big_supported(const GemmProb &p) {
  if (!gemm_mfma_supported(p)) return false;
  if (p.form != FORM_DW && (p.K & 7)) return false;
  const int64_t a_rows = p.form == FORM_DW ? p.K : p.M, b_rows = p.form == FORM_FWD ? p.N : p.K;
  if (a_rows * p.lda * 2 >= 0xffffff00ll || b_rows * p.ldb * 2 >= 0xffffff00ll) return false;
  return true;
}
// Tile shape for a launch: 256 (256 x 256, eight waves), 128 (128 x 256, eight waves), 64 (128 x 128,
// four waves, three workgroups per compute unit), or 0 when the smaller tile kernel should run it.
// `tiles256` / `tiles128`: 256 x 256 / 128 x 256 tiles of the whole launch.  The eight-wave kernels
// hold one workgroup per compute unit, so they win only when every one of the 256 compute units gets
// the same whole number of tiles; in between, the co-resident small tiles do.  Measured, 4 branches of
// [2048 x N] outputs with contraction K, microseconds for tile 256 / 128 / 64:
//   forward N 4096 K 1024 (512 / 1024 tiles): 87 / 95 / 90      N 3072 K 1024 (384 / 768): 77 / 71 / 66
//   forward N 1024 K 4096 (128 / 256):       127 / 88 / 92      N 1024 K 1024 (128 / 256): 39 / 26 / 26
//   backward-weight [3072 x 1024], 2048 rows (192 / 384): 81 / 90 / 71     [1024 x 1024] (64 / 128): 73 / 46 / 38
int gemm_big_tile_rows(int form, int maxM, int maxN, int64_t launch_elems, int tiles256, int tiles128) {
  constexpr int CUS = 256;
  if (maxM < 128 || maxN < 128) return 0;
  if (launch_elems < (int64_t)128 * 128 * 128) return 0;
  if (maxM >= 256 && maxN >= 256 && tiles256 >= CUS && tiles256 % CUS == 0) return 256;
  // forward with the two-batch direct loop: a last round that still fills half of the compute units beats the
  // co-resident small tiles (4 x [2048 x 3072 x 1024], 384 tiles: 70 against 74 us)
  if (form == FORM_FWD && maxM >= 256 && maxN >= 256 && tiles256 >= CUS && tiles256 % CUS >= CUS / 2) return 256;
  if (maxN >= 256 && tiles128 == CUS) return 128;
  // the single-buffer small tiles hide their load latency only behind co-resident workgroups: with
  // fewer tiles than compute units (a lone [2048 x 1024 x 1024] problem: 28 us against 20 us) they lose
  // to the ring-buffered tile kernel
  if (2 * tiles128 < CUS) return 0;
  return 64;
}
int gemm_big_tiles_for(int tile_rows, int M, int N, int *tiles_n) {
  const int bn = tile_rows == 64 ? 128 : 256, bm = tile_rows == 64 ? 128 : tile_rows;
  if (tiles_n) *tiles_n = cdiv(N, bn);
  return cdiv(M, bm) * cdiv(N, bn);
}

template <int FORM>
static void launch_big_form(const GemmProb *probs, int n, int blocks, int acc, int tile_rows, int direct, const ExtPtrs &ext,
                            hipStream_t s) {
  const dim3 g(blocks), b(512);
  // direct: the forward form on both eight-wave tiles, backward-data on the 256 x 256 tile (its a operand is
  // k-contiguous); backward-weight always stages through registers
  constexpr int P256 = FORM == FORM_DW ? 0 : 2, P128 = FORM == FORM_FWD ? 1 : 0;
  if constexpr (P256 != 0) {
    if (tile_rows == 256 && direct) {
      hipLaunchKernelGGL((k_gemm_big<FORM, 4, 2, 2, P256, 2>), g, b, 0, s, probs, n, blocks, acc, ext);
      return;
    }
  }
  if constexpr (P128 != 0) {
    if (tile_rows == 128 && direct) {
      hipLaunchKernelGGL((k_gemm_big<FORM, 2, 2, 2, P128, 3>), g, b, 0, s, probs, n, blocks, acc, ext);
      return;
    }
  }
  if (tile_rows == 256) hipLaunchKernelGGL((k_gemm_big<FORM, 4, 2, 2, 0, 2>), g, b, 0, s, probs, n, blocks, acc, ext);
  else if (tile_rows == 128) hipLaunchKernelGGL((k_gemm_big<FORM, 2, 2, 2, 0, 2>), g, b, 0, s, probs, n, blocks, acc, ext);
  else hipLaunchKernelGGL((k_gemm_mid<FORM>), g, dim3(256), 0, s, probs, n, blocks, acc, ext);
}
// direct != 0: operands straight into LDS where the form has such a loop (every record must pass
// gemm_big_direct_ok); the other launches stage through registers
void launch_gemm_big(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int form, int tile_rows, int direct,
                     const ExtPtrs &ext, hipStream_t s) {
  if (total_blocks <= 0) return;
  if (form == FORM_FWD) launch_big_form<FORM_FWD>(probs, n, total_blocks, accumulate_dw, tile_rows, direct, ext, s);
  else if (form == FORM_DX) launch_big_form<FORM_DX>(probs, n, total_blocks, accumulate_dw, tile_rows, direct, ext, s);
  else launch_big_form<FORM_DW>(probs, n, total_blocks, accumulate_dw, tile_rows, direct, ext, s);
}

void launch_gemm_dw_group(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int tile_rows, const SlotGroup &grp,
                          hipStream_t s) {
  if (total_blocks <= 0 || grp.n <= 0) return;
  const dim3 g(total_blocks), b(512);
  if (tile_rows == 256) hipLaunchKernelGGL((k_gemm_big_dw_group<4, 2, 2>), g, b, 0, s, probs, n, total_blocks, accumulate_dw, grp);
  else if (tile_rows == 128) hipLaunchKernelGGL((k_gemm_big_dw_group<2, 2, 2>), g, b, 0, s, probs, n, total_blocks, accumulate_dw, grp);
  else hipLaunchKernelGGL(k_gemm_mid_dw_group, dim3(total_blocks), dim3(256), 0, s, probs, n, total_blocks, accumulate_dw, grp);
}

}  // namespace gpp
