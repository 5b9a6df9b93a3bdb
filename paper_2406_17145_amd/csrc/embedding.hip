// Sparse path of a DLRM-shaped stage, grouped over all embedding tables:
//   forward   coalesced embedding-bag gather with sum pooling
//   backward  deterministic sorted segment reduction:
//             stable LSD radix sort of (row, position) keys -> segment heads ->
//             per-row sums in sorted order -> one read-modify-write per distinct row
//   reset     clears only the rows the backward passes since the last reset touched
// No float atomics anywhere and every sum has a fixed association order, so two
// runs give bit-identical gradients.
#include "device_utils.h"

namespace gpp {

constexpr int RADIX_BITS = 9;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_CHUNK = 2048;   // keys per workgroup per pass (256 threads x 8 rounds)
constexpr int LONG_SEG = 256;      // slice length of the segments that are summed by whole workgroups
constexpr int SHORT_MAX = 32;      // segments up to this length are summed by one 16-lane group, serially:
                                   // the longest serial chain sets that kernel's duration, so it is kept short
constexpr int LOG_SLOTS = 4;       // backward passes whose touched-row lists are kept for the reset

int emb_sort_chunk() { return SORT_CHUNK; }
int emb_radix_bits() { return RADIX_BITS; }
int emb_long_segment() { return LONG_SEG; }
int emb_log_slots() { return LOG_SLOTS; }
int emb_fwd_blocks(int n_bags) { return (n_bags + 3) / 4; }

// number of index positions in use = last offset, clamped to the capacity
__device__ __forceinline__ int used_positions(const EmbProb &p) { return max(0, min(p.offsets[p.n_bags], p.capacity)); }
// out-of-range rows are sorted as the nearest valid row; the segment sum skips them
__device__ __forceinline__ int clamp_row(int r, int num_rows) { return max(0, min(r, num_rows - 1)); }

// lanes that share one table row in the vector kernels: dim/4 rounded up to a power of two
__device__ __forceinline__ int lanes_per_row(int dim) {
  int l = 1;
  while (l * 4 < dim) l <<= 1;
  return l;
}
__device__ __forceinline__ float4 f4_add(float4 a, float4 b) { return make_float4(a.x + b.x, a.y + b.y, a.z + b.z, a.w + b.w); }
__device__ __forceinline__ float4 f4_shfl_down(float4 v, int d) {
  return make_float4(__shfl_down(v.x, d, 64), __shfl_down(v.y, d, 64), __shfl_down(v.z, d, 64), __shfl_down(v.w, d, 64));
}
// four consecutive elements of a pooled-output (or its gradient) row as floats
__device__ __forceinline__ float4 load4(const void *base, int dtype, int64_t idx) {
  if (dtype == DT_BF16) {
    const uint2 u = *(const uint2 *)((const uint16_t *)base + idx);
    return make_float4(__uint_as_float(u.x << 16), __uint_as_float(u.x & 0xffff0000u), __uint_as_float(u.y << 16),
                       __uint_as_float(u.y & 0xffff0000u));
  }
  return *(const float4 *)((const float *)base + idx);
}
__device__ __forceinline__ void store4(void *base, int dtype, int64_t idx, float4 v) {
  if (dtype == DT_BF16) {
    uint2 u;
    u.x = (uint32_t)f32_to_bf16_bits(v.x) | ((uint32_t)f32_to_bf16_bits(v.y) << 16);
    u.y = (uint32_t)f32_to_bf16_bits(v.z) | ((uint32_t)f32_to_bf16_bits(v.w) << 16);
    *(uint2 *)((uint16_t *)base + idx) = u;
  } else {
    *(float4 *)((float *)base + idx) = v;
  }
}

// ------------------------------------------------------------------ forward
// generic: one wave per bag, a lane per column (any dimension up to 256)
__global__ __launch_bounds__(256) void k_emb_fwd(const EmbProb *__restrict__ probs, int n, StageFlags *flags) {
  const int pi = find_prob(probs, n, blockIdx.x);
  const EmbProb p = probs[pi];
  const int lane = threadIdx.x & 63;
  const int bag = (blockIdx.x - p.blk_begin) * 4 + (threadIdx.x >> 6);
  if (bag >= p.n_bags) return;
  int lo = p.offsets[bag], hi = p.offsets[bag + 1];
  bool bad = lo < 0 || hi < lo || hi > p.capacity;
  lo = max(0, min(lo, p.capacity));
  hi = max(lo, min(hi, p.capacity));
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int j = lo; j < hi; ++j) {
    const int r = p.indices[j];
    if (lane == 0) p.bag_of[j] = bag;
    if (r < 0 || r >= p.num_rows) {
      bad = true;
      continue;
    }
    const float *row = p.table + (int64_t)r * p.ld_table;
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int c = lane + 64 * q;
      if (c < p.dim) acc[q] += row[c];
    }
  }
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int c = lane + 64 * q;
    if (c < p.dim) store_from_f32(p.out, p.out_dtype, (int64_t)bag * p.ld_out + c, acc[q]);
  }
  if (bad && lane == 0) flags->index_error = 1;
}

// vector: one wave per bag; LPR lanes read one 16-byte piece of a row each, so a wave has
// 64/LPR rows in flight per load instruction.  FWD_UNROLL such instructions are issued back to back
// before any of them is consumed (a bag of 20 rows of 128 floats is then two batches: one memory
// round trip each instead of one per few rows); the loads are unconditional -- a lane without a row
// reads row 0 and discards it -- because a branch around a load would make the wave wait for the
// loads before it.  Sums run in index order within a sub-group; the sub-groups are combined in lane order.
constexpr int FWD_UNROLL = 8;
__global__ __launch_bounds__(256) void k_emb_fwd_vec(const EmbProb *__restrict__ probs, int n, StageFlags *flags) {
  const int pi = find_prob(probs, n, blockIdx.x);
  const EmbProb p = probs[pi];
  const int lane = threadIdx.x & 63;
  const int bag = (blockIdx.x - p.blk_begin) * 4 + (threadIdx.x >> 6);
  if (bag >= p.n_bags) return;
  int lo = p.offsets[bag], hi = p.offsets[bag + 1];
  bool bad = lo < 0 || hi < lo || hi > p.capacity;
  lo = max(0, min(lo, p.capacity));
  hi = max(lo, min(hi, p.capacity));
  const int lpr = lanes_per_row(p.dim), rpi = 64 / lpr;
  const int sub = lane / lpr, c4 = (lane % lpr) * 4;
  const bool col_ok = c4 < p.dim;
  const float *col_base = p.table + (col_ok ? c4 : 0);
  float4 acc = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  for (int base = lo; base < hi; base += 64) {
    const int cnt = min(64, hi - base);
    int my = -1;
    if (lane < cnt) {
      my = p.indices[base + lane];
      p.bag_of[base + lane] = bag;
      if (my < 0 || my >= p.num_rows) {
        bad = true;
        my = -1;
      }
    }
    for (int j0 = 0; j0 < cnt; j0 += rpi * FWD_UNROLL) {
      float4 v[FWD_UNROLL];
      bool ok[FWD_UNROLL];
#pragma unroll
      for (int u = 0; u < FWD_UNROLL; ++u) {
        const int j = j0 + u * rpi + sub;
        const int r = __shfl(my, min(j, 63), 64);
        ok[u] = j < cnt && r >= 0 && col_ok;
        v[u] = *(const float4 *)(col_base + (int64_t)(ok[u] ? r : 0) * p.ld_table);
      }
#pragma unroll
      for (int u = 0; u < FWD_UNROLL; ++u)
        if (ok[u]) acc = f4_add(acc, v[u]);
    }
  }
  for (int d = lpr; d < 64; d <<= 1) acc = f4_add(acc, f4_shfl_down(acc, d));
  if (sub == 0 && col_ok) store4(p.out, p.out_dtype, (int64_t)bag * p.ld_out + c4, acc);
  if (__any(bad) && lane == 0) flags->index_error = 1;
}

bool emb_vec_supported(const EmbProb &p) {
  if ((p.dim & 3) || p.dim > 256 || (p.ld_table & 3) || (p.ld_out & 3)) return false;
  if (((uintptr_t)p.table | (uintptr_t)p.dtable) & 15) return false;
  if ((uintptr_t)p.out & 15) return false;
  return true;
}
void launch_emb_fwd(const EmbProb *probs, int n, int total_blocks, int vec, StageFlags *flags, hipStream_t s) {
  if (total_blocks <= 0) return;
  if (vec) hipLaunchKernelGGL(k_emb_fwd_vec, dim3(total_blocks), dim3(256), 0, s, probs, n, flags);
  else hipLaunchKernelGGL(k_emb_fwd, dim3(total_blocks), dim3(256), 0, s, probs, n, flags);
}

// ------------------------------------------------------------------ stable radix sort by row
struct SortIo {
  const int32_t *src_keys;
  const int32_t *src_pos;  // null in pass 0: position = index
  int32_t *dst_keys, *dst_pos;
};
__device__ __forceinline__ SortIo sort_io(const EmbProb &p, int pass) {
  SortIo io;
  if (pass == 0) {
    io.src_keys = p.indices; io.src_pos = nullptr; io.dst_keys = p.keys_a; io.dst_pos = p.pos_a;
  } else if (pass & 1) {
    io.src_keys = p.keys_a; io.src_pos = p.pos_a; io.dst_keys = p.keys_b; io.dst_pos = p.pos_b;
  } else {
    io.src_keys = p.keys_b; io.src_pos = p.pos_b; io.dst_keys = p.keys_a; io.dst_pos = p.pos_a;
  }
  return io;
}

__global__ __launch_bounds__(256) void k_sort_hist(const EmbProb *__restrict__ probs, int pass) {
  __shared__ int hist[RADIX];
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks || pass >= p.passes) return;
  const int n_used = used_positions(p);
  const SortIo io = sort_io(p, pass);
  for (int d = threadIdx.x; d < RADIX; d += 256) hist[d] = 0;
  __syncthreads();
  const int base = blockIdx.x * SORT_CHUNK;
  for (int r = 0; r < SORT_CHUNK / 256; ++r) {
    const int j = base + r * 256 + threadIdx.x;
    if (j < n_used) {
      const int key = clamp_row(io.src_keys[j], p.num_rows);
      atomicAdd(&hist[(key >> (pass * RADIX_BITS)) & (RADIX - 1)], 1);
    }
  }
  __syncthreads();
  for (int d = threadIdx.x; d < RADIX; d += 256) p.hist[d * p.sort_blocks + blockIdx.x] = hist[d];
}

// Each workgroup first derives its own output offsets from the digit-major [RADIX][sort_blocks]
// count table (exclusive scan over digits of the per-digit totals, plus the counts of the blocks
// before it), then ranks its keys round by round, waves in order, so the scatter is stable.
__global__ __launch_bounds__(256) void k_sort_scatter(const EmbProb *__restrict__ probs, int pass) {
  __shared__ int next[RADIX];
  __shared__ int scan[256];
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks || pass >= p.passes) return;
  const int n_used = used_positions(p);
  const SortIo io = sort_io(p, pass);
  {
    int tot[RADIX / 256], mine[RADIX / 256], pair = 0;
#pragma unroll
    for (int k = 0; k < RADIX / 256; ++k) {
      const int d = threadIdx.x * (RADIX / 256) + k;
      int t = 0, m = 0;
      for (int b = 0; b < p.sort_blocks; ++b) {
        const int c = p.hist[d * p.sort_blocks + b];
        t += c;
        if (b < (int)blockIdx.x) m += c;
      }
      tot[k] = t;
      mine[k] = m;
      pair += t;
    }
    scan[threadIdx.x] = pair;
    __syncthreads();
    for (int o = 1; o < 256; o <<= 1) {
      const int v = (int)threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
      __syncthreads();
      scan[threadIdx.x] += v;
      __syncthreads();
    }
    int run = scan[threadIdx.x] - pair;
#pragma unroll
    for (int k = 0; k < RADIX / 256; ++k) {
      next[threadIdx.x * (RADIX / 256) + k] = run + mine[k];
      run += tot[k];
    }
  }
  __syncthreads();
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  const int base = blockIdx.x * SORT_CHUNK;
  for (int r = 0; r < SORT_CHUNK / 256; ++r) {
    const int j = base + r * 256 + threadIdx.x;
    const bool valid = j < n_used;
    int key = 0, pos = 0, digit = 0;
    if (valid) {
      key = clamp_row(io.src_keys[j], p.num_rows);
      pos = io.src_pos ? io.src_pos[j] : j;
      digit = (key >> (pass * RADIX_BITS)) & (RADIX - 1);
    }
    uint64_t peers = __ballot(valid);
#pragma unroll
    for (int b = 0; b < RADIX_BITS; ++b) {
      const bool bit = (digit >> b) & 1;
      const uint64_t m = __ballot(valid && bit);
      peers &= bit ? m : ~m;
    }
    const int rank = __popcll(peers & lt_mask);
    const int cnt = __popcll(peers);
    int dst = 0;
    for (int w = 0; w < 4; ++w) {   // waves in order: keeps the sort stable
      if (wave == w && valid) dst = next[digit] + rank;
      __syncthreads();
      if (wave == w && valid && rank == 0) next[digit] += cnt;
      __syncthreads();
    }
    if (valid) {
      io.dst_keys[dst] = key;
      io.dst_pos[dst] = pos;
    }
  }
}

// ------------------------------------------------------------------ segment heads
__device__ __forceinline__ const int32_t *sorted_keys(const EmbProb &p) { return (p.passes & 1) ? p.keys_a : p.keys_b; }
__device__ __forceinline__ const int32_t *sorted_pos(const EmbProb &p) { return (p.passes & 1) ? p.pos_a : p.pos_b; }
// bag id of every sorted position (-1 where the index was out of range), in the key buffer the sort
// no longer needs: the segment sums then read one array instead of chasing position -> index -> bag
__device__ __forceinline__ int32_t *sorted_bag(const EmbProb &p) { return (p.passes & 1) ? p.keys_b : p.keys_a; }

// heads per chunk of SORT_CHUNK sorted keys (stored in the first sort_blocks entries of `hist`)
__global__ __launch_bounds__(256) void k_seg_count(const EmbProb *__restrict__ probs, int slot) {
  __shared__ int red[4];
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks) return;
  const int n_used = used_positions(p);
  const int32_t *keys = sorted_keys(p);
  const int base = blockIdx.x * SORT_CHUNK + threadIdx.x * (SORT_CHUNK / 256);
  int s = 0;
#pragma unroll
  for (int e = 0; e < SORT_CHUNK / 256; ++e) {
    const int i = base + e;
    if (i < n_used && (i == 0 || keys[i] != keys[i - 1])) ++s;
  }
  {  // the gather list, coalesced: thread t takes positions chunk + t, chunk + t + 256, ...
    const int32_t *spos = sorted_pos(p);
    int32_t *sbag = sorted_bag(p);
#pragma unroll
    for (int e = 0; e < SORT_CHUNK / 256; ++e) {
      const int i = blockIdx.x * SORT_CHUNK + e * 256 + threadIdx.x;
      if (i < n_used) {
        const int pos = spos[i];
        const int r = p.indices[pos];
        sbag[i] = (r >= 0 && r < p.num_rows) ? p.bag_of[pos] : -1;
      }
    }
  }
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) {
    p.hist[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
    if (blockIdx.x == 0) p.counts[slot * 4 + 2] = 0;  // long-segment counter
  }
}

// unique_rows[slot], seg_offsets, counts[slot] = {n_used, n_unique, n_long}
__global__ __launch_bounds__(256) void k_seg_write(const EmbProb *__restrict__ probs, int slot) {
  __shared__ int scan[256];
  __shared__ int before_s, total_s;
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks) return;
  const int n_used = used_positions(p);
  const int32_t *keys = sorted_keys(p);
  int32_t *uniq = p.unique_rows + (int64_t)slot * p.capacity;
  if (threadIdx.x < 64) {   // one wave folds the per-chunk head counts
    int before = 0, total = 0;
    for (int b = threadIdx.x; b < p.sort_blocks; b += 64) {
      const int c = p.hist[b];
      total += c;
      if (b < (int)blockIdx.x) before += c;
    }
    for (int o = 32; o > 0; o >>= 1) {
      before += __shfl_xor(before, o, 64);
      total += __shfl_xor(total, o, 64);
    }
    if (threadIdx.x == 0) {
      before_s = before;
      total_s = total;
    }
  }
  const int base = blockIdx.x * SORT_CHUNK + threadIdx.x * (SORT_CHUNK / 256);
  int s = 0;
#pragma unroll
  for (int e = 0; e < SORT_CHUNK / 256; ++e) {
    const int i = base + e;
    if (i < n_used && (i == 0 || keys[i] != keys[i - 1])) ++s;
  }
  scan[threadIdx.x] = s;
  __syncthreads();
  for (int o = 1; o < 256; o <<= 1) {
    const int v = (int)threadIdx.x >= o ? scan[threadIdx.x - o] : 0;
    __syncthreads();
    scan[threadIdx.x] += v;
    __syncthreads();
  }
  int u = before_s + scan[threadIdx.x] - s;
#pragma unroll
  for (int e = 0; e < SORT_CHUNK / 256; ++e) {
    const int i = base + e;
    if (i < n_used && (i == 0 || keys[i] != keys[i - 1])) {
      uniq[u] = keys[i];
      p.seg_offsets[u] = i;
      ++u;
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    p.counts[slot * 4 + 0] = n_used;
    p.counts[slot * 4 + 1] = total_s;
    p.seg_offsets[total_s] = n_used;
  }
}

// ------------------------------------------------------------------ segment sums
// Vector path (dimension a multiple of 4, at most 256): a GROUP of 16 lanes owns one distinct row;
// lane l of the group holds columns 4 l + 64 k .. +3 for k < KV.  A wave therefore works on four
// rows at once and every lane has KV independent 16-byte loads in flight per position.
constexpr int GROUP = 16;
constexpr int KV_MAX = 4;
struct RowAcc {
  float4 v[KV_MAX];
};
__device__ __forceinline__ void acc_zero(RowAcc &a) {
#pragma unroll
  for (int k = 0; k < KV_MAX; ++k) a.v[k] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}
// a += pooled-output gradient row of `bag` (bag < 0: nothing)
__device__ __forceinline__ void acc_add_bag(RowAcc &a, const EmbProb &p, int bag, int l16) {
  if (bag < 0) return;
#pragma unroll
  for (int k = 0; k < KV_MAX; ++k) {
    const int c4 = 4 * l16 + 64 * k;
    if (c4 < p.dim) a.v[k] = f4_add(a.v[k], load4(p.out, p.out_dtype, (int64_t)bag * p.ld_out + c4));
  }
}
// sum over sorted positions lo, lo + stride, ... < hi, in that order, four positions in flight
__device__ __forceinline__ void acc_positions(RowAcc &a, const EmbProb &p, const int32_t *sbag, int lo, int hi, int stride, int l16) {
  int q = lo;
  for (; q + 3 * stride < hi; q += 4 * stride) {
    const int b0 = sbag[q], b1 = sbag[q + stride], b2 = sbag[q + 2 * stride], b3 = sbag[q + 3 * stride];
    RowAcc t0, t1;
    acc_zero(t0);
    acc_zero(t1);
    acc_add_bag(a, p, b0, l16);
    acc_add_bag(t0, p, b1, l16);
    acc_add_bag(t1, p, b2, l16);
    // fixed association: ((a + b0) + b1) + b2) + b3, with the loads issued together
#pragma unroll
    for (int k = 0; k < KV_MAX; ++k) a.v[k] = f4_add(f4_add(a.v[k], t0.v[k]), t1.v[k]);
    acc_add_bag(a, p, b3, l16);
  }
  for (; q < hi; q += stride) acc_add_bag(a, p, sbag[q], l16);
}
// `first`: no backward pass has touched the table since it was cleared, so every row still holds
// zeros and the sum is stored without reading the row
__device__ __forceinline__ void row_add(float *row, const RowAcc &a, int dim, int l16, bool first) {
#pragma unroll
  for (int k = 0; k < KV_MAX; ++k) {
    const int c4 = 4 * l16 + 64 * k;
    if (c4 < dim) {
      float4 *d = (float4 *)(row + c4);
      *d = first ? a.v[k] : f4_add(*d, a.v[k]);
    }
  }
}

// a group per distinct row; rows with more than SHORT_MAX positions are cut into slices of LONG_SEG
// and queued (entries (row id, slice) in consecutive list slots, slice order) for the two kernels below
__global__ __launch_bounds__(256) void k_emb_bwd_short(const EmbProb *__restrict__ probs, int slot, int first) {
  const EmbProb p = probs[blockIdx.y];
  const int l16 = threadIdx.x & (GROUP - 1);
  const int u = blockIdx.x * (256 / GROUP) + (threadIdx.x / GROUP);
  if (u >= p.counts[slot * 4 + 1]) return;
  const int lo = p.seg_offsets[u], hi = p.seg_offsets[u + 1];
  if (hi - lo > SHORT_MAX) {
    if (l16 == 0) {
      const int n_slices = (hi - lo + LONG_SEG - 1) / LONG_SEG;
      const int base = atomicAdd(&p.counts[slot * 4 + 2], n_slices);
      for (int sl = 0; sl < n_slices; ++sl) {
        p.long_list[2 * (base + sl)] = u;
        p.long_list[2 * (base + sl) + 1] = sl;
      }
    }
    return;
  }
  RowAcc a;
  acc_zero(a);
  acc_positions(a, p, sorted_bag(p), lo, hi, 1, l16);
  row_add(p.dtable + (int64_t)p.unique_rows[(int64_t)slot * p.capacity + u] * p.ld_table, a, p.dim, l16, first != 0);
}

// one workgroup of 16 groups per queued slice: group g sums positions g, g + 16, ... of the slice,
// the 16 partial rows are added in group order through LDS and stored as the slice's partial row
__global__ __launch_bounds__(256) void k_emb_bwd_long_partial(const EmbProb *__restrict__ probs, int slot) {
  __shared__ float4 part[256 / GROUP][KV_MAX][GROUP];
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.counts[slot * 4 + 2]) return;
  const int u = p.long_list[2 * blockIdx.x], sl = p.long_list[2 * blockIdx.x + 1];
  const int l16 = threadIdx.x & (GROUP - 1), g = threadIdx.x / GROUP;
  const int lo = p.seg_offsets[u] + sl * LONG_SEG, hi = min(p.seg_offsets[u + 1], lo + LONG_SEG);
  RowAcc a;
  acc_zero(a);
  acc_positions(a, p, sorted_bag(p), lo + g, hi, 256 / GROUP, l16);
#pragma unroll
  for (int k = 0; k < KV_MAX; ++k) part[g][k][l16] = a.v[k];
  __syncthreads();
  if (g == 0) {
    float *dst = p.partial + (int64_t)blockIdx.x * p.ld_table;
#pragma unroll
    for (int k = 0; k < KV_MAX; ++k) {
      const int c4 = 4 * l16 + 64 * k;
      if (c4 < p.dim) {
        float4 t = part[0][k][l16];
#pragma unroll
        for (int w = 1; w < 256 / GROUP; ++w) t = f4_add(t, part[w][k][l16]);
        *(float4 *)(dst + c4) = t;
      }
    }
  }
}
// a group per queued entry; the entry of a row's slice 0 adds that row's slice partials in slice order
__global__ __launch_bounds__(256) void k_emb_bwd_long_final(const EmbProb *__restrict__ probs, int slot, int first) {
  const EmbProb p = probs[blockIdx.y];
  const int e = blockIdx.x * (256 / GROUP) + (threadIdx.x / GROUP);
  if (e >= p.counts[slot * 4 + 2]) return;
  const int u = p.long_list[2 * e];
  if (p.long_list[2 * e + 1] != 0) return;
  const int l16 = threadIdx.x & (GROUP - 1);
  const int n_slices = (p.seg_offsets[u + 1] - p.seg_offsets[u] + LONG_SEG - 1) / LONG_SEG;
  RowAcc a;
  acc_zero(a);
  for (int sl = 0; sl < n_slices; ++sl) {
    const float *src = p.partial + (int64_t)(e + sl) * p.ld_table;
#pragma unroll
    for (int k = 0; k < KV_MAX; ++k) {
      const int c4 = 4 * l16 + 64 * k;
      if (c4 < p.dim) a.v[k] = f4_add(a.v[k], *(const float4 *)(src + c4));
    }
  }
  row_add(p.dtable + (int64_t)p.unique_rows[(int64_t)slot * p.capacity + u] * p.ld_table, a, p.dim, l16, first != 0);
}
// upper bound of queued slices: every segment longer than SHORT_MAX has at most len / LONG_SEG + 1 of them
int emb_long_entries(int capacity) { return capacity / SHORT_MAX + capacity / LONG_SEG + 2; }

// scalar fallback (dimension not a multiple of 4): one wave per distinct row, a lane per column
__global__ __launch_bounds__(256) void k_emb_bwd_generic(const EmbProb *__restrict__ probs, int slot) {
  const EmbProb p = probs[blockIdx.y];
  const int lane = threadIdx.x & 63;
  const int u = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (u >= p.counts[slot * 4 + 1]) return;
  const int32_t *spos = sorted_pos(p);
  const int lo = p.seg_offsets[u], hi = p.seg_offsets[u + 1];
  const int row = p.unique_rows[(int64_t)slot * p.capacity + u];
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int q = lo; q < hi; ++q) {
    const int pos = spos[q];
    const int r = p.indices[pos];
    if (r < 0 || r >= p.num_rows) continue;
    const int64_t go = (int64_t)p.bag_of[pos] * p.ld_out;
#pragma unroll
    for (int k = 0; k < 4; ++k) {
      const int c = lane + 64 * k;
      if (c < p.dim) acc[k] += load_as_f32(p.out, p.out_dtype, go + c);
    }
  }
  float *drow = p.dtable + (int64_t)row * p.ld_table;
#pragma unroll
  for (int k = 0; k < 4; ++k) {
    const int c = lane + 64 * k;
    if (c < p.dim) drow[c] += acc[k];
  }
}

int emb_bwd_num_launches(int max_passes, int vec) { return 2 * max_passes + 2 + (vec ? 3 : 1); }

int launch_emb_bwd(const EmbProb *probs, int n, int max_capacity, int max_sort_blocks, int max_passes, int vec,
                   int slot, int first, hipStream_t s) {
  if (n <= 0) return 0;
  for (int pass = 0; pass < max_passes; ++pass) {
    hipLaunchKernelGGL(k_sort_hist, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, pass);
    hipLaunchKernelGGL(k_sort_scatter, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, pass);
  }
  hipLaunchKernelGGL(k_seg_count, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, slot);
  hipLaunchKernelGGL(k_seg_write, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, slot);
  if (vec) {
    constexpr int GPB = 256 / GROUP;   // groups per workgroup
    hipLaunchKernelGGL(k_emb_bwd_short, dim3((max_capacity + GPB - 1) / GPB, n), dim3(256), 0, s, probs, slot, first);
    const int entries = emb_long_entries(max_capacity);
    hipLaunchKernelGGL(k_emb_bwd_long_partial, dim3(entries, n), dim3(256), 0, s, probs, slot);
    hipLaunchKernelGGL(k_emb_bwd_long_final, dim3((entries + GPB - 1) / GPB, n), dim3(256), 0, s, probs, slot, first);
  } else {
    hipLaunchKernelGGL(k_emb_bwd_generic, dim3((max_capacity + 3) / 4, n), dim3(256), 0, s, probs, slot);
  }
  return emb_bwd_num_launches(max_passes, vec);
}

// ------------------------------------------------------------------ gradient clear
// full clear of the table-gradient accumulators
__global__ __launch_bounds__(256) void k_emb_reset(const EmbProb *__restrict__ probs) {
  const EmbProb p = probs[blockIdx.y];
  const int64_t total = (int64_t)p.num_rows * p.ld_table / 4;  // ld_table is a multiple of 8
  float4 *d = (float4 *)p.dtable;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256)
    d[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}
// sparse clear: only the rows listed by the last `slots` backward passes (16 lanes per listed row)
__global__ __launch_bounds__(256) void k_emb_reset_rows(const EmbProb *__restrict__ probs) {
  const EmbProb p = probs[blockIdx.y];
  const int slot = blockIdx.z;
  const int u = blockIdx.x * 16 + (threadIdx.x >> 4);
  if (u >= p.counts[slot * 4 + 1]) return;
  float *drow = p.dtable + (int64_t)p.unique_rows[(int64_t)slot * p.capacity + u] * p.ld_table;
  if ((p.dim & 3) == 0 && (p.ld_table & 3) == 0) {
    for (int c = (threadIdx.x & 15) * 4; c < p.dim; c += 64) *(float4 *)(drow + c) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
  } else {
    for (int c = threadIdx.x & 15; c < p.dim; c += 16) drow[c] = 0.0f;
  }
}
void launch_emb_reset(const EmbProb *probs, int n, int max_capacity, int slots, hipStream_t s) {
  if (n <= 0) return;
  if (slots <= 0) hipLaunchKernelGGL(k_emb_reset, dim3(1024, n), dim3(256), 0, s, probs);
  else hipLaunchKernelGGL(k_emb_reset_rows, dim3((max_capacity + 15) / 16, n, slots), dim3(256), 0, s, probs);
}

}  // namespace gpp
