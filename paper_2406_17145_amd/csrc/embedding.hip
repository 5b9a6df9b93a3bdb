// Sparse path of a DLRM-shaped stage, grouped over all embedding tables:
//   forward   coalesced embedding-bag gather with sum pooling
//   backward  deterministic sorted segment reduction:
//             stable LSD radix sort of (row, position) keys -> per-row sums in sorted
//             order, started by the group that sits on a segment's first position ->
//             one read-modify-write per distinct row
//   reset     clears only the rows the backward passes since the last reset touched
// No float atomics anywhere and every sum has a fixed association order, so two
// runs give bit-identical gradients.
#include "device_utils.h"

namespace gpp {

constexpr int RADIX_BITS = 9;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_CHUNK = 1024;   // keys per workgroup per pass (four waves x 4 rounds of 64)
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
// Concatenated bag (one wave per bag): row j of the bag is copied to columns [j * dim, (j + 1) * dim) of
// the sample's output, slots beyond the bag's length are cleared.  VEC: dim is a multiple of 4 and the
// buffers are 16-byte aligned; dim / 4 lanes then move one row with one 16-byte load each, 64 / (dim / 4)
// rows per load instruction, CONCAT_UNROLL instructions requested before the first store.
constexpr int CONCAT_UNROLL = 8;
template <bool VEC>
__device__ __forceinline__ void emb_fwd_concat_body(const EmbProb &p, int bag, StageFlags *flags) {
  const int lane = threadIdx.x & 63;
  int lo = p.offsets[bag], hi = p.offsets[bag + 1];
  bool bad = lo < 0 || hi < lo || hi > p.capacity || hi - lo > p.bag_size || (bag == 0 && lo != 0);
  lo = max(0, min(lo, p.capacity));
  hi = max(lo, min(min(hi, p.capacity), lo + p.bag_size));
  const int len = hi - lo;
  const int64_t out0 = (int64_t)bag * p.ld_out;
  const int lpr = VEC ? max(1, p.dim >> 2) : 64, rpi = VEC ? max(1, 64 / lpr) : 1;
  const int sub = lane / lpr, c4 = (lane % lpr) * 4;
  for (int base = 0; base < len; base += 64) {
    const int cnt = min(64, len - base);
    int my = -1;
    if (lane < cnt) {
      my = p.indices[lo + base + lane];
      p.bag_of[lo + base + lane] = bag;
      if (my < 0 || my >= p.num_rows) {
        bad = true;
        my = -1;
      }
    }
    if (VEC) {
      for (int j0 = 0; j0 < cnt; j0 += rpi * CONCAT_UNROLL) {
        float4 v[CONCAT_UNROLL];
        bool none[CONCAT_UNROLL];
#pragma unroll
        for (int u = 0; u < CONCAT_UNROLL; ++u) {
          const int j = j0 + u * rpi + sub;
          const int r = __shfl(my, min(j, 63), 64);
          v[u] = *(const float4 *)(p.table + (int64_t)max(r, 0) * p.ld_table + (sub < rpi ? c4 : 0));
          none[u] = r < 0;       // (applied at the store: overwriting v[u] here would wait for its load, row by row)
        }
#pragma unroll
        for (int u = 0; u < CONCAT_UNROLL; ++u) {
          const int j = j0 + u * rpi + sub;
          // an index out of range leaves a zero row
          const float4 w = none[u] ? make_float4(0.0f, 0.0f, 0.0f, 0.0f) : v[u];
          if (j < cnt && sub < rpi) store4(p.out, p.out_dtype, out0 + (int64_t)(base + j) * p.dim + c4, w);
        }
      }
    } else {
      for (int j = 0; j < cnt; ++j) {
        const int r = __shfl(my, j, 64);
        for (int c = lane; c < p.dim; c += 64)
          store_from_f32(p.out, p.out_dtype, out0 + (int64_t)(base + j) * p.dim + c, r >= 0 ? p.table[(int64_t)r * p.ld_table + c] : 0.0f);
      }
    }
  }
  // slots the bag does not fill
  const int tail0 = len * p.dim, tail1 = p.bag_size * p.dim;
  if (VEC) {
    for (int c = tail0 + 4 * lane; c < tail1; c += 256) store4(p.out, p.out_dtype, out0 + c, make_float4(0.0f, 0.0f, 0.0f, 0.0f));
  } else {
    for (int c = tail0 + lane; c < tail1; c += 64) store_from_f32(p.out, p.out_dtype, out0 + c, 0.0f);
  }
  if (__any(bad) && lane == 0) flags->index_error = 1;
}

// generic: one wave per bag, a lane per column (any dimension up to 256)
__global__ __launch_bounds__(256) void k_emb_fwd(const EmbProb *__restrict__ probs, int n, StageFlags *flags) {
  const int pi = find_prob(probs, n, blockIdx.x);
  const EmbProb p = probs[pi];
  const int lane = threadIdx.x & 63;
  const int bag = (blockIdx.x - p.blk_begin) * 4 + (threadIdx.x >> 6);
  if (bag >= p.n_bags) return;
  if (p.concat) return emb_fwd_concat_body<false>(p, bag, flags);
  int lo = p.offsets[bag], hi = p.offsets[bag + 1];
  bool bad = lo < 0 || hi < lo || hi > p.capacity || (bag == 0 && lo != 0);   // offsets start at 0 and do not decrease
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
// before any of them is consumed (a bag of 20 rows of 128 floats is then ONE batch: one memory
// round trip instead of one per few rows; measured 57 -> 52 us against two batches of 16 and 4 rows); the loads are unconditional -- a lane without a row
// reads row 0 and discards it -- because a branch around a load would make the wave wait for the
// loads before it.  Sums run in index order within a sub-group; the sub-groups are combined in lane order.
constexpr int FWD_UNROLL = 10;
// Table -> XCD affinity of the gather (per_table > 0): hardware deals consecutive workgroup ids round-robin
// over the 8 XCDs, each with its own L2, and a popular row of a table is otherwise fetched from memory by
// every L2 whose workgroups meet it (measured on the recommendation workload: 254 MB fetched for 164 MB of
// distinct rows).  The first 8 * (n / 8) tables are served by one XCD each (table t by XCD t % 8: ids
// xcd + 8 * k, k = (t / 8) * per_table + block); the n % 8 tables left over keep consecutive ids, spread
// over all XCDs, so that every XCD has the same number of bags.  per_table = largest workgroup count of a table.
int emb_fwd_affinity_grid(int n, int per_table) { return n * per_table; }
__device__ __forceinline__ void emb_fwd_locate(int bid, int n, int per_table, int &table, int &blk) {
  const int full = (n / 8) * 8, split = full * per_table;
  if (bid < split) {
    const int k = bid >> 3;
    table = (bid & 7) + 8 * (k / per_table);
    blk = k % per_table;
  } else {
    table = full + (bid - split) / per_table;
    blk = (bid - split) % per_table;
  }
}
__global__ __launch_bounds__(256) void k_emb_fwd_vec(const EmbProb *__restrict__ probs, int n, int per_table, StageFlags *flags) {
  int pi, blk;
  if (per_table > 0) {
    emb_fwd_locate(blockIdx.x, n, per_table, pi, blk);
  } else {
    pi = find_prob(probs, n, blockIdx.x);
    blk = blockIdx.x - probs[pi].blk_begin;
  }
  const EmbProb p = probs[pi];
  const int lane = threadIdx.x & 63;
  const int bag = blk * 4 + (threadIdx.x >> 6);
  if (bag >= p.n_bags) return;
  if (p.concat) return emb_fwd_concat_body<true>(p, bag, flags);
  int lo = p.offsets[bag], hi = p.offsets[bag + 1];
  bool bad = lo < 0 || hi < lo || hi > p.capacity || (bag == 0 && lo != 0);   // offsets start at 0 and do not decrease
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
void launch_emb_fwd(const EmbProb *probs, int n, int total_blocks, int vec, int per_table, StageFlags *flags, hipStream_t s) {
  if (total_blocks <= 0) return;
  if (vec) hipLaunchKernelGGL(k_emb_fwd_vec, dim3(total_blocks), dim3(256), 0, s, probs, n, per_table, flags);
  else hipLaunchKernelGGL(k_emb_fwd, dim3(total_blocks), dim3(256), 0, s, probs, n, flags);
}

// ------------------------------------------------------------------ stable radix sort by row
// LSD radix sort of (row, position) with RADIX_BITS-bit digits.  A workgroup owns SORT_CHUNK
// consecutive keys, wave w of it the sub-range [256 w, 256 w + 256) in rounds of 64, so "key order"
// is wave-major and the scatter can rank its keys with three workgroup barriers in all: the waves
// count their digits privately, one pass turns the counts into per-wave start offsets (global
// base of the digit + the workgroups before this one + the waves before this one), then every wave
// walks its rounds alone.  The last pass writes the sorted rows into the log slot of this backward
// pass (the next gradient reset reads them there) and, next to the sorted positions, the bag id
// of every sorted position (-1 where the index was out of range), which is what the sums gather by.
struct SortIo {
  const int32_t *src_keys;
  const int32_t *src_pos;  // null in pass 0: position = index
  int32_t *dst_keys, *dst_pos;
};
__device__ __forceinline__ int32_t *log_keys(const EmbProb &p, int slot) { return p.unique_rows + (int64_t)slot * p.capacity; }
__device__ __forceinline__ SortIo sort_io(const EmbProb &p, int pass, int slot) {
  SortIo io;
  if (pass == 0) {
    io.src_keys = p.indices; io.src_pos = nullptr; io.dst_keys = p.keys_a; io.dst_pos = p.pos_a;
  } else if (pass & 1) {
    io.src_keys = p.keys_a; io.src_pos = p.pos_a; io.dst_keys = p.keys_b; io.dst_pos = p.pos_b;
  } else {
    io.src_keys = p.keys_b; io.src_pos = p.pos_b; io.dst_keys = p.keys_a; io.dst_pos = p.pos_a;
  }
  if (pass == p.passes - 1) io.dst_keys = log_keys(p, slot);
  return io;
}
constexpr int SORT_ROUNDS = SORT_CHUNK / 256;   // rounds of 64 keys per wave
// index of the key that lane `lane` of wave `wave` handles in round r of workgroup `blk`
__device__ __forceinline__ int sort_key_index(int blk, int wave, int r, int lane) {
  return blk * SORT_CHUNK + wave * (SORT_CHUNK / 4) + r * 64 + lane;
}

__global__ __launch_bounds__(256) void k_sort_hist(const EmbProb *__restrict__ probs, int pass, int slot) {
  __shared__ int hist[RADIX];
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks || pass >= p.passes) return;
  const int n_used = used_positions(p);
  const SortIo io = sort_io(p, pass, slot);
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (n_used <= 0) {   // nothing to sort: this workgroup's counts are zero (the whole workgroup takes this path)
    for (int d = threadIdx.x; d < RADIX; d += 256) p.hist[blockIdx.x * RADIX + d] = 0;
    return;
  }
  // loads without a branch around them (an index beyond the end reads the last key and drops it)
  int key[SORT_ROUNDS];
#pragma unroll
  for (int r = 0; r < SORT_ROUNDS; ++r) {
    const int j = sort_key_index(blockIdx.x, wave, r, lane);
    const int k = clamp_row(io.src_keys[min(j, n_used - 1)], p.num_rows);
    key[r] = j < n_used ? k : -1;
  }
  for (int d = threadIdx.x; d < RADIX; d += 256) hist[d] = 0;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < SORT_ROUNDS; ++r)
    if (key[r] >= 0) atomicAdd(&hist[(key[r] >> (pass * RADIX_BITS)) & (RADIX - 1)], 1);
  __syncthreads();
  for (int d = threadIdx.x; d < RADIX; d += 256) p.hist[blockIdx.x * RADIX + d] = hist[d];   // [block][digit]
}

// One workgroup per table turns the [block][digit] count table into output offsets, in place:
// entry [b][d] becomes the number of keys with digit d in the blocks before b, and row
// [sort_blocks] receives the exclusive scan over digits of the digit totals.  The scatter then needs
// two small loads per thread instead of the whole table per workgroup.
__global__ __launch_bounds__(256) void k_sort_offsets(const EmbProb *__restrict__ probs, int pass) {
  __shared__ int scan[4];
  const EmbProb p = probs[blockIdx.x];
  if (pass >= p.passes) return;
  static_assert(RADIX / 256 == 2, "two digits per thread");
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int run[2] = {0, 0};
  for (int b0 = 0; b0 < p.sort_blocks; b0 += 8) {   // eight rows of the table in flight
    int2 c[8];
#pragma unroll
    for (int u = 0; u < 8; ++u)
      c[u] = *(const int2 *)(p.hist + (int64_t)min(b0 + u, p.sort_blocks - 1) * RADIX + threadIdx.x * 2);
#pragma unroll
    for (int u = 0; u < 8; ++u) {
      if (b0 + u < p.sort_blocks) {
        *(int2 *)(p.hist + (int64_t)(b0 + u) * RADIX + threadIdx.x * 2) = make_int2(run[0], run[1]);
        run[0] += c[u].x;
        run[1] += c[u].y;
      }
    }
  }
  const int pair = run[0] + run[1];
  int incl = pair;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int v = __shfl_up(incl, o, 64);
    if (lane >= o) incl += v;
  }
  if (lane == 63) scan[wave] = incl;
  __syncthreads();
  int base = incl - pair;
  for (int w = 0; w < wave; ++w) base += scan[w];
  *(int2 *)(p.hist + (int64_t)p.sort_blocks * RADIX + threadIdx.x * 2) = make_int2(base, base + run[0]);
}

__global__ __launch_bounds__(256) void k_sort_scatter(const EmbProb *__restrict__ probs, int pass, int slot) {
  __shared__ int off[4][RADIX];   // per wave: digit counts, then the next output index of each digit
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks || pass >= p.passes) return;
  const int n_used = used_positions(p);
  const SortIo io = sort_io(p, pass, slot);
  const bool last = pass == p.passes - 1;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  if (n_used <= 0) {   // nothing to sort (the whole workgroup takes this path)
    if (last && blockIdx.x == 0 && threadIdx.x == 0) {
      p.counts[slot * 4 + 0] = 0;
      p.counts[slot * 4 + 2] = 0;
    }
    return;
  }
  // all of this thread's keys are requested before anything waits for them; no branch sits around a
  // load (an index beyond the end reads the last key and drops it)
  int key[SORT_ROUNDS], pos[SORT_ROUNDS];
#pragma unroll
  for (int r = 0; r < SORT_ROUNDS; ++r) {
    const int j = sort_key_index(blockIdx.x, wave, r, lane), jc = min(j, n_used - 1);
    const int k = clamp_row(io.src_keys[jc], p.num_rows);
    key[r] = j < n_used ? k : -1;
    pos[r] = jc;
  }
  if (io.src_pos) {
#pragma unroll
    for (int r = 0; r < SORT_ROUNDS; ++r) pos[r] = io.src_pos[pos[r]];
  }
  int bag[SORT_ROUNDS];
  if (last) {
#pragma unroll
    for (int r = 0; r < SORT_ROUNDS; ++r) {
      const int row = p.indices[pos[r]];
      const int b = p.bag_of[pos[r]];
      // a position that no bag of this micro-batch covers (offsets that break the contract; the forward pass has
      // flagged them) still holds what an earlier call wrote: only a real bag id is ever used as an index
      const bool b_ok = (unsigned)b < (unsigned)p.n_bags;
      // what the sums gather by: the bag, or, for concatenated bags, the slot of the position in the
      // gradient seen as [bags * bag_size, dim]
      const int slot_in_bag = p.concat ? pos[r] - p.offsets[b_ok ? b : 0] : 0;
      const int piece = p.concat ? b * p.bag_size + slot_in_bag : b;
      bag[r] = (b_ok && row >= 0 && row < p.num_rows && (unsigned)slot_in_bag < (unsigned)max(p.bag_size, 1)) ? piece : -1;
    }
  }
  for (int d = threadIdx.x; d < 4 * RADIX; d += 256) (&off[0][0])[d] = 0;
  __syncthreads();
#pragma unroll
  for (int r = 0; r < SORT_ROUNDS; ++r)
    if (key[r] >= 0) atomicAdd(&off[wave][(key[r] >> (pass * RADIX_BITS)) & (RADIX - 1)], 1);
  __syncthreads();
  {
    // thread t owns digits 2 t and 2 t + 1: first output index of the digit (whole table) plus the
    // keys with that digit in the workgroups before this one, then the waves in order
    static_assert(RADIX / 256 == 2, "two digits per thread");
    const int2 basev = *(const int2 *)(p.hist + (int64_t)p.sort_blocks * RADIX + threadIdx.x * 2);
    const int2 minev = *(const int2 *)(p.hist + (int64_t)blockIdx.x * RADIX + threadIdx.x * 2);
    const int start[2] = {basev.x + minev.x, basev.y + minev.y};
#pragma unroll
    for (int k = 0; k < RADIX / 256; ++k) {
      const int d = threadIdx.x * (RADIX / 256) + k;
      int next = start[k];
#pragma unroll
      for (int w = 0; w < 4; ++w) {
        const int c = off[w][d];
        off[w][d] = next;
        next += c;
      }
    }
  }
  __syncthreads();
  const uint64_t lt_mask = lane == 0 ? 0ull : (~0ull >> (64 - lane));
  int *mine_off = off[wave];
#pragma unroll
  for (int r = 0; r < SORT_ROUNDS; ++r) {
    const bool valid = key[r] >= 0;
    const int digit = valid ? (key[r] >> (pass * RADIX_BITS)) & (RADIX - 1) : 0;
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
    if (valid) dst = mine_off[digit] + rank;          // every lane of a digit reads before its first lane adds:
    __builtin_amdgcn_wave_barrier();                   // the wave executes these LDS accesses in program order
    if (valid && rank == 0) mine_off[digit] += cnt;
    __builtin_amdgcn_wave_barrier();
    if (valid) {
      io.dst_keys[dst] = key[r];
      io.dst_pos[dst] = pos[r];
      if (last) p.sbag[dst] = bag[r];
    }
  }
  if (last && blockIdx.x == 0 && threadIdx.x == 0) {
    p.counts[slot * 4 + 0] = n_used;
    p.counts[slot * 4 + 2] = 0;   // queue length of the long segments
  }
}

// ------------------------------------------------------------------ segment sums
// Vector path (dimension a multiple of 4, at most 256): a wave per 64 sorted positions finds the
// positions that start a segment (their row differs from the row before) and its four GROUPs of 16
// lanes sum those segments in sorted order, one read-modify-write of the gradient row each.  No
// prefix sum over segments is needed on this path.  Lane l of a group holds columns 4 l + 64 k ..
// +3 for k < KV, so a wave works on four rows at once and every lane has KV independent 16-byte
// loads in flight per position.
constexpr int GROUP = 16;
constexpr int KV_MAX = 4;
// KV = 16-byte pieces per lane = ceil(dimension / 64): a template parameter, so that the loads of a
// batch of rows are straight-line code, all requested before the first is used.  They are
// unconditional (a branch around a load makes the wave wait for the loads before it): a lane
// without a valid bag or column reads bag 0 / column 0 and discards the value.
template <int KV>
struct RowAcc {
  float4 v[KV];
};
template <int KV>
__device__ __forceinline__ void acc_zero(RowAcc<KV> &a) {
#pragma unroll
  for (int k = 0; k < KV; ++k) a.v[k] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}
// the pooled-output gradient rows of NB bags, requested together.  DT is that matrix's storage type
// as a template parameter (DT_F32 / DT_BF16; -1 = look at the record): a run-time test of the type
// in front of every load is a branch too, and would serialise the loads.
template <int KV, int NB, int DT>
__device__ __forceinline__ void rows_fetch(float4 (&r)[NB][KV], const EmbProb &p, const int (&bag)[NB], int l16) {
#pragma unroll
  for (int q = 0; q < NB; ++q)
#pragma unroll
    for (int k = 0; k < KV; ++k) {
      const int c4 = 4 * l16 + 64 * k;
      r[q][k] = load4(p.out, DT < 0 ? p.out_dtype : DT, (int64_t)max(bag[q], 0) * p.ld_out + (c4 < p.dim ? c4 : 0));
    }
}
// a = ((a + row 0) + row 1) + ... in that order; rows of bags < 0 (index out of range) are skipped
template <int KV, int NB>
__device__ __forceinline__ void rows_add(RowAcc<KV> &a, const float4 (&r)[NB][KV], const int (&bag)[NB]) {
#pragma unroll
  for (int q = 0; q < NB; ++q)
#pragma unroll
    for (int k = 0; k < KV; ++k)
      if (bag[q] >= 0) a.v[k] = f4_add(a.v[k], r[q][k]);
}
// sum over the positions whose bag ids are bags[lo], bags[lo + stride], ... (index < hi), in that
// order, four rows in flight; `bags` may be LDS or global memory
template <int KV, int DT>
__device__ __forceinline__ void acc_positions(RowAcc<KV> &a, const EmbProb &p, const int32_t *bags, int lo, int hi, int stride, int l16) {
  for (int q = lo; q < hi; q += 4 * stride) {
    int bag[4];
#pragma unroll
    for (int u = 0; u < 4; ++u) {
      const int b = bags[min(q + u * stride, hi - 1)];   // no branch around the load
      bag[u] = q + u * stride < hi ? b : -1;
    }
    float4 r[4][KV];
    rows_fetch<KV, 4, DT>(r, p, bag, l16);
    rows_add<KV, 4>(a, r, bag);
  }
}
// `first`: no backward pass has touched the table since it was cleared, so every row still holds
// zeros and the sum is stored without reading the row
template <int KV>
__device__ __forceinline__ void row_add(float *row, const RowAcc<KV> &a, int dim, int l16, bool first) {
#pragma unroll
  for (int k = 0; k < KV; ++k) {
    const int c4 = 4 * l16 + 64 * k;
    if (c4 < dim) {
      float4 *d = (float4 *)(row + c4);
      *d = first ? a.v[k] : f4_add(*d, a.v[k]);
    }
  }
}

// queue entry of a slice of a long segment: (first sorted position, positions, row, slices of the
// row when this is its first slice else 0); a row's entries are consecutive, in slice order
struct LongEntry {
  int32_t start, count, row, n_slices;
};

// A wave looks at 64 consecutive sorted positions: lane j loads the row of position base + j
// (coalesced), the positions whose row differs from the row before start a
// segment, and their lane numbers are listed, in order, in the wave's corner of LDS.  Returns the
// number of segment starts in the window.
// The rows themselves go to `wkey` (the groups of a wave run out of step afterwards, and a lane
// shuffle cannot read from a lane that has already left a loop; LDS can).
__device__ __forceinline__ int window_heads(const int32_t *keys, int base, int n_used, int lane, int *wkey, uint8_t *list) {
  const int i = base + lane;
  const int key = i < n_used ? keys[i] : -1;
  wkey[lane] = key;
  const int before = base > 0 ? keys[base - 1] : -1;           // same address for the whole wave
  int prev = __shfl_up(key, 1, 64);
  if (lane == 0) prev = before;
  const bool head = i < n_used && key != prev;
  const uint64_t hm = __ballot(head);
  if (head) list[__popcll(hm & (lane == 0 ? 0ull : (~0ull >> (64 - lane))))] = (uint8_t)lane;
  __builtin_amdgcn_wave_barrier();
  return __popcll(hm);
}
// end (exclusive) of the segment of row k0 that is known to reach position lo - 1: 16-ary search by
// a group of 16 lanes (`gl` = the group's first lane).  Invariant: row(lo - 1) == k0, and row(hi) != k0
// or hi == n_used.
__device__ __forceinline__ int segment_end(const int32_t *keys, int k0, int lo, int n_used, int l16, int gl) {
  int hi = n_used;
  while (lo < hi) {
    const int step = (hi - lo + 15) / 16;
    const int q = lo + l16 * step;
    const bool same = q < hi && keys[q] == k0;
    const int cnt = __popc((unsigned)(__ballot(same) >> gl) & 0xffffu);
    if (cnt == 0) {
      hi = lo;
    } else {
      hi = min(hi, lo + cnt * step);
      lo = lo + (cnt - 1) * step + 1;
    }
  }
  return lo;
}

// Table -> XCD affinity for launches whose workgroups of one table re-read that table's slice of a
// shared matrix: hardware deals consecutive workgroup ids of a 1-D grid round-robin over the 8
// XCDs, so workgroup id b runs on XCD b % 8; table t is served only by XCD t % 8, and that L2 then
// holds the slices of its three or four tables instead of all of them.  Grid: 8 * ceil(n / 8) *
// per_table workgroups; returns false for the ids beyond the last table.
__device__ __forceinline__ bool xcd_table(int bid, int n, int per_table, int &table, int &blk) {
  const int xcd = bid & 7, k = bid >> 3;
  table = xcd + 8 * (k / per_table);
  blk = k % per_table;
  return table < n;
}
int emb_xcd_grid(int n, int per_table) { return 8 * ((n + 7) / 8) * per_table; }

template <int KV, int DT>
__global__ __launch_bounds__(256) void k_emb_bwd_sum(const EmbProb *__restrict__ probs, int n, int per_table, int slot, int first) {
  __shared__ uint8_t heads[4][64];
  __shared__ int wkey[4][64], wbag[4][64];
  int table, blk;
  if (!xcd_table(blockIdx.x, n, per_table, table, blk)) return;
  const EmbProb p = probs[table];
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & (GROUP - 1), gl = lane & ~(GROUP - 1), g = lane / GROUP;
  const int base = (blk * 4 + wave) * 64;
  const int n_used = used_positions(p);
  if (base >= n_used) return;
  const int32_t *keys = log_keys(p, slot);
  const int32_t *sbag = p.sbag;
  wbag[wave][lane] = base + lane < n_used ? sbag[base + lane] : -1;
  const int n_heads = window_heads(keys, base, n_used, lane, wkey[wave], heads[wave]);
  const int *bagw = wbag[wave];
  const int window_end = min(64, n_used - base);
  const int after = base + 64 < n_used ? keys[base + 64] : -1;   // row of the position behind the window
  // The wave's four groups take the segments of the window in turn, SEGS at a time each: the rows
  // of the first two positions of all SEGS segments are requested together and their sums stored
  // together, because a wave gets its memory replies in order -- a store between two batches of loads
  // makes the second batch wait for the store's acknowledgement.  Most segments of a Zipf-distributed
  // table have one or two positions; the rest of a longer one follows, four rows in flight.
  constexpr int SEGS = 4, NG = 64 / GROUP;
  for (int o0 = 0; o0 < n_heads; o0 += NG * SEGS) {
    int h[SEGS], k0[SEGS], len[SEGS], bag[2 * SEGS];
#pragma unroll
    for (int u = 0; u < SEGS; ++u) {
      const int o = o0 + u * NG + g;
      const bool act = o < n_heads;
      h[u] = act ? (int)heads[wave][o] : 0;                          // lane of the segment's first position
      k0[u] = wkey[wave][h[u]];
      len[u] = act ? (o + 1 < n_heads ? (int)heads[wave][o + 1] : window_end) - h[u] : 0;
      if (act && o + 1 == n_heads && k0[u] == after)                 // runs on beyond the window
        len[u] = segment_end(keys, k0[u], base + 64, n_used, l16, gl) - (base + h[u]);
      if (len[u] > SHORT_MAX) {
        if (l16 == 0) {
          const int i = base + h[u];
          const int n_slices = (len[u] + LONG_SEG - 1) / LONG_SEG;
          const int qb = atomicAdd(&p.counts[slot * 4 + 2], n_slices);
          LongEntry *q = (LongEntry *)p.long_list + qb;
          for (int sl = 0; sl < n_slices; ++sl) {
            LongEntry e;
            e.start = i + sl * LONG_SEG;
            e.count = min(LONG_SEG, len[u] - sl * LONG_SEG);
            e.row = k0[u];
            e.n_slices = sl == 0 ? n_slices : 0;
            q[sl] = e;
          }
        }
        len[u] = 0;
      }
#pragma unroll
      for (int t = 0; t < 2; ++t) bag[2 * u + t] = (t < len[u] && h[u] + t < 64) ? bagw[h[u] + t] : -1;
    }
    float4 r[2 * SEGS][KV];
    rows_fetch<KV, 2 * SEGS, DT>(r, p, bag, l16);
    RowAcc<KV> a[SEGS];
#pragma unroll
    for (int u = 0; u < SEGS; ++u) {
      acc_zero(a[u]);
#pragma unroll
      for (int t = 0; t < 2; ++t)
#pragma unroll
        for (int k = 0; k < KV; ++k)
          if (bag[2 * u + t] >= 0) a[u].v[k] = f4_add(a[u].v[k], r[2 * u + t][k]);
    }
#pragma unroll
    for (int u = 0; u < SEGS; ++u) {
      if (len[u] > 2 || (len[u] == 2 && h[u] == 63)) {
        // positions inside the window take their bag ids from the wave's LDS copy, the rest from memory
        const int in_window = min(len[u], 64 - h[u]);
        if (in_window > 2) acc_positions<KV, DT>(a[u], p, bagw, h[u] + 2, h[u] + in_window, 1, l16);
        if (len[u] > in_window) acc_positions<KV, DT>(a[u], p, sbag, base + h[u] + in_window, base + h[u] + len[u], 1, l16);
      }
    }
#pragma unroll
    for (int u = 0; u < SEGS; ++u)
      if (len[u] > 0) row_add<KV>(p.dtable + (int64_t)k0[u] * p.ld_table, a[u], p.dim, l16, first != 0);
  }
}

// one workgroup of 16 groups per queued slice: group g sums positions g, g + 16, ... of the slice,
// the 16 partial rows are added in group order through LDS and stored as the slice's partial row
template <int KV, int DT>
__global__ __launch_bounds__(256) void k_emb_bwd_long_partial(const EmbProb *__restrict__ probs, int slot) {
  __shared__ float4 part[256 / GROUP][KV][GROUP];
  const EmbProb p = probs[blockIdx.y];
  const int n_long = p.counts[slot * 4 + 2];
  const int l16 = threadIdx.x & (GROUP - 1), g = threadIdx.x / GROUP;
  for (int e = blockIdx.x; e < n_long; e += gridDim.x) {
    const LongEntry le = ((const LongEntry *)p.long_list)[e];
    RowAcc<KV> a;
    acc_zero(a);
    acc_positions<KV, DT>(a, p, p.sbag, le.start + g, le.start + le.count, 256 / GROUP, l16);
    __syncthreads();   // `part` is free again
#pragma unroll
    for (int k = 0; k < KV; ++k) part[g][k][l16] = a.v[k];
    __syncthreads();
    if (g == 0) {
      float *dst = p.partial + (int64_t)e * p.ld_table;
#pragma unroll
      for (int k = 0; k < KV; ++k) {
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
}
// a group per queued entry; the entry of a row's slice 0 adds that row's slice partials in slice order
template <int KV>
__global__ __launch_bounds__(256) void k_emb_bwd_long_final(const EmbProb *__restrict__ probs, int slot, int first) {
  const EmbProb p = probs[blockIdx.y];
  const int n_long = p.counts[slot * 4 + 2];
  const int l16 = threadIdx.x & (GROUP - 1);
  for (int e = blockIdx.x * (256 / GROUP) + (threadIdx.x / GROUP); e < n_long; e += gridDim.x * (256 / GROUP)) {
    const LongEntry le = ((const LongEntry *)p.long_list)[e];
    if (le.n_slices == 0) continue;
    RowAcc<KV> a;
    acc_zero(a);
    for (int sl = 0; sl < le.n_slices; ++sl) {
      const float *src = p.partial + (int64_t)(e + sl) * p.ld_table;
#pragma unroll
      for (int k = 0; k < KV; ++k) {
        const int c4 = 4 * l16 + 64 * k;
        if (c4 < p.dim) a.v[k] = f4_add(a.v[k], *(const float4 *)(src + c4));
      }
    }
    row_add<KV>(p.dtable + (int64_t)le.row * p.ld_table, a, p.dim, l16, first != 0);
  }
}
// upper bound of queued slices: every segment longer than SHORT_MAX has at most len / LONG_SEG + 1 of them
int emb_long_entries(int capacity) { return capacity / SHORT_MAX + capacity / LONG_SEG + 2; }

// ------------------------------------------------------------------ segment table
// distinct rows, segment offsets and their count: needed by the scalar fallback below and handed
// out for inspection; the vector path does not use them.
__device__ __forceinline__ const int32_t *sorted_pos(const EmbProb &p) { return (p.passes & 1) ? p.pos_a : p.pos_b; }

// heads per chunk of SORT_CHUNK sorted keys (stored in the first sort_blocks entries of `hist`)
__global__ __launch_bounds__(256) void k_seg_count(const EmbProb *__restrict__ probs, int slot) {
  __shared__ int red[4];
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks) return;
  const int n_used = used_positions(p);
  const int32_t *keys = log_keys(p, slot);
  const int base = blockIdx.x * SORT_CHUNK + threadIdx.x * (SORT_CHUNK / 256);
  int s = 0;
#pragma unroll
  for (int e = 0; e < SORT_CHUNK / 256; ++e) {
    const int i = base + e;
    if (i < n_used && (i == 0 || keys[i] != keys[i - 1])) ++s;
  }
  for (int o = 32; o > 0; o >>= 1) s += __shfl_xor(s, o, 64);
  if ((threadIdx.x & 63) == 0) red[threadIdx.x >> 6] = s;
  __syncthreads();
  if (threadIdx.x == 0) p.hist[blockIdx.x] = red[0] + red[1] + red[2] + red[3];
}

// seg_rows, seg_offsets, counts[slot][1] = number of distinct rows
__global__ __launch_bounds__(256) void k_seg_write(const EmbProb *__restrict__ probs, int slot) {
  __shared__ int scan[256];
  __shared__ int before_s, total_s;
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks) return;
  const int n_used = used_positions(p);
  const int32_t *keys = log_keys(p, slot);
  int32_t *uniq = p.seg_rows;
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
    p.counts[slot * 4 + 1] = total_s;
    p.seg_offsets[total_s] = n_used;
  }
}
void launch_emb_segments(const EmbProb *probs, int n, int max_sort_blocks, int slot, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(k_seg_count, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, slot);
  hipLaunchKernelGGL(k_seg_write, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, slot);
}

// scalar fallback (dimension not a multiple of 4): one wave per distinct row, a lane per column
__global__ __launch_bounds__(256) void k_emb_bwd_generic(const EmbProb *__restrict__ probs, int slot) {
  const EmbProb p = probs[blockIdx.y];
  const int lane = threadIdx.x & 63;
  const int u = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (u >= p.counts[slot * 4 + 1]) return;
  const int lo = p.seg_offsets[u], hi = p.seg_offsets[u + 1];
  const int row = p.seg_rows[u];
  float acc[4] = {0.0f, 0.0f, 0.0f, 0.0f};
  for (int q = lo; q < hi; ++q) {
    const int bag = p.sbag[q];
    if (bag < 0) continue;
    const int64_t go = (int64_t)bag * p.ld_out;
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

template <int KV, int DT>
static void launch_sums_typed(const EmbProb *probs, int n, int per_table, dim3 g_sum, dim3 g_part, dim3 g_fin, int slot, int first,
                              hipStream_t s) {
  hipLaunchKernelGGL((k_emb_bwd_sum<KV, DT>), g_sum, dim3(256), 0, s, probs, n, per_table, slot, first);
  hipLaunchKernelGGL((k_emb_bwd_long_partial<KV, DT>), g_part, dim3(256), 0, s, probs, slot);
  hipLaunchKernelGGL((k_emb_bwd_long_final<KV>), g_fin, dim3(256), 0, s, probs, slot, first);
}
template <int KV>
static void launch_sums_kv(const EmbProb *probs, int n, int per_table, int out_dtype, dim3 g_sum, dim3 g_part, dim3 g_fin, int slot,
                           int first, hipStream_t s) {
  if (out_dtype == DT_BF16) launch_sums_typed<KV, DT_BF16>(probs, n, per_table, g_sum, g_part, g_fin, slot, first, s);
  else if (out_dtype == DT_F32) launch_sums_typed<KV, DT_F32>(probs, n, per_table, g_sum, g_part, g_fin, slot, first, s);
  else launch_sums_typed<KV, -1>(probs, n, per_table, g_sum, g_part, g_fin, slot, first, s);
}
static void launch_sums(const EmbProb *probs, int n, int per_table, int kv, int out_dtype, dim3 g_sum, dim3 g_part, dim3 g_fin,
                        int slot, int first, hipStream_t s) {
  if (kv <= 1) launch_sums_kv<1>(probs, n, per_table, out_dtype, g_sum, g_part, g_fin, slot, first, s);
  else if (kv == 2) launch_sums_kv<2>(probs, n, per_table, out_dtype, g_sum, g_part, g_fin, slot, first, s);
  else launch_sums_kv<4>(probs, n, per_table, out_dtype, g_sum, g_part, g_fin, slot, first, s);
}

int emb_bwd_num_launches(int max_passes, int vec) { return 3 * max_passes + (vec ? 3 : 3); }

int launch_emb_bwd(const EmbProb *probs, int n, int max_capacity, int max_sort_blocks, int max_passes, int vec, int max_dim,
                   int out_dtype, int slot, int first, hipStream_t s) {
  if (n <= 0) return 0;
  for (int pass = 0; pass < max_passes; ++pass) {
    hipLaunchKernelGGL(k_sort_hist, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, pass, slot);
    hipLaunchKernelGGL(k_sort_offsets, dim3(n), dim3(256), 0, s, probs, pass);
    hipLaunchKernelGGL(k_sort_scatter, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, pass, slot);
  }
  if (vec) {
    // the queue of long segments is short (a few hundred slices for a Zipf-distributed table):
    // fixed grids that loop over it
    const int entries = emb_long_entries(max_capacity);
    const int per_table = (max_capacity + 255) / 256;
    const dim3 g_sum(emb_xcd_grid(n, per_table)), g_part(entries < 256 ? entries : 256, n), g_fin(16, n);
    launch_sums(probs, n, per_table, (max_dim + 63) / 64, out_dtype, g_sum, g_part, g_fin, slot, first, s);
  } else {
    launch_emb_segments(probs, n, max_sort_blocks, slot, s);
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
// sparse clear: only the rows that the logged backward passes touched.  A wave per 64 sorted
// positions of a log slot; the positions that start a segment are listed and their rows cleared by
// the wave's four 16-lane groups in turn.
__global__ __launch_bounds__(256) void k_emb_reset_rows(const EmbProb *__restrict__ probs) {
  __shared__ uint8_t heads[4][64];
  __shared__ int wkey[4][64];
  const EmbProb p = probs[blockIdx.y];
  const int slot = blockIdx.z;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6, l16 = lane & 15, g = lane >> 4;
  const int base = (blockIdx.x * 4 + wave) * 64;
  const int n_used = min(p.counts[slot * 4 + 0], p.capacity);
  if (base >= n_used) return;
  const int n_heads = window_heads(log_keys(p, slot), base, n_used, lane, wkey[wave], heads[wave]);
  for (int o = g; o < n_heads; o += 4) {
    const int row = wkey[wave][heads[wave][o]];
    float *drow = p.dtable + (int64_t)row * p.ld_table;
    if ((p.dim & 3) == 0 && (p.ld_table & 3) == 0) {
      for (int c = l16 * 4; c < p.dim; c += 64) *(float4 *)(drow + c) = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
    } else {
      for (int c = l16; c < p.dim; c += 16) drow[c] = 0.0f;
    }
  }
}
void launch_emb_reset(const EmbProb *probs, int n, int max_capacity, int slots, hipStream_t s) {
  if (n <= 0) return;
  if (slots <= 0) hipLaunchKernelGGL(k_emb_reset, dim3(1024, n), dim3(256), 0, s, probs);
  else hipLaunchKernelGGL(k_emb_reset_rows, dim3((max_capacity + 255) / 256, n, slots), dim3(256), 0, s, probs);
}

}  // namespace gpp
