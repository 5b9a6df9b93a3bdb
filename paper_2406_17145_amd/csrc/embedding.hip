// Sparse path of a DLRM-shaped stage, grouped over all embedding tables:
//   forward   coalesced embedding-bag gather with sum pooling
//   backward  deterministic sorted segment reduction:
//             stable LSD radix sort of (row, position) keys -> segment heads ->
//             per-row sums in sorted order -> one read-modify-write per distinct row
// plus the pairwise-dot feature interaction.  No float atomics anywhere, so two
// runs give bit-identical gradients.
#include "device_utils.h"

namespace gpp {

constexpr int RADIX_BITS = 9;
constexpr int RADIX = 1 << RADIX_BITS;
constexpr int SORT_CHUNK = 2048;  // keys per workgroup per pass (256 threads x 8 rounds)

int emb_sort_chunk() { return SORT_CHUNK; }
int emb_radix_bits() { return RADIX_BITS; }
int emb_fwd_blocks(int n_bags) { return (n_bags + 3) / 4; }

// ------------------------------------------------------------------ forward
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
void launch_emb_fwd(const EmbProb *probs, int n, int total_blocks, StageFlags *flags, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_emb_fwd, dim3(total_blocks), dim3(256), 0, s, probs, n, flags);
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
// number of index positions in use = last offset, clamped to the capacity
__device__ __forceinline__ int used_positions(const EmbProb &p) { return max(0, min(p.offsets[p.n_bags], p.capacity)); }
// out-of-range rows are sorted as the nearest valid row; the segment sum skips them
__device__ __forceinline__ int clamp_row(int r, int num_rows) { return max(0, min(r, num_rows - 1)); }

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

// exclusive scan over the digit-major [RADIX][sort_blocks] counts of one table
__global__ __launch_bounds__(1024) void k_sort_scan(const EmbProb *__restrict__ probs, int pass) {
  __shared__ int part[1024];
  const EmbProb p = probs[blockIdx.x];
  if (pass >= p.passes) return;
  const int total = RADIX * p.sort_blocks;
  const int per = (total + 1023) / 1024;
  const int lo = threadIdx.x * per, hi = min(total, lo + per);
  int s = 0;
  for (int i = lo; i < hi; ++i) s += p.hist[i];
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    int v = threadIdx.x >= o ? part[threadIdx.x - o] : 0;
    __syncthreads();
    part[threadIdx.x] += v;
    __syncthreads();
  }
  int run = part[threadIdx.x] - s;
  for (int i = lo; i < hi; ++i) {
    int c = p.hist[i];
    p.hist[i] = run;
    run += c;
  }
}

__global__ __launch_bounds__(256) void k_sort_scatter(const EmbProb *__restrict__ probs, int pass) {
  __shared__ int next[RADIX];
  const EmbProb p = probs[blockIdx.y];
  if ((int)blockIdx.x >= p.sort_blocks || pass >= p.passes) return;
  const int n_used = used_positions(p);
  const SortIo io = sort_io(p, pass);
  for (int d = threadIdx.x; d < RADIX; d += 256) next[d] = p.hist[d * p.sort_blocks + blockIdx.x];
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

// segment heads of the sorted keys -> unique_rows, seg_offsets, counts[1]
__global__ __launch_bounds__(1024) void k_segments(const EmbProb *__restrict__ probs) {
  __shared__ int part[1024];
  const EmbProb p = probs[blockIdx.x];
  const int n_used = used_positions(p);
  const int32_t *keys = (p.passes & 1) ? p.keys_a : p.keys_b;
  const int per = (n_used + 1023) / 1024;
  const int lo = min(n_used, (int)threadIdx.x * per), hi = min(n_used, lo + per);
  int s = 0;
  for (int i = lo; i < hi; ++i) s += (i == 0 || keys[i] != keys[i - 1]) ? 1 : 0;
  part[threadIdx.x] = s;
  __syncthreads();
  for (int o = 1; o < 1024; o <<= 1) {
    int v = threadIdx.x >= o ? part[threadIdx.x - o] : 0;
    __syncthreads();
    part[threadIdx.x] += v;
    __syncthreads();
  }
  int u = part[threadIdx.x] - s;
  for (int i = lo; i < hi; ++i)
    if (i == 0 || keys[i] != keys[i - 1]) {
      p.unique_rows[u] = keys[i];
      p.seg_offsets[u] = i;
      ++u;
    }
  if (threadIdx.x == 1023) {
    p.counts[0] = n_used;
    p.counts[1] = part[1023];
    p.seg_offsets[part[1023]] = n_used;
  }
}

// one wave per distinct row: sum the pooled-output gradients of its positions in sorted order
__global__ __launch_bounds__(256) void k_emb_bwd(const EmbProb *__restrict__ probs) {
  const EmbProb p = probs[blockIdx.y];
  const int lane = threadIdx.x & 63;
  const int u = blockIdx.x * 4 + (threadIdx.x >> 6);
  if (u >= p.counts[1]) return;
  const int32_t *spos = (p.passes & 1) ? p.pos_a : p.pos_b;
  const int lo = p.seg_offsets[u], hi = p.seg_offsets[u + 1];
  const int row = p.unique_rows[u];
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

int emb_bwd_num_launches(int max_passes) { return 3 * max_passes + 2; }

int launch_emb_bwd(const EmbProb *probs, int n, int max_capacity, int max_sort_blocks, int max_passes,
                   StageFlags *flags, hipStream_t s) {
  (void)flags;
  if (n <= 0) return 0;
  for (int pass = 0; pass < max_passes; ++pass) {
    hipLaunchKernelGGL(k_sort_hist, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, pass);
    hipLaunchKernelGGL(k_sort_scan, dim3(n), dim3(1024), 0, s, probs, pass);
    hipLaunchKernelGGL(k_sort_scatter, dim3(max_sort_blocks, n), dim3(256), 0, s, probs, pass);
  }
  hipLaunchKernelGGL(k_segments, dim3(n), dim3(1024), 0, s, probs);
  hipLaunchKernelGGL(k_emb_bwd, dim3((max_capacity + 3) / 4, n), dim3(256), 0, s, probs);
  return emb_bwd_num_launches(max_passes);
}

// clears the table-gradient accumulators (iteration boundary)
__global__ __launch_bounds__(256) void k_emb_reset(const EmbProb *__restrict__ probs) {
  const EmbProb p = probs[blockIdx.y];
  const int64_t total = (int64_t)p.num_rows * p.ld_table / 4;  // ld_table is a multiple of 8
  float4 *d = (float4 *)p.dtable;
  for (int64_t i = (int64_t)blockIdx.x * 256 + threadIdx.x; i < total; i += (int64_t)gridDim.x * 256)
    d[i] = make_float4(0.0f, 0.0f, 0.0f, 0.0f);
}
void launch_emb_reset(const EmbProb *probs, int n, hipStream_t s) {
  if (n <= 0) return;
  hipLaunchKernelGGL(k_emb_reset, dim3(1024, n), dim3(256), 0, s, probs);
}

// ------------------------------------------------------------------ pairwise-dot interaction
// one workgroup per sample; the F vectors sit in LDS
__device__ __forceinline__ void term_to_pair(int t, int &i, int &j) {
  i = (int)((1.0f + sqrtf(1.0f + 8.0f * (float)t)) * 0.5f);
  while (i * (i - 1) / 2 > t) --i;
  while ((i + 1) * i / 2 <= t) ++i;
  j = t - i * (i - 1) / 2;
}

__global__ __launch_bounds__(256) void k_interact_fwd(const InteractProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const InteractProb p = probs[pi];
  const int s = blockIdx.x - p.blk_begin;
  const int st = p.d + 1;
  for (int e = threadIdx.x; e < p.F * p.d; e += 256)
    lds[(e / p.d) * st + (e % p.d)] = load_as_f32(p.x, p.x_dtype, (int64_t)s * p.ld_x + e);
  __syncthreads();
  for (int c = threadIdx.x; c < p.d; c += 256) store_from_f32(p.y, p.y_dtype, (int64_t)s * p.ld_y + c, lds[c]);
  const int terms = p.F * (p.F - 1) / 2;
  for (int t = threadIdx.x; t < terms; t += 256) {
    int i, j;
    term_to_pair(t, i, j);
    float a = 0.0f;
    for (int c = 0; c < p.d; ++c) a += lds[i * st + c] * lds[j * st + c];
    store_from_f32(p.y, p.y_dtype, (int64_t)s * p.ld_y + p.d + t, a);
  }
}

__global__ __launch_bounds__(256) void k_interact_bwd(const InteractProb *__restrict__ probs, int n) {
  extern __shared__ float lds[];
  const int pi = find_prob(probs, n, blockIdx.x);
  const InteractProb p = probs[pi];
  const int s = blockIdx.x - p.blk_begin;
  const int st = p.d + 1;
  float *T = lds;
  float *G = lds + p.F * st;  // symmetric F x F, zero diagonal
  for (int e = threadIdx.x; e < p.F * p.d; e += 256)
    T[(e / p.d) * st + (e % p.d)] = load_as_f32(p.x, p.x_dtype, (int64_t)s * p.ld_x + e);
  for (int e = threadIdx.x; e < p.F; e += 256) G[e * p.F + e] = 0.0f;
  const int terms = p.F * (p.F - 1) / 2;
  for (int t = threadIdx.x; t < terms; t += 256) {
    int i, j;
    term_to_pair(t, i, j);
    float g = load_as_f32(p.dy, p.dy_dtype, (int64_t)s * p.ld_dy + p.d + t);
    G[i * p.F + j] = g;
    G[j * p.F + i] = g;
  }
  __syncthreads();
  for (int e = threadIdx.x; e < p.F * p.d; e += 256) {
    const int i = e / p.d, c = e % p.d;
    float a = i == 0 ? load_as_f32(p.dy, p.dy_dtype, (int64_t)s * p.ld_dy + c) : 0.0f;
    for (int j = 0; j < p.F; ++j) a += G[i * p.F + j] * T[j * st + c];
    store_from_f32(p.y, p.y_dtype, (int64_t)s * p.ld_y + e, a);
  }
}

static size_t interact_lds(int F, int d) { return ((size_t)F * (d + 1) + (size_t)F * F) * sizeof(float); }
void launch_interact_fwd(const InteractProb *probs, int n, int total_blocks, int maxF, int maxd, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_interact_fwd, dim3(total_blocks), dim3(256), interact_lds(maxF, maxd), s, probs, n);
}
void launch_interact_bwd(const InteractProb *probs, int n, int total_blocks, int maxF, int maxd, hipStream_t s) {
  if (total_blocks <= 0) return;
  hipLaunchKernelGGL(k_interact_bwd, dim3(total_blocks), dim3(256), interact_lds(maxF, maxd), s, probs, n);
}
size_t interact_lds_bytes(int F, int d) { return interact_lds(F, d); }

}  // namespace gpp
