// Device-side problem records and launch entry points shared by the stage
// planner (host) and the HIP kernels.  One record describes one branch's share
// of a grouped launch: all independent operators of one topological level of
// the stage's operator graph run in one kernel, each workgroup finding its
// record through the per-record prefix sums (`blk_begin`).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

namespace gpp {

enum : int32_t { DT_F32 = 0, DT_BF16 = 1, DT_I32 = 2 };

// Every buffer a record names is device global memory.  The device pass is told so in the field types: a pointer
// that comes out of a record in memory otherwise has no known address space, and the compiler then uses flat
// loads and stores, which count on BOTH wait counters -- every wait for an LDS read (or for a cross-lane
// ds_bpermute) also waits for the global loads in flight, a whole memory round trip inside loops that meant
// to overlap them.  Same size and layout on the host, where the records are filled (the planner's source files
// hold no kernel and see the plain types in both compiler passes).
#if defined(__HIP_DEVICE_COMPILE__) && !defined(GPP_HOST_ONLY_UNIT)
#define GPP_G __attribute__((address_space(1)))
#else
#define GPP_G
#endif
enum : int32_t { ACT_NONE = 0, ACT_RELU = 1, ACT_GELU = 2 };
enum : int32_t { FORM_FWD = 0, FORM_DX = 1, FORM_DW = 2 };

// ---- grouped GEMM -----------------------------------------------------
// FORM_FWD  C[m,n] = act( sum_k A[m,k] * B[n,k] + bias[n] ) (+ res[m,n])      A = X, B = W
// FORM_DX   C[m,k] = ( sum_n A[m,n] * B[n,k] (+ res[m,k]) ) * act'(aux[m,k])   A = dZ, B = W
// FORM_DW   C[n,k] (+)= sum_m A[m,n] * B[m,k]                                  A = dZ, B = X
// M, N are the output's rows / columns, K the contraction length.
struct GemmProb {
  const GPP_G void *A, *B;
  GPP_G void *C;
  const GPP_G float *bias;
  GPP_G void *aux;        // FWD + GELU: stash of the activation derivative (written). DX: mask source / derivative (read).
  const GPP_G void *res;  // FWD: residual addend. DX: gradient addend (may equal C: accumulate).
  int64_t lda, ldb, ldc, ldaux, ldres;
  int32_t M, N, K;
  int32_t form, act;
  int32_t in_dtype;   // dtype of A and B (DT_F32 or DT_BF16)
  int32_t c_dtype, aux_dtype, res_dtype;
  int32_t blk_begin;  // first workgroup of this record
  int32_t tiles_n;    // tile columns of this record
  int32_t split_k;    // workgroups that share one output tile, each summing a slice of K
  GPP_G float *partial;     // split_k > 1: fp32 partial tiles [tile][split][tile elements + tile rows]
  GPP_G int32_t *counters;  // split_k > 1: arrival counter per tile (zero between launches)
  int32_t c_ext;      // > 0: C is entry c_ext - 1 of the launch's per-call pointer block (may be null: result not wanted)
};

// ---- 2-D copy / convert / accumulate / activation backward --------------
// dst[r,c] = cvt(src[r,c]) (+ addend[r,c]); rows x cols elements.
// mode 1 (act backward, in place on dst): dst[r,c] = dst[r,c] * act'(src[r,c])
// mode 2 (add): dst = src + addend
struct EltProb {
  const GPP_G void *src;
  GPP_G void *dst;
  const GPP_G void *addend;
  int64_t ld_src, ld_dst, ld_add;
  int32_t rows, cols;
  int32_t src_dtype, dst_dtype, add_dtype;
  int32_t mode, act;
  int32_t ext_src, ext_dst;  // >= 0: pointer comes from the per-call pointer block instead
  int32_t blk_begin;
};

// ---- column sums: out[c] (+)= sum_r src[r,c]  (bias gradients) ----------
struct ColsumProb {
  const GPP_G void *src;
  GPP_G float *out;
  int64_t ld;
  int32_t rows, cols, dtype;
  int32_t blk_begin;
};

// ---- LayerNorm ------------------------------------------------------------
struct LnProb {
  const GPP_G void *x;      // input rows
  GPP_G void *y;            // fwd: output; bwd: dx
  const GPP_G void *dy;     // bwd
  const GPP_G void *addend; // bwd: optional gradient addend for dx
  const GPP_G float *gamma, *beta;
  GPP_G float *mean, *rstd;        // per-row statistics (written fwd, read bwd)
  GPP_G float *dgamma, *dbeta;     // accumulators
  GPP_G float *partial;            // bwd scratch: [row_blocks, 2, d]
  int64_t ldx, ldy, lddy, ldadd;
  int32_t rows, d;
  int32_t x_dtype, y_dtype, dy_dtype, add_dtype;
  float eps;
  int32_t blk_begin;
  int32_t row_blocks;
};

// ---- attention -------------------------------------------------------------
struct AttnProb {
  const GPP_G void *qkv;   // [b*S, 3d]
  GPP_G void *out;         // fwd: O [b*S, d]; bwd: dqkv [b*S, 3d]
  const GPP_G void *dout;  // bwd: dO
  const GPP_G void *o;     // bwd: O (forward output)
  GPP_G float *lse;        // [b*heads, S] log-sum-exp of scaled scores
  GPP_G float *delta;      // [b*heads, S] rowsum(dO * O)
  int64_t ld_qkv, ld_out, ld_dout, ld_o;
  int32_t batch, heads, seq, dh;
  int32_t dtype, out_dtype;
  int32_t grad_dtype;  // bwd: dtype of dqkv
  int32_t blk_begin;
};

// ---- mean-pool over the sequence -------------------------------------------
struct PoolProb {
  const GPP_G void *src;
  GPP_G void *dst;
  int64_t ld_src, ld_dst;
  int32_t batch, seq, d;
  int32_t src_dtype, dst_dtype;
  int32_t backward;  // 0: dst[b,:] = mean_s src[b*S+s,:]; 1: dst[b*S+s,:] = src[b,:]/S
  int32_t blk_begin;
};

// ---- embedding bag ------------------------------------------------------------
struct EmbProb {
  const GPP_G float *table;
  GPP_G float *dtable;
  const GPP_G int32_t *indices;  // [capacity]
  const GPP_G int32_t *offsets;  // [n_bags+1]
  GPP_G void *out;               // fwd: pooled output; bwd: gradient w.r.t. pooled output (read)
  GPP_G int32_t *bag_of;         // [capacity] bag id of each index position (written fwd)
  GPP_G int32_t *keys_a, *keys_b, *pos_a, *pos_b;  // sort ping-pong buffers [capacity]
  GPP_G int32_t *hist;           // [radix, sort_blocks]
  GPP_G int32_t *unique_rows;    // [log_slots][capacity]: the SORTED rows of the last backward passes, one log slot each
                           // (a position whose row differs from the row before starts a distinct row)
  GPP_G int32_t *sbag;           // [capacity]: bag id of every sorted position (-1: index out of range)
  GPP_G int32_t *seg_rows;       // [capacity]: distinct rows in ascending order (scalar path and inspection only)
  GPP_G int32_t *seg_offsets;    // [capacity+1]: first sorted position of every distinct row (same)
  GPP_G int32_t *counts;         // [log_slots][4]: n_used, n_unique (inspection only), queued slices, -
  GPP_G int32_t *long_list;      // [emb_long_entries][4]: queued slices of long segments (start, count, row, slices)
  GPP_G float *partial;          // [emb_long_entries][ld_table]: partial row of each queued slice
  int64_t ld_table, ld_out;
  int32_t n_bags, capacity, dim, num_rows;
  int32_t out_dtype;
  int32_t sort_blocks, passes;
  int32_t blk_begin;
  // concat != 0: the rows of a bag are concatenated instead of summed.  Forward: row j of bag s goes to
  // out[s, j * dim ..]; backward: `out` is the gradient seen as [n_bags * bag_size, dim] (ld_out = dim) and
  // sbag holds s * bag_size + j, so the segment sums read one piece per position exactly as they read one
  // pooled row per position when summing
  int32_t concat, bag_size;
};

// ---- pairwise-dot interaction --------------------------------------------------
struct InteractProb {
  const GPP_G void *x;   // [b, F*d]
  GPP_G void *y;         // fwd: [b, d + F(F-1)/2]; bwd: dx [b, F*d]
  const GPP_G void *dy;  // bwd
  int64_t ld_x, ld_y, ld_dy;
  int32_t batch, F, d;
  int32_t x_dtype, y_dtype, dy_dtype;
  int32_t blk_begin;
};

// ---- loss heads -------------------------------------------------------------------
struct LossProb {
  const GPP_G void *y;        // prediction
  const GPP_G void *target;   // f32 targets or i32 labels
  GPP_G float *loss;          // fwd: scalar out
  GPP_G void *dy;             // bwd: gradient out
  int64_t ld_y, ld_t, ld_dy;
  int32_t rows, cols, kind;   // kind = gpp_op_kind_t value
  int32_t y_dtype, dy_dtype;
  float scale;
  int32_t blk_begin;
};

// A one-column head: Linear(K -> 1) without activation whose only consumer is an element-wise loss,
// with everything of it that depends on forward values alone, in one launch of one workgroup.
struct HeadProb {
  const GPP_G void *x;        // [rows x K] bf16: the head's input
  const GPP_G void *w;        // [K] bf16: the Linear's weight row
  const GPP_G float *bias;    // one float, or null
  const GPP_G void *target;   // [rows] f32, stride ld_t
  const GPP_G void *mask;     // [rows x K] bf16: what the derivative of x's activation is taken from, or null
  GPP_G void *y;              // [rows] prediction out, stride ld_y
  GPP_G void *dy;             // [rows] loss gradient out, stride ld_dy
  GPP_G void *dx;             // [rows x K] bf16: gradient of x (times the derivative of its activation) out
  GPP_G float *partials;      // tall heads (more rows than one workgroup sums): one partial loss per 8 rows, summed by the loss-sum launch
  int64_t ld_x, ld_t, ld_mask, ld_y, ld_dy, ld_dx;
  int32_t rows, K, kind;      // kind = gpp_op_kind_t value of the loss
  int32_t y_dtype, dy_dtype, act;
  float scale;
};

constexpr int HEAD_GROUP_MAX = 16;
struct HeadOuts {
  GPP_G float *p[HEAD_GROUP_MAX];   // where each member's loss sum goes
};

struct ExtPtrs {
  GPP_G void *p[64];
};

// per-stage device flags
struct StageFlags {
  int32_t index_error;    // an embedding index, a bag offset or a class label was out of range
};

// ---- launch entry points (defined next to the kernels) -------------------------
void launch_gemm_generic(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int in_dtype, hipStream_t s);
void launch_gemm_mfma(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int form, int tile,
                      const ExtPtrs &ext, hipStream_t s);
// tile geometry used by the planner to count workgroups
int gemm_generic_tiles(int M, int N, int *tiles_n);
int gemm_mfma_group_tile(int form, int maxM, int maxN);
int gemm_mfma_tiles_for(int tile, int M, int N, int *tiles_n);
int gemm_mfma_partial_floats(int tile);
// large-tile kernels: 256 x 256 or 128 x 256 outputs per workgroup of eight waves (tile_rows 256 / 128),
// 128 x 128 outputs per workgroup of four waves, three workgroups per compute unit (tile_rows 64)
void launch_gemm_big(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int form, int tile_rows, int direct,
                     const ExtPtrs &ext, hipStream_t s);
bool gemm_big_supported(const GemmProb &p);
bool gemm_big_direct_ok(const GemmProb &p);
// Backward-weight whose contraction runs over the rows of `n` stash slots, starting at slot `first` and
// wrapping at `total`; slot s lies s * stride bytes behind slot 0, whose addresses the records hold.
struct SlotGroup {
  int32_t first = 0, n = 1, total = 1, pad = 0;
  int64_t stride = 0;
};
void launch_gemm_dw_group(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int tile_rows, const SlotGroup &grp,
                          hipStream_t s);
int gemm_big_tile_rows(int form, int maxM, int maxN, int64_t launch_elems, int tiles256, int tiles128);
int gemm_big_tiles_for(int tile_rows, int M, int N, int *tiles_n);
// backward-weight for small weight matrices and many rows: 64 x 64 tiles, the contraction split over the waves
void launch_gemm_dw_ksplit(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, hipStream_t s);
int gemm_dw_ksplit_blocks(int M, int N);
// few-row (micro-batch <= 256 rows) forward / backward-data kernel
// members > 1: a group launch (the records are member 0's; member i's slot memory lies i * member_stride_bytes
// further, its per-call pointers i * member_ext_stride entries further); total_blocks counts one member
void launch_gemm_skinny(const GemmProb *probs, int n, int total_blocks, int form, int row_tiles, int col_tiles, int waves,
                        const ExtPtrs &ext, hipStream_t s, int members = 1, int64_t member_stride_bytes = 0,
                        int member_ext_stride = 0);
// backward of a level with few rows in one launch: records of form DX (few-row body) first, then
// records of form DW (tile body, two tiles per workgroup)
void launch_gemm_bwd_merged(const GemmProb *probs, int n, int total_blocks, int row_tiles, int col_tiles,
                            int accumulate_dw, const ExtPtrs &ext, hipStream_t s);
int gemm_bwd_merged_dw_tile();
int gemm_bwd_merged_ksplit_mark();   // split_k value of a backward-weight record that runs the contraction-split body
int gemm_bwd_merged_dw_blocks(int M, int N);
int gemm_skinny_blocks(int M, int N, int row_tiles, int col_tiles);
int gemm_skinny_row_tiles(int M);
int gemm_skinny_col_tiles(int blocks_at_64_columns);
int gemm_mfma_pick_split(int tile, int launch_tiles, int rows_in_tile, int K);
bool gemm_mfma_supported(const GemmProb &p);

void launch_elt(const EltProb *probs, int n, int total_blocks, const ExtPtrs &ext, hipStream_t s);
int elt_blocks(int rows, int cols);
void launch_colsum(const ColsumProb *probs, int n, int total_blocks, int accumulate, hipStream_t s);
int colsum_blocks(int cols);

// vec: 0 = generic kernel, else 8-column chunks per lane (1, 2, 4) of the bf16 vector kernel
void launch_ln_fwd(const LnProb *probs, int n, int total_blocks, int vec, hipStream_t s);
bool ln_fwd_vec_supported(const LnProb &p);
void launch_ln_bwd(const LnProb *probs, int n, int total_blocks, int max_d, int vec, hipStream_t s);
bool ln_bwd_vec_supported(const LnProb &p);
int ln_bwd_rows_per_block();
int ln_bwd_max_d();
void launch_ln_bwd_params(const LnProb *probs, int n, int total_blocks, int accumulate, hipStream_t s);
int ln_rows_per_block();
int ln_param_blocks(int d);

int attn_blocks(int batch, int heads, int seq);

void launch_pool(const PoolProb *probs, int n, int total_blocks, hipStream_t s);
int pool_blocks(const PoolProb &p);

void launch_emb_fwd(const EmbProb *probs, int n, int total_blocks, int vec, int per_table, StageFlags *flags, hipStream_t s);
int emb_fwd_affinity_grid(int n, int per_table);
int emb_fwd_blocks(int n_bags);
bool emb_vec_supported(const EmbProb &p);
// sort + segment heads + segment sums into log slot `slot`; returns the number of launches it enqueues
// `first`: the gradient tables are all zero (no backward since they were cleared): sums are stored, not added
// `max_dim`: largest embedding dimension among the tables (vector path: picks the lane layout);
// `out_dtype`: storage type of the pooled-output gradients when all tables share it, else -1
int launch_emb_bwd(const EmbProb *probs, int n, int max_capacity, int max_sort_blocks, int max_passes, int vec, int max_dim,
                   int out_dtype, int slot, int first, hipStream_t s);
int emb_bwd_num_launches(int max_passes, int vec);
// distinct rows, segment offsets and their count of log slot `slot` (the vector path does not need them)
void launch_emb_segments(const EmbProb *probs, int n, int max_sort_blocks, int slot, hipStream_t s);
int emb_sort_chunk();
int emb_radix_bits();
int emb_long_segment();
int emb_long_entries(int capacity);
int emb_log_slots();
// slots <= 0: clear whole tables; otherwise only the rows logged in slots [0, slots)
void launch_emb_reset(const EmbProb *probs, int n, int max_capacity, int slots, hipStream_t s);

void launch_loss_fwd(const LossProb *probs, int n, int total_blocks, StageFlags *flags, hipStream_t s);
int loss_fwd_blocks(const LossProb &p);
// every loss of the stage and their sum in one single-workgroup launch (rows x cols summed over the
// records at most loss_small_limit()); a null `out` skips the launch
void launch_loss_fwd_small(const LossProb *probs, int n, float *out, StageFlags *flags, hipStream_t s);
int loss_small_limit();
int loss_ce_row_limit();   // longest softmax cross-entropy row whose gradient the forward kernels can write
bool head_loss_supported(int64_t rows, int64_t K);
bool head_loss_is_tall(int64_t rows, int64_t K);
int head_loss_parts(int64_t rows);
void launch_head_loss(const HeadProb *prob, int members, int rows, int K, const HeadOuts &outs, hipStream_t s);
void launch_loss_bwd(const LossProb *probs, int n, int total_blocks, hipStream_t s);
int loss_bwd_blocks(const LossProb &p);

void launch_fill_zero(void *ptr, size_t bytes, hipStream_t s);

}  // namespace gpp
