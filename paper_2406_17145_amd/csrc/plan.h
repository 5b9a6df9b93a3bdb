// Host-side stage planner: turns the operator DAG G_i of one GPP stage into
// an ordered list of grouped kernel launches (one per operator kind per
// topological level) plus the device tables those launches read.
#pragma once
#include <stdint.h>

#include <string>
#include <vector>

#include "../../include/gpp.h"
#define GPP_HOST_ONLY_UNIT      // host code only in the files that include this header: records with plain pointers
#include "kernels.h"

namespace gpp {

enum Space : int32_t { SP_NONE = -1, SP_SLOT = 0, SP_SHARED = 1, SP_ABS = 2 };

// A 2-D view of device memory, resolved to a pointer once the workspace base
// and the slot are known.
struct Buf {
  int32_t space = SP_NONE;
  int64_t off = 0;   // bytes from the start of its space (SP_ABS: the pointer itself)
  int64_t ld = 0;    // elements
  int32_t dtype = DT_F32;
  bool valid() const { return space != SP_NONE; }
};

enum Kern : int32_t {
  K_ELT, K_GEMM_GENERIC, K_GEMM_MFMA, K_COLSUM, K_LN_FWD, K_LN_BWD, K_LN_BWD_PARAMS, K_ATTN_FWD, K_ATTN_DQ,
  K_ATTN_DKV, K_POOL, K_EMB_FWD, K_EMB_BWD, K_INTERACT_FWD, K_INTERACT_BWD, K_LOSS_FWD, K_LOSS_BWD, K_LOSS_SUM,
  K_GEMM_SKINNY, K_GEMM_BWD_MERGED, K_LOSS_FWD_SMALL, K_GEMM_BIG, K_GEMM_DW_KSPLIT, K_GEMM_DW_GROUP, K_FORK, K_JOIN,
  K_HEAD_LOSS
};
enum ExtKind : int32_t { EXT_NONE = 0, EXT_INPUTS, EXT_OUTPUTS, EXT_GRAD_OUTPUTS, EXT_GRAD_INPUTS };

struct Step {
  int32_t kern;
  int64_t table_off;  // bytes into the slot's table blob
  int32_t n;          // records
  int32_t blocks;     // workgroups
  int32_t a0, a1, a2, a3; // kernel-specific launch arguments
  int32_t ext_kind, ext_base;
  int32_t launches;   // kernel launches this step enqueues
  int32_t lane;       // 0: the caller's stream; 1: the stage's side stream (between a K_FORK and a K_JOIN)
};

struct Node {
  gpp_op_desc_t d;
  std::vector<int> in, users;
  int level = 0;
  int64_t rows = 0, feat = 0;
  bool is_loss = false, is_output = false, wants_grad = false;
  int input_index = -1, output_index = -1;
  Buf val, aux, stat0, stat1, gout, extra;
  std::vector<Buf> more;     // embedding scratch
  int32_t gdtype = DT_F32;
  int fused_add = -1;        // LINEAR: ADD op performed in its epilogue
  int fused_by = -1;         // ADD: the LINEAR that performs it
  int val_parent = -1;       // value lives inside this CONCAT's buffer
  int gout_parent = -1;      // gradient is a view of this consumer's gradient
  int64_t val_col = 0, gout_col = 0;
  int loss_index = -1;
  int emb_passes = 0, emb_sort_blocks = 0;
  bool grad_direct = false;  // input: its gradient is written straight into the caller's buffer by the producing GEMM
};

struct Plan {
  std::vector<Node> nodes;
  std::vector<int> order;            // topological
  std::vector<std::vector<int>> by_level;
  std::vector<int> input_ops, output_ops, loss_ops;
  int64_t micro_batch = 0;
  int32_t slots = 1, flags = 0;
  int64_t slot_bytes = 0, shared_bytes = 0, table_bytes = 0, tmp_bytes = 0;
  int64_t gemm_partial_bytes = 0, gemm_counter_bytes = 0;   // split-K partial tiles and arrival counters
  int64_t off_flags = 0, off_tables = 0, off_group_tables = 0, off_slots = 0, off_shared = 0, total_bytes = 0;
  // group launches (flag bits 8-11 = L): a second copy of the launch tables in which the records of the slots
  // l, l + L, l + 2L, ... follow each other, one table per lane l, so that ONE launch covers a step of several
  // micro-batches of a kFkB group; 0 = none
  int32_t group_lanes = 0;
  Buf loss_scalars;                  // f32 partial losses per slot
  int loss_parts = 0;
  std::vector<Step> fwd, bwd;
  bool lanes = false;                // the step lists hold side-stream steps: the stage needs its side streams
  // the forward (backward) steps touch workspace memory that all slots share: passes of different
  // micro-batches must then run one after the other
  bool fwd_shared = false, bwd_shared = false;
  std::vector<Step> dwg;             // weight gradients of a group of backward passes (flag bit 2), slot 0's tables
  std::vector<uint8_t> blob;         // tables of the slot being emitted
  std::string error;

  gpp_status_t analyse(const gpp_stage_desc_t *desc);
  // emits steps + tables for `slot` against workspace base `ws` (may be null for sizing)
  gpp_status_t emit(int slot, char *ws);
  void layout();
};

}  // namespace gpp
