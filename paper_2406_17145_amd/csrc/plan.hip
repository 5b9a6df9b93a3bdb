// Stage planner (host code).  See plan.h.
#include "plan.h"

#include <algorithm>
#include <cstring>
#include <functional>

namespace gpp {

// launch helpers defined next to their kernels
int attn_max_seq();
int attn_mfma_blocks(int batch, int heads, int seq);
bool attn_mfma_supported(const AttnProb &p);
size_t interact_lds_bytes(int F, int d);

static int64_t align_up(int64_t v, int64_t a) { return (v + a - 1) / a * a; }
static int64_t ld_of(int64_t features) { return align_up(features, 64); }
static int64_t esize(int32_t dt) { return dt == DT_BF16 ? 2 : 4; }
static bool is_float(int32_t dt) { return dt == DT_F32 || dt == DT_BF16; }

#define FAIL(code, msg)      \
  do {                       \
    error = (msg);           \
    return (code);           \
  } while (0)

// ===========================================================================
// analysis: validation (condition C1: the stage's sub-graph is a DAG), shapes,
// levels, fusion and aliasing decisions, buffer allocation
// ===========================================================================
gpp_status_t Plan::analyse(const gpp_stage_desc_t *desc) {
  if (!desc || !desc->ops) FAIL(GPP_ERR_INVALID_ARG, "null descriptor");
  if (desc->n_ops <= 0 || desc->n_ops > 65536) FAIL(GPP_ERR_INVALID_ARG, "n_ops out of range");
  if (desc->micro_batch <= 0 || desc->micro_batch > (1 << 24)) FAIL(GPP_ERR_INVALID_ARG, "micro_batch out of range");
  if (desc->in_flight_slots <= 0 || desc->in_flight_slots > 1024) FAIL(GPP_ERR_INVALID_ARG, "in_flight_slots out of range");
  micro_batch = desc->micro_batch;
  slots = desc->in_flight_slots;
  flags = desc->flags;
  group_lanes = (flags >> 8) & 15;
  if (group_lanes > 0 && (slots % group_lanes != 0 || slots / group_lanes < 2 || !(flags & 4))) group_lanes = 0;
  const int n = desc->n_ops;
  nodes.assign(n, Node());
  for (int i = 0; i < n; ++i) {
    Node &nd = nodes[i];
    nd.d = desc->ops[i];
    if (nd.d.kind < GPP_OP_INPUT || nd.d.kind > GPP_OP_EMBEDDING_BAG_CONCAT) FAIL(GPP_ERR_INVALID_ARG, "unknown operator kind");
    if (nd.d.n_in < 0 || nd.d.n_in > 4096 || (nd.d.n_in > 0 && !nd.d.in)) FAIL(GPP_ERR_INVALID_ARG, "bad producer list");
    for (int k = 0; k < nd.d.n_in; ++k) {
      int p = nd.d.in[k];
      if (p < 0 || p >= n) FAIL(GPP_ERR_BAD_GRAPH, "dangling edge: producer id out of range");
      nd.in.push_back(p);
    }
    nd.d.in = nullptr;
  }
  for (int i = 0; i < n; ++i)
    for (int p : nodes[i].in) nodes[p].users.push_back(i);

  // arity
  for (int i = 0; i < n; ++i) {
    const Node &nd = nodes[i];
    int want = -1;
    switch (nd.d.kind) {
      case GPP_OP_INPUT: want = 0; break;
      case GPP_OP_LINEAR: case GPP_OP_LAYERNORM: case GPP_OP_ATTENTION: case GPP_OP_MEANPOOL_SEQ:
      case GPP_OP_DOT_INTERACT: want = 1; break;
      case GPP_OP_ADD: case GPP_OP_EMBEDDING_BAG_SUM: case GPP_OP_EMBEDDING_BAG_CONCAT: case GPP_OP_LOSS_MSE: case GPP_OP_LOSS_CE:
      case GPP_OP_LOSS_BCE_LOGITS: want = 2; break;
      default: break;
    }
    if (want >= 0 && (int)nd.in.size() != want) FAIL(GPP_ERR_BAD_GRAPH, "operator has the wrong number of producers");
    if (nd.d.kind == GPP_OP_CONCAT && nd.in.empty()) FAIL(GPP_ERR_BAD_GRAPH, "concat without producers");
  }

  // topological order (Kahn); leftovers mean a cycle
  {
    std::vector<int> indeg(n);
    for (int i = 0; i < n; ++i) indeg[i] = (int)nodes[i].in.size();
    std::vector<int> ready;
    for (int i = 0; i < n; ++i)
      if (!indeg[i]) ready.push_back(i);
    size_t head = 0;
    while (head < ready.size()) {
      int i = ready[head++];
      order.push_back(i);
      for (int u : nodes[i].users)
        if (--indeg[u] == 0) ready.push_back(u);
    }
    if ((int)order.size() != n) FAIL(GPP_ERR_BAD_GRAPH, "operator graph has a cycle");
  }

  // shapes, dtypes, levels
  int max_level = 0;
  for (int i : order) {
    Node &nd = nodes[i];
    const gpp_op_desc_t &d = nd.d;
    auto in = [&](int k) -> Node & { return nodes[nd.in[k]]; };
    nd.level = 0;
    for (int p : nd.in) nd.level = std::max(nd.level, nodes[p].level + 1);
    max_level = std::max(max_level, nd.level);
    nd.is_loss = d.kind >= GPP_OP_LOSS_MSE && d.kind <= GPP_OP_LOSS_BCE_LOGITS;
    if (!nd.is_loss && (d.out_features <= 0 || d.out_features > (1ll << 31) - 64)) FAIL(GPP_ERR_SHAPE, "out_features out of range");
    if (d.dtype < GPP_F32 || d.dtype > GPP_I32) FAIL(GPP_ERR_INVALID_ARG, "bad dtype");
    for (int p : nd.in)
      if (nodes[p].is_loss) FAIL(GPP_ERR_BAD_GRAPH, "a loss operator cannot feed another operator");
    nd.feat = d.out_features;
    switch (d.kind) {
      case GPP_OP_INPUT:
        if (d.seq_len <= 0 || d.rows_extra < 0) FAIL(GPP_ERR_SHAPE, "input: seq_len must be >= 1, rows_extra >= 0");
        nd.rows = micro_batch * d.seq_len + d.rows_extra;
        if (d.requires_grad && !is_float(d.dtype)) FAIL(GPP_ERR_INVALID_ARG, "integer input cannot require a gradient");
        break;
      case GPP_OP_LINEAR:
        nd.rows = in(0).rows;
        if (in(0).feat != d.in_features) FAIL(GPP_ERR_SHAPE, "linear: in_features differs from the producer's features");
        if (!is_float(d.dtype) || !is_float(d.param_dtype)) FAIL(GPP_ERR_UNSUPPORTED, "linear: float dtypes only");
        if (in(0).d.dtype != d.param_dtype) FAIL(GPP_ERR_UNSUPPORTED, "linear: weight dtype must equal the producer's dtype");
        if (d.act < GPP_ACT_NONE || d.act > GPP_ACT_GELU_ERF) FAIL(GPP_ERR_INVALID_ARG, "linear: bad activation");
        break;
      case GPP_OP_LAYERNORM:
        nd.rows = in(0).rows;
        if (in(0).feat != d.out_features) FAIL(GPP_ERR_SHAPE, "layernorm: feature count differs from the producer's");
        if (!is_float(d.dtype) || !is_float(in(0).d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "layernorm: float dtypes only");
        if (!(d.eps > 0)) FAIL(GPP_ERR_INVALID_ARG, "layernorm: eps must be positive");
        break;
      case GPP_OP_ATTENTION:
        nd.rows = in(0).rows;
        if (in(0).feat != 3 * d.out_features) FAIL(GPP_ERR_SHAPE, "attention: producer must have 3*out_features columns (Q|K|V)");
        if (d.heads <= 0 || d.out_features % d.heads) FAIL(GPP_ERR_SHAPE, "attention: heads must divide out_features");
        if (d.seq_len <= 0 || nd.rows != micro_batch * d.seq_len) FAIL(GPP_ERR_SHAPE, "attention: rows must equal micro_batch*seq_len");
        if (d.out_features / d.heads > 128) FAIL(GPP_ERR_UNSUPPORTED, "attention: head dimension above 128");
        if (d.seq_len > attn_max_seq()) FAIL(GPP_ERR_UNSUPPORTED, "attention: sequence too long for this build");
        if (!is_float(d.dtype) || !is_float(in(0).d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "attention: float dtypes only");
        break;
      case GPP_OP_ADD:
        nd.rows = in(0).rows;
        if (in(0).rows != in(1).rows || in(0).feat != in(1).feat || in(0).feat != d.out_features)
          FAIL(GPP_ERR_SHAPE, "add: operand shapes differ");
        if (!is_float(d.dtype) || !is_float(in(0).d.dtype) || !is_float(in(1).d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "add: float dtypes only");
        break;
      case GPP_OP_MEANPOOL_SEQ:
        if (d.seq_len <= 0 || in(0).rows != micro_batch * d.seq_len) FAIL(GPP_ERR_SHAPE, "meanpool: producer rows must equal micro_batch*seq_len");
        if (in(0).feat != d.out_features) FAIL(GPP_ERR_SHAPE, "meanpool: feature count differs");
        if (!is_float(d.dtype) || !is_float(in(0).d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "meanpool: float dtypes only");
        nd.rows = micro_batch;
        break;
      case GPP_OP_CONCAT: {
        int64_t w = 0;
        nd.rows = in(0).rows;
        for (size_t k = 0; k < nd.in.size(); ++k) {
          if (in(k).rows != nd.rows) FAIL(GPP_ERR_SHAPE, "concat: producers have different row counts");
          if (in(k).d.dtype != d.dtype) FAIL(GPP_ERR_UNSUPPORTED, "concat: producers must share the concat's dtype");
          w += in(k).feat;
        }
        if (w != d.out_features) FAIL(GPP_ERR_SHAPE, "concat: out_features is not the sum of the producers' features");
        if (!is_float(d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "concat: float dtypes only");
        break;
      }
      case GPP_OP_EMBEDDING_BAG_SUM:
      case GPP_OP_EMBEDDING_BAG_CONCAT:
        nd.rows = micro_batch;
        if (d.kind == GPP_OP_EMBEDDING_BAG_CONCAT) {
          if (d.in_features <= 0 || d.in_features > 256) FAIL(GPP_ERR_UNSUPPORTED, "embedding bag: row width must be 1..256");
          if (d.out_features != d.bag_size * d.in_features) FAIL(GPP_ERR_SHAPE, "concatenated embedding bag: out_features must be bag_size * in_features");
          if (d.out_features % 64) FAIL(GPP_ERR_UNSUPPORTED, "concatenated embedding bag: bag_size * in_features must be a multiple of 64");
        }
        if (in(0).d.kind != GPP_OP_INPUT || in(1).d.kind != GPP_OP_INPUT || in(0).d.dtype != GPP_I32 || in(1).d.dtype != GPP_I32)
          FAIL(GPP_ERR_BAD_GRAPH, "embedding bag: producers must be i32 inputs (indices, offsets)");
        if (d.bag_size <= 0 || in(0).feat != d.bag_size || in(0).rows != micro_batch) FAIL(GPP_ERR_SHAPE, "embedding bag: indices input must be [micro_batch, bag_size]");
        if (in(1).feat != 1 || in(1).rows != micro_batch + 1) FAIL(GPP_ERR_SHAPE, "embedding bag: offsets input must have micro_batch+1 entries");
        if (d.num_rows <= 0 || d.num_rows > (1ll << 31) - 1) FAIL(GPP_ERR_SHAPE, "embedding bag: num_rows out of range");
        if (d.kind == GPP_OP_EMBEDDING_BAG_SUM && d.out_features > 256) FAIL(GPP_ERR_UNSUPPORTED, "embedding bag: dimension above 256");
        if (micro_batch * d.bag_size > (1ll << 30)) FAIL(GPP_ERR_UNSUPPORTED, "embedding bag: too many indices");
        if (!is_float(d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "embedding bag: float output only");
        break;
      case GPP_OP_DOT_INTERACT: {
        nd.rows = in(0).rows;
        if (d.in_features <= 0 || in(0).feat % d.in_features) FAIL(GPP_ERR_SHAPE, "interaction: producer features must be a multiple of the vector width");
        int64_t F = in(0).feat / d.in_features;
        if (d.out_features != d.in_features + F * (F - 1) / 2) FAIL(GPP_ERR_SHAPE, "interaction: out_features must be d + F(F-1)/2");
        if (interact_lds_bytes((int)F, (int)d.in_features) > 60000) FAIL(GPP_ERR_UNSUPPORTED, "interaction: F*d too large");
        if (!is_float(d.dtype) || !is_float(in(0).d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "interaction: float dtypes only");
        break;
      }
      case GPP_OP_LOSS_MSE: case GPP_OP_LOSS_BCE_LOGITS:
        if (in(1).d.kind != GPP_OP_INPUT || in(1).d.dtype != GPP_F32) FAIL(GPP_ERR_BAD_GRAPH, "loss: target must be an f32 input");
        if (in(0).rows != in(1).rows || in(0).feat != in(1).feat) FAIL(GPP_ERR_SHAPE, "loss: prediction and target shapes differ");
        if (!is_float(in(0).d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "loss: float prediction only");
        break;
      case GPP_OP_LOSS_CE:
        if (in(1).d.kind != GPP_OP_INPUT || in(1).d.dtype != GPP_I32) FAIL(GPP_ERR_BAD_GRAPH, "cross-entropy: labels must be an i32 input");
        if (in(0).rows != in(1).rows || in(1).feat != 1) FAIL(GPP_ERR_SHAPE, "cross-entropy: labels must be [rows, 1]");
        if (!is_float(in(0).d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "loss: float prediction only");
        break;
    }
    if (nd.rows > (1ll << 31) - 64) FAIL(GPP_ERR_SHAPE, "too many rows");
  }
  by_level.assign(max_level + 1, {});
  for (int i : order) by_level[nodes[i].level].push_back(i);
  for (auto &v : by_level) std::sort(v.begin(), v.end());

  // roles
  for (int i = 0; i < n; ++i) {
    Node &nd = nodes[i];
    if (nd.d.kind == GPP_OP_INPUT) {
      nd.input_index = (int)input_ops.size();
      input_ops.push_back(i);
      if (nd.users.empty()) FAIL(GPP_ERR_BAD_GRAPH, "an input has no consumer");
    } else if (nd.is_loss) {
      nd.loss_index = (int)loss_ops.size();
      loss_ops.push_back(i);
    } else if (nd.users.empty()) {
      nd.is_output = true;
      nd.output_index = (int)output_ops.size();
      output_ops.push_back(i);
      if (!is_float(nd.d.dtype)) FAIL(GPP_ERR_UNSUPPORTED, "stage outputs must be float tensors");
    }
  }
  if (loss_ops.empty() && output_ops.empty()) FAIL(GPP_ERR_BAD_GRAPH, "stage has neither an output nor a loss");
  for (int i : order) {
    Node &nd = nodes[i];
    const int k = nd.d.kind;
    nd.wants_grad = (k == GPP_OP_INPUT) ? nd.d.requires_grad != 0
                                        : (k == GPP_OP_LINEAR || k == GPP_OP_LAYERNORM || k == GPP_OP_EMBEDDING_BAG_SUM || k == GPP_OP_EMBEDDING_BAG_CONCAT);
    if (k != GPP_OP_INPUT && !nd.is_loss)
      for (int p : nd.in) nd.wants_grad = nd.wants_grad || nodes[p].wants_grad;
    if (nd.is_loss) nd.wants_grad = false;
    nd.gdtype = (k == GPP_OP_LINEAR) ? nd.d.param_dtype : nd.d.dtype;
  }

  // ---- fusion / aliasing decisions -------------------------------------
  for (int i = 0; i < n; ++i) {
    Node &nd = nodes[i];
    // a LINEAR without activation whose only consumer is an ADD performs the add in its epilogue
    if (nd.d.kind == GPP_OP_LINEAR && nd.d.act == GPP_ACT_NONE && nd.users.size() == 1) {
      Node &a = nodes[nd.users[0]];
      if (a.d.kind == GPP_OP_ADD && a.fused_by < 0 && a.in[0] != a.in[1]) {
        int other = a.in[0] == i ? a.in[1] : a.in[0];
        if (nodes[other].level < nd.level && nodes[other].d.kind != GPP_OP_INPUT) {
          nd.fused_add = nd.users[0];
          a.fused_by = i;
        } else if (nodes[other].level < nd.level) {  // inputs are staged before level 1, also fine
          nd.fused_add = nd.users[0];
          a.fused_by = i;
        }
      }
    }
  }
  for (int i = 0; i < n; ++i) {
    Node &c = nodes[i];
    if (c.d.kind != GPP_OP_CONCAT) continue;
    int64_t col = 0;
    for (int p : c.in) {
      Node &m = nodes[p];
      const bool sole = m.users.size() == 1 && std::count(c.in.begin(), c.in.end(), p) == 1;
      if (sole && m.fused_add < 0 && m.d.kind != GPP_OP_CONCAT) {
        m.val_parent = i;
        m.val_col = col;
      }
      // (a concatenated embedding bag reads its gradient as a dense [b * bag_size, d] matrix: own buffer)
      if (sole && m.gdtype == c.gdtype && m.wants_grad && m.d.kind != GPP_OP_EMBEDDING_BAG_CONCAT) {
        m.gout_parent = i;
        m.gout_col = col;
      }
      col += m.feat;
    }
  }
  for (int i = 0; i < n; ++i) {
    Node &a = nodes[i];
    if (a.d.kind != GPP_OP_ADD || a.in[0] == a.in[1]) continue;
    for (int p : a.in) {
      Node &m = nodes[p];
      const bool plain = !(m.d.kind == GPP_OP_LINEAR && m.d.act != GPP_ACT_NONE);
      if (m.users.size() == 1 && plain && m.gdtype == a.gdtype && m.wants_grad && m.d.kind != GPP_OP_INPUT &&
          m.d.kind != GPP_OP_EMBEDDING_BAG_CONCAT) {
        m.gout_parent = i;
        m.gout_col = 0;
      }
    }
  }

  // ---- buffers ----------------------------------------------------------
  int64_t slot_top = 0, shared_top = 0;
  auto alloc = [&](int32_t space, int64_t rows, int64_t cols, int32_t dt) {
    Buf b;
    b.space = space;
    b.ld = ld_of(cols);
    b.dtype = dt;
    int64_t &top = space == SP_SLOT ? slot_top : shared_top;
    b.off = top;
    top = align_up(top + rows * b.ld * esize(dt), 256);
    return b;
  };
  // values: parents (concats) first so members can alias into them
  std::function<void(int)> alloc_val = [&](int i) {
    Node &nd = nodes[i];
    if (nd.val.valid() || nd.is_loss) return;
    if (nd.d.kind == GPP_OP_LINEAR && nd.fused_add >= 0) return;  // lives in the ADD's buffer
    if (nd.val_parent >= 0) {
      alloc_val(nd.val_parent);
      const Node &c = nodes[nd.val_parent];
      nd.val = c.val;
      nd.val.off += nd.val_col * esize(c.val.dtype);
      return;
    }
    nd.val = alloc(SP_SLOT, nd.rows, nd.feat, nd.d.dtype);
    if (nd.d.dtype == DT_I32) nd.val.ld = nd.feat;  // index / offset / label lists stay dense
  };
  for (int i = 0; i < n; ++i) alloc_val(i);
  std::function<void(int)> alloc_gout = [&](int i) {
    Node &nd = nodes[i];
    if (nd.gout.valid() || nd.is_loss || !nd.wants_grad) return;
    if (nd.gout_parent >= 0) {
      alloc_gout(nd.gout_parent);
      const Node &c = nodes[nd.gout_parent];
      nd.gout = c.gout;
      nd.gout.off += nd.gout_col * esize(c.gout.dtype);
      return;
    }
    // grouped weight gradients read dZ of several in-flight micro-batches at once: a copy per slot
    nd.gout = alloc((flags & 4) ? SP_SLOT : SP_SHARED, nd.rows, nd.feat, nd.gdtype);
  };
  for (int i = 0; i < n; ++i) alloc_gout(i);
  for (int i = 0; i < n; ++i) {
    Node &nd = nodes[i];
    const gpp_op_desc_t &d = nd.d;
    if (d.kind == GPP_OP_LINEAR && d.act == GPP_ACT_GELU_ERF) nd.aux = alloc(SP_SLOT, nd.rows, nd.feat, d.dtype);
    if (d.kind == GPP_OP_LAYERNORM) {
      nd.stat0 = alloc(SP_SLOT, 1, nd.rows, DT_F32);
      nd.stat1 = alloc(SP_SLOT, 1, nd.rows, DT_F32);
      if (nd.feat <= ln_bwd_max_d()) {  // per-row-block partial sums of the gamma / beta gradients
        const int64_t rb = (nd.rows + ln_bwd_rows_per_block() - 1) / ln_bwd_rows_per_block();
        nd.extra = alloc(SP_SHARED, 1, rb * 2 * nd.feat, DT_F32);
      }
    }
    if (d.kind == GPP_OP_ATTENTION) {
      nd.stat0 = alloc(SP_SLOT, 1, micro_batch * d.heads * d.seq_len, DT_F32);    // log-sum-exp
      nd.stat1 = alloc(SP_SHARED, 1, micro_batch * d.heads * d.seq_len, DT_F32);  // rowsum(dO*O)
    }
    if (d.kind == GPP_OP_EMBEDDING_BAG_SUM || d.kind == GPP_OP_EMBEDDING_BAG_CONCAT) {
      const int64_t cap = micro_batch * d.bag_size;
      const int64_t row_width = d.kind == GPP_OP_EMBEDDING_BAG_CONCAT ? d.in_features : nd.feat;
      nd.extra = alloc(SP_SLOT, 1, cap, DT_I32);  // bag id of each position
      int bits = 0;
      while ((1ll << bits) < d.num_rows) ++bits;
      const int passes = std::max(1, (bits + emb_radix_bits() - 1) / emb_radix_bits());
      const int sort_blocks = (int)((cap + emb_sort_chunk() - 1) / emb_sort_chunk());
      nd.more.clear();
      for (int k = 0; k < 4; ++k) nd.more.push_back(alloc(SP_SHARED, 1, cap, DT_I32));            // keys a/b, pos a/b
      nd.more.push_back(alloc(SP_SHARED, 1, (int64_t)(1 << emb_radix_bits()) * (sort_blocks + 1), DT_I32));  // digit counts per block + digit bases
      nd.more.push_back(alloc(SP_SHARED, 1, cap * emb_log_slots(), DT_I32));  // sorted rows per log slot
      nd.more.push_back(alloc(SP_SHARED, 1, cap + 1, DT_I32));                // segment offsets
      nd.more.push_back(alloc(SP_SHARED, 1, 4 * emb_log_slots(), DT_I32));    // counts per log slot
      nd.more.push_back(alloc(SP_SHARED, 1, 4 * (int64_t)emb_long_entries((int)cap), DT_I32));       // queued slices of long segments
      nd.more.push_back(alloc(SP_SHARED, emb_long_entries((int)cap), ld_of(row_width), DT_F32));     // their partial rows
      nd.more.push_back(alloc(SP_SHARED, 1, cap, DT_I32));                    // bag id of every sorted position
      nd.more.push_back(alloc(SP_SHARED, 1, cap, DT_I32));                    // distinct rows (scalar path, inspection)
      nd.emb_passes = passes;
      nd.emb_sort_blocks = sort_blocks;
    }
  }
  {  // one partial loss per four prediction rows; the egress kernel folds them
    int64_t parts = 0;
    for (int i : loss_ops) {
      nodes[i].loss_index = (int)parts;
      parts += (nodes[nodes[i].in[0]].rows + 3) / 4;
    }
    loss_parts = (int)parts;
    loss_scalars = alloc(SP_SLOT, 1, std::max<int64_t>(1, parts), DT_F32);
  }
  slot_bytes = align_up(slot_top, 256);
  shared_bytes = align_up(shared_top, 256);
  return GPP_OK;
}

void Plan::layout() {
  off_flags = 0;
  off_tables = 256;
  off_group_tables = align_up(off_tables + (int64_t)slots * table_bytes, 256);
  off_slots = align_up(off_group_tables + (group_lanes > 0 ? (int64_t)slots * table_bytes : 0), 256);
  off_shared = off_slots + (int64_t)slots * slot_bytes;
  total_bytes = off_shared + shared_bytes + tmp_bytes + gemm_partial_bytes + gemm_counter_bytes;
}

// ===========================================================================
// emission
// ===========================================================================
namespace {

struct Emitter {
  Plan &pl;
  int slot;
  char *ws;
  std::vector<Step> *steps = nullptr;
  // gradient assembly state per node
  enum { G_EMPTY, G_ADDEND, G_WRITTEN };
  std::vector<int> gstate;
  std::vector<Buf> gaddend;
  std::vector<char> dz_ready;
  int64_t part_need = 0, cnt_need = 0;  // split-K scratch high-water marks over all launches
  std::vector<LnProb> ln_fold_later;    // LayerNorm parameter folds of the whole backward pass (see backward())
  std::vector<GemmProb> dw_group;   // backward-weight records left to the launch over a group of slots
  std::vector<char> loss_fused;     // per node: this loss's gradient is written by the forward pass
  std::vector<int> head_loss;       // per LINEAR node: the loss that computes it (one-column head fused into its loss), or -1
  // Embedding bags next to dense branches: the gather (forward) and the sort + segment sums (backward) are long
  // chains of launches that nothing on the dense side depends on until the branches merge.  They run on the
  // stage's side stream: K_FORK (side stream waits for what has been issued), the steps with lane 1, K_JOIN
  // before the first step that needs them.  emb_level = level of the first real consumer of a bag's output.
  int emb_level = -1;
  bool fork_open = false;
  std::vector<char> emb_hoisted;    // per node: its backward was issued early, on the side stream
  std::vector<int> written_level;   // level whose launches first wrote the node's gradient
  int cur_level = 0;
  int64_t shared_tmp_top;

  Emitter(Plan &p, int s, char *w) : pl(p), slot(s), ws(w) { shared_tmp_top = 0; }

  void *ptr(const Buf &b) const {
    if (!b.valid()) return nullptr;
    if (b.space == SP_ABS) return (void *)b.off;
    if (b.space == SP_SLOT) return ws + pl.off_slots + (int64_t)slot * pl.slot_bytes + b.off;
    // memory every slot shares: passes of different slots that use it may not overlap
    if (steps == &pl.fwd) pl.fwd_shared = true;
    else if (steps == &pl.bwd) pl.bwd_shared = true;
    return ws + pl.off_shared + b.off;
  }
  template <typename T>
  int64_t push_table(const std::vector<T> &recs) {
    int64_t off = align_up((int64_t)pl.blob.size(), 64);
    pl.blob.resize(off + recs.size() * sizeof(T));
    if (!recs.empty()) memcpy(pl.blob.data() + off, recs.data(), recs.size() * sizeof(T));
    return off;
  }
  Step &add_step(int kern, int64_t table_off, int n, int blocks) {
    Step s;
    memset(&s, 0, sizeof(s));
    s.kern = kern;
    s.table_off = table_off;
    s.n = n;
    s.blocks = blocks;
    s.launches = 1;
    steps->push_back(s);
    return steps->back();
  }

  void fork() {
    add_step(K_FORK, 0, 0, 0).launches = 0;
    fork_open = true;
    pl.lanes = true;
  }
  void join() {
    if (!fork_open) return;
    add_step(K_JOIN, 0, 0, 0).launches = 0;
    fork_open = false;
  }
  // level of the first operator that really reads node i's value (a concat the node is written into in place
  // is looked through)
  int consumer_level(int i) const {
    int m = 1 << 30;
    for (int u : pl.nodes[i].users) {
      const Node &c = pl.nodes[u];
      m = std::min(m, (c.d.kind == GPP_OP_CONCAT && pl.nodes[i].val_parent == u) ? consumer_level(u) : c.level);
    }
    return m;
  }
  void find_emb_level() {
    emb_level = -1;
    if (!(pl.flags & 8)) return;     // opt-in: measured -5 % at 128-512 rows, +3 % at 2048 rows per micro-batch
    bool dense = false;
    int lvl = 1 << 30;
    for (size_t i = 0; i < pl.nodes.size(); ++i) {
      const int k = pl.nodes[i].d.kind;
      if (k == GPP_OP_LINEAR) dense = true;
      if (k == GPP_OP_EMBEDDING_BAG_SUM || k == GPP_OP_EMBEDDING_BAG_CONCAT) lvl = std::min(lvl, consumer_level((int)i));
    }
    if (dense && lvl < (1 << 30)) emb_level = lvl;
  }

  EmbProb emb_bwd_record(int i) {
    auto &N = pl.nodes;
    Node &nd = N[i];
    const gpp_op_desc_t &d = nd.d;
    EmbProb e;
    memset(&e, 0, sizeof(e));
    e.concat = d.kind == GPP_OP_EMBEDDING_BAG_CONCAT;
    e.bag_size = (int32_t)d.bag_size;
    e.dim = (int32_t)(e.concat ? d.in_features : nd.feat);
    e.table = (const float *)d.param[0];
    e.dtable = (float *)d.grad[0];
    e.ld_table = ld_of(e.dim);
    e.indices = (const int32_t *)ptr(N[nd.in[0]].val);
    e.offsets = (const int32_t *)ptr(N[nd.in[1]].val);
    e.out = ptr(nd.gout);
    // concatenated bags: bag_size * dim is a multiple of 64, so the gradient rows carry no padding and
    // the matrix is also [micro_batch * bag_size, dim] with leading dimension dim
    e.ld_out = e.concat ? e.dim : nd.gout.ld;
    e.out_dtype = nd.gout.dtype;
    e.bag_of = (int32_t *)ptr(nd.extra);
    e.keys_a = (int32_t *)ptr(nd.more[0]);
    e.keys_b = (int32_t *)ptr(nd.more[1]);
    e.pos_a = (int32_t *)ptr(nd.more[2]);
    e.pos_b = (int32_t *)ptr(nd.more[3]);
    e.hist = (int32_t *)ptr(nd.more[4]);
    e.unique_rows = (int32_t *)ptr(nd.more[5]);
    e.seg_offsets = (int32_t *)ptr(nd.more[6]);
    e.counts = (int32_t *)ptr(nd.more[7]);
    e.long_list = (int32_t *)ptr(nd.more[8]);
    e.partial = (float *)ptr(nd.more[9]);
    e.sbag = (int32_t *)ptr(nd.more[10]);
    e.seg_rows = (int32_t *)ptr(nd.more[11]);
    e.n_bags = (int32_t)pl.micro_batch;
    e.capacity = (int32_t)(pl.micro_batch * d.bag_size);
    e.num_rows = (int32_t)d.num_rows;
    e.passes = nd.emb_passes;
    e.sort_blocks = nd.emb_sort_blocks;
    return e;
  }
  void emit_emb_bwd(std::vector<EmbProb> &embs, int lane) {
    if (embs.empty()) return;
    int cap = 0, sb = 0, ps = 0, md = 0, odt = embs[0].out_dtype;
    for (auto &e : embs) {
      cap = std::max(cap, e.capacity);
      sb = std::max(sb, e.sort_blocks);
      ps = std::max(ps, e.passes);
      md = std::max(md, e.dim);
      if (e.out_dtype != odt) odt = 3;   // mixed
    }
    bool vec = true;
    for (auto &e : embs) vec = vec && emb_vec_supported(e);
    pl.bwd_shared = true;   // accumulates parameter gradients in the order of the backward passes
    Step &s = add_step(K_EMB_BWD, push_table(embs), (int)embs.size(), 0);
    s.a0 = cap;
    s.a1 = sb;
    s.a2 = ps | (vec ? 256 : 0) | (odt << 9) | (md << 11);   // passes (8 bits), vector path, gradient dtype (2 bits), largest dimension
    s.launches = emb_bwd_num_launches(ps, vec ? 1 : 0);
    s.lane = lane;
  }

  // ---- elementwise helper ------------------------------------------------
  EltProb elt(const Buf &src, const Buf &dst, int64_t rows, int64_t cols) {
    EltProb e;
    memset(&e, 0, sizeof(e));
    e.src = ptr(src);
    e.dst = ptr(dst);
    e.ld_src = src.ld;
    e.ld_dst = dst.ld;
    e.rows = (int32_t)rows;
    e.cols = (int32_t)cols;
    e.src_dtype = src.dtype;
    e.dst_dtype = dst.dtype;
    e.ext_src = e.ext_dst = -1;
    return e;
  }
  void with_addend(EltProb &e, const Buf &a) {
    e.addend = ptr(a);
    e.ld_add = a.ld;
    e.add_dtype = a.dtype;
  }
  void emit_elt(std::vector<EltProb> &recs, int ext_kind = EXT_NONE, int ext_base = 0) {
    if (recs.empty()) return;
    int blocks = 0;
    for (auto &e : recs) {
      e.blk_begin = blocks;
      blocks += elt_blocks(e.rows, e.cols);
    }
    Step &s = add_step(K_ELT, push_table(recs), (int)recs.size(), blocks);
    s.ext_kind = ext_kind;
    s.ext_base = ext_base;
    recs.clear();
  }

  // ---- gradient targets ----------------------------------------------------
  struct Target {
    Buf dst, addend;      // addend valid: kernel must add it (may equal dst)
    bool post = false;    // kernel wrote into a temporary `dst`; accumulate into `final` afterwards
    Buf final_dst;
  };
  std::vector<EltProb> post_copies;

  Buf tmp_like(const Node &nd) {
    Buf b = nd.gout;
    b.space = SP_SHARED;
    b.ld = ld_of(nd.feat);
    b.off = pl.shared_bytes + shared_tmp_top;  // temporaries sit behind the planned shared region
    shared_tmp_top = align_up(shared_tmp_top + nd.rows * b.ld * esize(b.dtype), 256);
    return b;
  }
  void copy_now(const Buf &src, const Buf &dst, const Node &nd, bool accumulate) {
    std::vector<EltProb> r;
    EltProb e = elt(src, dst, nd.rows, nd.feat);
    if (accumulate) with_addend(e, dst);
    r.push_back(e);
    emit_elt(r);
  }
  Target acquire(int p, bool can_addend) {
    Node &nd = pl.nodes[p];
    Target t;
    t.dst = nd.gout;
    if (gstate[p] == G_ADDEND && !can_addend) {
      copy_now(gaddend[p], nd.gout, nd, false);
      gstate[p] = G_WRITTEN;
      written_level[p] = cur_level + 1;   // already launched
    }
    if (gstate[p] == G_EMPTY) {
      gstate[p] = G_WRITTEN;
      written_level[p] = cur_level;
    } else if (gstate[p] == G_ADDEND) {
      t.addend = gaddend[p];
      gstate[p] = G_WRITTEN;
      written_level[p] = cur_level;
    } else if (can_addend && written_level[p] != cur_level) {
      t.addend = nd.gout;   // accumulate in place: every earlier writer ran in an earlier launch
    } else {                // a launch of this same level also writes it: go through a temporary
      t.post = true;
      t.final_dst = nd.gout;
      t.dst = tmp_like(nd);
      EltProb e = elt(t.dst, t.final_dst, nd.rows, nd.feat);
      with_addend(e, t.final_dst);
      post_copies.push_back(e);
    }
    return t;
  }
  // accumulate-copies run after the level's kernels; two copies into one destination never share a launch
  void flush_post() {
    while (!post_copies.empty()) {
      std::vector<EltProb> now, later;
      for (auto &e : post_copies) {
        bool clash = false;
        for (auto &o : now) clash = clash || o.dst == e.dst;
        (clash ? later : now).push_back(e);
      }
      emit_elt(now);
      post_copies.swap(later);
    }
  }
  // a consumer hands `view` through unchanged (ADD, CONCAT)
  void pass_through(int p, const Buf &view) {
    Node &nd = pl.nodes[p];
    if (!nd.wants_grad || nd.gout_parent >= 0) return;
    if (gstate[p] == G_EMPTY) {
      gstate[p] = G_ADDEND;
      gaddend[p] = view;
      return;
    }
    if (gstate[p] == G_ADDEND) {
      copy_now(gaddend[p], nd.gout, nd, false);
      gstate[p] = G_WRITTEN;
      written_level[p] = cur_level + 1;   // already launched
    }
    if (written_level[p] == cur_level) {  // first writer is a kernel of this level, not launched yet
      EltProb e = elt(view, nd.gout, nd.rows, nd.feat);
      with_addend(e, nd.gout);
      post_copies.push_back(e);
    } else {
      copy_now(view, nd.gout, nd, true);
    }
  }

  // ---- GEMM grouping ---------------------------------------------------------
  void emit_gemms(std::vector<GemmProb> &recs) {
    if (recs.empty()) return;
    // split by kernel and operand dtype; each group is one launch
    auto on_mfma = [&](const GemmProb &r) { return !(pl.flags & 1) && r.in_dtype == DT_BF16 && gemm_mfma_supported(r); };
    auto wants_ext = [](const std::vector<GemmProb> &g) {
      for (auto &r : g)
        if (r.c_ext > 0) return true;
      return false;
    };
    // few rows, backward: both consumers of a level's dZ (dX and dW) share one launch
    bool merged_bwd = false;
    {
      std::vector<GemmProb> dx, dw;
      int max_m = 0;
      for (auto &r : recs)
        if (on_mfma(r)) {
          if (r.form == FORM_DX) {
            dx.push_back(r);
            max_m = std::max(max_m, r.M);
          } else if (r.form == FORM_DW) {
            dw.push_back(r);
          }
        }
      int row_tiles = dx.empty() ? 0 : gemm_skinny_row_tiles(max_m);
      // many rows but a small level (the MLPs of the recommendation workload): backward-data by the
      // contraction-splitting few-row body over 64-row blocks, backward-weight by the 64 x 64 tiles
      // whose waves split the long contraction -- the same two bodies the stand-alone launches
      // would use, in one launch instead of two
      bool dw_ksplit = false;
      if (!dx.empty() && !dw.empty() && row_tiles == 0 && !(pl.flags & 2)) {
        int64_t elems = 0;
        int tiles128 = 0, min_k = 1 << 30;
        for (auto &r : dx) elems += (int64_t)r.M * r.N;
        for (auto &r : dw) {
          tiles128 += gemm_mfma_tiles_for(128, r.M, r.N, nullptr);
          min_k = std::min(min_k, r.K);
        }
        if (elems < (int64_t)128 * 128 * 256 && min_k >= 512 && tiles128 < 192) {
          row_tiles = 2;
          dw_ksplit = true;
        }
      }
      if (!dx.empty() && !dw.empty() && row_tiles > 0 && !(pl.flags & 2)) {
        int blocks = 0, col_tiles = 2;
        skinny_pick_tiles(dx, row_tiles, col_tiles, false);
        for (auto &r : dx) {
          r.blk_begin = blocks;
          r.split_k = 1;
          blocks += gemm_skinny_blocks(r.M, r.N, row_tiles, col_tiles);
        }
        for (auto &r : dw) {
          r.blk_begin = blocks;
          if (dw_ksplit) {
            r.split_k = gemm_bwd_merged_ksplit_mark();
            blocks += gemm_dw_ksplit_blocks(r.M, r.N);
          } else {
            r.split_k = 1;
            r.tiles_n = (r.N + gemm_bwd_merged_dw_tile() - 1) / gemm_bwd_merged_dw_tile();
            blocks += gemm_bwd_merged_dw_blocks(r.M, r.N);
          }
        }
        const bool ext = wants_ext(dx);
        dx.insert(dx.end(), dw.begin(), dw.end());
        Step &s = add_step(K_GEMM_BWD_MERGED, push_table(dx), (int)dx.size(), blocks);
        s.a1 = col_tiles;
        s.a2 = row_tiles;
        if (ext) s.ext_kind = EXT_GRAD_INPUTS;
        merged_bwd = true;
      }
    }
    for (int use_mfma = 0; use_mfma < 2; ++use_mfma)
      for (int dt = 0; dt < 2; ++dt)
        for (int form = 0; form < 3; ++form) {
          std::vector<GemmProb> g;
          for (auto &r : recs) {
            bool m = on_mfma(r);
            if ((int)m == use_mfma && r.in_dtype == dt && (r.form == form || !use_mfma)) g.push_back(r);
          }
          if (!use_mfma && form > 0) continue;  // the generic kernel mixes forms in one launch
          if (use_mfma && form > 0 && merged_bwd) continue;
          if (g.empty()) continue;
          int blocks = 0, tile = 0, max_m = 0, max_n = 0;
          for (auto &r : g) {
            max_m = std::max(max_m, r.M);
            max_n = std::max(max_n, r.N);
          }
          if (use_mfma) tile = gemm_mfma_group_tile(form, max_m, max_n);
          // few rows: the weight-streaming kernel (forward and backward-data only)
          int row_tiles = (use_mfma && form != FORM_DW) ? gemm_skinny_row_tiles(max_m) : 0;
          // many rows but a small launch (fewer 128 x 128 tiles than compute units, e.g. the MLPs of the
          // recommendation workload at 2048 rows): the tiled kernels would run one workgroup on half of
          // the compute units with a barrier per k-step; the kernel whose waves split the contraction
          // covers the matrix with 64-row blocks instead (measured at [2048 x 1024 x 1024]: 14.8 us
          // against 20.7 us forward, 15.4 against 26.7 backward-data)
          if (use_mfma && form != FORM_DW && row_tiles == 0 && !(pl.flags & 2)) {
            int64_t elems = 0;
            for (auto &r : g) elems += (int64_t)r.M * r.N;
            if (elems < (int64_t)128 * 128 * 256) row_tiles = 2;
          }
          if (row_tiles > 0) {
            int blocks = 0, col_tiles = 2;
            // (group launches cover several micro-batches: the launch is large without the smaller row tile, and
            // 64-row tiles fetch each weight tile once per micro-batch: 1.73 M -> 2.02 M samples/s on the feature towers)
            skinny_pick_tiles(g, row_tiles, col_tiles, pl.group_lanes == 0);
            for (auto &r : g) {
              r.blk_begin = blocks;
              r.split_k = 1;
              blocks += gemm_skinny_blocks(r.M, r.N, row_tiles, col_tiles);
            }
            Step &s = add_step(K_GEMM_SKINNY, push_table(g), (int)g.size(), blocks);
            s.a0 = col_tiles;
            s.a1 = form;
            s.a2 = row_tiles;
            // waves per workgroup: four where the launch shares the GPU (flag bit 4) and has at most 64 rows
            // (measured on the feature-tower workload with four streams: 64 rows +21 %, 96 rows -6 %; keeping
            // eight waves for the launches with long contractions lowers their latency but the step gets 2 % slower)
            s.a3 = ((pl.flags & 16) && max_m <= 64) ? 4 : 8;
            if (wants_ext(g)) s.ext_kind = EXT_GRAD_INPUTS;
            continue;
          }
          // many rows and columns: the large-tile kernel
          if (use_mfma && !(pl.flags & 2)) {
            bool ok = true;
            int64_t elems = 0;
            int tiles256 = 0, tiles128 = 0;
            for (auto &r : g) {
              ok = ok && gemm_big_supported(r);
              elems += (int64_t)r.M * r.N;
              tiles256 += ((r.M + 255) / 256) * ((r.N + 255) / 256);
              tiles128 += ((r.M + 127) / 128) * ((r.N + 255) / 256);
            }
            int tile_rows = ok ? gemm_big_tile_rows(form, max_m, max_n, elems, tiles256, tiles128) : 0;
            if (tile_rows > 0) {
              // backward-data whose epilogue streams a second matrix (the stashed derivative or the mask source):
              // the 256 x 256 tiles' epilogues all fall together at the end of a round of tiles; three co-resident
              // 128 x 128 workgroups hide them behind each other's k-loops (measured cold on 4 x [2048 x 4096 x 1024]
              // with the GELU derivative: 119 -> 106 us)
              if (form == FORM_DX && tile_rows == 256) {
                bool second = true;
                for (auto &r : g) second = second && r.act != ACT_NONE;
                if (second) tile_rows = 64;
              }
              // operands copied straight into LDS (software-pipelined loops of the eight-wave tiles) where the
              // a operand is k-contiguous and the tile has such a loop: forward on both tiles (4 x [2048 x 4096 x
              // 1024] cold: 83 staged, 82 plain direct loop, 78 pipelined), backward-data on the 256 x 256 tile
              // (4 x [2048 x 4096 x 4096]: 336 staged, 297 pipelined; on the 128 x 256 tile the two 8-byte transposing
              // reads per fragment of W keep the staged loop ahead: 96 against 112 us)
              bool direct = form == FORM_FWD || (form == FORM_DX && tile_rows == 256);
              for (auto &r : g) direct = direct && gemm_big_direct_ok(r);
              int blocks = 0;
              for (auto &r : g) {
                r.blk_begin = blocks;
                r.split_k = 1;
                blocks += gemm_big_tiles_for(tile_rows, r.M, r.N, &r.tiles_n);
              }
              Step &s = add_step(K_GEMM_BIG, push_table(g), (int)g.size(), blocks);
              s.a0 = direct ? 1 : 0;
              s.a1 = form;
              s.a2 = tile_rows;
              if (wants_ext(g)) s.ext_kind = EXT_GRAD_INPUTS;
              continue;
            }
          }
          // backward-weight with a long contraction and too few 128 x 128 tiles to fill the chip:
          // small tiles, the contraction split over the waves of each workgroup
          if (use_mfma && form == FORM_DW && !(pl.flags & 2)) {
            int tiles128 = 0, min_k = 1 << 30;
            for (auto &r : g) {
              tiles128 += gemm_mfma_tiles_for(128, r.M, r.N, nullptr);
              min_k = std::min(min_k, r.K);
            }
            if (min_k >= 512 && tiles128 < 192) {
              int blocks = 0;
              for (auto &r : g) {
                r.blk_begin = blocks;
                r.split_k = 1;
                blocks += gemm_dw_ksplit_blocks(r.M, r.N);
              }
              add_step(K_GEMM_DW_KSPLIT, push_table(g), (int)g.size(), blocks);
              continue;
            }
          }
          int launch_tiles = 0;
          if (use_mfma)
            for (auto &r : g) launch_tiles += gemm_mfma_tiles_for(tile, r.M, r.N, nullptr);
          int64_t part_off = 0, cnt_off = 0;
          for (auto &r : g) {
            r.blk_begin = blocks;
            r.split_k = 1;
            if (!use_mfma) {
              blocks += gemm_generic_tiles(r.M, r.N, &r.tiles_n);
              continue;
            }
            const int tiles = gemm_mfma_tiles_for(tile, r.M, r.N, &r.tiles_n);
            // rows of the streamed operands that one tile covers: the output's rows for FWD / DX
            r.split_k = (pl.flags & 2) ? gemm_mfma_pick_split(tile, launch_tiles, form == FORM_DW ? tile : r.M, r.K) : 1;
            if (r.split_k > 1) {  // partial tiles and arrival counters live behind the shared region
              pl.fwd_shared = pl.bwd_shared = true;
              r.partial = (float *)(ws + pl.off_shared + pl.shared_bytes + pl.tmp_bytes + part_off);
              r.counters = (int32_t *)(ws + pl.off_shared + pl.shared_bytes + pl.tmp_bytes + pl.gemm_partial_bytes + cnt_off);
              part_off += (int64_t)tiles * r.split_k * gemm_mfma_partial_floats(tile) * 4;
              cnt_off += align_up((int64_t)tiles * 4, 256);
            }
            blocks += tiles * r.split_k;
          }
          part_need = std::max(part_need, align_up(part_off, 256));
          cnt_need = std::max(cnt_need, cnt_off);
          Step &s = add_step(use_mfma ? K_GEMM_MFMA : K_GEMM_GENERIC, push_table(g), (int)g.size(), blocks);
          s.a0 = dt;
          s.a1 = form;
          s.a2 = tile;
          if (use_mfma && wants_ext(g)) s.ext_kind = EXT_GRAD_INPUTS;
        }
    recs.clear();
  }

  // Tile shape of a few-row launch: `row_tiles` comes in as the largest row tile the rows allow.  The
  // work is streaming weights, so the launch wants more than one workgroup per compute unit: first
  // the column tile shrinks (64 -> 32 columns), then -- in the stand-alone launches -- the row tile
  // (64 -> 32 rows; the row blocks of a column block re-read its weights from one L2).  Measured on
  // the feature-tower workload: forward launches 16.1 -> 12.6 us; in the merged backward launch the
  // extra backward-data workgroups take compute units from the backward-weight tiles (17.7 -> 20.6 us),
  // so there the row tile stays.
  static void skinny_pick_tiles(const std::vector<GemmProb> &g, int &row_tiles, int &col_tiles, bool shrink_rows) {
    auto count = [&](int rt, int ct) {
      int b = 0;
      for (auto &r : g) b += gemm_skinny_blocks(r.M, r.N, rt, ct);
      return b;
    };
    col_tiles = gemm_skinny_col_tiles(count(row_tiles, 2));
    // up to 64 rows a workgroup's k-loop is the whole launch: 32 columns halve it, as long as the launch
    // stays at two workgroups per compute unit (branches of 256 ... 4096 columns, 304 workgroups: +15 % at
    // 64 rows, +7 % at 16 rows, -11 % at 128 rows; seven branches of 4096 columns, 896 workgroups: -8 %)
    int max_m = 0;
    for (auto &r : g) max_m = std::max(max_m, r.M);
    if (max_m <= 64 && count(row_tiles, 1) <= 512) col_tiles = 1;
    if (shrink_rows && col_tiles == 1 && row_tiles == 2 && count(2, 1) <= 256) row_tiles = 1;
  }

  gpp_status_t run();
  void forward();
  void backward();
};

// ---------------------------------------------------------------------------
void Emitter::forward() {
  steps = &pl.fwd;
  steps->clear();
  bool loss_summed = false;
  auto &N = pl.nodes;
  loss_fused.assign(N.size(), 0);
  // One-column heads: Linear(K -> 1) without activation feeding nothing but an element-wise loss, in a stage
  // with per-slot gradient buffers (grouped weight gradients).  The loss's launch then also computes the
  // Linear itself, the loss gradient and the gradient of the Linear's input (all of which depend on forward
  // values only): three launches of a micro-batch's chain become one.
  head_loss.assign(N.size(), -1);
  if ((pl.flags & 4) && !(pl.flags & 1) && pl.loss_ops.size() == 1) {
    const int li = pl.loss_ops[0];
    const Node &ls = N[li];
    const int yi = ls.in[0];
    const Node &y = N[yi];
    bool ok = ls.d.kind != GPP_OP_LOSS_CE && y.d.kind == GPP_OP_LINEAR && y.feat == 1 && y.d.act == GPP_ACT_NONE &&
              y.d.param_dtype == GPP_BF16 && y.wants_grad && y.users.size() == 1 && y.gout_parent < 0 && y.val_parent < 0 &&
              y.fused_add < 0 && !y.is_output && y.gout.space == SP_SLOT && y.rows <= loss_small_limit();
    if (ok) {
      const Node &x = N[y.in[0]];
      ok = x.d.kind == GPP_OP_LINEAR && x.wants_grad && x.users.size() == 1 && x.gout_parent < 0 && x.val_parent < 0 && x.fused_add < 0 && x.fused_by < 0 &&
           x.input_index < 0 && x.gout.space == SP_SLOT && x.val.dtype == DT_BF16 && x.gout.dtype == DT_BF16 && x.rows == y.rows &&
           head_loss_supported(x.rows, x.feat) && (x.val.ld & 7) == 0 && (x.gout.ld & 7) == 0 &&
           (x.d.act == GPP_ACT_NONE || (x.d.act == GPP_ACT_GELU_ERF ? x.aux : x.val).dtype == DT_BF16);
    }
    if (ok) head_loss[yi] = li;
  }
  find_emb_level();
  fork_open = false;

  // ingest: copy the caller's dense inputs into the (padded) stash buffers
  {
    std::vector<EltProb> recs;
    int base = 0;
    for (size_t k = 0; k < pl.input_ops.size(); ++k) {
      Node &nd = N[pl.input_ops[k]];
      if ((int)k - base == 64) {
        emit_elt(recs, EXT_INPUTS, base);
        base = (int)k;
      }
      Buf src;
      src.space = SP_ABS;
      src.ld = nd.feat;
      src.dtype = nd.d.dtype;
      EltProb e = elt(src, nd.val, nd.rows, nd.feat);
      e.ext_src = (int32_t)(k - base);
      recs.push_back(e);
    }
    emit_elt(recs, EXT_INPUTS, base);
  }

  for (size_t L = 1; L < pl.by_level.size(); ++L) {
    if ((int)L == emb_level) join();     // the first operator that reads a bag's output is on this level
    std::vector<GemmProb> gemms;
    std::vector<LnProb> lns;
    std::vector<AttnProb> attns;
    std::vector<EltProb> elts;
    std::vector<PoolProb> pools;
    std::vector<EmbProb> embs;
    std::vector<InteractProb> inters;
    std::vector<LossProb> losses;
    std::vector<HeadProb> heads;
    for (int i : pl.by_level[L]) {
      Node &nd = N[i];
      const gpp_op_desc_t &d = nd.d;
      switch (d.kind) {
        case GPP_OP_LINEAR: {
          if (head_loss[i] >= 0) break;      // computed by its loss's launch
          const Node &x = N[nd.in[0]];
          GemmProb g;
          memset(&g, 0, sizeof(g));
          g.form = FORM_FWD;
          g.A = ptr(x.val);
          g.lda = x.val.ld;
          g.B = d.param[0];
          g.ldb = ld_of(d.in_features);
          g.bias = d.has_bias ? (const float *)d.param[1] : nullptr;
          g.M = (int32_t)nd.rows;
          g.N = (int32_t)nd.feat;
          g.K = (int32_t)d.in_features;
          g.act = d.act;
          g.in_dtype = d.param_dtype;
          Buf out = nd.val;
          if (nd.fused_add >= 0) {
            const Node &a = N[nd.fused_add];
            const Node &r = N[a.in[0] == i ? a.in[1] : a.in[0]];
            out = a.val;
            g.res = ptr(r.val);
            g.ldres = r.val.ld;
            g.res_dtype = r.val.dtype;
          }
          g.C = ptr(out);
          g.ldc = out.ld;
          g.c_dtype = out.dtype;
          if (nd.aux.valid()) {
            g.aux = ptr(nd.aux);
            g.ldaux = nd.aux.ld;
            g.aux_dtype = nd.aux.dtype;
          }
          gemms.push_back(g);
          break;
        }
        case GPP_OP_LAYERNORM: {
          const Node &x = N[nd.in[0]];
          LnProb l;
          memset(&l, 0, sizeof(l));
          l.x = ptr(x.val);
          l.ldx = x.val.ld;
          l.x_dtype = x.val.dtype;
          l.y = ptr(nd.val);
          l.ldy = nd.val.ld;
          l.y_dtype = nd.val.dtype;
          l.gamma = (const float *)d.param[0];
          l.beta = (const float *)d.param[1];
          l.mean = (float *)ptr(nd.stat0);
          l.rstd = (float *)ptr(nd.stat1);
          l.rows = (int32_t)nd.rows;
          l.d = (int32_t)nd.feat;
          l.eps = (float)d.eps;
          lns.push_back(l);
          break;
        }
        case GPP_OP_ATTENTION: {
          const Node &x = N[nd.in[0]];
          AttnProb a;
          memset(&a, 0, sizeof(a));
          a.qkv = ptr(x.val);
          a.ld_qkv = x.val.ld;
          a.dtype = x.val.dtype;
          a.out = ptr(nd.val);
          a.ld_out = nd.val.ld;
          a.out_dtype = nd.val.dtype;
          a.lse = (float *)ptr(nd.stat0);
          a.batch = (int32_t)pl.micro_batch;
          a.heads = d.heads;
          a.seq = d.seq_len;
          a.dh = (int32_t)(nd.feat / d.heads);
          attns.push_back(a);
          break;
        }
        case GPP_OP_ADD: {
          if (nd.fused_by >= 0) break;
          EltProb e = elt(N[nd.in[0]].val, nd.val, nd.rows, nd.feat);
          with_addend(e, N[nd.in[1]].val);
          elts.push_back(e);
          break;
        }
        case GPP_OP_MEANPOOL_SEQ: {
          const Node &x = N[nd.in[0]];
          PoolProb p;
          memset(&p, 0, sizeof(p));
          p.src = ptr(x.val);
          p.ld_src = x.val.ld;
          p.src_dtype = x.val.dtype;
          p.dst = ptr(nd.val);
          p.ld_dst = nd.val.ld;
          p.dst_dtype = nd.val.dtype;
          p.batch = (int32_t)pl.micro_batch;
          p.seq = d.seq_len;
          p.d = (int32_t)nd.feat;
          pools.push_back(p);
          break;
        }
        case GPP_OP_CONCAT: {
          int64_t col = 0;
          for (int p : nd.in) {
            const Node &m = N[p];
            if (m.val_parent != i) {  // member could not be produced in place
              Buf dst = nd.val;
              dst.off += col * esize(dst.dtype);
              elts.push_back(elt(m.fused_add >= 0 ? N[m.fused_add].val : m.val, dst, m.rows, m.feat));
            }
            col += m.feat;
          }
          break;
        }
        case GPP_OP_EMBEDDING_BAG_SUM:
        case GPP_OP_EMBEDDING_BAG_CONCAT: {
          EmbProb e;
          memset(&e, 0, sizeof(e));
          e.concat = d.kind == GPP_OP_EMBEDDING_BAG_CONCAT;
          e.bag_size = (int32_t)d.bag_size;
          e.dim = (int32_t)(e.concat ? d.in_features : nd.feat);
          e.table = (const float *)d.param[0];
          e.ld_table = ld_of(e.dim);
          e.indices = (const int32_t *)ptr(N[nd.in[0]].val);
          e.offsets = (const int32_t *)ptr(N[nd.in[1]].val);
          e.out = ptr(nd.val);
          e.ld_out = nd.val.ld;
          e.out_dtype = nd.val.dtype;
          e.bag_of = (int32_t *)ptr(nd.extra);
          e.n_bags = (int32_t)pl.micro_batch;
          e.capacity = (int32_t)(pl.micro_batch * d.bag_size);
          e.num_rows = (int32_t)d.num_rows;
          embs.push_back(e);
          break;
        }
        case GPP_OP_DOT_INTERACT: {
          const Node &x = N[nd.in[0]];
          InteractProb p;
          memset(&p, 0, sizeof(p));
          p.x = ptr(x.val);
          p.ld_x = x.val.ld;
          p.x_dtype = x.val.dtype;
          p.y = ptr(nd.val);
          p.ld_y = nd.val.ld;
          p.y_dtype = nd.val.dtype;
          p.batch = (int32_t)nd.rows;
          p.d = (int32_t)d.in_features;
          p.F = (int32_t)(x.feat / d.in_features);
          inters.push_back(p);
          break;
        }
        case GPP_OP_LOSS_MSE: case GPP_OP_LOSS_CE: case GPP_OP_LOSS_BCE_LOGITS: {
          const Node &y = N[nd.in[0]];
          const Node &t = N[nd.in[1]];
          const Buf &yv = y.fused_add >= 0 ? N[y.fused_add].val : y.val;
          if (head_loss[nd.in[0]] == i) {     // the one-column head and its loss in one launch
            const Node &x = N[y.in[0]];
            HeadProb h;
            memset(&h, 0, sizeof(h));
            h.x = ptr(x.val);
            h.ld_x = x.val.ld;
            h.w = y.d.param[0];
            h.bias = y.d.has_bias ? (const float *)y.d.param[1] : nullptr;
            h.target = ptr(t.val);
            h.ld_t = t.val.ld;
            if (x.d.act != GPP_ACT_NONE) {
              const Buf &ms = x.d.act == GPP_ACT_GELU_ERF ? x.aux : x.val;
              h.mask = ptr(ms);
              h.ld_mask = ms.ld;
              h.act = x.d.act;
            }
            h.y = ptr(y.val);
            h.ld_y = y.val.ld;
            h.y_dtype = y.val.dtype;
            h.dy = ptr(y.gout);
            h.ld_dy = y.gout.ld;
            h.dy_dtype = y.gout.dtype;
            h.dx = ptr(x.gout);
            h.ld_dx = x.gout.ld;
            h.rows = (int32_t)y.rows;
            h.K = (int32_t)x.feat;
            // tall heads leave the sum of their per-workgroup partial losses to the loss-sum launch
            if (head_loss_is_tall(y.rows, x.feat)) h.partials = (float *)ptr(pl.loss_scalars) + nd.loss_index;
            h.kind = d.kind;
            h.scale = (float)d.loss_scale;
            heads.push_back(h);
            loss_fused[i] = 1;
            break;
          }
          LossProb l;
          memset(&l, 0, sizeof(l));
          l.y = ptr(yv);
          l.ld_y = yv.ld;
          l.y_dtype = yv.dtype;
          l.target = ptr(t.val);
          l.ld_t = t.val.ld;
          l.loss = (float *)ptr(pl.loss_scalars) + nd.loss_index;
          l.rows = (int32_t)y.rows;
          l.cols = (int32_t)y.feat;
          l.kind = d.kind;
          l.scale = (float)d.loss_scale;
          // per-slot gradient buffers (grouped weight gradients): an element-wise loss whose prediction
          // has no other consumer writes its gradient in the forward pass, one launch less per backward
          // (the softmax cross-entropy too, where its kernels keep a whole row of logits in registers)
          if ((pl.flags & 4) && (d.kind != GPP_OP_LOSS_CE || y.feat <= loss_ce_row_limit()) && y.wants_grad && y.users.size() == 1 &&
              y.gout_parent < 0 && y.fused_add < 0 && y.gout.space == SP_SLOT) {
            l.dy = ptr(y.gout);
            l.ld_dy = y.gout.ld;
            l.dy_dtype = y.gout.dtype;
            loss_fused[i] = 1;
          }
          losses.push_back(l);
          break;
        }
        default: break;
      }
    }
    // the gather first: on the side stream it runs next to everything else of this and the next levels
    if (!embs.empty()) {
      int blocks = 0;
      for (auto &e : embs) {
        e.blk_begin = blocks;
        blocks += emb_fwd_blocks(e.n_bags);
      }
      bool vec = true;
      for (auto &e : embs) vec = vec && emb_vec_supported(e);
      // vector kernel with eight or more tables: table -> XCD affinity (see emb_fwd_affinity_grid); a1 = the
      // largest workgroup count of a table, the grid is then laid out per table instead of by prefix sums
      int per_table = 0;
      for (auto &e : embs) per_table = std::max(per_table, emb_fwd_blocks(e.n_bags));
      const bool affinity = vec && embs.size() >= 8;
      const bool side = emb_level > (int)L;     // something else can run before the bags are needed
      if (side && !fork_open) fork();
      Step &se = add_step(K_EMB_FWD, push_table(embs), (int)embs.size(), affinity ? emb_fwd_affinity_grid((int)embs.size(), per_table) : blocks);
      se.a0 = vec ? 1 : 0;
      se.a1 = affinity ? per_table : 0;
      se.lane = side ? 1 : 0;
    }
    emit_gemms(gemms);
    if (!lns.empty()) {
      int blocks = 0;
      for (auto &l : lns) {
        l.blk_begin = blocks;
        blocks += (l.rows + ln_rows_per_block() - 1) / ln_rows_per_block();
      }
      bool vec = true;
      int widest = 0;
      for (auto &l : lns) {
        vec = vec && ln_fwd_vec_supported(l);
        widest = std::max(widest, l.d);
      }
      Step &st = add_step(K_LN_FWD, push_table(lns), (int)lns.size(), blocks);
      st.a0 = !vec ? 0 : (widest <= 512 ? 1 : (widest <= 1024 ? 2 : 4));
    }
    if (!attns.empty()) {
      int blocks = 0, ms = 0;
      bool mfma = !(pl.flags & 1);
      for (auto &a : attns) mfma = mfma && attn_mfma_supported(a);
      for (auto &a : attns) {
        a.blk_begin = blocks;
        blocks += mfma ? attn_mfma_blocks(a.batch, a.heads, a.seq) : attn_blocks(a.batch, a.heads, a.seq);
        ms = std::max(ms, a.seq);
      }
      Step &s = add_step(K_ATTN_FWD, push_table(attns), (int)attns.size(), blocks);
      s.a0 = ms;
      s.a1 = mfma ? 1 : 0;
    }
    emit_elt(elts);
    if (!pools.empty()) {
      int blocks = 0;
      for (auto &p : pools) {
        p.blk_begin = blocks;
        blocks += pool_blocks(p);
      }
      add_step(K_POOL, push_table(pools), (int)pools.size(), blocks);
    }
    if (!inters.empty()) {
      int blocks = 0, mf = 0, md = 0;
      for (auto &p : inters) {
        p.blk_begin = blocks;
        blocks += p.batch;
        mf = std::max(mf, p.F);
        md = std::max(md, p.d);
      }
      Step &s = add_step(K_INTERACT_FWD, push_table(inters), (int)inters.size(), blocks);
      s.a0 = mf;
      s.a1 = md;
    }
    if (!heads.empty()) {      // (the stage's only loss)
      Step &sh = add_step(K_HEAD_LOSS, push_table(heads), 1, 1);
      sh.a0 = heads[0].rows;
      sh.a1 = heads[0].K;
      loss_summed = heads[0].partials == nullptr;
    }
    if (!losses.empty()) {
      int blocks = 0;
      int64_t elems = 0;
      for (auto &l : losses) {
        l.blk_begin = blocks;
        blocks += loss_fwd_blocks(l);
        elems += (int64_t)l.rows * l.cols;
      }
      // the one-workgroup kernel: few elements in few rows (rows are padded to 64 elements, so a tall one-column
      // prediction is a cache line per element: 2048 x 1 took 18 us there, 7 + 6 us with the row-parallel kernel
      // and the sum)
      int max_rows = 0;
      for (auto &l : losses) max_rows = std::max(max_rows, l.rows);
      if (losses.size() == pl.loss_ops.size() && elems <= loss_small_limit() && max_rows <= 512) {
        add_step(K_LOSS_FWD_SMALL, push_table(losses), (int)losses.size(), 1);   // value and sum in one launch
        loss_summed = true;
      } else {
        add_step(K_LOSS_FWD, push_table(losses), (int)losses.size(), blocks);   // (writes the gradients its records name, too)
      }
    }
  }

  join();
  // egress: stage outputs to the caller's dense buffers, loss scalars summed
  {
    std::vector<EltProb> recs;
    int base = 0;
    for (size_t k = 0; k < pl.output_ops.size(); ++k) {
      Node &nd = N[pl.output_ops[k]];
      if ((int)k - base == 64) {
        emit_elt(recs, EXT_OUTPUTS, base);
        base = (int)k;
      }
      Buf dst;
      dst.space = SP_ABS;
      dst.ld = nd.feat;
      dst.dtype = nd.d.dtype;
      const Buf &v = nd.fused_add >= 0 ? N[nd.fused_add].val : nd.val;
      EltProb e = elt(v, dst, nd.rows, nd.feat);
      e.ext_dst = (int32_t)(k - base);
      recs.push_back(e);
    }
    emit_elt(recs, EXT_OUTPUTS, base);
    if (!loss_summed) add_step(K_LOSS_SUM, 0, pl.loss_parts, 1);
  }
}

// ---------------------------------------------------------------------------
void Emitter::backward() {
  steps = &pl.bwd;
  steps->clear();
  auto &N = pl.nodes;
  const int n = (int)N.size();
  gstate.assign(n, G_EMPTY);
  gaddend.assign(n, Buf());
  dz_ready.assign(n, 0);
  written_level.assign(n, -1);
  post_copies.clear();
  emb_hoisted.assign(n, 0);
  fork_open = false;

  // ingest the caller's output gradients
  {
    std::vector<EltProb> recs;
    int base = 0;
    for (size_t k = 0; k < pl.output_ops.size(); ++k) {
      Node &nd = N[pl.output_ops[k]];
      if ((int)k - base == 64) {
        emit_elt(recs, EXT_GRAD_OUTPUTS, base);
        base = (int)k;
      }
      if (!nd.wants_grad) continue;
      Buf src;
      src.space = SP_ABS;
      src.ld = nd.feat;
      src.dtype = nd.d.dtype;
      EltProb e = elt(src, nd.gout, nd.rows, nd.feat);
      e.ext_src = (int32_t)(k - base);
      recs.push_back(e);
      gstate[pl.output_ops[k]] = G_WRITTEN;
      written_level[pl.output_ops[k]] = (int)pl.by_level.size();
    }
    emit_elt(recs, EXT_GRAD_OUTPUTS, base);
  }

  auto mask_source = [&](const Node &p) -> Buf { return p.d.act == GPP_ACT_GELU_ERF ? p.aux : p.val; };
  // every member of concat `c` is a ReLU layer stored in place whose only consumer is the concat and
  // whose gradient is a view of the concat's gradient
  auto concat_relu_members = [&](int c) -> bool {
    for (int m : N[c].in) {
      const Node &mm = N[m];
      if (mm.d.kind != GPP_OP_LINEAR || mm.d.act != GPP_ACT_RELU || mm.users.size() != 1 || mm.val_parent != c ||
          mm.gout_parent != c || mm.fused_add >= 0 || dz_ready[m])
        return false;
    }
    return true;
  };
  // a member that shares its consumer's gradient buffer is "written" once the consumer is
  std::function<int(int)> state_of = [&](int i) -> int {
    return N[i].gout_parent >= 0 ? state_of(N[i].gout_parent) : gstate[i];
  };

  for (int L = (int)pl.by_level.size() - 1; L >= 0; --L) {
    cur_level = L;
    // 1. losses seed the gradient of their prediction
    {
      std::vector<LossProb> losses;
      int blocks = 0;
      for (int i : pl.by_level[L]) {
        Node &nd = N[i];
        if (!nd.is_loss) continue;
        Node &y = N[nd.in[0]];
        if (!y.wants_grad) continue;
        const Node &t = N[nd.in[1]];
        const Buf &yv = y.fused_add >= 0 ? N[y.fused_add].val : y.val;
        Target tg = acquire(nd.in[0], false);
        // written by the forward pass already (the prediction's only consumer is this loss, so the
        // gradient buffer itself is the target and nothing is added to it)
        if (loss_fused[i] && !tg.post && !tg.addend.valid() && tg.dst.space == y.gout.space && tg.dst.off == y.gout.off) continue;
        LossProb l;
        memset(&l, 0, sizeof(l));
        l.y = ptr(yv);
        l.ld_y = yv.ld;
        l.y_dtype = yv.dtype;
        l.target = ptr(t.val);
        l.ld_t = t.val.ld;
        l.dy = ptr(tg.dst);
        l.ld_dy = tg.dst.ld;
        l.dy_dtype = tg.dst.dtype;
        l.rows = (int32_t)y.rows;
        l.cols = (int32_t)y.feat;
        l.kind = nd.d.kind;
        l.scale = (float)nd.d.loss_scale;
        blocks += loss_bwd_blocks(l);
        losses.push_back(l);
      }
      if (!losses.empty()) add_step(K_LOSS_BWD, push_table(losses), (int)losses.size(), blocks);
      flush_post();
    }

    // 2. complete the gradients of this level's operators
    std::vector<int> live;
    {
      std::vector<EltProb> copies, masks;
      for (int i : pl.by_level[L]) {
        Node &nd = N[i];
        if (nd.is_loss || !nd.wants_grad) continue;
        if (nd.gout_parent < 0 && gstate[i] == G_ADDEND) {
          copies.push_back(elt(gaddend[i], nd.gout, nd.rows, nd.feat));
          gstate[i] = G_WRITTEN;
        }
        if (state_of(i) != G_WRITTEN) continue;  // no gradient reaches this operator
        live.push_back(i);
        if (nd.d.kind == GPP_OP_LINEAR && nd.d.act != GPP_ACT_NONE && !dz_ready[i]) {
          EltProb e = elt(mask_source(nd), nd.gout, nd.rows, nd.feat);
          e.mode = 1;
          e.act = nd.d.act;
          masks.push_back(e);
        }
      }
      emit_elt(copies);
      emit_elt(masks);
    }

    // 3. per-kind grouped backward launches
    std::vector<ColsumProb> colsums;
    std::vector<GemmProb> gemms;
    std::vector<LnProb> lns;
    std::vector<AttnProb> attns;
    std::vector<PoolProb> pools;
    std::vector<EmbProb> embs;
    std::vector<InteractProb> inters;
    for (int i : live) {
      Node &nd = N[i];
      const gpp_op_desc_t &d = nd.d;
      switch (d.kind) {
        case GPP_OP_LINEAR: {
          const Node &x = N[nd.in[0]];
          GemmProb w;
          memset(&w, 0, sizeof(w));
          w.form = FORM_DW;
          w.A = ptr(nd.gout);
          w.lda = nd.gout.ld;
          w.B = ptr(x.val);
          w.ldb = x.val.ld;
          w.C = d.grad[0];
          w.ldc = ld_of(d.in_features);
          w.c_dtype = DT_F32;
          w.M = (int32_t)nd.feat;           // rows of dW = out_features
          w.N = (int32_t)d.in_features;     // columns of dW
          w.K = (int32_t)nd.rows;           // contraction over the micro-batch rows
          w.in_dtype = d.param_dtype;
          // on the matrix-core path the bias gradient rides along in the backward-weight launch
          bool fuse_db = d.has_bias && !(pl.flags & 1) && w.in_dtype == DT_BF16 && gemm_mfma_supported(w);
          // grouped weight gradients: this record waits for the launch that contracts over every slot of
          // a group of backward passes (both operands sit at the same offsets in every slot)
          const bool grouped = (pl.flags & 4) && !(pl.flags & 1) && w.in_dtype == DT_BF16 && gemm_big_supported(w) &&
                               nd.gout.space == SP_SLOT && x.val.space == SP_SLOT;
          if (grouped) fuse_db = d.has_bias;
          if (fuse_db) w.bias = (const float *)d.grad[1];
          if (grouped) dw_group.push_back(w);
          if (!grouped && d.has_bias && !fuse_db) {
            ColsumProb c;
            memset(&c, 0, sizeof(c));
            c.src = ptr(nd.gout);
            c.ld = nd.gout.ld;
            c.dtype = nd.gout.dtype;
            c.out = (float *)d.grad[1];
            c.rows = (int32_t)nd.rows;
            c.cols = (int32_t)nd.feat;
            colsums.push_back(c);
          }
          if (!grouped) {
            gemms.push_back(w);
            pl.bwd_shared = true;   // accumulates into the parameter's gradient: backward passes stay in order
          }
          if (head_loss[i] >= 0) {
            // the forward pass wrote the input's gradient, activation derivative included (its only consumer
            // is this head, so the gradient buffer itself was the target)
            (void)acquire(nd.in[0], true);
            if (x.d.act != GPP_ACT_NONE) dz_ready[nd.in[0]] = 1;
            break;
          }
          if (x.wants_grad) {
            Target tg = acquire(nd.in[0], true);
            GemmProb g;
            memset(&g, 0, sizeof(g));
            g.form = FORM_DX;
            g.A = ptr(nd.gout);
            g.lda = nd.gout.ld;
            g.B = d.param[0];
            g.ldb = ld_of(d.in_features);
            g.C = ptr(tg.dst);
            g.ldc = tg.dst.ld;
            g.c_dtype = tg.dst.dtype;
            g.M = (int32_t)nd.rows;
            g.N = (int32_t)d.in_features;
            g.K = (int32_t)nd.feat;
            g.in_dtype = d.param_dtype;
            if (tg.addend.valid()) {
              g.res = ptr(tg.addend);
              g.ldres = tg.addend.ld;
              g.res_dtype = tg.addend.dtype;
            }
            // a stage input with this single consumer: the matrix-core kernels store its gradient
            // straight into the caller's dense buffer, no export copy
            if (x.input_index >= 0 && x.input_index < 64 && x.users.size() == 1 && !tg.addend.valid() && !tg.post &&
                !(pl.flags & 1) && g.in_dtype == DT_BF16 && gemm_mfma_supported(g)) {
              g.C = nullptr;
              g.c_ext = x.input_index + 1;
              g.ldc = x.feat;
              g.c_dtype = x.d.dtype;
              N[nd.in[0]].grad_direct = true;
            }
            // a concat of ReLU layers written in place: the members' activation derivative is one mask
            // over the whole merge buffer (the sign of the stored outputs), applied in this epilogue
            if (x.d.kind == GPP_OP_CONCAT && x.users.size() == 1 && concat_relu_members(nd.in[0])) {
              g.act = ACT_RELU;
              g.aux = ptr(x.val);
              g.ldaux = x.val.ld;
              g.aux_dtype = x.val.dtype;
              for (int m : x.in) dz_ready[m] = 1;
            }
            // fold the producer's activation derivative into this epilogue when we are its only consumer
            if (x.d.kind == GPP_OP_LINEAR && x.d.act != GPP_ACT_NONE && x.users.size() == 1 && x.gout_parent < 0) {
              Buf ms = mask_source(x);
              g.act = x.d.act;
              g.aux = ptr(ms);
              g.ldaux = ms.ld;
              g.aux_dtype = ms.dtype;
              dz_ready[nd.in[0]] = 1;
            }
            gemms.push_back(g);
          }
          break;
        }
        case GPP_OP_LAYERNORM: {
          const Node &x = N[nd.in[0]];
          LnProb l;
          memset(&l, 0, sizeof(l));
          l.x = ptr(x.val);
          l.ldx = x.val.ld;
          l.x_dtype = x.val.dtype;
          l.dy = ptr(nd.gout);
          l.lddy = nd.gout.ld;
          l.dy_dtype = nd.gout.dtype;
          l.gamma = (const float *)d.param[0];
          l.mean = (float *)ptr(nd.stat0);
          l.rstd = (float *)ptr(nd.stat1);
          l.dgamma = (float *)d.grad[0];
          l.dbeta = (float *)d.grad[1];
          l.partial = (float *)ptr(nd.extra);
          l.rows = (int32_t)nd.rows;
          l.d = (int32_t)nd.feat;
          l.eps = (float)d.eps;
          if (x.wants_grad) {
            Target tg = acquire(nd.in[0], true);
            l.y = ptr(tg.dst);
            l.ldy = tg.dst.ld;
            l.y_dtype = tg.dst.dtype;
            if (tg.addend.valid()) {
              l.addend = ptr(tg.addend);
              l.ldadd = tg.addend.ld;
              l.add_dtype = tg.addend.dtype;
            }
          }
          lns.push_back(l);
          break;
        }
        case GPP_OP_ATTENTION: {
          const Node &x = N[nd.in[0]];
          if (!x.wants_grad) break;
          Target tg = acquire(nd.in[0], false);
          AttnProb a;
          memset(&a, 0, sizeof(a));
          a.qkv = ptr(x.val);
          a.ld_qkv = x.val.ld;
          a.dtype = x.val.dtype;
          a.out = ptr(tg.dst);
          a.ld_out = tg.dst.ld;
          a.grad_dtype = tg.dst.dtype;
          a.dout = ptr(nd.gout);
          a.ld_dout = nd.gout.ld;
          a.o = ptr(nd.val);
          a.ld_o = nd.val.ld;
          a.out_dtype = nd.val.dtype;
          a.lse = (float *)ptr(nd.stat0);
          a.delta = (float *)ptr(nd.stat1);
          a.batch = (int32_t)pl.micro_batch;
          a.heads = d.heads;
          a.seq = d.seq_len;
          a.dh = (int32_t)(nd.feat / d.heads);
          attns.push_back(a);
          break;
        }
        case GPP_OP_ADD:
          pass_through(nd.in[0], nd.gout);
          pass_through(nd.in[1], nd.gout);
          break;
        case GPP_OP_CONCAT: {
          int64_t col = 0;
          for (int p : nd.in) {
            Buf view = nd.gout;
            view.off += col * esize(view.dtype);
            pass_through(p, view);
            col += N[p].feat;
          }
          break;
        }
        case GPP_OP_MEANPOOL_SEQ: {
          const Node &x = N[nd.in[0]];
          if (!x.wants_grad) break;
          Target tg = acquire(nd.in[0], false);
          PoolProb p;
          memset(&p, 0, sizeof(p));
          p.backward = 1;
          p.src = ptr(nd.gout);
          p.ld_src = nd.gout.ld;
          p.src_dtype = nd.gout.dtype;
          p.dst = ptr(tg.dst);
          p.ld_dst = tg.dst.ld;
          p.dst_dtype = tg.dst.dtype;
          p.batch = (int32_t)pl.micro_batch;
          p.seq = d.seq_len;
          p.d = (int32_t)nd.feat;
          pools.push_back(p);
          break;
        }
        case GPP_OP_EMBEDDING_BAG_SUM:
        case GPP_OP_EMBEDDING_BAG_CONCAT: {
          if (emb_hoisted[i]) break;          // issued early, on the side stream
          embs.push_back(emb_bwd_record(i));
          break;
        }
        case GPP_OP_DOT_INTERACT: {
          const Node &x = N[nd.in[0]];
          if (!x.wants_grad) break;
          Target tg = acquire(nd.in[0], false);
          InteractProb p;
          memset(&p, 0, sizeof(p));
          p.x = ptr(x.val);
          p.ld_x = x.val.ld;
          p.x_dtype = x.val.dtype;
          p.dy = ptr(nd.gout);
          p.ld_dy = nd.gout.ld;
          p.dy_dtype = nd.gout.dtype;
          p.y = ptr(tg.dst);
          p.ld_y = tg.dst.ld;
          p.y_dtype = tg.dst.dtype;
          p.batch = (int32_t)nd.rows;
          p.d = (int32_t)d.in_features;
          p.F = (int32_t)(x.feat / d.in_features);
          inters.push_back(p);
          break;
        }
        default: break;
      }
    }
    if (!colsums.empty()) {
      int blocks = 0;
      for (auto &c : colsums) {
        c.blk_begin = blocks;
        blocks += colsum_blocks(c.cols);
      }
      pl.bwd_shared = true;   // accumulates parameter gradients in the order of the backward passes
      add_step(K_COLSUM, push_table(colsums), (int)colsums.size(), blocks);
    }
    emit_gemms(gemms);
    if (!lns.empty()) {
      // first kernel: dx rows and per-row-block partial parameter sums; operators without partial
      // scratch and without a dx consumer skip it
      std::vector<LnProb> dx;
      int blocks = 0, max_d = 0;
      for (auto &l : lns)
        if (l.y || l.partial) {
          l.row_blocks = (l.rows + ln_bwd_rows_per_block() - 1) / ln_bwd_rows_per_block();
          LnProb c = l;
          c.blk_begin = blocks;
          blocks += l.row_blocks;
          max_d = std::max(max_d, l.partial ? l.d : 0);
          dx.push_back(c);
        }
      if (!dx.empty()) {
        bool vec = true;
        int widest = 0;
        for (auto &l : dx) {
          vec = vec && ln_bwd_vec_supported(l) && l.partial;
          widest = std::max(widest, l.d);
        }
        Step &st = add_step(K_LN_BWD, push_table(dx), (int)dx.size(), blocks);
        st.a0 = max_d;
        st.a1 = !vec ? 0 : (widest <= 512 ? 1 : (widest <= 1024 ? 2 : 4));
      }
      // second kernel: the fold into the parameter gradients.  Operators with partial sums (a buffer of their
      // own in the shared region, read by nothing else) are folded by ONE launch at the end of the backward
      // pass instead of one per level (four launches of 6 us in the two-layer transformer stage); the others read
      // x and dy, which later levels may overwrite, and are folded here.
      std::vector<LnProb> now;
      for (auto &l : lns) (l.partial ? ln_fold_later : now).push_back(l);
      pl.bwd_shared = true;   // accumulates parameter gradients in the order of the backward passes
      if (!now.empty()) {
        blocks = 0;
        for (auto &l : now) {
          l.blk_begin = blocks;
          blocks += ln_param_blocks(l.d);
        }
        add_step(K_LN_BWD_PARAMS, push_table(now), (int)now.size(), blocks);
      }
    }
    if (!attns.empty()) {
      int blocks = 0, ms = 0;
      bool mfma = !(pl.flags & 1);
      for (auto &a : attns) mfma = mfma && attn_mfma_supported(a) && a.grad_dtype == DT_BF16;
      for (auto &a : attns) {
        a.blk_begin = blocks;
        blocks += mfma ? attn_mfma_blocks(a.batch, a.heads, a.seq) : attn_blocks(a.batch, a.heads, a.seq);
        ms = std::max(ms, a.seq);
      }
      int64_t off = push_table(attns);
      Step &s1 = add_step(K_ATTN_DQ, off, (int)attns.size(), blocks);
      s1.a0 = ms;
      s1.a1 = mfma ? 1 : 0;
      Step &s2 = add_step(K_ATTN_DKV, off, (int)attns.size(), blocks);
      s2.a0 = ms;
      s2.a1 = mfma ? 1 : 0;
    }
    if (!pools.empty()) {
      int blocks = 0;
      for (auto &p : pools) {
        p.blk_begin = blocks;
        blocks += pool_blocks(p);
      }
      add_step(K_POOL, push_table(pools), (int)pools.size(), blocks);
    }
    emit_emb_bwd(embs, 0);
    if (!inters.empty()) {
      int blocks = 0, mf = 0, md = 0;
      for (auto &p : inters) {
        p.blk_begin = blocks;
        blocks += p.batch;
        mf = std::max(mf, p.F);
        md = std::max(md, p.d);
      }
      Step &s = add_step(K_INTERACT_BWD, push_table(inters), (int)inters.size(), blocks);
      s.a0 = mf;
      s.a1 = md;
    }
    flush_post();
    // bags whose gradient is complete now (it is a slice of the merge buffer that this level's operators
    // have just written) start their sort and segment sums on the side stream, next to the backward
    // passes of the dense branches
    // (all bags or none: the gradient reset works from ONE table of all embedding records)
    if (L == emb_level && L > 1) {
      std::vector<int> bags, ready;
      for (size_t i = 0; i < N.size(); ++i) {
        const int k = N[i].d.kind;
        if (k != GPP_OP_EMBEDDING_BAG_SUM && k != GPP_OP_EMBEDDING_BAG_CONCAT) continue;
        bags.push_back((int)i);
        if (N[i].gout_parent >= 0 && N[i].level < L && N[i].wants_grad && state_of((int)i) == G_WRITTEN && consumer_level((int)i) == L)
          ready.push_back((int)i);
      }
      if (!ready.empty() && ready.size() == bags.size()) {
        std::vector<EmbProb> early;
        for (int i : ready) {
          early.push_back(emb_bwd_record(i));
          emb_hoisted[i] = 1;
        }
        fork();
        emit_emb_bwd(early, 1);
      }
    }
  }
  join();
  if (!ln_fold_later.empty()) {
    int blocks = 0;
    for (auto &l : ln_fold_later) {
      l.blk_begin = blocks;
      blocks += ln_param_blocks(l.d);
    }
    add_step(K_LN_BWD_PARAMS, push_table(ln_fold_later), (int)ln_fold_later.size(), blocks);
    ln_fold_later.clear();
  }

  // egress: input gradients to the caller's dense buffers
  {
    std::vector<EltProb> recs;
    int base = 0;
    for (size_t k = 0; k < pl.input_ops.size(); ++k) {
      Node &nd = N[pl.input_ops[k]];
      if ((int)k - base == 64) {
        emit_elt(recs, EXT_GRAD_INPUTS, base);
        base = (int)k;
      }
      if (!nd.wants_grad || nd.grad_direct || state_of(pl.input_ops[k]) != G_WRITTEN) continue;
      Buf dst;
      dst.space = SP_ABS;
      dst.ld = nd.feat;
      dst.dtype = nd.d.dtype;
      EltProb e = elt(nd.gout, dst, nd.rows, nd.feat);
      e.ext_dst = (int32_t)(k - base);
      recs.push_back(e);
    }
    emit_elt(recs, EXT_GRAD_INPUTS, base);
  }

  // the weight gradients left to the group launch: every layer of the stage in ONE launch (they depend
  // on nothing but the stashed operands), tiles chosen as for any large-tile launch
  steps = &pl.dwg;
  steps->clear();
  if (!dw_group.empty()) {
    // (a launch of their own for the largest layers with 256 x 256 tiles, which win on those shapes alone --
    // 98 against 112 us on 4 x [4096 x 1024] over 2048 rows -- measured no faster for the step: 515 against
    // 502 us for the transformer stage; one launch lets the co-resident tiles of all layers fill each other's tails)
    int64_t elems = 0;
    int tiles256 = 0, tiles128 = 0, max_m = 0, max_n = 0;
    for (auto &r : dw_group) {
      elems += (int64_t)r.M * r.N;
      tiles256 += ((r.M + 255) / 256) * ((r.N + 255) / 256);
      tiles128 += ((r.M + 127) / 128) * ((r.N + 255) / 256);
      max_m = std::max(max_m, r.M);
      max_n = std::max(max_n, r.N);
    }
    int tile_rows = gemm_big_tile_rows(FORM_DW, max_m, max_n, elems, tiles256, tiles128);
    if (tile_rows == 0) tile_rows = 64;
    int blocks = 0;
    for (auto &r : dw_group) {
      r.blk_begin = blocks;
      r.split_k = 1;
      blocks += gemm_big_tiles_for(tile_rows, r.M, r.N, &r.tiles_n);
    }
    // (contraction-major operands: staged through registers, see emit_gemms)
    Step &sg = add_step(K_GEMM_DW_GROUP, push_table(dw_group), (int)dw_group.size(), blocks);
    sg.a2 = tile_rows;
  }
  steps = &pl.bwd;
}

}  // namespace

gpp_status_t Plan::emit(int slot, char *ws) {
  blob.clear();
  Emitter em(*this, slot, ws);
  em.forward();
  em.backward();
  table_bytes = std::max<int64_t>(table_bytes, align_up((int64_t)blob.size(), 256));
  // temporaries requested during emission extend the shared region (same for every slot)
  tmp_bytes = std::max<int64_t>(tmp_bytes, em.shared_tmp_top);
  gemm_partial_bytes = std::max<int64_t>(gemm_partial_bytes, em.part_need);
  gemm_counter_bytes = std::max<int64_t>(gemm_counter_bytes, em.cnt_need);
  return GPP_OK;
}

}  // namespace gpp
