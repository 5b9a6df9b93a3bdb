// C ABI of the GPP stage library: descriptor validation, planning, the
// micro-batch state machine (ordering condition C4 of the paper's problem
// formulation) and the launch loop.  Everything numeric runs in the HIP kernels.
#include <hip/hip_runtime.h>

#include <cstdio>
#include <cstring>
#include <deque>
#include <mutex>
#include <new>
#include <string>

#include "plan.h"

using namespace gpp;

namespace gpp {
void launch_gemm_generic(const GemmProb *probs, int n, int total_blocks, int accumulate_dw, int in_dtype, hipStream_t s);
void launch_attn_fwd(const AttnProb *probs, int n, int total_blocks, int max_seq, hipStream_t s);
void launch_attn_bwd_dq(const AttnProb *probs, int n, int total_blocks, int max_seq, hipStream_t s);
void launch_attn_bwd_dkv(const AttnProb *probs, int n, int total_blocks, int max_seq, hipStream_t s);
void launch_attn_fwd_mfma(const AttnProb *probs, int n, int total_blocks, hipStream_t s);
void launch_attn_bwd_dq_mfma(const AttnProb *probs, int n, int total_blocks, hipStream_t s);
void launch_attn_bwd_dkv_mfma(const AttnProb *probs, int n, int total_blocks, hipStream_t s);
void launch_interact_fwd(const InteractProb *probs, int n, int total_blocks, int maxF, int maxd, hipStream_t s);
void launch_interact_bwd(const InteractProb *probs, int n, int total_blocks, int maxF, int maxd, hipStream_t s);
void launch_loss_sum(const float *losses, int n, float *out, hipStream_t s);
}  // namespace gpp

static thread_local std::string g_last_error;
static gpp_status_t fail(gpp_status_t st, const std::string &msg) {
  g_last_error = msg;
  return st;
}
namespace gpp {
gpp_status_t report_error(gpp_status_t st, const std::string &msg) { return fail(st, msg); }
}

struct gpp_stage {
  Plan plan;
  char *ws = nullptr;
  std::vector<char> slot_busy;
  std::deque<int> fifo;          // slots in the order their forwards were issued
  std::deque<int> pending;       // grouped weight gradients: backpropagated slots whose operands are still needed
  bool fresh = true;             // no backward since the last grad_reset: next one overwrites dense accumulators
  bool fresh_w = true;           // no grouped weight-gradient launch since the last grad_reset
  bool emb_clear_pending = true; // table accumulators not yet cleared since create
  int64_t emb_table_off = -1;    // table of all embedding records (slot 0) for the clear kernel
  int emb_count = 0;
  int emb_capacity = 0;          // largest index capacity among the tables
  int emb_logged = 0;            // backward passes since the last reset whose touched rows are logged
  bool emb_log_overflow = false; // more passes than log slots: the next reset clears whole tables
  int emb_last_slot = 0;
  const void *emb_last_table = nullptr;  // device records of the last embedding backward (its stash slot's copy)
  int emb_sort_blocks = 0;
  // optional per-step timing (HIP events on the caller's stream)
  bool prof_on = false;
  int prof_repeat = 1;               // timing mode: GEMM steps are launched this many times inside their bracket
  std::vector<hipEvent_t> prof_ev;   // pairs (begin, end)
  std::vector<int> prof_tag;         // tag of each recorded pair
  size_t prof_used = 0;
  double prof_ms[GPP_PROFILE_TAGS] = {0};
  int64_t prof_launches[GPP_PROFILE_TAGS] = {0};
  // events of the schedule executor (created on first use, two per micro-batch, no timing)
  std::vector<hipEvent_t> sched_ev;
  bool group_ok = false;     // group tables are in place (see Plan::group_lanes)
  // side streams (one for forward calls, one for backward calls) and their fork / join events, created with the
  // stage when its plan runs embedding bags next to dense branches
  hipStream_t lane_stream[2] = {nullptr, nullptr};
  hipEvent_t lane_fork[2] = {nullptr, nullptr}, lane_join[2] = {nullptr, nullptr};
  int static_device = -1;    // >= 0: the workspace is the library's static device array of that GPU (gpp_stage_create_static)
};

// ---- the static workspace of gpp_stage_create_static: device memory that exists as soon as the library is
// loaded on a GPU, so that a stage can be created without any allocation.  In host code the array's name is a
// stand-in, not a device address: the address of THIS GPU's copy is asked for once per device and kept.
static __device__ __align__(256) unsigned char scratch[GPP_STATIC_WORKSPACE_BYTES];
constexpr int STATIC_MAX_DEVICES = 64;
static std::mutex g_static_mutex;
static void *g_static_ptr[STATIC_MAX_DEVICES] = {nullptr};          // per device: address of its copy of `scratch`
static const gpp_stage *g_static_owner[STATIC_MAX_DEVICES] = {nullptr};   // per device: the stage that holds it

static bool gemm_step(const Step &sp) {
  return sp.kern == K_GEMM_MFMA || sp.kern == K_GEMM_BIG || sp.kern == K_GEMM_SKINNY || sp.kern == K_GEMM_BWD_MERGED ||
         sp.kern == K_GEMM_DW_KSPLIT || sp.kern == K_GEMM_DW_GROUP;
}

// profile tag of a step: grouped-GEMM steps are split by form, element-wise steps by direction
static int step_tag(const Step &sp, bool backward) {
  switch (sp.kern) {
    case K_GEMM_MFMA: return 1 + sp.a1;                    // 1 fwd, 2 dx, 3 dw
    case K_GEMM_BIG: return 28 + sp.a1;                    // 28 fwd, 29 dx, 30 dw
    case K_GEMM_SKINNY: return 25 + sp.a1;                 // 25 fwd, 26 dx
    case K_GEMM_BWD_MERGED: return 27;
    case K_GEMM_DW_KSPLIT: return 31;
    case K_GEMM_DW_GROUP: return 30;
    case K_LOSS_FWD_SMALL: return 21;
    case K_HEAD_LOSS: return 21;
    case K_GEMM_GENERIC: return backward ? 5 : 4;
    case K_ELT: return backward ? 7 : 6;
    case K_COLSUM: return 8;
    case K_LN_FWD: return 9;
    case K_LN_BWD: return 10;
    case K_LN_BWD_PARAMS: return 11;
    case K_ATTN_FWD: return 12;
    case K_ATTN_DQ: return 13;
    case K_ATTN_DKV: return 14;
    case K_POOL: return backward ? 16 : 15;
    case K_EMB_FWD: return 17;
    case K_EMB_BWD: return 18;
    case K_INTERACT_FWD: return 19;
    case K_INTERACT_BWD: return 20;
    case K_LOSS_FWD: return 21;
    case K_LOSS_BWD: return 22;
    case K_LOSS_SUM: return 23;
    default: return 0;
  }
}
static const char *const kTagNames[GPP_PROFILE_TAGS] = {
    "other", "gemm_mfma_fwd", "gemm_mfma_dx", "gemm_mfma_dw", "gemm_generic_fwd", "gemm_generic_bwd", "elt_fwd", "elt_bwd",
    "colsum_bias_grad", "layernorm_fwd", "layernorm_bwd_dx", "layernorm_bwd_params", "attention_fwd", "attention_bwd_dq",
    "attention_bwd_dkv", "meanpool_fwd", "meanpool_bwd", "embedding_fwd", "embedding_bwd_sort_segsum", "interact_fwd",
    "interact_bwd", "loss_fwd", "loss_bwd", "loss_sum", "embedding_grad_clear", "gemm_skinny_fwd", "gemm_skinny_dx", "gemm_bwd_merged_dx_dw", "gemm_big_fwd", "gemm_big_dx", "gemm_big_dw",
    "gemm_dw_ksplit"};

// Group launches: one launch for a step of several micro-batches (the records of their slots one after the
// other).  Possible where every step is one of the kinds below, runs on the caller's stream, touches slot
// memory only, and the per-call pointers of all members fit one pointer block.
static size_t group_record_bytes(int kern) {
  return kern == K_ELT ? sizeof(EltProb) : kern == K_GEMM_SKINNY ? sizeof(GemmProb) : kern == K_HEAD_LOSS ? sizeof(HeadProb) : 0;
}
// (the loss sum has no records: one small launch per member adds that member's partial losses)
static bool group_form(const Step &sp) { return group_record_bytes(sp.kern) != 0 || sp.kern == K_LOSS_SUM; }
static bool group_supported(const Plan &pl) {
  if (pl.group_lanes <= 0 || pl.fwd_shared || pl.bwd_shared || pl.lanes) return false;
  const int G = pl.slots / pl.group_lanes;
  if (G > HEAD_GROUP_MAX) return false;
  for (const std::vector<Step> *list : {&pl.fwd, &pl.bwd})
    for (const Step &sp : *list) {
      if (!group_form(sp) || sp.lane != 0 || sp.launches != 1) return false;
      if (sp.ext_kind != EXT_NONE) {
        const int total = (sp.ext_kind == EXT_INPUTS || sp.ext_kind == EXT_GRAD_INPUTS) ? (int)pl.input_ops.size() : (int)pl.output_ops.size();
        if (sp.ext_base != 0 || G * total > 64) return false;
      }
    }
  return true;
}

extern "C" {

int64_t gpp_ld(int64_t features) { return (features + 63) / 64 * 64; }

const char *gpp_last_error(void) { return g_last_error.c_str(); }

static gpp_status_t build_plan(const gpp_stage_desc_t *desc, Plan &pl) {
  gpp_status_t st = pl.analyse(desc);
  if (st != GPP_OK) return st;
  pl.layout();
  st = pl.emit(0, nullptr);  // sizing pass: table and temporary sizes
  if (st != GPP_OK) return st;
  pl.layout();
  return GPP_OK;
}

gpp_status_t gpp_stage_workspace_bytes(const gpp_stage_desc_t *desc, size_t *bytes) {
  if (!bytes) return fail(GPP_ERR_INVALID_ARG, "bytes is null");
  Plan pl;
  gpp_status_t st = build_plan(desc, pl);
  if (st != GPP_OK) return fail(st, pl.error);
  *bytes = (size_t)pl.total_bytes;
  return GPP_OK;
}

// workspace == nullptr: take the static workspace of the current device (gpp_stage_create_static)
static gpp_status_t stage_create(const gpp_stage_desc_t *desc, void *workspace, size_t workspace_bytes, gpp_stage_t **out) {
  if (!out) return fail(GPP_ERR_INVALID_ARG, "out is null");
  const bool use_static = workspace == nullptr;
  int dev = -1;
  if (use_static) {
    hipError_t he = hipGetDevice(&dev);
    if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP: ") + hipGetErrorString(he));
    if (dev < 0 || dev >= STATIC_MAX_DEVICES) return fail(GPP_ERR_UNSUPPORTED, "device ordinal beyond the static workspace table");
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (!g_static_ptr[dev]) {     // once per device, with that device current
      void *ptr = nullptr;
      he = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
      if (he != hipSuccess || !ptr) return fail(GPP_ERR_DEVICE, std::string("HIP: static workspace: ") + hipGetErrorString(he));
      g_static_ptr[dev] = ptr;
    }
    if (g_static_owner[dev]) return fail(GPP_ERR_ORDER, "the static workspace of this GPU is held by another stage (destroy it first)");
    workspace = g_static_ptr[dev];
    workspace_bytes = GPP_STATIC_WORKSPACE_BYTES;
  }
  gpp_stage *st = new (std::nothrow) gpp_stage();
  if (!st) return fail(GPP_ERR_INVALID_ARG, "out of host memory");
  gpp_status_t rc = build_plan(desc, st->plan);
  if (rc != GPP_OK) {
    std::string e = st->plan.error;
    delete st;
    return fail(rc, e);
  }
  Plan &pl = st->plan;
  // parameters must be present
  for (size_t i = 0; i < pl.nodes.size(); ++i) {
    const gpp_op_desc_t &d = pl.nodes[i].d;
    bool need2 = (d.kind == GPP_OP_LINEAR && d.has_bias) || d.kind == GPP_OP_LAYERNORM;
    bool need1 = d.kind == GPP_OP_LINEAR || d.kind == GPP_OP_LAYERNORM || d.kind == GPP_OP_EMBEDDING_BAG_SUM || d.kind == GPP_OP_EMBEDDING_BAG_CONCAT;
    if ((need1 && (!d.param[0] || !d.grad[0])) || (need2 && (!d.param[1] || !d.grad[1]))) {
      delete st;
      return fail(GPP_ERR_INVALID_ARG, "operator " + std::to_string(i) + ": parameter or gradient pointer is null");
    }
    for (int k = 0; k < 2; ++k)
      if (((uintptr_t)d.param[k] | (uintptr_t)d.grad[k]) & 15) {
        delete st;
        return fail(GPP_ERR_INVALID_ARG, "operator " + std::to_string(i) + ": parameter pointers must be 16-byte aligned");
      }
  }
  if (!workspace || ((uintptr_t)workspace & 255)) {
    delete st;
    return fail(GPP_ERR_WORKSPACE, "workspace is null or not 256-byte aligned");
  }
  if (workspace_bytes < (size_t)pl.total_bytes) {
    const int64_t need = pl.total_bytes;
    delete st;
    return fail(GPP_ERR_WORKSPACE, (use_static ? "the stage needs more than the static workspace holds: need " : "workspace too small: need ") +
                                       std::to_string(need) + " bytes, have " + std::to_string(workspace_bytes));
  }
  if (use_static && pl.lanes) {      // the side stream and its events would have to be created here
    delete st;
    return fail(GPP_ERR_UNSUPPORTED, "stage flag bit 3 (side stream) is not available with the static workspace");
  }
  st->ws = (char *)workspace;
  hipError_t he = hipMemset(workspace, 0, (size_t)pl.total_bytes);
  std::vector<std::vector<uint8_t>> blobs;
  for (int s = 0; he == hipSuccess && s < pl.slots; ++s) {
    rc = pl.emit(s, st->ws);
    if (rc != GPP_OK) break;
    if (!pl.blob.empty())
      he = hipMemcpy(st->ws + pl.off_tables + (int64_t)s * pl.table_bytes, pl.blob.data(), pl.blob.size(), hipMemcpyHostToDevice);
    if (pl.group_lanes > 0) blobs.push_back(pl.blob);
  }
  if (he == hipSuccess && rc == GPP_OK && pl.group_lanes > 0 && group_supported(pl)) {
    const int L = pl.group_lanes, G = pl.slots / L;
    for (int l = 0; l < L && he == hipSuccess; ++l) {
      std::vector<uint8_t> gb((size_t)G * pl.table_bytes, 0);
      for (int i = 0; i < G; ++i) {
        const std::vector<uint8_t> &src = blobs[l + L * i];
        for (const std::vector<Step> *list : {&pl.fwd, &pl.bwd})
          for (const Step &sp : *list) {
            const size_t rec = group_record_bytes(sp.kern);
            uint8_t *dst = gb.data() + (size_t)G * sp.table_off + (size_t)i * sp.n * rec;
            // (few-row GEMM steps need no copy: their group launch reads the first slot's records and reaches the
            // other members by the slot stride, see run_steps_group)
            if (sp.n <= 0 || rec == 0 || sp.kern == K_GEMM_SKINNY) continue;
            memcpy(dst, src.data() + sp.table_off, (size_t)sp.n * rec);
            const int ext_total = sp.ext_kind == EXT_NONE ? 0
                                  : ((sp.ext_kind == EXT_INPUTS || sp.ext_kind == EXT_GRAD_INPUTS) ? (int)pl.input_ops.size()
                                                                                                   : (int)pl.output_ops.size());
            for (int r = 0; r < sp.n; ++r) {     // member i's workgroups and per-call pointers follow those of members 0 .. i-1
              if (sp.kern == K_ELT) {
                EltProb *e = (EltProb *)dst + r;
                e->blk_begin += i * sp.blocks;
                if (e->ext_src >= 0) e->ext_src += i * ext_total;
                if (e->ext_dst >= 0) e->ext_dst += i * ext_total;
              }
            }
          }
      }
      he = hipMemcpy(st->ws + pl.off_group_tables + (int64_t)l * G * pl.table_bytes, gb.data(), gb.size(), hipMemcpyHostToDevice);
    }
    st->group_ok = he == hipSuccess;
  }
  if (he == hipSuccess) he = hipDeviceSynchronize();
  if (he != hipSuccess || rc != GPP_OK) {
    std::string e = he != hipSuccess ? std::string("HIP: ") + hipGetErrorString(he) : pl.error;
    delete st;
    return fail(he != hipSuccess ? GPP_ERR_DEVICE : rc, e);
  }
  st->slot_busy.assign(pl.slots, 0);
  if (pl.lanes) {
    for (int k = 0; k < 2 && he == hipSuccess; ++k) {
      he = hipStreamCreateWithFlags(&st->lane_stream[k], hipStreamNonBlocking);      // default priority
      if (he == hipSuccess) he = hipEventCreateWithFlags(&st->lane_fork[k], hipEventDisableTiming);
      if (he == hipSuccess) he = hipEventCreateWithFlags(&st->lane_join[k], hipEventDisableTiming);
    }
    if (he != hipSuccess) {
      const std::string e = std::string("HIP: ") + hipGetErrorString(he);
      gpp_stage_destroy(st);
      return fail(GPP_ERR_DEVICE, e);
    }
  }
  for (const Step &s : pl.bwd)
    if (s.kern == K_EMB_BWD) {
      st->emb_table_off = s.table_off;
      st->emb_count = s.n;
      st->emb_capacity = s.a0;
    }
  if (use_static) {
    std::lock_guard<std::mutex> lock(g_static_mutex);
    if (g_static_owner[dev]) {     // another thread took it meanwhile
      delete st;
      return fail(GPP_ERR_ORDER, "the static workspace of this GPU is held by another stage (destroy it first)");
    }
    g_static_owner[dev] = st;
    st->static_device = dev;
  }
  *out = st;
  return GPP_OK;
}

gpp_status_t gpp_stage_create(const gpp_stage_desc_t *desc, void *workspace, size_t workspace_bytes, gpp_stage_t **out) {
  if (!workspace) return fail(GPP_ERR_WORKSPACE, "workspace is null or not 256-byte aligned");
  return stage_create(desc, workspace, workspace_bytes, out);
}

gpp_status_t gpp_stage_create_static(const gpp_stage_desc_t *desc, gpp_stage_t **out) { return stage_create(desc, nullptr, 0, out); }

gpp_status_t gpp_stage_destroy(gpp_stage_t *stage) {
  if (stage) {
    for (hipEvent_t e : stage->prof_ev) (void)hipEventDestroy(e);
    for (hipEvent_t e : stage->sched_ev) (void)hipEventDestroy(e);
    for (int k = 0; k < 2; ++k) {
      if (stage->lane_fork[k]) (void)hipEventDestroy(stage->lane_fork[k]);
      if (stage->lane_join[k]) (void)hipEventDestroy(stage->lane_join[k]);
      if (stage->lane_stream[k]) (void)hipStreamDestroy(stage->lane_stream[k]);
    }
    if (stage->static_device >= 0) {
      std::lock_guard<std::mutex> lock(g_static_mutex);
      if (g_static_owner[stage->static_device] == stage) g_static_owner[stage->static_device] = nullptr;
    }
  }
  delete stage;
  return GPP_OK;
}

int32_t gpp_stage_num_inputs(const gpp_stage_t *s) { return s ? (int32_t)s->plan.input_ops.size() : -1; }
int32_t gpp_stage_num_outputs(const gpp_stage_t *s) { return s ? (int32_t)s->plan.output_ops.size() : -1; }
int32_t gpp_stage_input_op(const gpp_stage_t *s, int32_t i) {
  return (s && i >= 0 && i < (int32_t)s->plan.input_ops.size()) ? s->plan.input_ops[i] : -1;
}
int32_t gpp_stage_output_op(const gpp_stage_t *s, int32_t i) {
  return (s && i >= 0 && i < (int32_t)s->plan.output_ops.size()) ? s->plan.output_ops[i] : -1;
}
gpp_status_t gpp_stage_info(const gpp_stage_t *s, int64_t *micro_batch, int32_t *in_flight_slots, int32_t *flags) {
  if (!s) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  if (micro_batch) *micro_batch = s->plan.micro_batch;
  if (in_flight_slots) *in_flight_slots = s->plan.slots;
  if (flags) *flags = s->plan.flags;
  return GPP_OK;
}
gpp_status_t gpp_stage_lanes(const gpp_stage_t *s, int32_t *forward_ok, int32_t *backward_ok) {
  if (!s) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  if (forward_ok) *forward_ok = !(s->plan.fwd_shared || s->plan.lanes);
  if (backward_ok) *backward_ok = !(s->plan.bwd_shared || s->plan.lanes);
  return GPP_OK;
}
gpp_status_t gpp_stage_group_launches(const gpp_stage_t *s, int32_t *lanes, int32_t *members) {
  if (!s) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  if (lanes) *lanes = s->group_ok ? s->plan.group_lanes : 0;
  if (members) *members = s->group_ok ? s->plan.slots / s->plan.group_lanes : 0;
  return GPP_OK;
}
gpp_status_t gpp_stage_io_info(const gpp_stage_t *s, int32_t is_output, int32_t index, int64_t *rows, int64_t *features,
                               int32_t *dtype, int32_t *has_grad) {
  if (!s) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  const std::vector<int> &ids = is_output ? s->plan.output_ops : s->plan.input_ops;
  if (index < 0 || index >= (int32_t)ids.size()) return fail(GPP_ERR_INVALID_ARG, "input / output index out of range");
  const Node &nd = s->plan.nodes[ids[index]];
  if (rows) *rows = nd.rows;
  if (features) *features = nd.feat;
  if (dtype) *dtype = nd.d.dtype;
  if (has_grad) *has_grad = nd.wants_grad ? 1 : 0;
  return GPP_OK;
}
int32_t gpp_stage_num_launches(const gpp_stage_t *s, int32_t backward) {
  if (!s) return -1;
  int32_t n = 0;
  for (const Step &st : backward == 2 ? s->plan.dwg : (backward ? s->plan.bwd : s->plan.fwd)) n += st.launches;
  return n;
}

}  // extern "C"

// ---------------------------------------------------------------------------
static gpp_status_t run_steps(gpp_stage *st, const std::vector<Step> &steps, int slot, const void *const *ext_in,
                              void *const *ext_out, float *loss_out, int accumulate, hipStream_t s,
                              const SlotGroup *grp = nullptr) {
  Plan &pl = st->plan;
  const char *tables = st->ws + pl.off_tables + (int64_t)slot * pl.table_bytes;
  StageFlags *flags = (StageFlags *)(st->ws + pl.off_flags);
  const bool is_bwd = &steps == &pl.bwd;
  const int side = is_bwd ? 1 : 0;
  hipStream_t caller = s;
  for (const Step &sp : steps) {
    // side-stream steps: the fork makes the side stream wait for everything issued so far on the caller's
    // stream, the join makes the caller's stream wait for the side stream (default priorities; under graph
    // capture the two waits pull the side stream into the capture and back out)
    if (sp.kern == K_FORK || sp.kern == K_JOIN) {
      if (!st->lane_stream[side]) return fail(GPP_ERR_UNSUPPORTED, "internal: side stream missing");
      hipError_t he;
      if (sp.kern == K_FORK) {
        he = hipEventRecord(st->lane_fork[side], caller);
        if (he == hipSuccess) he = hipStreamWaitEvent(st->lane_stream[side], st->lane_fork[side], 0);
      } else {
        he = hipEventRecord(st->lane_join[side], st->lane_stream[side]);
        if (he == hipSuccess) he = hipStreamWaitEvent(caller, st->lane_join[side], 0);
      }
      if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP event: ") + hipGetErrorString(he));
      continue;
    }
    s = sp.lane ? st->lane_stream[side] : caller;
    const void *tab = tables + sp.table_off;
    hipEvent_t ev_end = nullptr;
    if (st->prof_on) {
      if (st->prof_used + 2 > st->prof_ev.size()) {
        for (int k = 0; k < 2; ++k) {
          hipEvent_t e;
          if (hipEventCreate(&e) != hipSuccess) return fail(GPP_ERR_DEVICE, "hipEventCreate failed");
          st->prof_ev.push_back(e);
        }
      }
      (void)hipEventRecord(st->prof_ev[st->prof_used], s);
      ev_end = st->prof_ev[st->prof_used + 1];
      st->prof_tag.resize(st->prof_used / 2 + 1);
      st->prof_tag[st->prof_used / 2] = step_tag(sp, is_bwd) | ((sp.launches * (gemm_step(sp) ? st->prof_repeat : 1)) << 8);
      st->prof_used += 2;
    }
    // per-call pointers the step's records refer to by index
    ExtPtrs ext;
    memset(&ext, 0, sizeof(ext));
    if (sp.ext_kind != EXT_NONE) {
      const bool in_side = sp.ext_kind == EXT_INPUTS || sp.ext_kind == EXT_GRAD_OUTPUTS;
      const int total = (sp.ext_kind == EXT_INPUTS || sp.ext_kind == EXT_GRAD_INPUTS) ? (int)pl.input_ops.size()
                                                                                     : (int)pl.output_ops.size();
      for (int k = 0; k < 64 && sp.ext_base + k < total; ++k) {
        if (in_side)
          ext.p[k] = ext_in ? (void *)ext_in[sp.ext_base + k] : nullptr;
        else
          ext.p[k] = ext_out ? ext_out[sp.ext_base + k] : nullptr;
      }
    }
    // timing mode: a bracket of two events costs about two microseconds of dispatch latency, a quarter of a
    // few-row GEMM launch; such steps are launched several times back to back inside one bracket (they
    // only read their operands and tables; accumulating ones add again, which the timing pass ignores)
    const int reps = (st->prof_on && gemm_step(sp)) ? st->prof_repeat : 1;
    for (int rep = 0; rep < reps; ++rep)
    switch (sp.kern) {
      case K_ELT: launch_elt((const EltProb *)tab, sp.n, sp.blocks, ext, s); break;
      case K_GEMM_GENERIC: launch_gemm_generic((const GemmProb *)tab, sp.n, sp.blocks, accumulate, sp.a0, s); break;
      case K_GEMM_MFMA: launch_gemm_mfma((const GemmProb *)tab, sp.n, sp.blocks, accumulate, sp.a1, sp.a2, ext, s); break;
      case K_GEMM_BIG: launch_gemm_big((const GemmProb *)tab, sp.n, sp.blocks, accumulate, sp.a1, sp.a2, sp.a0, ext, s); break;
      case K_GEMM_DW_KSPLIT: launch_gemm_dw_ksplit((const GemmProb *)tab, sp.n, sp.blocks, accumulate, s); break;
      case K_GEMM_DW_GROUP:
        if (!grp) return fail(GPP_ERR_UNSUPPORTED, "internal: group launch without a group");
        launch_gemm_dw_group((const GemmProb *)tab, sp.n, sp.blocks, accumulate, sp.a2, *grp, s);
        break;
      case K_GEMM_SKINNY: launch_gemm_skinny((const GemmProb *)tab, sp.n, sp.blocks, sp.a1, sp.a2, sp.a0, sp.a3, ext, s); break;
      case K_GEMM_BWD_MERGED: launch_gemm_bwd_merged((const GemmProb *)tab, sp.n, sp.blocks, sp.a2, sp.a1, accumulate, ext, s); break;
      case K_HEAD_LOSS: {   // always runs: it also writes the prediction and two gradients
        float *sink = loss_out ? loss_out : (float *)(st->ws + pl.off_slots + (int64_t)slot * pl.slot_bytes + pl.loss_scalars.off);
        HeadOuts ho;
        memset(&ho, 0, sizeof(ho));
        ho.p[0] = sink;
        launch_head_loss((const HeadProb *)tab, 1, sp.a0, sp.a1, ho, s);
        break;
      }
      case K_LOSS_FWD_SMALL: {
        // the launch may also write the loss gradient (per-slot gradient buffers), so it runs without a
        // loss_out too: the sum then goes to the slot's own loss scalars
        float *sink = loss_out ? loss_out : (float *)(st->ws + pl.off_slots + (int64_t)slot * pl.slot_bytes + pl.loss_scalars.off);
        launch_loss_fwd_small((const LossProb *)tab, sp.n, sink, flags, s);
        break;
      }
      case K_COLSUM: launch_colsum((const ColsumProb *)tab, sp.n, sp.blocks, accumulate, s); break;
      case K_LN_FWD: launch_ln_fwd((const LnProb *)tab, sp.n, sp.blocks, sp.a0, s); break;
      case K_LN_BWD: launch_ln_bwd((const LnProb *)tab, sp.n, sp.blocks, sp.a0, sp.a1, s); break;
      case K_LN_BWD_PARAMS: launch_ln_bwd_params((const LnProb *)tab, sp.n, sp.blocks, accumulate, s); break;
      case K_ATTN_FWD:
        if (sp.a1) launch_attn_fwd_mfma((const AttnProb *)tab, sp.n, sp.blocks, s);
        else launch_attn_fwd((const AttnProb *)tab, sp.n, sp.blocks, sp.a0, s);
        break;
      case K_ATTN_DQ:
        if (sp.a1) launch_attn_bwd_dq_mfma((const AttnProb *)tab, sp.n, sp.blocks, s);
        else launch_attn_bwd_dq((const AttnProb *)tab, sp.n, sp.blocks, sp.a0, s);
        break;
      case K_ATTN_DKV:
        if (sp.a1) launch_attn_bwd_dkv_mfma((const AttnProb *)tab, sp.n, sp.blocks, s);
        else launch_attn_bwd_dkv((const AttnProb *)tab, sp.n, sp.blocks, sp.a0, s);
        break;
      case K_POOL: launch_pool((const PoolProb *)tab, sp.n, sp.blocks, s); break;
      case K_EMB_FWD: launch_emb_fwd((const EmbProb *)tab, sp.n, sp.blocks, sp.a0, sp.a1, flags, s); break;
      case K_EMB_BWD: {
        if (st->emb_clear_pending) {
          launch_emb_reset((const EmbProb *)tab, sp.n, sp.a0, 0, s);
          st->emb_clear_pending = false;
        }
        // the rows this pass touches are logged so that the next reset clears only those
        if (st->emb_logged >= emb_log_slots()) st->emb_log_overflow = true;
        const int slot = st->emb_logged < emb_log_slots() ? st->emb_logged : emb_log_slots() - 1;
        launch_emb_bwd((const EmbProb *)tab, sp.n, sp.a0, sp.a1, sp.a2 & 255, (sp.a2 >> 8) & 1, sp.a2 >> 11,
                       ((sp.a2 >> 9) & 3) == 3 ? -1 : ((sp.a2 >> 9) & 3), slot, st->emb_logged == 0 ? 1 : 0, s);
        st->emb_last_slot = slot;
        st->emb_last_table = tab;
        st->emb_sort_blocks = sp.a1;
        st->emb_logged++;
        break;
      }
      case K_INTERACT_FWD: launch_interact_fwd((const InteractProb *)tab, sp.n, sp.blocks, sp.a0, sp.a1, s); break;
      case K_INTERACT_BWD: launch_interact_bwd((const InteractProb *)tab, sp.n, sp.blocks, sp.a0, sp.a1, s); break;
      case K_LOSS_FWD: launch_loss_fwd((const LossProb *)tab, sp.n, sp.blocks, flags, s); break;
      case K_LOSS_BWD: launch_loss_bwd((const LossProb *)tab, sp.n, sp.blocks, s); break;
      case K_LOSS_SUM:
        if (loss_out) {
          Buf b = pl.loss_scalars;
          const float *ls = (const float *)(st->ws + pl.off_slots + (int64_t)slot * pl.slot_bytes + b.off);
          launch_loss_sum(ls, sp.n, loss_out, s);
        }
        break;
      default: return fail(GPP_ERR_UNSUPPORTED, "internal: unknown step");
    }
    if (ev_end) (void)hipEventRecord(ev_end, s);
  }
  hipError_t he = hipGetLastError();
  if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP launch: ") + hipGetErrorString(he));
  return GPP_OK;
}

// One launch per step for the micro-batches `members` (ids into io) of lane `lane`: their slots are
// lane, lane + L, lane + 2 L, ... in this order (the caller has checked it).
static gpp_status_t run_steps_group(gpp_stage *st, const std::vector<Step> &steps, int lane, const std::vector<int64_t> &members,
                                    const gpp_microbatch_io_t *io, hipStream_t s) {
  Plan &pl = st->plan;
  const int G = pl.slots / pl.group_lanes, m = (int)members.size();
  const char *tables = st->ws + pl.off_group_tables + (int64_t)lane * G * pl.table_bytes;
  const bool is_bwd = &steps == &pl.bwd;
  for (const Step &sp : steps) {
    const void *tab = tables + (int64_t)G * sp.table_off;
    ExtPtrs ext;
    memset(&ext, 0, sizeof(ext));
    if (sp.ext_kind != EXT_NONE) {
      const int total = (sp.ext_kind == EXT_INPUTS || sp.ext_kind == EXT_GRAD_INPUTS) ? (int)pl.input_ops.size()
                                                                                     : (int)pl.output_ops.size();
      for (int i = 0; i < m; ++i) {
        const gpp_microbatch_io_t &mb = io[members[i]];
        for (int k = 0; k < total; ++k) {
          const void *ptr = nullptr;
          switch (sp.ext_kind) {
            case EXT_INPUTS: ptr = mb.inputs ? mb.inputs[k] : nullptr; break;
            case EXT_OUTPUTS: ptr = mb.outputs ? mb.outputs[k] : nullptr; break;
            case EXT_GRAD_OUTPUTS: ptr = mb.grad_outputs ? mb.grad_outputs[k] : nullptr; break;
            default: ptr = mb.grad_inputs ? mb.grad_inputs[k] : nullptr; break;
          }
          ext.p[i * total + k] = (void *)ptr;
        }
      }
    }
    hipEvent_t ev_end = nullptr;
    if (st->prof_on) {       // as in run_steps: a bracket of two events per step, GEMM steps repeated inside it
      if (st->prof_used + 2 > st->prof_ev.size()) {
        for (int k = 0; k < 2; ++k) {
          hipEvent_t e;
          if (hipEventCreate(&e) != hipSuccess) return fail(GPP_ERR_DEVICE, "hipEventCreate failed");
          st->prof_ev.push_back(e);
        }
      }
      (void)hipEventRecord(st->prof_ev[st->prof_used], s);
      ev_end = st->prof_ev[st->prof_used + 1];
      st->prof_tag.resize(st->prof_used / 2 + 1);
      st->prof_tag[st->prof_used / 2] = step_tag(sp, is_bwd) | ((sp.launches * (gemm_step(sp) ? st->prof_repeat : 1)) << 8);
      st->prof_used += 2;
    }
    const int reps = (st->prof_on && gemm_step(sp)) ? st->prof_repeat : 1;
    for (int rep = 0; rep < reps; ++rep)
    switch (sp.kern) {
      case K_ELT: launch_elt((const EltProb *)tab, m * sp.n, m * sp.blocks, ext, s); break;
      case K_GEMM_SKINNY: {
        // the records of the lane's first slot; the other members are that many further row blocks, their slot
        // memory L slots further each (the weight tile of a column block then serves all members from one L2)
        const void *tab0 = st->ws + pl.off_tables + (int64_t)lane * pl.table_bytes + sp.table_off;
        const int ext_total = sp.ext_kind == EXT_NONE ? 0
                              : ((sp.ext_kind == EXT_INPUTS || sp.ext_kind == EXT_GRAD_INPUTS) ? (int)pl.input_ops.size()
                                                                                               : (int)pl.output_ops.size());
        launch_gemm_skinny((const GemmProb *)tab0, sp.n, sp.blocks, sp.a1, sp.a2, sp.a0, sp.a3, ext, s, m,
                           (int64_t)pl.group_lanes * pl.slot_bytes, ext_total);
        break;
      }
      case K_HEAD_LOSS: {
        HeadOuts ho;
        memset(&ho, 0, sizeof(ho));
        for (int i = 0; i < m; ++i) {
          const int slot = lane + pl.group_lanes * i;
          float *lo = io[members[i]].loss_out;
          ho.p[i] = lo ? lo : (float *)(st->ws + pl.off_slots + (int64_t)slot * pl.slot_bytes + pl.loss_scalars.off);
        }
        launch_head_loss((const HeadProb *)tab, m, sp.a0, sp.a1, ho, s);
        break;
      }
      case K_LOSS_SUM:       // per member: its partial losses (none: zero) to where the caller wants the loss value
        for (int i = 0; i < m; ++i)
          if (io[members[i]].loss_out) {
            const int slot = lane + pl.group_lanes * i;
            const float *ls = (const float *)(st->ws + pl.off_slots + (int64_t)slot * pl.slot_bytes + pl.loss_scalars.off);
            launch_loss_sum(ls, sp.n, io[members[i]].loss_out, s);
          }
        break;
      default: return fail(GPP_ERR_UNSUPPORTED, "internal: step without a group form");
    }
    if (ev_end) (void)hipEventRecord(ev_end, s);
  }
  hipError_t he = hipGetLastError();
  if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP launch: ") + hipGetErrorString(he));
  return GPP_OK;
}

extern "C" {

gpp_status_t gpp_stage_forward(gpp_stage_t *st, int32_t slot, const void *const *inputs, void *const *outputs,
                               float *loss_out, void *hip_stream) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  Plan &pl = st->plan;
  if (slot < 0 || slot >= pl.slots) return fail(GPP_ERR_INVALID_ARG, "slot out of range");
  if (!inputs) return fail(GPP_ERR_INVALID_ARG, "inputs is null");
  for (size_t k = 0; k < pl.input_ops.size(); ++k)
    if (!inputs[k] || ((uintptr_t)inputs[k] & 3)) return fail(GPP_ERR_INVALID_ARG, "input " + std::to_string(k) + " is null or misaligned");
  if (!pl.output_ops.empty() && !outputs) return fail(GPP_ERR_INVALID_ARG, "outputs is null but the stage has outputs");
  if (st->slot_busy[slot] == 2)
    return fail(GPP_ERR_ORDER, "slot " + std::to_string(slot) + " waits for gpp_stage_backward_weights (grouped weight gradients)");
  if (st->slot_busy[slot]) return fail(GPP_ERR_ORDER, "slot " + std::to_string(slot) + " still holds a micro-batch in flight");
  gpp_status_t rc = run_steps(st, pl.fwd, slot, inputs, outputs, loss_out, 0, (hipStream_t)hip_stream);
  if (rc != GPP_OK) return rc;
  st->slot_busy[slot] = 1;
  st->fifo.push_back(slot);
  return GPP_OK;
}

gpp_status_t gpp_stage_backward(gpp_stage_t *st, int32_t slot, const void *const *grad_outputs, void *const *grad_inputs,
                                void *hip_stream) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  Plan &pl = st->plan;
  if (slot < 0 || slot >= pl.slots) return fail(GPP_ERR_INVALID_ARG, "slot out of range");
  if (st->slot_busy[slot] != 1) return fail(GPP_ERR_ORDER, "backward before forward on slot " + std::to_string(slot) + " (C4: fw_k precedes bw_k)");
  if (st->fifo.empty() || st->fifo.front() != slot)
    return fail(GPP_ERR_ORDER, "backward out of order (C4: bw_k precedes bw_{k+1}); oldest forward is in slot " +
                                   std::to_string(st->fifo.empty() ? -1 : st->fifo.front()));
  if (!pl.output_ops.empty()) {
    if (!grad_outputs) return fail(GPP_ERR_INVALID_ARG, "grad_outputs is null but the stage has outputs");
    for (size_t k = 0; k < pl.output_ops.size(); ++k)
      if (pl.nodes[pl.output_ops[k]].wants_grad && !grad_outputs[k]) return fail(GPP_ERR_INVALID_ARG, "grad_outputs[" + std::to_string(k) + "] is null");
  }
  gpp_status_t rc = run_steps(st, pl.bwd, slot, grad_outputs, grad_inputs, nullptr, st->fresh ? 0 : 1, (hipStream_t)hip_stream);
  if (rc != GPP_OK) return rc;
  st->fresh = false;
  st->fifo.pop_front();
  if (pl.dwg.empty()) {
    st->slot_busy[slot] = 0;
  } else {   // its stashed operands feed the weight-gradient launch of the group
    st->slot_busy[slot] = 2;
    st->pending.push_back(slot);
  }
  return GPP_OK;
}

gpp_status_t gpp_stage_backward_weights(gpp_stage_t *st, void *hip_stream) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  Plan &pl = st->plan;
  // one launch per run of consecutive slots (wrapping at the number of slots), in backward order
  while (!st->pending.empty()) {
    SlotGroup g;
    g.first = st->pending.front();
    g.total = pl.slots;
    g.stride = pl.slot_bytes;
    g.n = 1;
    while (g.n < (int)st->pending.size() && g.n < pl.slots && st->pending[g.n] == (g.first + g.n) % pl.slots) ++g.n;
    gpp_status_t rc = run_steps(st, pl.dwg, 0, nullptr, nullptr, nullptr, st->fresh_w ? 0 : 1, (hipStream_t)hip_stream, &g);
    if (rc != GPP_OK) return rc;
    st->fresh_w = false;
    for (int k = 0; k < g.n; ++k) {
      st->slot_busy[st->pending.front()] = 0;
      st->pending.pop_front();
    }
  }
  return GPP_OK;
}

gpp_status_t gpp_stage_grad_reset(gpp_stage_t *st, void *hip_stream) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  if (!st->fifo.empty()) return fail(GPP_ERR_ORDER, "grad_reset while a micro-batch is in flight");
  if (!st->pending.empty()) return fail(GPP_ERR_ORDER, "grad_reset before gpp_stage_backward_weights (grouped weight gradients pending)");
  st->fresh = true;
  st->fresh_w = true;
  if (st->emb_count > 0) {
    const char *tables = st->ws + st->plan.off_tables;  // slot 0's records carry the same accumulators
    const EmbProb *recs = (const EmbProb *)(tables + st->emb_table_off);
    if (st->emb_clear_pending || st->emb_log_overflow)
      launch_emb_reset(recs, st->emb_count, st->emb_capacity, 0, (hipStream_t)hip_stream);
    else if (st->emb_logged > 0)
      launch_emb_reset(recs, st->emb_count, st->emb_capacity, st->emb_logged, (hipStream_t)hip_stream);
    st->emb_clear_pending = false;
    st->emb_log_overflow = false;
    st->emb_logged = 0;
    hipError_t he = hipGetLastError();
    if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP launch: ") + hipGetErrorString(he));
  }
  return GPP_OK;
}

gpp_status_t gpp_stage_memory(const gpp_stage_t *st, size_t *slot_bytes, size_t *shared_bytes, size_t *total_bytes) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  if (slot_bytes) *slot_bytes = (size_t)st->plan.slot_bytes;
  if (shared_bytes) *shared_bytes = (size_t)(st->plan.total_bytes - (int64_t)st->plan.slots * st->plan.slot_bytes);
  if (total_bytes) *total_bytes = (size_t)st->plan.total_bytes;
  return GPP_OK;
}

// One mini-batch under a task list.  The whole list is checked against C4 and the number of stash
// slots before the first kernel is enqueued, so a refused list leaves the stage untouched.
//
// Lanes: forward pass j goes to forward stream j mod nf, backward pass j to backward stream j mod nb.
// Passes of different micro-batches have no data in common when the stage's steps use slot memory
// only (and, for backward passes, leave every parameter gradient to the group launch), so several
// lanes only change WHEN the kernels run: the task list still fixes the order of issue, the use of
// the stash slots, and the order in which the group launches add into the accumulators.
// Events per micro-batch j: 3j forward done, 3j+1 slot free again, 3j+2 backward done.
static gpp_status_t run_schedule_lanes(gpp_stage_t *st, const int32_t *tasks, int64_t n_tasks, const gpp_microbatch_io_t *io,
                                       int64_t n_micro, void *const *streams_forward, int32_t nf, void *const *streams_backward,
                                       int32_t nb) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  if (n_micro < 0 || n_tasks != 2 * n_micro) return fail(GPP_ERR_INVALID_ARG, "a mini-batch of n micro-batches has 2n tasks");
  if (n_micro > 0 && (!tasks || !io)) return fail(GPP_ERR_INVALID_ARG, "tasks or io is null");
  if (nf < 1 || nb < 1 || nf > 16 || nb > 16 || !streams_forward || !streams_backward)
    return fail(GPP_ERR_INVALID_ARG, "1 to 16 forward streams and 1 to 16 backward streams");
  if (!st->fifo.empty() || !st->pending.empty()) return fail(GPP_ERR_ORDER, "run_schedule while a micro-batch is in flight");
  const Plan &pl = st->plan;
  if (nf > 1 && (pl.fwd_shared || pl.lanes))
    return fail(GPP_ERR_UNSUPPORTED, "forward passes of this stage use memory that its slots share: one forward stream only");
  if (nb > 1 && (pl.bwd_shared || pl.lanes))
    return fail(GPP_ERR_UNSUPPORTED,
                "backward passes of this stage accumulate parameter gradients or use memory that its slots share "
                "(grouped weight gradients, stage flag bit 2, lift this for Linear layers): one backward stream only");
  const int slots = pl.slots;
  {
    int64_t f = 0, b = 0;   // forward / backward passes seen so far
    for (int64_t t = 0; t < n_tasks; ++t) {
      const int64_t v = tasks[t];
      if (v > 0) {
        if (v - 1 != f) return fail(GPP_ERR_ORDER, "task " + std::to_string(t) + ": forward passes must come in micro-batch order (C4)");
        if (f - b >= slots)
          return fail(GPP_ERR_ORDER, "task " + std::to_string(t) + ": more micro-batches in flight than the stage has stash slots (" +
                                         std::to_string(slots) + ")");
        ++f;
      } else if (v < 0) {
        if (-v - 1 != b) return fail(GPP_ERR_ORDER, "task " + std::to_string(t) + ": backward passes must come in micro-batch order (C4)");
        if (b >= f) return fail(GPP_ERR_ORDER, "task " + std::to_string(t) + ": backward pass before its forward pass (C4)");
        ++b;
      } else {
        return fail(GPP_ERR_INVALID_ARG, "task " + std::to_string(t) + " is zero");
      }
    }
  }
  bool two = false;   // more than one stream in play: order across streams comes from events
  for (int k = 0; k < nf; ++k) two = two || streams_forward[k] != streams_forward[0];
  for (int k = 0; k < nb; ++k) two = two || streams_backward[k] != streams_forward[0];
  if (two) {
    while ((int64_t)st->sched_ev.size() < 3 * n_micro) {
      hipEvent_t e;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return fail(GPP_ERR_DEVICE, "hipEventCreate failed");
      st->sched_ev.push_back(e);
    }
  }
  gpp_status_t rc = gpp_stage_grad_reset(st, streams_backward[0]);
  if (rc != GPP_OK) return rc;
  int64_t last_group = -1;   // micro-batch whose slot-free event follows the latest group launch of weight gradients
  hipError_t he = hipSuccess;
  const int L = pl.group_lanes;

  // after the last backward pass of a run (micro-batches j - run + 1 .. j, the last one on stream sb): the
  // grouped weight gradients, which follow every backward pass of the run (other lanes: their events) and the
  // group launch before it (both add into the same accumulators); only then are the run's slots free
  auto finish_backward_run = [&](int64_t j, hipStream_t sb) -> gpp_status_t {
    const int64_t run = (int64_t)st->pending.size();
    for (int64_t q = j - run + 1; q < j && he == hipSuccess; ++q)
      if (two && nb > 1 && streams_backward[q % nb] != (void *)sb) he = hipStreamWaitEvent(sb, st->sched_ev[3 * q + 2], 0);
    if (two && nb > 1 && last_group >= 0 && he == hipSuccess) he = hipStreamWaitEvent(sb, st->sched_ev[3 * last_group + 1], 0);
    if (he == hipSuccess) {
      gpp_status_t r = gpp_stage_backward_weights(st, sb);
      if (r != GPP_OK) return r;
    }
    if (two)
      for (int64_t q = j - run + 1; q <= j && he == hipSuccess; ++q) he = hipEventRecord(st->sched_ev[3 * q + 1], sb);
    last_group = j;
    return GPP_OK;
  };

  for (int64_t t = 0; t < n_tasks;) {
    const bool fwd = tasks[t] > 0;
    int64_t e = t + 1;
    while (e < n_tasks && (tasks[e] > 0) == fwd) ++e;
    const int64_t j0 = (fwd ? tasks[t] : -tasks[t]) - 1, m = e - t;     // the run: micro-batches j0 .. j0 + m - 1

    // ---- group launches: per lane, ONE launch per step for all micro-batches of the run on that lane
    bool grouped_run = st->group_ok && m >= 2 && L == (fwd ? nf : nb);
    std::vector<std::vector<int64_t>> members(grouped_run ? L : 0);
    if (grouped_run) {
      for (int64_t j = j0; j < j0 + m; ++j) members[j % L].push_back(j);
      for (int l = 0; l < L && grouped_run; ++l)
        for (size_t i = 0; i < members[l].size(); ++i)
          if ((int)(members[l][i] % slots) != l + L * (int)i) grouped_run = false;    // not the slots the lane's table holds, in its order
    }
    if (grouped_run && fwd) {
      for (int64_t j = j0; j < j0 + m; ++j) {
        const gpp_microbatch_io_t &mb = io[j];
        if (!mb.inputs) return fail(GPP_ERR_INVALID_ARG, "inputs is null");
        for (size_t k = 0; k < pl.input_ops.size(); ++k)
          if (!mb.inputs[k] || ((uintptr_t)mb.inputs[k] & 3)) return fail(GPP_ERR_INVALID_ARG, "input " + std::to_string(k) + " is null or misaligned");
        if (!pl.output_ops.empty() && !mb.outputs) return fail(GPP_ERR_INVALID_ARG, "outputs is null but the stage has outputs");
        if (st->slot_busy[j % slots]) return fail(GPP_ERR_ORDER, "slot " + std::to_string(j % slots) + " still holds a micro-batch in flight");
      }
      for (int l = 0; l < L && he == hipSuccess; ++l) {
        if (members[l].empty()) continue;
        hipStream_t sf = (hipStream_t)streams_forward[l];
        for (int64_t j : members[l])
          if (two && j >= slots && he == hipSuccess) he = hipStreamWaitEvent(sf, st->sched_ev[3 * (j - slots) + 1], 0);
        if (he != hipSuccess) break;
        rc = run_steps_group(st, pl.fwd, l, members[l], io, sf);
        if (rc != GPP_OK) return rc;
        for (int64_t j : members[l])
          if (two && he == hipSuccess) he = hipEventRecord(st->sched_ev[3 * j], sf);
      }
      for (int64_t j = j0; j < j0 + m; ++j) {
        st->slot_busy[j % slots] = 1;
        st->fifo.push_back((int32_t)(j % slots));
      }
    } else if (grouped_run) {
      for (int64_t j = j0; j < j0 + m; ++j) {
        const gpp_microbatch_io_t &mb = io[j];
        if (!pl.output_ops.empty()) {
          if (!mb.grad_outputs) return fail(GPP_ERR_INVALID_ARG, "grad_outputs is null but the stage has outputs");
          for (size_t k = 0; k < pl.output_ops.size(); ++k)
            if (pl.nodes[pl.output_ops[k]].wants_grad && !mb.grad_outputs[k]) return fail(GPP_ERR_INVALID_ARG, "grad_outputs[" + std::to_string(k) + "] is null");
        }
        if (st->slot_busy[j % slots] != 1 || (int64_t)st->fifo.size() <= j - j0 || st->fifo[j - j0] != (int32_t)(j % slots))
          return fail(GPP_ERR_ORDER, "backward out of order (C4)");
      }
      for (int l = 0; l < L && he == hipSuccess; ++l) {
        if (members[l].empty()) continue;
        hipStream_t sb = (hipStream_t)streams_backward[l];
        for (int64_t j : members[l])
          if (two && (void *)sb != streams_forward[j % nf] && he == hipSuccess) he = hipStreamWaitEvent(sb, st->sched_ev[3 * j], 0);
        if (he != hipSuccess) break;
        rc = run_steps_group(st, pl.bwd, l, members[l], io, sb);
        if (rc != GPP_OK) return rc;
        for (int64_t j : members[l])
          if (two && nb > 1 && he == hipSuccess) he = hipEventRecord(st->sched_ev[3 * j + 2], sb);
      }
      st->fresh = false;
      for (int64_t j = j0; j < j0 + m; ++j) {
        st->fifo.pop_front();
        if (pl.dwg.empty()) {
          st->slot_busy[j % slots] = 0;
        } else {
          st->slot_busy[j % slots] = 2;
          st->pending.push_back((int32_t)(j % slots));
        }
      }
      const int64_t jl = j0 + m - 1;
      hipStream_t sl = (hipStream_t)streams_backward[jl % nb];
      if (he == hipSuccess) {
        if (!st->pending.empty()) {
          rc = finish_backward_run(jl, sl);
          if (rc != GPP_OK) return rc;
        } else if (two) {     // no grouped weight gradients: every slot is free after its lane's launch
          for (int64_t j = j0; j < j0 + m && he == hipSuccess; ++j) he = hipEventRecord(st->sched_ev[3 * j + 1], (hipStream_t)streams_backward[j % nb]);
        }
      }
    } else {
      // ---- one micro-batch at a time
      for (int64_t u = t; u < e; ++u) {
        const int64_t j = (tasks[u] > 0 ? tasks[u] : -tasks[u]) - 1;
        const int32_t slot = (int32_t)(j % slots);
        const gpp_microbatch_io_t &mb = io[j];
        if (fwd) {
          hipStream_t sf = (hipStream_t)streams_forward[j % nf];
          // the slot's previous micro-batch must have been consumed by its backward pass
          if (two && j >= slots) he = hipStreamWaitEvent(sf, st->sched_ev[3 * (j - slots) + 1], 0);
          if (he == hipSuccess) {
            rc = gpp_stage_forward(st, slot, mb.inputs, mb.outputs, mb.loss_out, sf);
            if (rc != GPP_OK) return rc;
            if (two) he = hipEventRecord(st->sched_ev[3 * j], sf);
          }
        } else {
          hipStream_t sb = (hipStream_t)streams_backward[j % nb];
          // (a backward pass on its forward pass's own stream follows it there without an event)
          if (two && (void *)sb != streams_forward[j % nf]) he = hipStreamWaitEvent(sb, st->sched_ev[3 * j], 0);
          if (he == hipSuccess) {
            rc = gpp_stage_backward(st, slot, mb.grad_outputs, mb.grad_inputs, sb);
            if (rc != GPP_OK) return rc;
            // grouped weight gradients: one launch after the last backward pass of a run of backward
            // tasks; only then are the run's slots free for the forward passes that wait for them
            if (st->pending.empty()) {
              if (two) he = hipEventRecord(st->sched_ev[3 * j + 1], sb);
            } else if (u + 1 < e) {
              if (two && nb > 1) he = hipEventRecord(st->sched_ev[3 * j + 2], sb);
            } else {
              rc = finish_backward_run(j, sb);
              if (rc != GPP_OK) return rc;
            }
          }
        }
        if (he != hipSuccess) break;
      }
    }
    if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP event: ") + hipGetErrorString(he));
    t = e;
  }
  return GPP_OK;
}

gpp_status_t gpp_stage_run_schedule(gpp_stage_t *st, const int32_t *tasks, int64_t n_tasks, const gpp_microbatch_io_t *io,
                                    int64_t n_micro, void *stream_forward, void *stream_backward) {
  return run_schedule_lanes(st, tasks, n_tasks, io, n_micro, &stream_forward, 1, &stream_backward, 1);
}

gpp_status_t gpp_stage_run_schedule_lanes(gpp_stage_t *st, const int32_t *tasks, int64_t n_tasks, const gpp_microbatch_io_t *io,
                                          int64_t n_micro, void *const *streams_forward, int32_t n_forward,
                                          void *const *streams_backward, int32_t n_backward) {
  return run_schedule_lanes(st, tasks, n_tasks, io, n_micro, streams_forward, n_forward, streams_backward, n_backward);
}

gpp_status_t gpp_stage_sync_status(gpp_stage_t *st, void *hip_stream) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  hipError_t he = hipStreamSynchronize((hipStream_t)hip_stream);
  StageFlags f;
  if (he == hipSuccess) he = hipMemcpy(&f, st->ws + st->plan.off_flags, sizeof(f), hipMemcpyDeviceToHost);
  if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP: ") + hipGetErrorString(he));
  if (f.index_error) {
    hipMemset(st->ws + st->plan.off_flags, 0, sizeof(f));
    return fail(GPP_ERR_INDEX, "an embedding index or offset was out of range");
  }
  return GPP_OK;
}

gpp_status_t gpp_stage_profile_enable(gpp_stage_t *st, int32_t enable) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  st->prof_on = enable != 0;
  st->prof_repeat = enable > 1 ? (enable < 64 ? enable : 64) : 1;
  return GPP_OK;
}

gpp_status_t gpp_stage_profile_read(gpp_stage_t *st, double *ms, int64_t *launches, int32_t reset) {
  if (!st || !ms || !launches) return fail(GPP_ERR_INVALID_ARG, "null argument");
  for (size_t k = 0; k + 1 < st->prof_used; k += 2) {
    if (hipEventSynchronize(st->prof_ev[k + 1]) != hipSuccess) return fail(GPP_ERR_DEVICE, "hipEventSynchronize failed");
    float t = 0.0f;
    if (hipEventElapsedTime(&t, st->prof_ev[k], st->prof_ev[k + 1]) != hipSuccess) return fail(GPP_ERR_DEVICE, "hipEventElapsedTime failed");
    const int tag = st->prof_tag[k / 2] & 255;
    st->prof_ms[tag] += t;
    st->prof_launches[tag] += st->prof_tag[k / 2] >> 8;
  }
  st->prof_used = 0;
  for (int k = 0; k < GPP_PROFILE_TAGS; ++k) {
    ms[k] = st->prof_ms[k];
    launches[k] = st->prof_launches[k];
    if (reset) {
      st->prof_ms[k] = 0.0;
      st->prof_launches[k] = 0;
    }
  }
  return GPP_OK;
}

const char *gpp_profile_tag_name(int32_t tag) { return (tag >= 0 && tag < GPP_PROFILE_TAGS) ? kTagNames[tag] : ""; }

gpp_status_t gpp_stage_embedding_sort_result(gpp_stage_t *st, int32_t op, const int32_t **sorted_pos, const int32_t **unique_rows,
                                             const int32_t **seg_offsets, const int32_t **counts) {
  if (!st) return fail(GPP_ERR_INVALID_ARG, "stage is null");
  Plan &pl = st->plan;
  if (op < 0 || op >= (int32_t)pl.nodes.size() || (pl.nodes[op].d.kind != GPP_OP_EMBEDDING_BAG_SUM && pl.nodes[op].d.kind != GPP_OP_EMBEDDING_BAG_CONCAT))
    return fail(GPP_ERR_INVALID_ARG, "op is not an embedding bag");
  const Node &nd = pl.nodes[op];
  if (!st->emb_last_table) return fail(GPP_ERR_ORDER, "no backward pass has run yet");
  // the hot path sums segments without a table of distinct rows: build it now, for all tables,
  // from the sorted rows the last backward pass left in its log slot, and wait for it
  launch_emb_segments((const EmbProb *)st->emb_last_table, st->emb_count, st->emb_sort_blocks, st->emb_last_slot, nullptr);
  hipError_t he = hipDeviceSynchronize();
  if (he != hipSuccess) return fail(GPP_ERR_DEVICE, std::string("HIP: ") + hipGetErrorString(he));
  auto sh = [&](const Buf &b) { return (const int32_t *)(st->ws + pl.off_shared + b.off); };
  if (sorted_pos) *sorted_pos = sh((nd.emb_passes & 1) ? nd.more[2] : nd.more[3]);
  if (unique_rows) *unique_rows = sh(nd.more[11]);
  if (seg_offsets) *seg_offsets = sh(nd.more[6]);
  if (counts) *counts = sh(nd.more[7]) + st->emb_last_slot * 4;
  return GPP_OK;
}

}  // extern "C"
