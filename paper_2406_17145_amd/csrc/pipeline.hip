// Several stages of one stage graph G_S on ONE GPU, each stage on its own pair of HIP streams (the
// streams stand in for the stage's devices): every stage runs its own micro-batch task list, and the
// edges of G_S become events between the streams (paper section 3: an edge (S_i, S_j) of E_S orders
// the two stages; section 2: independent stages run concurrently).  Host code over the stage calls.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <string>
#include <vector>

#include "../../include/gpp.h"

namespace gpp {
gpp_status_t report_error(gpp_status_t st, const std::string &msg);
}
using gpp::report_error;

namespace {
struct Port {            // one input or output of a stage
  int edge = -1;         // data edge attached to it, or -1: the caller's pointer is used
  size_t bytes = 0;
};
struct PStage {
  gpp_stage_t *h = nullptr;
  int slots = 1;
  bool grouped = false;                   // weight gradients per run of backward passes (stage flag bit 2)
  std::vector<int64_t> freed_by;          // per micro-batch: the backward pass whose event says that its slot is free
  int64_t cap = 1, k = 1;                 // micro-batches it may hold, group size
  std::vector<Port> in, out;
  std::vector<int> pred, succ;            // stages ordered before / after it (data and order edges)
  std::vector<hipEvent_t> ev;             // 2 per micro-batch: after fw_j, after bw_j (and its weight gradients)
};
struct Edge {
  gpp_pipeline_edge_t e;
  size_t bytes = 0;       // one micro-batch of the tensor
  int copies = 1;         // in-flight micro-batches of the producer
  char *act = nullptr, *grad = nullptr;
};
size_t align256(size_t v) { return (v + 255) / 256 * 256; }
}  // namespace

struct gpp_pipeline {
  std::vector<PStage> st;
  std::vector<Edge> ed;
  int64_t b = 0;
};

static gpp_status_t build(gpp_pipeline &P, int32_t n_stages, gpp_stage_t *const *stages, int32_t n_edges,
                          const gpp_pipeline_edge_t *edges, const int64_t *in_flight, const int64_t *k, size_t *bytes) {
  if (n_stages <= 0 || !stages || n_edges < 0 || (n_edges > 0 && !edges) || !in_flight || !k)
    return report_error(GPP_ERR_INVALID_ARG, "pipeline: null argument or no stage");
  P.st.assign(n_stages, PStage());
  for (int s = 0; s < n_stages; ++s) {
    PStage &S = P.st[s];
    S.h = stages[s];
    int64_t b = 0;
    int32_t slots = 0, flags = 0;
    if (gpp_stage_info(S.h, &b, &slots, &flags) != GPP_OK) return GPP_ERR_INVALID_ARG;
    S.grouped = (flags & 4) != 0;
    if (s == 0) P.b = b;
    if (b != P.b) return report_error(GPP_ERR_UNSUPPORTED, "pipeline: all stages must use one micro-batch size (the paper's default configuration)");
    if (in_flight[s] <= 0 || k[s] <= 0) return report_error(GPP_ERR_INVALID_ARG, "pipeline: in-flight samples and k must be positive");
    S.slots = slots;
    S.cap = std::max<int64_t>(1, in_flight[s] / b);
    S.k = k[s];
    if (S.cap > slots)
      return report_error(GPP_ERR_ORDER, "pipeline: stage " + std::to_string(s) + " holds " + std::to_string(S.cap) +
                                             " micro-batches in flight but has " + std::to_string(slots) + " stash slots");
    S.in.assign(gpp_stage_num_inputs(S.h), Port());
    S.out.assign(gpp_stage_num_outputs(S.h), Port());
  }
  P.ed.assign(n_edges, Edge());
  size_t total = 0;
  for (int e = 0; e < n_edges; ++e) {
    Edge &E = P.ed[e];
    E.e = edges[e];
    const int x = E.e.from_stage, y = E.e.to_stage;
    if (x < 0 || x >= n_stages || y < 0 || y >= n_stages || x == y) return report_error(GPP_ERR_INVALID_ARG, "pipeline: edge endpoint out of range");
    P.st[x].succ.push_back(y);
    P.st[y].pred.push_back(x);
    if (E.e.from_output < 0 && E.e.to_input < 0) continue;   // order-only edge
    if (E.e.from_output < 0 || E.e.from_output >= (int)P.st[x].out.size() || E.e.to_input < 0 || E.e.to_input >= (int)P.st[y].in.size())
      return report_error(GPP_ERR_INVALID_ARG, "pipeline: edge names an output or input the stage does not have");
    if (P.st[x].out[E.e.from_output].edge >= 0 || P.st[y].in[E.e.to_input].edge >= 0)
      return report_error(GPP_ERR_UNSUPPORTED, "pipeline: an output feeds one input, an input has one producer (fan-out lives inside a stage)");
    int64_t ro, fo, ri, fi;
    int32_t dto, dti, go, gi;
    gpp_stage_io_info(P.st[x].h, 1, E.e.from_output, &ro, &fo, &dto, &go);
    gpp_stage_io_info(P.st[y].h, 0, E.e.to_input, &ri, &fi, &dti, &gi);
    if (ro != ri || fo != fi || dto != dti)
      return report_error(GPP_ERR_SHAPE, "pipeline: edge " + std::to_string(e) + " joins tensors of different shape or type");
    if (go && !gi)
      return report_error(GPP_ERR_BAD_GRAPH, "pipeline: edge " + std::to_string(e) + ": the producer expects a gradient the consumer's input does not return");
    E.bytes = align256((size_t)ro * fo * (dto == GPP_F32 || dto == GPP_I32 ? 4 : 2));
    E.copies = (int)P.st[x].cap;
    P.st[x].out[E.e.from_output].edge = e;
    P.st[y].in[E.e.to_input].edge = e;
    total += 2 * E.bytes * E.copies;
  }
  // the stage graph must be acyclic (C2 orders the stages)
  {
    std::vector<int> indeg(n_stages, 0), ready;
    for (auto &S : P.st) for (int y : S.succ) ++indeg[y];
    for (int s = 0; s < n_stages; ++s) if (!indeg[s]) ready.push_back(s);
    int done = 0;
    while (!ready.empty()) {
      const int s = ready.back();
      ready.pop_back();
      ++done;
      for (int y : P.st[s].succ) if (--indeg[y] == 0) ready.push_back(y);
    }
    if (done != n_stages) return report_error(GPP_ERR_BAD_GRAPH, "pipeline: the stage graph has a cycle");
  }
  if (bytes) *bytes = std::max<size_t>(total, 256);
  return GPP_OK;
}

// Issue order over all stages: a task is issued once the tasks of other stages it waits for have been
// issued (their events exist then).  `issue` = nullptr: dry run that only checks that every task can
// be issued (the in-flight counts of the stages fit each other).
template <typename F>
static bool sweep(const gpp_pipeline &P, const std::vector<std::vector<int32_t>> &tasks, F issue) {
  const int n = (int)P.st.size();
  std::vector<size_t> pos(n, 0);
  std::vector<int64_t> fdone(n, 0), bdone(n, 0);   // forward / backward passes issued per stage
  for (;;) {
    bool progress = false, all = true;
    for (int s = 0; s < n; ++s) {
      while (pos[s] < tasks[s].size()) {
        const int32_t t = tasks[s][pos[s]];
        const int64_t j = (t > 0 ? t : -t) - 1;
        bool ok = true;
        if (t > 0) for (int p : P.st[s].pred) ok = ok && fdone[p] > j;
        else       for (int q : P.st[s].succ) ok = ok && bdone[q] > j;
        if (!ok) break;
        const bool run_ends = pos[s] + 1 == tasks[s].size() || tasks[s][pos[s] + 1] > 0;
        if (!issue(s, t, j, run_ends)) return false;
        (t > 0 ? fdone[s] : bdone[s])++;
        ++pos[s];
        progress = true;
      }
      all = all && pos[s] == tasks[s].size();
    }
    if (all) return true;
    if (!progress) return false;
  }
}

extern "C" {

gpp_status_t gpp_pipeline_workspace_bytes(int32_t n_stages, gpp_stage_t *const *stages, int32_t n_edges,
                                          const gpp_pipeline_edge_t *edges, const int64_t *in_flight, const int64_t *k,
                                          size_t *bytes) {
  if (!bytes) return report_error(GPP_ERR_INVALID_ARG, "bytes is null");
  gpp_pipeline P;
  return build(P, n_stages, stages, n_edges, edges, in_flight, k, bytes);
}

gpp_status_t gpp_pipeline_create(int32_t n_stages, gpp_stage_t *const *stages, int32_t n_edges, const gpp_pipeline_edge_t *edges,
                                 const int64_t *in_flight, const int64_t *k, void *workspace, size_t workspace_bytes,
                                 gpp_pipeline_t **out) {
  if (!out) return report_error(GPP_ERR_INVALID_ARG, "out is null");
  gpp_pipeline *P = new gpp_pipeline();
  size_t need = 0;
  gpp_status_t rc = build(*P, n_stages, stages, n_edges, edges, in_flight, k, &need);
  if (rc == GPP_OK && (!workspace || workspace_bytes < need || ((uintptr_t)workspace & 255)))
    rc = report_error(GPP_ERR_WORKSPACE, "pipeline: workspace missing, misaligned or smaller than " + std::to_string(need) + " bytes");
  if (rc != GPP_OK) {
    delete P;
    return rc;
  }
  char *w = (char *)workspace;
  for (Edge &E : P->ed) {
    if (!E.bytes) continue;
    E.act = w;
    w += E.bytes * E.copies;
    E.grad = w;
    w += E.bytes * E.copies;
  }
  *out = P;
  return GPP_OK;
}

gpp_status_t gpp_pipeline_destroy(gpp_pipeline_t *P) {
  if (P)
    for (auto &S : P->st)
      for (hipEvent_t e : S.ev) (void)hipEventDestroy(e);
  delete P;
  return GPP_OK;
}

gpp_status_t gpp_pipeline_run(gpp_pipeline_t *P, int64_t n_micro, const gpp_microbatch_io_t *const *io,
                              void *const *streams_forward, void *const *streams_backward) {
  if (!P || !io || !streams_forward || !streams_backward) return report_error(GPP_ERR_INVALID_ARG, "pipeline_run: null argument");
  if (n_micro < 0 || n_micro > (1 << 24)) return report_error(GPP_ERR_INVALID_ARG, "pipeline_run: bad number of micro-batches");
  const int n = (int)P->st.size();
  std::vector<std::vector<int32_t>> tasks(n);
  for (int s = 0; s < n; ++s) {
    if (n_micro > 0 && !io[s]) return report_error(GPP_ERR_INVALID_ARG, "pipeline_run: io[" + std::to_string(s) + "] is null");
    tasks[s].resize(2 * n_micro);
    gpp_status_t rc = gpp_schedule_tasks(n_micro, P->st[s].cap * P->b, P->st[s].k, P->b, tasks[s].data());
    if (rc != GPP_OK) return rc;
  }
  // dry run: nothing is enqueued unless every task of every stage can be
  if (!sweep(*P, tasks, [](int, int32_t, int64_t, bool) { return true; }))
    return report_error(GPP_ERR_ORDER, "pipeline_run: the stages' task lists wait for each other (in-flight counts too small for this stage graph)");
  for (auto &S : P->st) S.freed_by.assign(n_micro, -1);
  for (auto &S : P->st)
    while ((int64_t)S.ev.size() < 2 * n_micro) {
      hipEvent_t e;
      if (hipEventCreateWithFlags(&e, hipEventDisableTiming) != hipSuccess) return report_error(GPP_ERR_DEVICE, "hipEventCreate failed");
      S.ev.push_back(e);
    }
  for (int s = 0; s < n; ++s) {
    gpp_status_t rc = gpp_stage_grad_reset(P->st[s].h, streams_backward[s]);
    if (rc != GPP_OK) return rc;
  }
  gpp_status_t status = GPP_OK;
  std::vector<const void *> in_ptrs;
  std::vector<void *> out_ptrs;
  auto issue = [&](int s, int32_t t, int64_t j, bool run_ends) {
    PStage &S = P->st[s];
    hipStream_t sf = (hipStream_t)streams_forward[s], sb = (hipStream_t)streams_backward[s];
    const int32_t slot = (int32_t)(j % S.slots);
    const gpp_microbatch_io_t &m = io[s][j];
    hipError_t he = hipSuccess;
    auto wait = [&](hipStream_t on, hipEvent_t ev) {
      if (he == hipSuccess) he = hipStreamWaitEvent(on, ev, 0);
    };
    if (t > 0) {
      for (int p : S.pred) wait(sf, P->st[p].ev[2 * j]);                 // the producers' fw_j
      if (j >= S.slots) wait(sf, S.ev[2 * S.freed_by[j - S.slots] + 1]);  // the slot's previous micro-batch
      in_ptrs.assign(S.in.size(), nullptr);
      out_ptrs.assign(S.out.size(), nullptr);
      for (size_t q = 0; q < S.in.size(); ++q) {
        const int e = S.in[q].edge;
        in_ptrs[q] = e >= 0 ? P->ed[e].act + (j % P->ed[e].copies) * P->ed[e].bytes : (m.inputs ? m.inputs[q] : nullptr);
      }
      for (size_t q = 0; q < S.out.size(); ++q) {
        const int e = S.out[q].edge;
        out_ptrs[q] = e >= 0 ? (void *)(P->ed[e].act + (j % P->ed[e].copies) * P->ed[e].bytes) : (m.outputs ? m.outputs[q] : nullptr);
      }
      if (he == hipSuccess) status = gpp_stage_forward(S.h, slot, in_ptrs.data(), out_ptrs.data(), m.loss_out, sf);
      if (status != GPP_OK) return false;
      if (he == hipSuccess) he = hipEventRecord(S.ev[2 * j], sf);
    } else {
      wait(sb, S.ev[2 * j]);                                             // its own fw_j
      for (int q : S.succ) wait(sb, P->st[q].ev[2 * j + 1]);             // the consumers' bw_j
      in_ptrs.assign(S.out.size(), nullptr);                             // gradients w.r.t. the outputs
      out_ptrs.assign(S.in.size(), nullptr);                             // gradients w.r.t. the inputs
      for (size_t q = 0; q < S.out.size(); ++q) {
        const int e = S.out[q].edge;
        in_ptrs[q] = e >= 0 ? P->ed[e].grad + (j % P->ed[e].copies) * P->ed[e].bytes : (m.grad_outputs ? m.grad_outputs[q] : nullptr);
      }
      for (size_t q = 0; q < S.in.size(); ++q) {
        const int e = S.in[q].edge;
        out_ptrs[q] = e >= 0 ? (void *)(P->ed[e].grad + (j % P->ed[e].copies) * P->ed[e].bytes) : (m.grad_inputs ? m.grad_inputs[q] : nullptr);
      }
      if (he == hipSuccess) status = gpp_stage_backward(S.h, slot, in_ptrs.data(), out_ptrs.data(), sb);
      if (status != GPP_OK) return false;
      // grouped weight gradients run with the last backward pass of a run; a stage without them records
      // the event at once.  The event after bw_j also tells the producers that the gradient is there.
      if (run_ends) {
        status = gpp_stage_backward_weights(S.h, sb);
        if (status != GPP_OK) return false;
      }
      if (he == hipSuccess) he = hipEventRecord(S.ev[2 * j + 1], sb);
      // a slot is free after its own backward pass, or, with grouped weight gradients, after the run's launch
      if (!S.grouped) S.freed_by[j] = j;
      else if (run_ends)
        for (int64_t q = j; q >= 0 && S.freed_by[q] < 0; --q) S.freed_by[q] = j;
    }
    if (he != hipSuccess) {
      status = report_error(GPP_ERR_DEVICE, std::string("pipeline_run: HIP event: ") + hipGetErrorString(he));
      return false;
    }
    return true;
  };
  if (!sweep(*P, tasks, issue) && status == GPP_OK) status = report_error(GPP_ERR_ORDER, "pipeline_run: internal: issue order diverged from the dry run");
  return status;
}

}  // extern "C"
