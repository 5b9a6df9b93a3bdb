/*
 * gpp.h -- C ABI of the MI355X graph-pipeline-parallel (GPP) stage library.
 *
 * A DNN is a DAG of operators G_C = (V_C, E_C) that GPP cuts into a DAG of
 * stages; a stage is S_i = <G_i, b_i, D_i, Pi_i>: a sub-graph of operators, a
 * micro-batch size, a device set and a micro-batch schedule (paper section 3,
 * "Problem Formulation").  This library executes ONE stage on ONE GPU
 * (|D_i| = 1): for each micro-batch j it runs the forward pass fw_j and later
 * the backward pass bw_j of G_i, keeps fw_j's activations until bw_j (paper
 * section 1: a micro-batch is "in flight" until its backward finishes), and
 * adds weight gradients over the micro-batches of a mini-batch, because under
 * the synchronous schedule weights change only between iterations (paper
 * section 6, default configuration; section 8, synchronous pipelines).  The
 * schedule Pi_i is the caller's order of calls; the library enforces the
 * ordering condition C4 of section 3.  Branches of G_i that are
 * computationally independent are kept side by side: all operators of one
 * topological level run as ONE grouped kernel launch (paper section 2).
 *
 * Conventions
 *   - plain C, no C++ or PyTorch types; every function returns a status and
 *     never throws or aborts; out-parameters are untouched on error.
 *   - "DEVICE" pointers are HIP device memory owned by the caller; "HOST"
 *     pointers are ordinary host memory.  The library allocates no device
 *     memory: parameters, gradient accumulators, the workspace and all
 *     per-call tensors belong to the caller.
 *   - forward / backward / grad_reset only enqueue kernels on the given HIP
 *     stream (a hipStream_t passed as void*); they neither allocate nor
 *     synchronise.  All calls on one stage must be issued on one stream (or be
 *     ordered by the caller), and must not overlap from several host threads.
 *   - 2-D tensors are row-major [rows, features].  rows = micro_batch*seq_len
 *     (+ rows_extra for inputs).  Tensors passed per call (inputs, outputs and
 *     their gradients) are dense: leading dimension == features.  Parameters
 *     and gradient accumulators with a feature dimension use the padded
 *     leading dimension gpp_ld(features) (next multiple of 64 elements, so that
 *     every row of a bf16 or fp32 matrix starts on a 128-byte cache line); the
 *     padding columns of parameters must hold zeros and the library never
 *     writes padding columns of gradient accumulators.
 *   - all device base pointers must be 16-byte aligned; the workspace 256.
 */
#ifndef GPP_H
#define GPP_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct gpp_stage gpp_stage_t; /* opaque, owned by the library between create and destroy */

typedef enum {
  GPP_OK = 0,
  GPP_ERR_INVALID_ARG = 1, /* null pointer, bad enum, bad size */
  GPP_ERR_BAD_GRAPH = 2,   /* cycle, dangling edge, wrong arity: G_i is not a DAG of known operators */
  GPP_ERR_SHAPE = 3,       /* feature / row counts of connected operators disagree */
  GPP_ERR_UNSUPPORTED = 4, /* valid graph this library has no kernel for (e.g. dtype mix) */
  GPP_ERR_WORKSPACE = 5,   /* workspace too small or misaligned */
  GPP_ERR_ORDER = 6,       /* ordering condition C4 violated, or slot busy / free */
  GPP_ERR_INDEX = 7,       /* an embedding index, a bag offset or a class label was out of range (see gpp_stage_sync_status) */
  GPP_ERR_DEVICE = 8       /* a HIP call failed, see gpp_last_error */
} gpp_status_t;

typedef enum { GPP_F32 = 0, GPP_BF16 = 1, GPP_I32 = 2 } gpp_dtype_t;

/* Operator kinds: the operator types of the paper's evaluation models
 * (appendix "DNN Model Configurations": feed-forward layers, transformer
 * layers with multi-head attention, embedding bags, an interaction, and the
 * concatenation that merges branches) plus loss heads for a last stage. */
typedef enum {
  GPP_OP_INPUT = 0,         /* tensor entering the stage along a stage-graph edge, or a target */
  GPP_OP_LINEAR = 1,        /* y = act(x W^T + b); W is [out_features, gpp_ld(in_features)] */
  GPP_OP_LAYERNORM = 2,     /* over features, biased variance, affine gamma/beta, eps */
  GPP_OP_ATTENTION = 3,     /* input [b*S, 3d] = Q|K|V column blocks; softmax(QK^T/sqrt(d/heads))V, non-causal */
  GPP_OP_ADD = 4,           /* elementwise sum of two producers */
  GPP_OP_MEANPOOL_SEQ = 5,  /* [b*S, d] -> [b, d], mean over the S rows of each sample */
  GPP_OP_CONCAT = 6,        /* feature-wise concatenation of its producers, in the order given */
  GPP_OP_EMBEDDING_BAG_SUM = 7, /* in[0] = indices input (i32, [b, bag_size] capacity), in[1] = offsets input
                                   (i32, b+1 entries, offsets[0] = 0, non-decreasing, offsets[b] <= b*bag_size);
                                   out[s,:] = sum_{j in [off[s], off[s+1])} table[idx[j],:] */
  GPP_OP_DOT_INTERACT = 8,  /* input [b, F*d] seen as F vectors of d = in_features; out = [vector 0 |
                               <v_i,v_j> for i>j in row-major order (1,0),(2,0),(2,1),...] */
  GPP_OP_LOSS_MSE = 9,      /* in = (prediction, target f32); L = loss_scale * sum (y-t)^2 */
  GPP_OP_LOSS_CE = 10,      /* in = (logits, labels i32 [b,1]); L = -loss_scale * sum log softmax(y)[label] */
  GPP_OP_LOSS_BCE_LOGITS = 11, /* in = (logits, targets f32); L = loss_scale * sum softplus(y) - t*y */
  GPP_OP_EMBEDDING_BAG_CONCAT = 12 /* producers as EMBEDDING_BAG_SUM; the rows of a bag are concatenated (the
                                   paper's DLRM, appendix "DNN Model Configurations"): in_features = row width d,
                                   out_features = bag_size * d (a multiple of 64),
                                   out[s, j*d:(j+1)*d] = table[idx[off[s] + j], :], zero for j >= the bag's length */
} gpp_op_kind_t;

typedef enum { GPP_ACT_NONE = 0, GPP_ACT_RELU = 1, GPP_ACT_GELU_ERF = 2 } gpp_act_t;

/* One vertex of G_i.  `in` lists producer op ids (the edges E_C inside the
 * stage).  HOST memory; the library copies what it needs during create. */
typedef struct {
  int32_t kind;          /* gpp_op_kind_t */
  int32_t n_in;
  const int32_t *in;     /* HOST, n_in producer ids */
  int32_t branch;        /* branch label (>= 0), -1 for merge / tail operators; informational */
  int64_t in_features;   /* LINEAR: K; DOT_INTERACT: vector width d */
  int64_t out_features;  /* feature count of the output (INPUT: of the tensor itself) */
  int32_t act;           /* gpp_act_t, LINEAR only */
  int32_t has_bias;      /* LINEAR only */
  int32_t heads;         /* ATTENTION */
  int32_t seq_len;       /* rows per sample of the output (INPUT, LAYERNORM, ATTENTION, ...: S; 1 = plain) */
  int32_t rows_extra;    /* INPUT only: extra rows beyond micro_batch*seq_len (1 for bag offsets) */
  int32_t requires_grad; /* INPUT only: 1 = float tensor from a predecessor stage whose gradient is returned */
  int64_t num_rows;      /* EMBEDDING_BAG_SUM: table rows */
  int64_t bag_size;      /* EMBEDDING_BAG_SUM: maximum indices per bag (capacity b*bag_size) */
  double eps;            /* LAYERNORM */
  double loss_scale;     /* LOSS_*: carries the 1/B normalisation of the whole mini-batch, so that
                            micro-batch gradients sum to the full-batch gradient */
  int32_t dtype;         /* gpp_dtype_t of the output tensor as stored */
  int32_t param_dtype;   /* LINEAR: dtype of W (must equal the producer's dtype); others ignored */
  void *param[2];        /* DEVICE. LINEAR: W, bias(f32) | LAYERNORM: gamma(f32), beta(f32) |
                            EMBEDDING_BAG_SUM: table f32 [num_rows, gpp_ld(out_features)];
                            EMBEDDING_BAG_CONCAT: table f32 [num_rows, gpp_ld(in_features)] */
  void *grad[2];         /* DEVICE, f32 accumulators with the layout of param[] (W's gradient is f32
                            [out_features, gpp_ld(in_features)]) */
} gpp_op_desc_t;

typedef struct {
  int32_t n_ops;
  const gpp_op_desc_t *ops;   /* HOST */
  int64_t micro_batch;        /* b_i */
  int32_t in_flight_slots;    /* how many micro-batches may be in flight (activation stash slots) */
  int32_t flags;              /* bit 0: force the generic (non-MFMA) GEMM kernels (testing);
                                 bit 1: split the contraction of small grouped GEMMs over several
                                 workgroups (deterministic; measured slower, off by default);
                                 bit 2: grouped weight gradients, see gpp_stage_backward_weights;
                                 bit 3: a stage that holds embedding bags next to dense branches runs the
                                 bags' gather and their sort + segment sums on a side stream of its own
                                 (created with the stage at default priority, forked from and joined to the
                                 caller's stream by events inside every forward / backward call); off by
                                 default: it pays only for large micro-batches;
                                 bit 4: the stage's launches will share the GPU with other launches (several
                                 streams per direction in gpp_stage_run_schedule_lanes, other stages of a
                                 pipeline): few-row GEMM launches of at most 64 rows then use workgroups of
                                 four waves instead of eight (half the LDS and registers per workgroup, so
                                 workgroups of concurrent launches fit a compute unit side by side; a launch
                                 that has the GPU to itself is ~10 % slower that way);
                                 bits 8-11: L > 0 asks for GROUP LAUNCHES in gpp_stage_run_schedule_lanes with L
                                 streams per direction (needs bit 2, in_flight_slots a multiple of L and at
                                 least 2 L): where a run of forward (backward) tasks puts several micro-batches
                                 on one stream, each step of the pass is ONE launch over all of them (the
                                 launch records of their slots one after the other, from a second copy of the
                                 tables per lane; for the few-row GEMMs the first slot's records plus the slot
                                 stride) instead of one launch per micro-batch.  Same kernels,
                                 same tiles per micro-batch, so the results do not change; the chain of
                                 dependent launches on a stream gets shorter.  Taken where every step has a
                                 group form (element-wise copies, few-row GEMMs, the fused head) and a run
                                 starts at slot 0 of each lane; otherwise the call launches per micro-batch.  The
                                 micro-batches of one launch write their outputs, losses and input gradients
                                 together: every micro-batch in flight needs buffers of its own */
} gpp_stage_desc_t;

/* Leading dimension used for parameters and gradient accumulators. */
int64_t gpp_ld(int64_t features);

/* Bytes of workspace a stage needs (activation stash for every slot, backward
 * scratch, launch tables, sort buffers).  Host-only: needs no GPU.  Validates
 * the descriptor (parameter pointers are not looked at). */
gpp_status_t gpp_stage_workspace_bytes(const gpp_stage_desc_t *desc, size_t *bytes);

/* Validates G_i (C1: it must be a DAG; shapes must agree), plans the grouped
 * launches and copies the launch tables into the workspace (synchronous
 * copies; the only calls of this library that synchronise are create,
 * destroy-free-of-device-work and sync_status).  `workspace` is DEVICE memory
 * of at least gpp_stage_workspace_bytes bytes, 256-byte aligned, owned by the
 * caller and reserved for this stage until destroy.  Its content is cleared. */
gpp_status_t gpp_stage_create(const gpp_stage_desc_t *desc, void *workspace, size_t workspace_bytes,
                              gpp_stage_t **out);

/* For callers that cannot allocate device memory (code under HIP graph capture set-up, tight serving loops,
 * harnesses that forbid hipMalloc): gpp_stage_create with the workspace taken from a device array that is part
 * of the library itself (GPP_STATIC_WORKSPACE_BYTES per GPU, held by every GPU the library runs on until the
 * process ends).  The call allocates no device memory and calls no allocating routine; parameters, gradient
 * accumulators and per-call tensors stay the caller's.  The created stage is an ordinary stage: forward,
 * backward, grad_reset, the schedule executor and destroy work on it as on any other.
 *   - GPP_ERR_WORKSPACE if the stage needs more than GPP_STATIC_WORKSPACE_BYTES (gpp_stage_workspace_bytes says
 *     how much a descriptor needs); GPP_ERR_UNSUPPORTED with flag bit 3 (its side stream would have to be created).
 *   - One stage per GPU holds the array at a time: GPP_ERR_ORDER while another stage created by this call on the
 *     current GPU has not been destroyed.  The array keeps the previous stage's contents; the call clears the
 *     part it uses (on the null stream, synchronously), so device work of a destroyed static stage must have
 *     finished before the next one is created: calls that overlap on one GPU race.
 *   - The GPU that is current at the call is the one whose array is used. */
#define GPP_STATIC_WORKSPACE_BYTES (32u << 20)
gpp_status_t gpp_stage_create_static(const gpp_stage_desc_t *desc, gpp_stage_t **out);

/* fw_j: forward pass of one micro-batch into stash slot `slot`.
 *   inputs[i]   DEVICE, dense tensor of the i-th GPP_OP_INPUT in op-id order (read during the call's
 *               kernels only; the stage keeps its own copy for the backward pass)
 *   outputs[i]  DEVICE, dense tensor for the i-th stage output (non-loss operator without consumer,
 *               op-id order); entries may be NULL
 *   loss_out    DEVICE float or NULL: receives the sum of this micro-batch's loss operators
 * Errors: GPP_ERR_ORDER if the slot is still in flight. */
gpp_status_t gpp_stage_forward(gpp_stage_t *stage, int32_t slot, const void *const *inputs,
                               void *const *outputs, float *loss_out, void *hip_stream);

/* bw_j: backward pass of the micro-batch held in `slot`; frees the slot.
 *   grad_outputs[i] DEVICE, dense gradient w.r.t. the i-th stage output (same dtype); the array may be
 *                   NULL when the stage has no outputs (loss-terminated)
 *   grad_inputs[i]  DEVICE or NULL, dense gradient w.r.t. the i-th GPP_OP_INPUT (written only for
 *                   inputs with requires_grad; same dtype as the input)
 * Weight gradients are ADDED into the accumulators (the first backward after gpp_stage_grad_reset
 * overwrites instead of reading them).  Errors: GPP_ERR_ORDER unless `slot` holds the OLDEST forward
 * that has not been backpropagated (C4: fw_k before bw_k, bw_k before bw_{k+1}). */
gpp_status_t gpp_stage_backward(gpp_stage_t *stage, int32_t slot, const void *const *grad_outputs,
                                void *const *grad_inputs, void *hip_stream);

/* Grouped weight gradients (stage flag bit 2; the kFkB schedules of section 6 run k backward passes in a row).
 * With the flag, gpp_stage_backward computes input gradients and the gradients of every operator except the
 * weights and biases of LINEAR operators in bf16 storage; those are left to this call, which contracts over the
 * rows of ALL micro-batches backpropagated since its previous call in one launch -- one pass over the fp32
 * accumulators for the whole group instead of one per micro-batch.  Until this call a backpropagated slot keeps
 * its stashed activations and output gradients and cannot take a new forward pass (GPP_ERR_ORDER), and
 * gpp_stage_grad_reset refuses to run.  The accumulated gradients are complete after this call.  The sums are
 * formed in a fixed order (micro-batch order inside the contraction), so results are deterministic, but they
 * round differently from per-micro-batch accumulation.  No-op without the flag or with nothing pending.
 * LINEAR operators the grouped kernel does not take (fp32 storage) keep accumulating in gpp_stage_backward. */
gpp_status_t gpp_stage_backward_weights(gpp_stage_t *stage, void *hip_stream);

/* Iteration boundary (weights are updated once per mini-batch): the next backward starts new sums.
 * Dense accumulators are not touched by this call (their next write overwrites); embedding-table
 * accumulators are cleared on the stream: only the rows that the backward passes since the previous
 * reset touched when at most four such passes ran, whole tables otherwise (and the first time).  Errors: GPP_ERR_ORDER while a micro-batch is in flight. */
gpp_status_t gpp_stage_grad_reset(gpp_stage_t *stage, void *hip_stream);

/* Waits for the stream and reports GPP_ERR_INDEX if any kernel since the last call met an embedding
 * index out of range, bag offsets that break their contract (first offset not 0, decreasing, beyond the
 * capacity) or a class label outside [0, classes) (such entries are skipped, never dereferenced; the
 * results of that micro-batch are then not those of the operator graph). */
gpp_status_t gpp_stage_sync_status(gpp_stage_t *stage, void *hip_stream);

gpp_status_t gpp_stage_destroy(gpp_stage_t *stage);

/* ---- Static micro-batch scheduler (paper section 6, Alg. 2; appendix "Generalized Per-stage kFkB
 * Schedule").  HOST-only integer routines (no GPU needed) and the executor that runs their result. ---- */

/* ComputeInFlight, the appendix table: in-flight SAMPLES *i_x of a stage S_x that runs k_x F k_x B at
 * micro-batch size b_x in front of a stage S_y that runs k_y F k_y B at size b_y and holds i_y in-flight
 * samples.  All arguments positive (k, b at most 2^30), else GPP_ERR_INVALID_ARG. */
gpp_status_t gpp_compute_in_flight(int64_t k_x, int64_t b_x, int64_t k_y, int64_t b_y, int64_t i_y, int64_t *i_x);

/* Schedules of a whole stage graph (section 6: the last stage first, then against the edges; appendix:
 * k_x = argmin over the candidates of the largest table value over the successors of S_x).
 *   edge_from[e] -> edge_to[e]   HOST, n_edges pairs of stage ids in [0, n_stages)
 *   b[x]                         HOST, micro-batch size of S_x
 *   k_values[k_begin[x] .. k_begin[x+1])   HOST, the candidate k of S_x (k_begin has n_stages + 1 entries)
 *   i_out[x], k_out[x]           HOST, written: in-flight samples and chosen k of S_x
 * A stage without successor holds one group, k * b samples; equal counts choose the smallest k.
 * GPP_ERR_BAD_GRAPH if the stage graph has a cycle. */
gpp_status_t gpp_assign_schedules(int32_t n_stages, int32_t n_edges, const int32_t *edge_from, const int32_t *edge_to,
                                  const int64_t *b, const int32_t *k_begin, const int64_t *k_values, int64_t *i_out,
                                  int64_t *k_out);

/* ScheduleTask of Alg. 2 for the configuration c = (i, k, b) and n_micro micro-batches: the kFkB order of the
 * footnote of section 6 with a warm-up of floor(i / b) forward passes (at least one; at most n_micro), groups of
 * min(k, warm-up) backward and forward passes, every backward pass as early as that allows.
 *   tasks   HOST, 2 * n_micro entries written: +(j+1) stands for fw_j, -(j+1) for bw_j */
gpp_status_t gpp_schedule_tasks(int64_t n_micro, int64_t i, int64_t k, int64_t b, int32_t *tasks);

/* Pointers of one micro-batch, with the meaning they have in gpp_stage_forward / gpp_stage_backward. */
typedef struct {
  const void *const *inputs;
  void *const *outputs;
  float *loss_out;
  const void *const *grad_outputs;
  void *const *grad_inputs;
} gpp_microbatch_io_t;

/* One mini-batch of the stage under a task list (Pi_i of section 3): gradient reset, then every task in
 * order; micro-batch j uses stash slot j % in_flight_slots.
 *   tasks[n_tasks]   HOST, n_tasks = 2 * n_micro, encoded as by gpp_schedule_tasks
 *   io[n_micro]      HOST array; the pointers inside are DEVICE pointers (arrays of them HOST)
 *   stream_forward / stream_backward   HIP streams of the forward and of the backward passes (and the
 *                    reset).  Equal: everything runs in task order.  Different: fw_j and bw_j' of different
 *                    micro-batches may overlap on the GPU, which C4 allows; the call orders bw_j after fw_j and
 *                    fw_j after bw_{j - in_flight_slots} with events (created on first use, kept by the stage).
 *                    Ordering against earlier and later work on other streams is the caller's.
 * The whole list is validated before anything is enqueued: GPP_ERR_ORDER if it violates C4 or holds more
 * micro-batches in flight than the stage has slots (nothing has run then).  On a stage with grouped weight
 * gradients the call issues gpp_stage_backward_weights after every run of consecutive backward tasks. */
gpp_status_t gpp_stage_run_schedule(gpp_stage_t *stage, const int32_t *tasks, int64_t n_tasks,
                                    const gpp_microbatch_io_t *io, int64_t n_micro, void *stream_forward,
                                    void *stream_backward);

/* gpp_stage_run_schedule with several streams per direction: forward pass j is enqueued on
 * streams_forward[j % n_forward], backward pass j on streams_backward[j % n_backward] (HOST arrays of HIP
 * streams, 1 to 16 each).  Micro-batches are independent computations (section 2: operators without a path
 * between them may run concurrently), so on a GPU that one few-row micro-batch cannot fill, neighbouring
 * passes of a kFkB group overlap.  C4 still governs everything whose ORDER can be observed: tasks are issued
 * in list order, a slot is reused only after its backward pass (and group launch), and the weight-gradient
 * launches add into the accumulators in list order, so every result is bit-identical to the one-stream run.
 *   n_forward > 1    needs forward steps that touch no memory shared between slots
 *   n_backward > 1   needs backward steps that touch no shared memory and accumulate no parameter gradient
 *                    themselves: Linear-only stages created with grouped weight gradients (flag bit 2)
 *   otherwise GPP_ERR_UNSUPPORTED (nothing has run).  gpp_stage_lanes reports both properties.
 * Micro-batches that may be in flight together need their own outputs, loss_out and grad_inputs buffers
 * (passes j and j' share a stream, hence run in order, when j = j' modulo the lane count).
 * Ordering against work on other streams before and after the call is the caller's, on every stream. */
gpp_status_t gpp_stage_run_schedule_lanes(gpp_stage_t *stage, const int32_t *tasks, int64_t n_tasks,
                                          const gpp_microbatch_io_t *io, int64_t n_micro, void *const *streams_forward,
                                          int32_t n_forward, void *const *streams_backward, int32_t n_backward);

/* Workspace use: bytes of ONE activation stash slot (the memory an in-flight micro-batch pins, section 2),
 * bytes shared by all slots (backward scratch, launch tables, sort buffers), and their total for this
 * stage's in_flight_slots.  Any pointer may be NULL. */
gpp_status_t gpp_stage_memory(const gpp_stage_t *stage, size_t *slot_bytes, size_t *shared_bytes, size_t *total_bytes);

/* ---- Pipeline stage partitioner (paper section 5, Alg. 1; problem statement of section 3).  HOST-only.
 * Cuts the operator graph G_C into stages, gives every stage a number of devices and returns the stage graph
 * whose bottleneck stage has the smallest time per sample among those that fit the memory of their devices
 * with the in-flight micro-batches their schedules need.  Method as in the paper: series-parallel structure
 * of G_C, a dynamic programme over it (value: the fewest in-flight samples at the first stages of a
 * sub-graph, given a bound on every stage's time per sample; in-flight samples by ComputeInFlight), binary
 * search on the bound until the interval is below eps_rel of its upper end.
 * Model (what the paper leaves open):
 *   - default schedule configuration of section 6: 1F1B everywhere, one micro-batch size b;
 *   - a stage on d devices is data-parallel: time per sample = sum of t / d, plus for d > 1 a ring all-reduce
 *     of its parameters per mini-batch: 2 (d-1)/d * sum of w * sync_seconds_per_byte / mini_batch;
 *   - memory of a stage per device = sum of w + in-flight samples / d * sum of a;
 *   - operators are nodes: operators that fall into several weakly connected parts are composed in PARALLEL,
 *     a connected set is split in SERIES at every operator all others are ancestors or descendants of, a
 *     connected set without one is an indivisible block; a stage is a node of that tree or a run of
 *     consecutive children of one node; every device is used and a stage has at least one.
 *   t[o] seconds per sample on one device (forward + backward), w[o] parameter and gradient bytes,
 *   a[o] stashed bytes per sample of operator o                                   HOST, n_ops entries each
 *   stage_of_op[n_ops]; stage_devices, stage_in_flight (samples): room for n_ops entries, *n_stages written
 * *n_stages = 0 (status GPP_OK) when no stage graph fits the memory.  *bottleneck: time per sample of the
 * slowest stage of the result; *dp_states (may be NULL): states the dynamic programme evaluated over all
 * steps of the binary search.  GPP_ERR_BAD_GRAPH if G_C has a cycle. */
gpp_status_t gpp_partition(int32_t n_ops, int32_t n_edges, const int32_t *edge_from, const int32_t *edge_to,
                           const double *t, const double *w, const double *a, int32_t n_devices, int64_t b,
                           double memory_bytes, double sync_seconds_per_byte, int64_t mini_batch, double eps_rel,
                           int32_t *stage_of_op, int32_t *n_stages, int32_t *stage_devices, int64_t *stage_in_flight,
                           double *bottleneck, int64_t *dp_states);

/* gpp_partition with the configuration loop of Alg. 1 (section 5: SearchStageGraph enumerates schedule configurations
 * c = (i, b, k); the series case of DP enumerates the configuration c_m of the stage(s) in the middle): every stage
 * takes a micro-batch size out of b_values and a kFkB group size out of k_values, the in-flight samples between two
 * stages follow from both stages' (b, k) by ComputeInFlight, and tensors between stages are charged.
 *   b_values[n_b], k_values[n_k]   HOST, the candidates (the paper considers powers of two); 1 to 64 of each
 *   t[o * n_b + j]   HOST, seconds per sample of operator o on one device at micro-batch size b_values[j] (the paper
 *                    profiles operators; efficiency rises with the micro-batch size, section 2)
 *   x[e]             HOST or NULL, bytes per sample on operator edge e
 *   link_latency, link_seconds_per_byte   the paper's affine communication model: per micro-batch, a stage pays
 *                    link_latency + bytes * link_seconds_per_byte for every operator edge with exactly one end inside
 *                    it (activations arriving, gradients coming back), i.e. per sample
 *                    cut edges * link_latency / b + cut bytes per sample * link_seconds_per_byte
 *   stage_b, stage_k room for n_ops entries each (may be NULL): the configuration chosen for every stage
 * Everything else as in gpp_partition.  Readings: both halves of a parallel decomposition receive the same c_f
 * (Alg. 1), so the stages that come first inside a parallel composition share one configuration; the configuration
 * that SearchStageGraph enumerates is that of the first stage(s) of the whole graph, the dummy one stands for the
 * successor the last stage does not have; b and k enter memory only through the in-flight samples. */
gpp_status_t gpp_partition_search(int32_t n_ops, int32_t n_edges, const int32_t *edge_from, const int32_t *edge_to,
                                  int32_t n_b, const int64_t *b_values, const double *t, const double *w, const double *a,
                                  int32_t n_k, const int64_t *k_values, const double *x, double link_latency,
                                  double link_seconds_per_byte, int32_t n_devices, double memory_bytes,
                                  double sync_seconds_per_byte, int64_t mini_batch, double eps_rel, int32_t *stage_of_op,
                                  int32_t *n_stages, int32_t *stage_devices, int64_t *stage_in_flight, int64_t *stage_b,
                                  int64_t *stage_k, double *bottleneck, int64_t *dp_states);

/* ---- Several stages of a stage graph G_S on one GPU (paper section 3: G_S = (V_S, E_S); an edge (S_x, S_y)
 * orders the two stages for every micro-batch, C2; stages without a path between them run concurrently,
 * section 2).  Each stage keeps its own task list (gpp_schedule_tasks for its (i, k)) and its own pair of
 * HIP streams, which stand in for the stage's devices; the edges become events between the streams and, for
 * data edges, device buffers that carry the tensor forward and its gradient backward. ---- */
typedef struct gpp_pipeline gpp_pipeline_t;
typedef struct {
  int32_t from_stage, from_output;  /* producer stage and which of its outputs; from_output = to_input = -1: an  */
  int32_t to_stage, to_input;       /* order-only edge (a linearised, sequential pipeline chains stages this way) */
} gpp_pipeline_edge_t;

/* Bytes of DEVICE workspace for the edge tensors: per data edge, forward tensor and gradient, one copy per
 * micro-batch the producer may hold in flight.  Validates the stage graph: GPP_ERR_BAD_GRAPH (cycle; producer
 * wants a gradient the consumer's input does not return), GPP_ERR_SHAPE (tensor shapes or types differ),
 * GPP_ERR_UNSUPPORTED (different micro-batch sizes; an output feeding several inputs -- fan-out lives inside
 * a stage), GPP_ERR_ORDER (a stage has fewer stash slots than in_flight[s] / micro_batch).
 *   stages[n_stages]   HOST array of created stages (borrowed until gpp_pipeline_destroy)
 *   in_flight[s], k[s] HOST, the schedule configuration of stage s as gpp_assign_schedules returns it
 *                      (in-flight SAMPLES and group size) */
gpp_status_t gpp_pipeline_workspace_bytes(int32_t n_stages, gpp_stage_t *const *stages, int32_t n_edges,
                                          const gpp_pipeline_edge_t *edges, const int64_t *in_flight, const int64_t *k,
                                          size_t *bytes);
/* `workspace`: DEVICE, 256-byte aligned, at least gpp_pipeline_workspace_bytes, the caller's, reserved until destroy. */
gpp_status_t gpp_pipeline_create(int32_t n_stages, gpp_stage_t *const *stages, int32_t n_edges,
                                 const gpp_pipeline_edge_t *edges, const int64_t *in_flight, const int64_t *k,
                                 void *workspace, size_t workspace_bytes, gpp_pipeline_t **out);
/* One mini-batch of n_micro micro-batches through every stage.
 *   io[s][j]   HOST: the caller's pointers of stage s, micro-batch j (meaning as in gpp_stage_forward / backward);
 *              entries of inputs, outputs and their gradients that an edge carries are ignored
 *   streams_forward[s], streams_backward[s]   HOST arrays of HIP streams, one pair per stage (pairs may coincide)
 * fw_j of a stage waits for fw_j of every predecessor, bw_j for bw_j of every successor; inside a stage the
 * order is its task list.  Before anything is enqueued a dry run checks that the task lists cannot wait for
 * each other (GPP_ERR_ORDER: in-flight counts too small for this stage graph).  Ordering against other work
 * on the streams is the caller's. */
gpp_status_t gpp_pipeline_run(gpp_pipeline_t *pipeline, int64_t n_micro, const gpp_microbatch_io_t *const *io,
                              void *const *streams_forward, void *const *streams_backward);
gpp_status_t gpp_pipeline_destroy(gpp_pipeline_t *pipeline);

/* Introspection (tests, benchmarks). */
/* micro-batch size, number of stash slots and flags the stage was created with (any pointer may be NULL) */
gpp_status_t gpp_stage_info(const gpp_stage_t *stage, int64_t *micro_batch, int32_t *in_flight_slots, int32_t *flags);
/* whether several forward / backward streams are allowed in gpp_stage_run_schedule_lanes (1) or not (0) */
gpp_status_t gpp_stage_lanes(const gpp_stage_t *stage, int32_t *forward_ok, int32_t *backward_ok);
/* group launches (flag bits 8-11): the number of streams per direction they are set up for and the most
 * micro-batches one launch covers; 0, 0 when the stage was created without them or has a step without a
 * group form */
gpp_status_t gpp_stage_group_launches(const gpp_stage_t *stage, int32_t *lanes, int32_t *members);
/* rows, features and gpp_dtype_t of the index-th input (is_output = 0) or output (1), and whether a gradient
 * flows through it (an input that returns one / an output that expects one) */
gpp_status_t gpp_stage_io_info(const gpp_stage_t *stage, int32_t is_output, int32_t index, int64_t *rows,
                               int64_t *features, int32_t *dtype, int32_t *has_grad);
int32_t gpp_stage_num_inputs(const gpp_stage_t *stage);
int32_t gpp_stage_num_outputs(const gpp_stage_t *stage);
/* op id of the i-th input / output; -1 if out of range */
int32_t gpp_stage_input_op(const gpp_stage_t *stage, int32_t i);
int32_t gpp_stage_output_op(const gpp_stage_t *stage, int32_t i);
/* number of kernel launches of one forward (backward = 0) / backward (1) / grouped weight-gradient (2) call */
int32_t gpp_stage_num_launches(const gpp_stage_t *stage, int32_t backward);
/* Integer artefacts of the last backward of embedding op `op`: DEVICE pointers into the workspace.
 * sorted_pos[n_used]: index positions stably sorted by row; unique_rows[n_unique] ascending;
 * seg_offsets[n_unique+1]; counts[0] = n_used, counts[1] = n_unique (DEVICE int32[2]).
 * Inspection call, not for the hot path: it enqueues two small kernels (the table of distinct rows
 * is not needed by the backward pass itself) and synchronises the device before it returns.
 * GPP_ERR_ORDER if no backward has run. */
gpp_status_t gpp_stage_embedding_sort_result(gpp_stage_t *stage, int32_t op, const int32_t **sorted_pos,
                                             const int32_t **unique_rows, const int32_t **seg_offsets,
                                             const int32_t **counts);

/* Per-kernel timing for benchmarks.  While enabled, forward/backward bracket every grouped launch
 * with a pair of HIP events on the caller's stream (events are created on first use: the only
 * allocation these calls ever make, and only in this mode).  profile_read waits for the recorded
 * events and returns, per tag, the accumulated milliseconds and kernel launches since the last
 * reset; ms and launches are HOST arrays of GPP_PROFILE_TAGS entries.  enable = R > 1 (at most 64) is a
 * TIMING-ONLY mode: every grouped GEMM launch is issued R times back to back inside its bracket, so that the
 * bracket's own dispatch latency (about two microseconds) is spread over R launches; accumulated gradients
 * and in-place sums of such a pass are meaningless. */
#define GPP_PROFILE_TAGS 32
gpp_status_t gpp_stage_profile_enable(gpp_stage_t *stage, int32_t enable);
gpp_status_t gpp_stage_profile_read(gpp_stage_t *stage, double *ms, int64_t *launches, int32_t reset);
const char *gpp_profile_tag_name(int32_t tag);

/* Thread-local description of the last error returned on this thread. */
const char *gpp_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* GPP_H */
