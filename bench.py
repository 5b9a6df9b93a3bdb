#!/usr/bin/env python3
"""Benchmark: forward+backward samples/s of one GPP stage on one MI355X.

A "step" is one pass of the whole hot path over one mini-batch of synthetic
input: grad_reset, then for each of the workload's micro-batches fw_j and bw_j
(weight gradients accumulate across them).  Inputs are resident in HBM before
the timed region.

Without --config the line's headline (`value`, `roofline`, `cpu_baseline`) is the
multi-modal-transformer-shaped stage (micro-batch 4, the largest single-GPU
workload and the only one bound by the matrix cores), and the key `configs`
carries the other four workloads measured the same way in the same process:
samples/s, median / min / max milliseconds per step, the dominant kernel and its
fraction of the published peak; for the heterogeneous stage also the sweep over
micro-batch sizes 1 ... 128, for the feature-tower stage also the schedules with
two micro-batches in flight.  With --config NAME only that workload runs.

Prints ONE JSON line.  Besides the driver's fields it carries
  roofline      the dominant kernel's algorithmic bytes (or flops) per launch over its average
                launch duration, measured with HIP events on the launch stream, one launch per
                event bracket, in an instrumented pass over the same steps; `traffic` is read
                from profiles/kernel_traffic.txt (written from rocprofv3 counter runs by
                paper_2406_17145_amd/profile_summary.py), null when that file has no entry
  cpu_baseline  the CPU oracle timed on this host on a bounded sample of the same workload
  kernels       per-kernel breakdown of the instrumented pass
  step_ms       median / min / max / spread of per-step times (HIP events around every step)
"""
import argparse
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
sys.path.insert(0, ROOT)

HBM_PEAK_GBS = 8000.0          # MI355X HBM3E, published
MFMA_BF16_PEAK_TFLOPS = 2500.0  # dense bf16, published


def gemm_traffic(wl):
    """Algorithmic bytes and flops of the three grouped-GEMM roles for ONE micro-batch.

    Per parameter of a bf16 Linear: forward reads W once (2 B); backward-data reads W once (2 B);
    backward-weight reads and writes the fp32 accumulator (8 B; 4 B on the first micro-batch after
    a reset, which overwrites).  Activations: every operand/result matrix once, in its storage type.
    """
    b = wl.micro_batch
    rows = {}
    for i, op in enumerate(wl.ops):
        if op["kind"] == "input":
            rows[i] = b * op.get("seq_len", 1) + op.get("rows_extra", 0)
        elif op["kind"] in ("meanpool", "embedding_bag_sum", "embedding_bag_concat"):
            rows[i] = b
        elif op["kind"].startswith("loss"):
            rows[i] = 0
        else:
            rows[i] = rows[op["inputs"][0]]
    out = {"fwd": [0, 0], "dx": [0, 0], "dw": [0, 0], "dw_first": [0, 0], "params": 0}
    for i, op in enumerate(wl.ops):
        if op["kind"] != "linear":
            continue
        es = 2 if op["dtype"] == "bf16" else 4
        m, k, n = rows[i], op["in_features"], op["out_features"]
        p = k * n
        out["params"] += p
        fl = 2 * m * k * n
        out["fwd"][0] += p * es + m * k * es + m * n * es
        out["fwd"][1] += fl
        needs_dx = wl.ops[op["inputs"][0]]["kind"] != "input" or wl.ops[op["inputs"][0]].get("role") == "data"
        if needs_dx:
            out["dx"][0] += p * es + m * n * es + m * k * es
            out["dx"][1] += fl
        out["dw"][0] += p * 8 + m * n * es + m * k * es
        out["dw_first"][0] += p * 4 + m * n * es + m * k * es
        out["dw"][1] += fl
        out["dw_first"][1] += fl
    return out


def other_traffic(wl):
    """Algorithmic (bytes, flops) per micro-batch of the non-GEMM kernels that can dominate a workload.

    embedding forward   compulsory HBM bytes: every distinct table row of the micro-batch once, the index
                        and offset arrays once, the pooled output once (the logical gather, one row read
                        per index, is reported beside it as `logical`)
    embedding backward  pooled-output gradient once, index array once, every distinct row of the fp32
                        gradient table read and written once
    attention           forward 4*S*S*dh flops per (sample, head): QK^T and PV; backward 8: dV, dP, dQ, dK
    """
    import numpy as np
    out = {}
    emb_ops = [(i, op) for i, op in enumerate(wl.ops) if op["kind"] == "embedding_bag_sum"]
    if emb_ops:
        mb = wl.batches[0]
        fwd = bwd = logical = 0
        for i, op in emb_ops:
            ins = op["inputs"]
            idx, off = np.asarray(mb[ins[0]]), np.asarray(mb[ins[1]])
            n_used = int(off[-1])
            uniq = int(np.unique(idx[:n_used]).size)
            dim = op["out_features"]
            es_out = 2 if op.get("dtype", "f32") == "bf16" else 4
            pooled = wl.micro_batch * dim * es_out
            fwd += uniq * dim * 4 + n_used * 4 + off.size * 4 + pooled
            logical += n_used * dim * 4 + n_used * 4 + off.size * 4 + pooled
            bwd += pooled + n_used * 4 + 2 * uniq * dim * 4
        out["embedding_fwd"] = (fwd, 0, logical)
        out["embedding_bwd_sort_segsum"] = (bwd, 0, bwd)
    att = [op for op in wl.ops if op["kind"] == "attention"]
    if att:
        fl = sum(wl.micro_batch * op["seq_len"] ** 2 * op["out_features"] for op in att)   # heads * dh = d_model
        by = sum(wl.micro_batch * op["seq_len"] * op["out_features"] * 2 * 4 for op in att)   # q, k, v, o in bf16
        out["attention_fwd"] = (by, 4 * fl, by)
        out["attention_bwd_dq"] = (by, 4 * fl, by)
        out["attention_bwd_dkv"] = (by, 4 * fl, by)
    return out


AUTO_SHARED_LANES = True   # fw_j and bw_j of a micro-batch on one stream: a chain of launches per micro-batch
AUTO_LANES = (2, 2)     # --lanes auto, where the stage allows several streams per direction

TRAFFIC_FILE = os.path.join(ROOT, "profiles", "kernel_traffic.txt")


def measured_traffic(config, kernel):
    """HBM bytes per launch of a kernel family of a workload, from two rocprofv3 --pmc runs (FETCH_SIZE, then
    WRITE_SIZE) scaled by what the same counters read for a copy of known size; the table is written by
    paper_2406_17145_amd/profile_summary.py next to the summaries it comes from.  None where not measured."""
    try:
        with open(TRAFFIC_FILE) as f:
            for line in f:
                part = [v.strip() for v in line.split("|")]
                if len(part) >= 3 and part[0] == config and part[1] == kernel:
                    return float(part[2])
    except OSError:
        pass
    return None


CONFIG_NAMES = ["tiny_mlp", "candle_uno", "mmt", "dlrm", "hetero", "paper_mmt", "paper_candle", "paper_dlrm"]


def build_parser():
    ap = argparse.ArgumentParser()
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=200)
    ap.add_argument("--warmup", type=int, default=20)
    ap.add_argument("--config", default="all", choices=["all"] + CONFIG_NAMES,
                    help="all (default): headline mmt, the other four workloads under the key `configs`")
    ap.add_argument("--micro-batch", type=int, default=0, help="override the config's micro-batch size")
    ap.add_argument("--in-flight", type=int, default=0, metavar="M",
                    help="--schedule kfkb: micro-batches the stage may hold (its stash slots; i = M * micro-batch samples); "
                         "0 = all micro-batches of a step, at most 8")
    ap.add_argument("--k", type=int, default=0, help="--schedule kfkb: group size k of the kFkB order; 0 = M")
    ap.add_argument("--grouped-dw", default="auto", choices=["auto", "on", "off"],
                    help="weight gradients of each run of backward passes in one launch over the run's stash slots "
                         "(gpp_stage_backward_weights); auto: on")
    ap.add_argument("--lanes", default="auto", metavar="F,B",
                    help="--schedule kfkb: streams for the forward and for the backward passes (pass j on stream j mod F / B); "
                         "auto: 2,2 where the stage allows several streams per direction (gpp_stage_lanes), else 1")
    ap.add_argument("--shared-lanes", default="auto", choices=["auto", "on", "off"],
                    help="--lanes F,F: the backward passes use the forward streams (one chain of launches per micro-batch)")
    ap.add_argument("--shared-gpu", default="auto", choices=["auto", "on", "off"],
                    help="stage flag bit 4 (workgroup sizes for launches that share the GPU); auto: on when several "
                         "streams per direction are used; on: also for a one-stream profiling run of the same kernels")
    ap.add_argument("--group-launches", default="auto", choices=["auto", "on", "off"],
                    help="stage flag bits 8-11: the micro-batches that a run of tasks puts on one stream share one launch per step")
    ap.add_argument("--same-stream", action="store_true",
                    help="--schedule kfkb: the calls of all lanes (and their group launches) on ONE stream: the launches of the "
                         "timed configuration one after the other, for kernel traces")
    ap.add_argument("--one-stream", action="store_true", help="--schedule kfkb: all tasks on one stream, in task order")
    ap.add_argument("--schedule", default="auto", choices=["auto", "serial", "overlap", "kfkb"],
                    help="micro-batch schedule of a step: serial = fw_k bw_k in turn on one stream; overlap = fw_{k+1} "
                         "runs while bw_k runs (a slot per micro-batch, two streams, enqueued by the Python binding); "
                         "kfkb = the scheduler's kFkB task list for c = (i, k, b), run by the library's executor "
                         "(forward and backward passes on two streams); auto = kfkb when the workload has at least "
                         "two micro-batches per step, else serial")
    ap.add_argument("--graph", default="auto", choices=["auto", "on", "off"],
                    help="on: the step (all its launches on both streams) is captured once into a HIP graph and "
                         "replayed; off: every step is enqueued from the host; auto: on with the two-stream schedules "
                         "when the stage has a slot per micro-batch of the step (a captured forward pass cannot wait "
                         "for a backward pass), off with the serial one (measured: replay is 1-3 %% slower than eager "
                         "launches there)")
    ap.add_argument("--side-stream", action="store_true",
                    help="stage flag bit 3: the embedding bags' launches on a side stream of the stage, next to the dense branches")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--no-serial-reference", action="store_true",
                    help="skip the untimed-in-value reference pass that runs the same steps eagerly in serial order "
                         "(keeps a kernel trace of the run to the launches of the timed schedule)")
    ap.add_argument("--no-kernel-pass", action="store_true", help="skip the event-instrumented pass")
    ap.add_argument("--no-step-times", action="store_true",
                    help="skip the pass that brackets every step with events (keeps a kernel trace to warm-up + steps)")
    ap.add_argument("--copy-calibration", type=int, default=0, metavar="MIB",
                    help="before the steps, run 3 plain elementwise copies of MIB mebibytes (counter calibration)")
    return ap


def run_one(args):
    """One workload in one launch configuration: returns the JSON object of its line."""
    import numpy as np
    import torch
    from paper_2406_17145_amd import binding as B
    from paper_2406_17145_amd import workloads as W

    kw = {}
    if args.micro_batch:
        kw["micro_batch"] = args.micro_batch
    wl = W.CONFIGS[args.config](**kw)
    kernels, roofline = {}, None
    from paper_2406_17145_amd.schedule import GraphedMinibatch, OverlapSchedule, SerialSchedule, TaskSchedule
    kfkb = args.schedule == "kfkb" or (args.schedule == "auto" and wl.n_micro >= 2)
    overlap = args.schedule == "overlap"
    if kfkb:
        args.in_flight = args.in_flight or min(wl.n_micro, 8)
        args.k = args.k or args.in_flight
    # overlapped schedule: one stash slot per micro-batch of the step (at most 8), so that no forward
    # call waits for a backward call (the form a HIP graph can hold, see schedule.py)
    n_slots = min(wl.n_micro, 8) if overlap else (max(1, min(args.in_flight, wl.n_micro)) if kfkb else 1)
    # (also with one micro-batch per step: the weight gradients of all layers then share one launch that no
    # backward-data launch waits for; measured +15 % on dlrm, +5 % on hetero, +3 % on mmt)
    grouped = args.grouped_dw != "off"
    base_flags = (B.FLAG_GROUPED_DW if grouped else 0) | (B.FLAG_SIDE_STREAM if args.side_stream else 0)
    # several streams per direction (decided below): the stage's launches then share the GPU, and it is created
    # with the workgroup sizes for that; whether the stage allows such streams is known once it exists
    want_lanes = kfkb and not args.one_stream and n_slots > 1 and args.lanes != "1,1"
    shared_gpu = args.shared_gpu == "on" or (args.shared_gpu == "auto" and want_lanes)
    # group launches: the micro-batches that a run of tasks puts on one stream share one launch per step
    group_flag = 0
    if kfkb and not args.one_stream and n_slots > 1 and args.group_launches != "off":
        n_l = AUTO_LANES[0] if args.lanes == "auto" else int(args.lanes.split(",")[0])
        if n_slots % n_l == 0 and n_slots // n_l >= 2:
            group_flag = B.flag_group_launches(n_l)
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=n_slots, flags=base_flags | group_flag | (B.FLAG_SHARED_GPU if shared_gpu else 0))
    lanes_refused = args.shared_gpu == "auto" and want_lanes and args.lanes == "auto" and not any(B.gpp_stage_lanes(st.handle))
    if lanes_refused or (group_flag and B.gpp_stage_group_launches(st.handle) == (0, 0)):
        # the stage has steps without a group form, or allows no lanes at all: created again without what it cannot use
        st.close()
        group_flag = 0
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=n_slots,
                     flags=base_flags | (B.FLAG_SHARED_GPU if shared_gpu and not lanes_refused else 0))
    dev_batches = [st.stage_inputs(mb) for mb in wl.batches]       # resident in HBM
    outs = [st.alloc_outputs() for _ in range(max(n_slots, 2))]    # one set per in-flight slot
    gins = st.alloc_grad_inputs()
    gouts = [torch.zeros_like(o) for o in outs[0]] if outs[0] else None
    losses = [torch.zeros(1, dtype=torch.float32, device=st.dev) for _ in range(max(n_slots, 2))]
    serial = SerialSchedule(st)
    sched = OverlapSchedule(st) if overlap else serial
    lanes = (1, 1)
    if kfkb and not args.one_stream:
        ok_f, ok_b = B.gpp_stage_lanes(st.handle)
        if args.lanes == "auto":
            lanes = (AUTO_LANES[0] if ok_f else 1, AUTO_LANES[1] if ok_b else 1)
        else:
            lanes = tuple(int(v) for v in args.lanes.split(","))
        lanes = (max(1, min(lanes[0], n_slots)), max(1, min(lanes[1], n_slots)))
    shared_lanes = lanes[0] == lanes[1] and lanes[0] > 1 and (args.shared_lanes == "on" or (args.shared_lanes == "auto" and AUTO_SHARED_LANES))
    gins_sched = gins
    if lanes[1] > 1:     # backward passes on different streams may overlap: a set of gradient-input buffers each
        gins_sched = [gins] + [st.alloc_grad_inputs() for _ in range(lanes[1] - 1)]
    if (B.gpp_stage_info(st.handle)[2] >> 8) & 15:     # group launches: a set per micro-batch in flight
        gins_sched = [gins] + [st.alloc_grad_inputs() for _ in range(n_slots - 1)]
    if kfkb:
        sched = TaskSchedule(st, n_slots * wl.micro_batch, args.k, two_streams=not (args.one_stream or args.same_stream), lanes=lanes,
                             shared_lanes=shared_lanes and not args.same_stream, same_stream=args.same_stream)

    def eager_step(schedule=None):
        schedule = schedule or sched
        if schedule is serial:
            schedule.minibatch(dev_batches, outputs=outs[0], grad_outputs=gouts, grad_inputs=gins, losses=losses[:1])
        else:
            schedule.minibatch(dev_batches, outputs=outs, grad_outputs=gouts,
                               grad_inputs=gins_sched if isinstance(schedule, TaskSchedule) else gins, losses=losses)

    step = eager_step

    graphed = None
    if (args.graph == "on" or (args.graph == "auto" and (overlap or kfkb))) and (wl.n_micro <= max(n_slots, 1) or (kfkb and args.one_stream)):
        eager_step()                # one eager step first (see GraphedMinibatch)
        torch.cuda.synchronize()
        if sched is serial:
            graphed = GraphedMinibatch(sched, dev_batches, outputs=outs[0], grad_outputs=gouts, grad_inputs=gins, losses=losses[:1])
        else:
            graphed = GraphedMinibatch(sched, dev_batches, outputs=outs, grad_outputs=gouts, grad_inputs=gins_sched, losses=losses)
        step = graphed.replay       # the timed steps replay the graph

    if args.copy_calibration:
        # a copy of known size: reads MIB and writes MIB per launch (torch's elementwise kernel)
        src = torch.ones(args.copy_calibration * (1 << 18), dtype=torch.float32, device=st.dev)
        dst = torch.empty_like(src)
        for _ in range(3):
            torch.mul(src, 1.0, out=dst)
        torch.cuda.synchronize()
        del src, dst

    # ---- instrumented pass (before the timed region: it is set-up as far as the timed steps are concerned, and
    # the GPU's clocks have settled by the time they start): per-kernel durations from HIP events on the launch stream
    if not args.no_kernel_pass:
        # Two passes.  One launch per event bracket: this is the figure every rate below uses (it agrees with the
        # rocprofv3 kernel trace from about 20 us per launch on; below that the bracket's own dispatch latency of
        # about 2 us shows, so short launches read a little SLOWER here than in the trace).  GEMM launches issued 8
        # times inside each bracket: reported beside it as `avg_launch_us_back_to_back` only -- a repeated launch
        # finds its weights in the last-level cache, which flatters launches that stream tens of megabytes.
        REP = 8
        k_steps = max(1, min(args.steps, 20))
        # per-kernel durations are taken with the calls back to back on ONE stream, eagerly: in serial order, or,
        # with grouped weight gradients (whose kernels depend on the grouping), in the timed task order
        inst = TaskSchedule(st, n_slots * wl.micro_batch, args.k, two_streams=False, lanes=lanes, same_stream=True) if (kfkb and grouped) else serial

        for _ in range(max(3, min(args.warmup, 20))):     # clocks and caches as in the timed steps
            eager_step(inst)
        torch.cuda.synchronize()

        def kernel_pass(rep):
            st.profile_enable(rep)
            for _ in range(k_steps):
                eager_step(inst)
            torch.cuda.synchronize()
            got = st.profile_read()
            st.profile_enable(False)
            # back to one launch per planned launch
            return {name: ((ms / rep, launches / rep) if name.startswith("gemm_") and not name.startswith("gemm_generic") else (ms, launches))
                    for name, (ms, launches) in got.items()}
        single, repeated = kernel_pass(1), kernel_pass(REP)
        prof = dict(single)
        total_ms = sum(v[0] for v in prof.values())
        for name, (ms, launches) in sorted(prof.items(), key=lambda kv: -kv[1][0]):
            kernels[name] = {"ms_per_step": ms / k_steps, "launches_per_step": launches / k_steps,
                             "avg_launch_us": 1e3 * ms / max(launches, 1), "share": ms / total_ms}
            if name in repeated and name.startswith("gemm_"):
                kernels[name]["avg_launch_us_back_to_back"] = 1e3 * repeated[name][0] / max(repeated[name][1], 1)
        tr = gemm_traffic(wl)
        nm = wl.n_micro
        # algorithmic bytes / flops per STEP of each GEMM role; a role's figure goes to the kernel family
        # that spends the most time on it (the planner may route a few small layers of a role elsewhere)
        role_alg = {
            "fwd": (tr["fwd"][0] * nm, tr["fwd"][1] * nm),
            "dx": (tr["dx"][0] * nm, tr["dx"][1] * nm),
            "dw": (tr["dw_first"][0] + tr["dw"][0] * (nm - 1), tr["dw"][1] * nm),
        }
        if grouped:
            # one pass over the fp32 accumulators per run of backward tasks (the first one of a step only
            # writes them); the operands of every micro-batch are read once
            tasks = sched.tasks(nm) if kfkb else [v for j in range(nm) for v in (j + 1, -(j + 1))]
            runs = sum(1 for t in range(len(tasks)) if tasks[t] < 0 and (t + 1 == len(tasks) or tasks[t + 1] > 0))
            act = tr["dw_first"][0] - 4 * tr["params"]
            role_alg["dw"] = (4 * tr["params"] * (2 * runs - 1) + act * nm, tr["dw"][1] * nm)
        role_alg["dx+dw"] = (role_alg["dx"][0] + role_alg["dw"][0], role_alg["dx"][1] + role_alg["dw"][1])
        role_tags = {
            "fwd": ["gemm_big_fwd", "gemm_mfma_fwd", "gemm_skinny_fwd", "gemm_generic_fwd"],
            "dx": ["gemm_big_dx", "gemm_mfma_dx", "gemm_skinny_dx"],
            "dw": ["gemm_big_dw", "gemm_mfma_dw", "gemm_dw_ksplit"],
            "dx+dw": ["gemm_bwd_merged_dx_dw", "gemm_generic_bwd"],
        }
        alg = {}
        for role, tags in role_tags.items():
            present = [t for t in tags if t in kernels]
            if role == "dx+dw" and present and any(t in kernels for t in role_tags["dx"] + role_tags["dw"]):
                continue   # split roles also ran: the merged launch holds only part of the traffic
            if present:
                alg[max(present, key=lambda t: kernels[t]["ms_per_step"])] = role_alg[role]
        logical = {}
        for name, (by, fl, lg) in other_traffic(wl).items():
            alg[name] = (by * nm, fl * nm)
            logical[name] = lg * nm
        dom = next(iter(kernels))
        if dom in alg:
            by, fl = alg[dom]
            k = kernels[dom]
            sec = k["ms_per_step"] * 1e-3
            gbs, tfl = by / sec / 1e9, fl / sec / 1e12
            # binding bound of this kernel: compare time at each peak
            hbm_bound = by / (HBM_PEAK_GBS * 1e9) >= fl / (MFMA_BF16_PEAK_TFLOPS * 1e12)
            if hbm_bound:
                roofline = {"bound": "hbm", "achieved": gbs, "peak": HBM_PEAK_GBS, "unit": "GB/s",
                            "frac": gbs / HBM_PEAK_GBS, "traffic": measured_traffic(args.config, dom)}
            else:
                roofline = {"bound": "mfma", "achieved": tfl, "peak": MFMA_BF16_PEAK_TFLOPS, "unit": "TFLOP/s",
                            "frac": tfl / MFMA_BF16_PEAK_TFLOPS, "traffic": measured_traffic(args.config, dom)}
            roofline.update({"kernel": dom, "avg_launch_us": k["avg_launch_us"],
                             "launches_per_step": k["launches_per_step"],
                             "algorithmic_bytes_per_launch": by / k["launches_per_step"],
                             "algorithmic_flops_per_launch": fl / k["launches_per_step"],
                             "other_fraction_tflops": tfl, "other_fraction_gbs": gbs})
            if dom in logical:
                roofline["logical_gbs"] = logical[dom] / sec / 1e9
        else:
            roofline = {"bound": "hbm", "achieved": None, "peak": HBM_PEAK_GBS, "unit": "GB/s", "frac": None,
                        "traffic": None, "kernel": dom}
        # the timed step as a whole: algorithmic bytes of every counted kernel over the step time.  The launch
        # durations above are each kernel ALONE on the GPU (one stream); in the timed step launches of
        # several streams overlap, so the step moves more bytes per second than its kernels do one by one
        step_bytes = sum(v[0] for v in alg.values())
        step_flops = sum(v[1] for v in alg.values())
        # every kernel with a known algorithmic count: achieved rates beside the durations
        for name, k in kernels.items():
            if name in alg and k["ms_per_step"] > 0:
                k["algorithmic_gbs"] = alg[name][0] / (k["ms_per_step"] * 1e-3) / 1e9
                k["algorithmic_tflops"] = alg[name][1] / (k["ms_per_step"] * 1e-3) / 1e12

    for _ in range(args.warmup):
        step()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(args.steps):
        step()
    torch.cuda.synchronize()
    dt = time.perf_counter() - t0
    st.sync_status()
    samples_per_step = wl.micro_batch * wl.n_micro
    value = args.steps * samples_per_step / dt
    # per-step times: a HIP event on the caller's stream in front of every step (every schedule starts and ends
    # a step on that stream), at least 50 steps; the difference of neighbouring events is one step
    n_ev = 1 if args.no_step_times else max(args.steps, 50)
    evs = [torch.cuda.Event(enable_timing=True) for _ in range(n_ev + 1)]
    for i in range(n_ev):
        evs[i].record()
        step()
    evs[n_ev].record()
    torch.cuda.synchronize()
    per_step = sorted(evs[i].elapsed_time(evs[i + 1]) for i in range(n_ev))
    med = per_step[n_ev // 2]
    step_ms = {"median": med, "min": per_step[0], "max": per_step[-1], "p10": per_step[n_ev // 10], "p90": per_step[(9 * n_ev) // 10],
               "spread_p10_p90": (per_step[(9 * n_ev) // 10] - per_step[n_ev // 10]) / med, "steps": n_ev,
               "samples_per_s_at_median": samples_per_step / (med * 1e-3)}
    serial_value = None
    if (overlap or kfkb or graphed is not None) and not args.no_serial_reference:   # the same steps enqueued from the host in serial order, for reference
        for _ in range(2):
            eager_step(serial)
        torch.cuda.synchronize()
        t1 = time.perf_counter()
        ref_steps = min(args.steps, 200)
        for _ in range(ref_steps):
            eager_step(serial)
        torch.cuda.synchronize()
        serial_value = ref_steps * samples_per_step / (time.perf_counter() - t1)

    if roofline is not None and not args.no_kernel_pass:
        roofline["step_algorithmic_gbs"] = step_bytes / (dt / args.steps) / 1e9
        roofline["step_frac_of_hbm_peak"] = roofline["step_algorithmic_gbs"] / HBM_PEAK_GBS
        roofline["step_algorithmic_tflops"] = step_flops / (dt / args.steps) / 1e12
        roofline["step_frac_of_mfma_peak"] = roofline["step_algorithmic_tflops"] / MFMA_BF16_PEAK_TFLOPS

    # ---- CPU oracle on this host, bounded sample --------------------------------------------
    cpu = None
    if not args.no_cpu_baseline:
        from oracle import gpp_oracle as O
        try:
            from threadpoolctl import threadpool_info
            cores = max([p.get("num_threads", 1) for p in threadpool_info()] + [1])
        except Exception:
            cores = os.cpu_count()
        # a bounded sample of the same workload: about 10-30 s of CPU work.  A workload whose micro-batch costs
        # more than that (the transformer stage: 1.3 TFLOP in fp64) is timed on ONE sample of it, once, cold
        heavy = 3 * gemm_traffic(wl)["fwd"][1] > 2e11
        cw = W.CONFIGS[args.config](micro_batch=1) if heavy else wl
        ost = O.OracleStage(cw.ops, cw.micro_batch, cw.params, model_storage=True)
        go = None
        if not heavy:
            s0 = ost.forward(cw.batches[0])        # warm-up
            go = {i: np.zeros((s0.values[i].shape)) for i in ost.output_ids}
            ost.backward(s0, go)
        n_done, t0 = 0, time.perf_counter()
        while True:
            mb = cw.batches[n_done % len(cw.batches)]
            s = ost.forward(mb)
            if go is None:
                go = {i: np.zeros((s.values[i].shape)) for i in ost.output_ids}
            ost.backward(s, go)
            n_done += 1
            el = time.perf_counter() - t0
            if el > 12.0 or n_done >= 64:
                break
        cpu = {"value": n_done * cw.micro_batch / el, "unit": "samples/s", "cores": cores, "kind": "oracle",
               "sample": f"{n_done} micro-batch(es) of {cw.micro_batch} sample(s) of the {args.config} workload, forward+backward, "
                         f"fp64 numpy, {el:.1f} s" + (" (one cold pass, no warm-up)" if heavy else "")}

    out = {
        "metric": "stage fwd+bwd samples/s", "value": value, "unit": "samples/s", "n_gpus": 1,
        "steps": args.steps, "warmup": args.warmup, "ms_per_step": 1e3 * dt / args.steps,
        "higher_is_better": True, "scaling": "weak", "vs_baseline": None,
        "dtype": "f32" if args.config == "tiny_mlp" else "bf16", "data": "synthetic",
        "config": {"workload": f"{args.config}: micro-batch {wl.micro_batch} x {wl.n_micro} micro-batches per step",
                   "micro_batch": wl.micro_batch, "micro_batches_per_step": wl.n_micro,
                   "schedule": (f"kFkB from the scheduler: i = {n_slots * wl.micro_batch} samples ({n_slots} micro-batches in flight), k = {args.k}, "
                                + ("one stream" if args.one_stream else
                                   (f"micro-batch j on stream j mod {lanes[0]} (forward and backward pass)"
                                    + (f", one launch per step for the {n_slots // lanes[0]} micro-batches of a stream" if group_flag else "")
                                    if shared_lanes else
                                    f"forward passes on {lanes[0]} stream(s), backward passes on {lanes[1]} other stream(s)"))) if kfkb else
                               (f"overlap: forward calls on one stream, backward calls on another, {n_slots} in-flight slots" if overlap else "serial"),
                   "stash_bytes_per_slot": B.gpp_stage_memory(st.handle)[0],
                   "peak_stash_bytes": n_slots * B.gpp_stage_memory(st.handle)[0],
                   "workspace_bytes": B.gpp_stage_memory(st.handle)[2],
                   "launch": "HIP graph replay of the whole step" if graphed is not None else "eager",
                   "launches_per_microbatch": st.num_launches(False) + st.num_launches(True),
                   "serial_eager_samples_per_s": serial_value},
        "roofline": roofline, "cpu_baseline": cpu, "step_ms": step_ms, "kernels": kernels,
    }
    st.close()
    return out


def summary(out):
    """The part of a workload's line that goes under `configs`."""
    r = out["roofline"] or {}
    keep = ("kernel", "bound", "achieved", "peak", "unit", "frac", "traffic", "avg_launch_us", "launches_per_step",
            "step_algorithmic_gbs", "step_frac_of_hbm_peak", "step_algorithmic_tflops", "step_frac_of_mfma_peak", "logical_gbs")
    top = sorted(out["kernels"].items(), key=lambda kv: -kv[1]["ms_per_step"])[:4]
    return {"workload": out["config"]["workload"], "samples_per_s": out["value"], "ms_per_step": out["ms_per_step"],
            "steps": out["steps"], "warmup": out["warmup"], "step_ms": out["step_ms"], "dtype": out["dtype"],
            "schedule": out["config"]["schedule"], "launch": out["config"]["launch"],
            "peak_stash_bytes": out["config"]["peak_stash_bytes"],
            "dominant_kernel": {k: r.get(k) for k in keep if k in r},
            "kernels": {name: {"avg_launch_us": k["avg_launch_us"], "launches_per_step": k["launches_per_step"], "share": k["share"],
                               **({"algorithmic_gbs": k["algorithmic_gbs"], "algorithmic_tflops": k["algorithmic_tflops"]}
                                  if "algorithmic_gbs" in k else {})} for name, k in top}}


def main():
    import copy
    # the two measurements around the stage path: --mode pipeline (several stages of a stage graph on one GPU) and
    # --mode partition (the partitioner on this build's operator graphs, host only) take their own flags
    if "--mode" in sys.argv[1:]:
        i = sys.argv.index("--mode")
        mode, rest = (sys.argv[i + 1] if i + 1 < len(sys.argv) else ""), sys.argv[1:i] + sys.argv[i + 2:]
        if mode == "pipeline":
            from paper_2406_17145_amd.bench_pipeline import main as run
            return run(rest)
        if mode == "partition":
            from paper_2406_17145_amd.bench_partition import main as run
            return run(rest)
        if mode != "stage":
            sys.exit("bench.py: --mode is one of stage (default), pipeline, partition")
        sys.argv = [sys.argv[0]] + rest
    args = build_parser().parse_args()
    if args.gpus != 1:
        print("bench.py: this build measures one stage on ONE GPU (no collectives, no sharding); "
              "--gpus must be 1", file=sys.stderr)
        sys.exit(2)
    if args.config != "all":
        print(json.dumps(run_one(args)))
        return

    def variant(config, **kw):
        a = copy.copy(args)
        a.config = config
        a.no_cpu_baseline = True
        # the driver may ask for few steps; the short-step workloads get enough of them for a stable median
        a.steps, a.warmup = max(args.steps, 200), max(args.warmup, 20)
        for k, v in kw.items():
            setattr(a, k, v)
        return a

    head = copy.copy(args)
    head.config = "mmt"
    out = run_one(head)
    configs = {"mmt": summary(out)}
    configs["candle_uno"] = summary(run_one(variant("candle_uno")))
    # the same stage with two micro-batches in flight (1F1B-like), beside the eight of the default: eager on two
    # streams (a captured step would need a slot per micro-batch), and captured on one stream
    two = run_one(variant("candle_uno", in_flight=2, k=1, no_kernel_pass=True, no_serial_reference=True))
    two1 = run_one(variant("candle_uno", in_flight=2, k=1, one_stream=True, no_kernel_pass=True, no_serial_reference=True))
    configs["candle_uno"]["two_in_flight"] = [
        {"samples_per_s": o["value"], "step_ms": o["step_ms"], "schedule": o["config"]["schedule"], "launch": o["config"]["launch"],
         "peak_stash_bytes": o["config"]["peak_stash_bytes"]} for o in (two, two1)]
    configs["dlrm"] = summary(run_one(variant("dlrm")))
    configs["hetero"] = summary(run_one(variant("hetero", micro_batch=128)))
    sweep = []
    for b in (1, 2, 4, 8, 16, 32, 64, 128):
        o = run_one(variant("hetero", micro_batch=b, no_kernel_pass=True, no_serial_reference=True))
        sweep.append({"micro_batch": b, "samples_per_s": o["value"], "ms_per_step": o["ms_per_step"], "median_ms": o["step_ms"]["median"],
                      "min_ms": o["step_ms"]["min"], "max_ms": o["step_ms"]["max"]})
    configs["hetero"]["micro_batch_sweep"] = sweep
    configs["tiny_mlp"] = summary(run_one(variant("tiny_mlp")))
    out["configs"] = configs
    print(json.dumps(out))


if __name__ == "__main__":
    main()
