"""Stage graph on one GPU: the CANDLE-Uno-shaped model cut into its four towers and a merge stage, run by the
library's pipeline executor as a GRAPH pipeline (towers side by side: stage graph of depth 2) and as a SEQUENTIAL
pipeline (the same stages chained: depth 5), the contrast of paper section 2 in miniature.

Prints one JSON line per variant: whole-mini-batch samples/s, and, per stage, the in-flight micro-batches the
scheduler assigns (gpp_assign_schedules) and the stash bytes they pin.  All stages share one GPU (their streams
stand in for devices), so the times show what the dependency structure allows on one chip, not a multi-GPU
speed-up; the in-flight counts and stash bytes are what the paper's memory argument is about.

  python bench.py --mode pipeline [--steps K] [--warmup W] [--micro-batch B] [--micro-batches N] [--k K] [--grouped-dw]
"""
import argparse
import json
import sys
import time


def main(argv=None):
    ap = argparse.ArgumentParser(prog="bench.py --mode pipeline")
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--warmup", type=int, default=10)
    ap.add_argument("--micro-batches", type=int, default=8)
    ap.add_argument("--micro-batch", type=int, default=64,
                    help="rows per micro-batch; at 64 every launch is a few microseconds and the host's launch rate "
                         "(about 3 us per launch or event) paces the eager pipeline, from about 1024 on the GPU does")
    ap.add_argument("--k", type=int, default=1, help="group size of every stage's kFkB list")
    ap.add_argument("--grouped-dw", action="store_true", help="stages with grouped weight gradients")
    args = ap.parse_args(argv)

    import torch
    from paper_2406_17145_amd import binding as B
    from paper_2406_17145_amd import workloads as W
    from paper_2406_17145_amd.schedule import StagePipeline

    wl = W.candle_uno(micro_batch=args.micro_batch, n_micro=args.micro_batches)
    n_towers = 1 + max(op["branch"] for op in wl.ops)
    stage_of = {i: (op["branch"] if op["branch"] >= 0 else n_towers) for i, op in enumerate(wl.ops) if op["kind"] != "input"}
    parts, edges = W.partition(wl, stage_of, n_towers + 1)
    chain = [(s, -1, s + 1, -1) for s in range(n_towers - 1)]
    b, n = wl.micro_batch, wl.n_micro
    for name, ed in (("graph pipeline (towers side by side)", edges), ("sequential pipeline (towers chained)", edges + chain)):
        caps, k = StagePipeline.in_flight_microbatches(len(parts), ed, b, [[args.k]] * len(parts))
        stages = [B.Stage(p.ops, b, p.params, slots=c, flags=B.FLAG_GROUPED_DW if args.grouped_dw else 0)
                  for p, c in zip(parts, caps)]
        pipe = StagePipeline(stages, ed, [c * b for c in caps], k)
        fed_in = {(e[2], e[3]) for e in ed if e[1] >= 0}
        fed_out = {(e[0], e[1]) for e in ed if e[1] >= 0}
        io = []
        for s, (st, p) in enumerate(zip(stages, parts)):
            gin = [None if (s, q) in fed_in else t for q, t in enumerate(st.alloc_grad_inputs())]
            rows = []
            for j in range(n):
                dev = {i: st.to_device(i, a) for i, a in p.batches[j].items()}     # resident in HBM
                inputs = [None if (s, q) in fed_in else dev[i] for q, i in enumerate(st.input_ids)]
                outs = [None if (s, q) in fed_out else t for q, t in enumerate(st.alloc_outputs())]
                rows.append((inputs, outs, torch.zeros(1, dtype=torch.float32, device=st.dev), None, gin))
            io.append(rows)
        for _ in range(args.warmup):
            pipe.minibatch(io)
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(args.steps):
            pipe.minibatch(io)
        torch.cuda.synchronize()
        dt = time.perf_counter() - t0
        for st in stages:
            st.sync_status()
        stash = pipe.stash_bytes()
        print(json.dumps({
            "metric": "stage-graph fwd+bwd samples/s", "variant": name, "value": args.steps * b * n / dt, "unit": "samples/s",
            "ms_per_step": 1e3 * dt / args.steps, "n_gpus": 1, "steps": args.steps, "warmup": args.warmup,
            "config": {"workload": f"candle_uno cut into {n_towers} tower stages + 1 merge stage: micro-batch {b} x {n} per step",
                       "k": k, "launch": "eager, a pair of streams per stage", "grouped_weight_gradients": args.grouped_dw},
            "in_flight_microbatches": caps, "stash_bytes": stash, "stash_bytes_total": sum(stash),
            "edge_buffer_bytes": pipe.ws_bytes}))
        sys.stdout.flush()
        pipe.close()
        for st in stages:
            st.close()
