"""Partitioner on the operator graphs of this build's workloads (host only, no GPU needed).

For every workload: per-operator costs from a two-term model (time per sample = max(flops / matrix-core rate,
bytes / memory rate) at the workload's micro-batch size, with the rates this build MEASURED on one MI355X for its
own kernels; parameter + gradient bytes; stashed bytes per sample), then gpp_partition for 1 .. 32 devices.
Prints one JSON line per (workload, devices): stages, devices per stage, in-flight micro-batches, bottleneck time
per sample, speed-up over one device, search time and dynamic-programme states.

  python bench.py --mode partition [--config NAME] [--memory-gb G]
"""
import argparse
import json
import time

MFMA_RATE = 700e12        # flop/s this build's large-tile GEMMs reach on the transformer workload
MEM_RATE = 3.0e12         # byte/s its weight-streaming and element-wise kernels reach
LINK_SECONDS_PER_BYTE = 1.0 / 150e9     # one xGMI link, for the data-parallel gradient all-reduce


def op_costs(wl):
    b = wl.micro_batch
    es = {"f32": 4, "bf16": 2, "i32": 4}
    rows, t, w, a = {}, [], [], []
    for i, op in enumerate(wl.ops):
        k = op["kind"]
        if k == "input":
            rows[i] = op.get("seq_len", 1) + op.get("rows_extra", 0) / b
        elif k in ("meanpool", "embedding_bag_sum"):
            rows[i] = 1
        elif op["inputs"]:
            rows[i] = rows[op["inputs"][0]]
        r = rows.get(i, 1)                                   # rows per sample
        feat = op.get("out_features", 1) or 1
        e = es[op.get("out_dtype", op.get("dtype", "f32"))]
        flops = bytes_ = params = 0.0
        if k == "linear":
            params = op["in_features"] * op["out_features"]
            flops = 6.0 * r * params                         # forward, backward-data, backward-weight
            bytes_ = (2 * 2 + 8) * params / b + 3 * r * (op["in_features"] + feat) * e
        elif k == "attention":
            s, d = op.get("seq_len", r), feat
            flops = 4.0 * 3.5 * s * s * d                    # forward + backward with recomputation
            bytes_ = 8 * r * d * e
        elif k == "embedding_bag_sum":
            bytes_ = 3 * op["bag_size"] * feat * 4
            params = op["num_rows"] * feat
        elif k != "input":
            bytes_ = 4 * r * feat * e
        t.append(max(flops / MFMA_RATE, bytes_ / MEM_RATE))
        w.append(params * (6 if k == "linear" else 8 if k == "embedding_bag_sum" else 0))
        a.append(0.0 if k.startswith("loss") else r * feat * e)
    edges = [(p, i) for i, op in enumerate(wl.ops) for p in op["inputs"]]
    return edges, t, w, a


def main(argv=None):
    ap = argparse.ArgumentParser(prog="bench.py --mode partition")
    ap.add_argument("--config", default="all")
    ap.add_argument("--memory-gb", type=float, default=288.0)
    args = ap.parse_args(argv)
    from paper_2406_17145_amd import binding as B
    from paper_2406_17145_amd import workloads as W
    names = ["candle_uno", "mmt", "dlrm", "hetero"] if args.config == "all" else [args.config]
    for name in names:
        wl = W.CONFIGS[name]()
        edges, t, w, a = op_costs(wl)
        base = None
        for d in (1, 2, 4, 8, 16, 32):
            t0 = time.perf_counter()
            got = B.gpp_partition(len(wl.ops), edges, t, w, a, d, wl.micro_batch, args.memory_gb * 1e9,
                                  LINK_SECONDS_PER_BYTE, 64 * wl.micro_batch, 1e-4)
            ms = 1e3 * (time.perf_counter() - t0)
            if got is None:
                print(json.dumps({"workload": name, "devices": d, "stages": 0, "search_ms": ms}))
                continue
            base = base or got["bottleneck"]
            print(json.dumps({"workload": name, "operators": len(wl.ops), "devices": d, "stages": len(got["devices"]),
                              "devices_per_stage": got["devices"],
                              "in_flight_microbatches": [i // wl.micro_batch for i in got["in_flight"]],
                              "bottleneck_us_per_sample": 1e6 * got["bottleneck"],
                              "speedup_over_one_device": base / got["bottleneck"], "search_ms": round(ms, 2),
                              "dp_states": got["dp_states"]}))
