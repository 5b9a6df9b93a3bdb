"""Writes config1_oracle.json from the oracle alone (never from the HIP path)."""
import json
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import gpp_oracle as O                      # noqa: E402
from paper_2406_17145_amd import workloads as W         # noqa: E402


def summary():
    wl = W.tiny_mlp()
    stage, res = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches)
    out = {"losses": [r[0].loss for r in res], "grad_l2": {}, "grad_first": {}}
    for i, g in stage.grads.items():
        for k, v in g.items():
            out["grad_l2"][f"{i}.{k}"] = float(np.sqrt((v * v).sum()))
            out["grad_first"][f"{i}.{k}"] = float(v.reshape(-1)[0])
    return out


if __name__ == "__main__":
    with open(os.path.join(os.path.dirname(__file__), "config1_oracle.json"), "w") as f:
        json.dump(summary(), f, indent=1, sort_keys=True)
