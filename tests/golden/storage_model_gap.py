"""Writes tests/golden/storage_model_gap.txt: per workload, how far the oracle's bf16 storage model
(operator outputs rounded to bf16, fp64 arithmetic inside an operator) is from the plain fp64 oracle, per tensor
class, as worst l2-relative difference.  This is the size of the numeric MODE (bf16 storage), not of any kernel:
the GPU parity tests compare against the storage-model run.  Calls only oracle/ and the input generators.

  python tests/golden/storage_model_gap.py [workload ...]
"""
import os
import sys

import numpy as np

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from oracle import gpp_oracle as O  # noqa: E402
from paper_2406_17145_amd import workloads as W  # noqa: E402


def rel(a, b):
    n = np.linalg.norm(a)
    return float(np.linalg.norm(a - b) / n) if n else float(np.linalg.norm(b))


def gap(wl):
    plain, res_p = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches)
    model, res_m = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches, model_storage=True)
    out = {"loss": max(abs(a[0].loss - b[0].loss) / abs(a[0].loss) for a, b in zip(res_p, res_m)),
           "input gradient": max([rel(a[1][i], b[1][i]) for a, b in zip(res_p, res_m) for i in a[1]] or [0.0])}
    for i in plain.grads:
        for k in plain.grads[i]:
            out["d" + k] = max(out.get("d" + k, 0.0), rel(plain.grads[i][k], model.grads[i][k]))
    return out


if __name__ == "__main__":
    names = sys.argv[1:] or ["candle_uno", "mmt", "dlrm", "hetero"]
    lines = ["# plain fp64 oracle against its own bf16 storage model (worst l2-relative difference per tensor class)",
             "# written by tests/golden/storage_model_gap.py"]
    for name in names:
        wl = W.CONFIGS[name]()
        g = gap(wl)
        lines.append(f"{name} b={wl.micro_batch} x{wl.n_micro} | " + " | ".join(f"{k} {v:.2e}" for k, v in sorted(g.items())))
        print(lines[-1], flush=True)
    with open(os.path.join(os.path.dirname(os.path.abspath(__file__)), "storage_model_gap.txt"), "w") as f:
        f.write("\n".join(lines) + "\n")
