"""Writes tests/golden/relu_spread.txt: for every full-size bf16 workload with ReLU layers, how far its input and
weight gradients move when only the float32 order of the Linear products changes (tests/relu_noise.py::measure:
the fp64 oracle against itself; nothing of the HIP path is involved).  The GPU parity bars of those tensors are
derived from these figures (tests/parity_bars.py).  The two BASELINE workloads are re-measured and checked
two-sidedly by the CPU suite (tests/test_oracle_pins.py::test_relu_mask_noise_floor); the paper-shaped ones take
minutes each (hundreds of millions of parameters in fp64) and are only written here.

  python tests/golden/make_relu_spread.py [workload ...]      (calls only oracle/ and the input generators)
"""
import os
import sys

ROOT = os.path.dirname(os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
sys.path.insert(0, ROOT)
from paper_2406_17145_amd import workloads as W  # noqa: E402
from tests.relu_noise import VARIANTS, measure  # noqa: E402

OUT = os.path.join(os.path.dirname(os.path.abspath(__file__)), "relu_spread.txt")
# the large workloads: two of the four orders (one BLAS order, one blocked order with bf16-stored gradients)
ORDERS = {"candle_uno": VARIANTS, "dlrm": ("blas", "blk64g"), "paper_candle": ("blas", "blk64g"), "paper_dlrm": ("blas", "blk64g")}

if __name__ == "__main__":
    names = sys.argv[1:] or list(ORDERS)
    old = {}
    if os.path.exists(OUT):
        for line in open(OUT):
            if not line.startswith("#") and "|" in line:
                old[line.split("|")[0].strip()] = line.rstrip("\n")
    for name in names:
        wl = W.CONFIGS[name]()
        m = measure(wl, ORDERS[name])
        key = f"{wl.name} {wl.micro_batch} {wl.n_micro} {len(wl.ops)}"
        old[key] = (f"{key} | l2 {m['l2']:.4e} | max {m['max']:.4e} | rows_over {m['rows_over']:.4e} | dw {m['dw']:.4e} | dt {m['dt']:.4e} | "
                    f"flips {m['flips']} of {m['decisions']} decisions, {m['near_zero']} within one bf16 step of zero | orders {','.join(ORDERS[name])}")
        print(old[key], flush=True)
        del wl
    with open(OUT, "w") as f:
        f.write("# workload micro-batch micro-batches operators | worst l2-relative / max-norm spread of an input gradient | share of\n"
                "# sample rows over 2e-2 | worst l2-relative spread of a weight or bias gradient | of a table gradient | ReLU decisions | float32 orders\n"
                "# written by tests/golden/make_relu_spread.py\n")
        for k in sorted(old):
            f.write(old[k] + "\n")
