"""The parity bars of the GPU tests and where each comes from.  No GPU code here.

Stated bars (per tensor, l2-relative ||gpu - ref|| / ||ref||): 1e-4 on the fp32 path,
2e-2 with bf16 storage and fp32 accumulation.  They hold for every output, every loss,
every gamma / beta / table gradient of every workload, and for every tensor of a graph
without ReLU.  The max-norm guard max|gpu - ref| / max|ref| is 1e-4 (fp32) and
5 x 2e-2 (bf16: a stored value is one rounding of 2^-9 relative, the guard looks for
errors of the size of the values).

ONE exception: bf16 graphs with ReLU layers.  tests/relu_noise.py explains the effect
(a ReLU mask decided from a rounded value: a handful of opposite decisions per
micro-batch, each worth a sample's whole gradient row) and measures it on the CPU from
the oracle alone: the spread of the gradients under re-ordered float32 sums.  The bar
of an INPUT gradient of such a graph is

    max(stated bar, BAND x measured spread)

for the l2 error and the max-norm guard, and the share of sample rows allowed over the
stated bar is BAND x measured share + one row.  WEIGHT and BIAS gradients of such a
graph get max(stated bar, BAND x their measured spread) too: summed over a mini-batch
of 512 samples the opposite decisions average out (the BASELINE workloads stay at the
stated 2e-2), over the 64 rows of one micro-batch of a 4096-wide stack they do not.
EMBEDDING-TABLE gradients of such a graph are the scattered gradients of the pooled
vectors, i.e. input gradients of the stack behind them: same rule, their own spread.
The measured spreads of the full-size workloads are stored in
tests/golden/relu_spread.txt (written by tests/golden/make_relu_spread.py from the
oracle); those of the two BASELINE workloads are re-measured and bracketed two-sidedly
(within [1/BAND, BAND]) by tests/test_oracle_pins.py::test_relu_mask_noise_floor; every
other workload is measured when its test runs (they are small).
"""
import os

BAND = 1.5
STATED_L2 = {"f32": 1e-4, "bf16": 2e-2}
STATED_MAX = {"f32": 1e-4, "bf16": 1e-1}
ROW_CHECK_MIN_WIDTH = 32    # narrower rows are a handful of numbers: no meaningful row norm


def _load():
    out = {}
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "relu_spread.txt")
    for line in open(path):
        if line.startswith("#") or "|" not in line:
            continue
        part = [v.strip() for v in line.split("|")]
        name, b, n, ops = part[0].split()
        vals = {v.split()[0]: float(v.split()[1]) for v in part[1:6]}
        out[(name, int(b), int(n), int(ops))] = vals
    return out


RELU_SPREAD_PINNED = _load()


def workload_key(wl):
    return (wl.name, wl.micro_batch, wl.n_micro, len(wl.ops))


def relu_gin_bars(spread, rows):
    """(l2 bar, max-norm bar, allowed share of rows over the stated bar) of an input gradient from a measured spread."""
    return (max(STATED_L2["bf16"], BAND * spread["l2"]),
            max(STATED_MAX["bf16"], BAND * spread["max"]),
            BAND * spread["rows_over"] + 1.0 / max(rows, 1))


def relu_dw_bar(spread, table=False):
    """l2 bar of a weight or bias gradient (table: of an embedding-table gradient) of a bf16 graph with ReLU layers."""
    return max(STATED_L2["bf16"], BAND * spread["dt" if table else "dw"])
