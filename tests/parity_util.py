"""Shared helpers of the GPU parity tests: run a workload through the HIP
library and through the oracle and compare every tensor.

Error measure, per tensor: "relative error" is the l2-relative error
||gpu-ref||_2 / ||ref||_2 and must stay under the numeric mode's tolerance
(1e-4 fp32 path, 2e-2 bf16 storage with fp32 accumulation).  Elementwise
relative error is ill-defined at the zeros that ReLU and sparse table gradients
produce, hence the norm-wise form.  A second, max-norm guard
max|gpu-ref| / max|ref| catches localised corruption (a wrong tile, a missed
tail): it uses the same tolerance in fp32 mode and 5x the tolerance in bf16
mode, because there a single ReLU mask decision that falls on the other side of
zero (fp32 vs fp64 accumulation, amplified at a bf16 rounding boundary of a
stored activation) legitimately moves one sample's whole gradient row.

Input gradients of bf16 graphs with ReLU layers are the one place where that
effect is not small: the masks of every layer between an input and the loss
multiply into its gradient, and a handful of opposite decisions per micro-batch
(each worth about 0.5% of a [64, 1000]-wide layer) already add up to 1-3% in
the l2 norm.  Two CPU runs of the oracle that differ only in the accumulation
precision of the matrix products (float32 vs float64) show the same spread
(tests/test_oracle_pins.py::test_relu_mask_noise_floor), so for those tensors
the bar is 5e-2; every other tensor of every graph stays at the stated 2e-2.
Their max-norm guard is 5x their own bar (0.25): one opposite mask decision
moves one sample's whole input-gradient row, which in a narrow input (a few
tens of columns, a few hundred rows) is one element at 10-15% of the tensor's
largest; the guard still catches what it is for, errors of the order of the
values themselves over a tile or a tail.
"""
import numpy as np

from oracle import gpp_oracle as O
from paper_2406_17145_amd import binding as B


def rel_errors(got, ref):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (got.shape, ref.shape)
    n = np.linalg.norm(ref)
    m = np.abs(ref).max() if ref.size else 0.0
    if n == 0.0:
        return (np.linalg.norm(got), np.abs(got).max() if got.size else 0.0)
    return np.linalg.norm(got - ref) / n, np.abs(got - ref).max() / m


def t2n(t):
    return t.float().cpu().numpy()


def run_gpu(wl, slots=1, flags=0, gouts=None, schedule=None, keep=False):
    """schedule: list of ("f", j) / ("b", j) over micro-batch ids; default fw_j, bw_j in turn.
    Micro-batch j uses slot j % slots."""
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=slots, flags=flags)
    st.grad_reset()
    n = len(wl.batches)
    schedule = schedule or [x for j in range(n) for x in (("f", j), ("b", j))]
    res = [dict() for _ in range(n)]
    import torch
    for what, j in schedule:
        if what == "f":
            loss = torch.zeros(1, dtype=torch.float32, device=st.dev)
            outs, _ = st.forward(j % slots, wl.batches[j], loss=loss)
            res[j]["loss"], res[j]["outs"] = loss, outs
        else:
            res[j]["gin"] = st.backward(j % slots, None if gouts is None else gouts[j])
    st.sync_status()
    out = []
    for r in res:
        out.append(dict(loss=float(r["loss"].cpu()[0]),
                        outs={i: t2n(t) for i, t in zip(st.output_ids, r["outs"])},
                        gin={i: t2n(t) for i, t in zip(st.input_ids, r["gin"]) if t is not None}))
    grads = st.grads_numpy()
    if keep:
        return out, grads, st
    st.close()
    return out, grads


def run_oracle(wl, gouts=None):
    # bf16-storage workloads: the oracle rounds stored operator outputs to bf16 as well, so that
    # ReLU masks are decided from the same stored values on both sides
    stage, res = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches, gouts, model_storage=True)
    return stage, res


def compare(wl, gpu_res, gpu_grads, ora_stage, ora_res, tol=None, label=""):
    tol = wl.tol if tol is None else tol
    tol_max = tol if tol <= 1e-3 else 5 * tol
    has_relu = any(op.get("act") == "relu" for op in wl.ops)
    tol_gin = 5e-2 if (tol > 1e-3 and has_relu) else tol
    worst = {}

    def chk(name, got, ref, t2=None):
        t2 = tol if t2 is None else t2
        e2, em = rel_errors(got, ref)
        worst[name] = (e2, em)
        tm = max(tol_max, 2 * t2) if t2 == tol else 5 * t2
        assert e2 <= t2 and em <= tm, f"{label} {name}: l2-rel {e2:.3e} (tol {t2}) max-rel {em:.3e} (tol {tm})"

    for j, (g, (st, gin)) in enumerate(zip(gpu_res, ora_res)):
        if ora_stage.ops and any(op["kind"].startswith("loss") for op in ora_stage.ops):
            assert abs(g["loss"] - st.loss) <= tol * max(abs(st.loss), 1e-30), (label, "loss", j, g["loss"], st.loss)
        for i in ora_stage.output_ids:
            chk(f"mb{j}.out{i}", g["outs"][i], st.values[i])
        assert set(g["gin"]) == set(gin), (set(g["gin"]), set(gin))
        for i, ref in gin.items():
            chk(f"mb{j}.gin{i}", g["gin"][i], ref, tol_gin)
    for i, gr in ora_stage.grads.items():
        for k, ref in gr.items():
            chk(f"op{i}.d{k}", gpu_grads[i][k], ref)
    return worst
