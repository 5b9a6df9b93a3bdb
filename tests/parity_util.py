"""Shared helpers of the GPU parity tests: run a workload through the HIP
library and through the oracle and compare every tensor.

Error measure, per tensor: "relative error" is the l2-relative error
||gpu-ref||_2 / ||ref||_2 and must stay under the numeric mode's tolerance
(1e-4 fp32 path, 2e-2 bf16 storage with fp32 accumulation).  Elementwise
relative error is ill-defined at the zeros that ReLU and sparse table gradients
produce, hence the norm-wise form.  A second, max-norm guard
max|gpu-ref| / max|ref| catches localised corruption (a wrong tile, a missed
tail).  The bars and the one exception (input gradients of bf16 graphs with ReLU
layers, whose bar is derived from a CPU measurement on the oracle) are stated in
tests/parity_bars.py.  Every comparison is also recorded (worst error per
workload and tensor class); tests/conftest.py writes the record out after a GPU
run.
"""
import numpy as np

from oracle import gpp_oracle as O
from paper_2406_17145_amd import binding as B
from tests import parity_bars as PB


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


# parameter counts of the workloads at the sizes the benchmark runs them: their comparisons are recorded one
# by one, every other workload of a family (small, ragged, degenerate cases) as one worst-case line
FULL_SIZE_PARAMETERS = {"tiny_mlp": 33152, "candle_uno": 18825001, "mmt": 105990120, "dlrm": 335168897, "hetero": 89558016,
                        "paper_candle": 587325441, "paper_mmt": 408299496, "paper_dlrm": 1235607553}
_SPREAD_CACHE = {}
RECORD = {}          # label -> tensor class -> [worst l2, worst max-norm, l2 bar]; conftest writes it out


def _relu_spread(wl):
    key = PB.workload_key(wl)
    if key in PB.RELU_SPREAD_PINNED:
        return PB.RELU_SPREAD_PINNED[key]
    key = key + (id(wl.ops),)
    if key not in _SPREAD_CACHE:
        from tests.relu_noise import measure
        n_par = sum(int(np.asarray(v).size) for p in wl.params.values() for v in p.values())
        # (a large workload that is not in the stored table: two of the four orders keep the test within minutes)
        _SPREAD_CACHE[key] = measure(wl) if n_par < 50_000_000 else measure(wl, ("blas", "blk64g"))
    return _SPREAD_CACHE[key]


def _tensor_class(name):
    if ".out" in name:
        return "output"
    if ".gin" in name:
        return "input gradient"
    return "d" + name.split(".d", 1)[1]


def compare(wl, gpu_res, gpu_grads, ora_stage, ora_res, tol=None, label=""):
    """Every tensor against the oracle.  Bars: tests/parity_bars.py (the stated ones, except the
    input gradients of bf16 graphs with ReLU, whose bars come from the spread the oracle itself
    shows under re-ordered float32 sums)."""
    tol = wl.tol if tol is None else tol
    mode = "f32" if tol <= 1e-3 else "bf16"
    tol_max = PB.STATED_MAX[mode] if tol == PB.STATED_L2[mode] else 5 * tol
    has_relu = any(op.get("act") == "relu" for op in wl.ops)
    worst = {}
    n_par = sum(int(np.asarray(v).size) for p in wl.params.values() for v in p.values())
    if FULL_SIZE_PARAMETERS.get(wl.name) == n_par:
        rec = RECORD.setdefault(f"{wl.name} full size, b={wl.micro_batch} x {wl.n_micro} micro-batches, {mode}", {})
    else:
        rec = RECORD.setdefault(f"{wl.name} small and ragged variants, {mode}", {})
        rec["(workloads compared)"] = [rec.get("(workloads compared)", [0, 0, 0])[0] + 1, 0.0, 0.0]

    def note(name, e2, em, bar):
        worst[name] = (e2, em)
        r = rec.setdefault(_tensor_class(name), [0.0, 0.0, bar])
        r[0], r[1], r[2] = max(r[0], e2), max(r[1], em), max(r[2], bar)

    def chk(name, got, ref):
        e2, em = rel_errors(got, ref)
        note(name, e2, em, tol)
        assert e2 <= tol and em <= tol_max, f"{label} {name}: l2-rel {e2:.3e} (bar {tol}) max-rel {em:.3e} (bar {tol_max})"

    def chk_relu_gin(name, got, ref):
        from tests.relu_noise import ROW_BAR, row_errors
        b2, bm, brows = PB.relu_gin_bars(_relu_spread(wl), ref.shape[0])
        e2, em = rel_errors(got, ref)
        note(name, e2, em, b2)
        assert e2 <= b2 and em <= bm, f"{label} {name}: l2-rel {e2:.3e} (bar {b2:.3e}) max-rel {em:.3e} (bar {bm:.3e})"
        if ref.size // ref.shape[0] >= PB.ROW_CHECK_MIN_WIDTH:
            over = float((row_errors(got, ref) > ROW_BAR).mean())
            r = rec.setdefault("input gradient: share of rows over %g" % ROW_BAR, [0.0, 0.0, brows])
            r[0], r[2] = max(r[0], over), max(r[2], brows)
            assert over <= brows, f"{label} {name}: {over:.3f} of the rows over {ROW_BAR} (allowed {brows:.3f})"

    for j, (g, (st, gin)) in enumerate(zip(gpu_res, ora_res)):
        if ora_stage.ops and any(op["kind"].startswith("loss") for op in ora_stage.ops):
            el = abs(g["loss"] - st.loss) / max(abs(st.loss), 1e-30)
            r = rec.setdefault("loss", [0.0, 0.0, tol])
            r[0] = r[1] = max(r[0], el)
            assert el <= tol, (label, "loss", j, g["loss"], st.loss)
        for i in ora_stage.output_ids:
            chk(f"mb{j}.out{i}", g["outs"][i], st.values[i])
        assert set(g["gin"]) == set(gin), (set(g["gin"]), set(gin))
        for i, ref in gin.items():
            if mode == "bf16" and has_relu:
                chk_relu_gin(f"mb{j}.gin{i}", g["gin"][i], ref)
            else:
                chk(f"mb{j}.gin{i}", g["gin"][i], ref)
    derived = mode == "bf16" and has_relu and tol == PB.STATED_L2[mode]
    for i, gr in ora_stage.grads.items():
        for k, ref in gr.items():
            bar = PB.relu_dw_bar(_relu_spread(wl), table=(k == "table")) if (derived and k in ("W", "b", "table")) else tol
            if bar != tol:
                e2, em = rel_errors(gpu_grads[i][k], ref)
                note(f"op{i}.d{k}", e2, em, bar)
                assert e2 <= bar and em <= 5 * bar, f"{label} op{i}.d{k}: l2-rel {e2:.3e} (bar {bar:.3e}) max-rel {em:.3e}"
            else:
                chk(f"op{i}.d{k}", gpu_grads[i][k], ref)
    return worst
