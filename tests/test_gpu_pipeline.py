"""Several stages of one stage graph on the GPU (the library's pipeline executor): a branchy model cut into
branch stages and a merge stage must give the gradients of the uncut model (the oracle runs the WHOLE graph
as one stage), whether the branch stages run side by side (graph pipeline) or chained (sequential pipeline)."""
import numpy as np
import pytest

from paper_2406_17145_amd import binding as B
from paper_2406_17145_amd import workloads as W
from paper_2406_17145_amd.schedule import StagePipeline
from tests.parity_util import rel_errors, run_gpu, run_oracle, t2n

pytestmark = pytest.mark.gpu


def _model(micro_batch=32, n_micro=6):
    wl = W.candle_uno(micro_batch=micro_batch, n_micro=n_micro, widths=(70, 131, 33), hidden=96, act="gelu")
    stage_of = {i: (op["branch"] if op["branch"] >= 0 else 3) for i, op in enumerate(wl.ops) if op["kind"] != "input"}
    parts, edges = W.partition(wl, stage_of, 4)
    return wl, parts, edges


def _run_pipeline(wl, parts, edges, in_flight=None, k=None, flags=0, reps=1):
    """Returns (losses per micro-batch, {global op id: {name: grad}}, {global input id: [grad per micro-batch]}, caps)."""
    import torch
    b, n = wl.micro_batch, wl.n_micro
    if in_flight is None:
        caps, k = StagePipeline.in_flight_microbatches(len(parts), edges, b)
        in_flight = [c * b for c in caps]
    caps = [max(1, i // b) for i in in_flight]
    stages = [B.Stage(p.ops, b, p.params, slots=c, flags=flags) for p, c in zip(parts, caps)]
    pipe = StagePipeline(stages, edges, in_flight, k)
    fed_in = {(e[2], e[3]) for e in edges if e[1] >= 0}
    fed_out = {(e[0], e[1]) for e in edges if e[1] >= 0}
    io, losses, gins = [], [], []
    for s, (st, p) in enumerate(zip(stages, parts)):
        rows, g_rows = [], []
        for j in range(n):
            dev = {i: st.to_device(i, a) for i, a in p.batches[j].items()}
            inputs = [None if (s, q) in fed_in else dev[i] for q, i in enumerate(st.input_ids)]
            outs = [None if (s, q) in fed_out else t for q, t in enumerate(st.alloc_outputs())]
            gin = [None if (s, q) in fed_in else t for q, t in enumerate(st.alloc_grad_inputs())]
            loss = torch.zeros(1, dtype=torch.float32, device=st.dev)
            rows.append((inputs, outs, loss, None, gin))
            g_rows.append(gin)
            if s == len(parts) - 1:
                losses.append(loss)
        io.append(rows)
        gins.append(g_rows)
    for _ in range(reps):
        pipe.minibatch(io)
    for st in stages:
        st.sync_status()
    grads, gin_out = {}, {}
    for s, (st, p) in enumerate(zip(stages, parts)):
        for l, g in st.grads_numpy().items():
            grads[p.global_of[l]] = g
        for q, i in enumerate(st.input_ids):
            if p.global_of[i] >= 0 and gins[s][0][q] is not None:
                gin_out[p.global_of[i]] = [t2n(gins[s][j][q]) for j in range(n)]
    out = ([float(l.cpu()[0]) for l in losses], grads, gin_out, caps, pipe.stash_bytes())
    pipe.close()
    for st in stages:
        st.close()
    return out


def _check_against_oracle(wl, losses, grads, gin, tol):
    ora_stage, ora_res = run_oracle(wl)
    for j, (st, g) in enumerate(ora_res):
        assert abs(losses[j] - st.loss) <= tol * abs(st.loss), (j, losses[j], st.loss)
        for i, ref in g.items():
            e2, em = rel_errors(gin[i][j], ref)
            assert e2 <= tol and em <= 5 * tol, ("input gradient", i, j, e2, em)
    assert set(grads) == set(ora_stage.grads)
    for i, gr in ora_stage.grads.items():
        for name, ref in gr.items():
            e2, em = rel_errors(grads[i][name], ref)
            assert e2 <= tol and em <= 5 * tol, ("weight gradient", i, name, e2, em)


def test_graph_pipeline_and_sequential_pipeline_match_the_uncut_model():
    wl, parts, edges = _model()
    print("[case] graph pipeline: three branch stages side by side, one merge stage", flush=True)
    l_g, g_g, gin_g, caps_g, stash_g = _run_pipeline(wl, parts, edges, reps=2)
    assert caps_g == [2, 2, 2, 1]                      # depth 2: the branch stages hold two micro-batches
    _check_against_oracle(wl, l_g, g_g, gin_g, wl.tol)
    print("[case] sequential pipeline: the same stages chained", flush=True)
    chain = edges + [(0, -1, 1, -1), (1, -1, 2, -1)]
    l_s, g_s, gin_s, caps_s, stash_s = _run_pipeline(wl, parts, chain, reps=2)
    assert caps_s == [4, 3, 2, 1]                      # depth 4
    assert stash_s[0] == 2 * stash_g[0]
    # the same kernels in the same per-stage order: bit-identical
    assert l_s == l_g
    for i in g_g:
        for name in g_g[i]:
            assert np.array_equal(g_g[i][name], g_s[i][name]), (i, name)
    # the uncut model as ONE stage on the GPU: same storage types at the cuts, so values agree closely
    _, g_one = run_gpu(wl)
    for i in g_one:
        for name in g_one[i]:
            e2, _ = rel_errors(g_g[i][name], g_one[i][name])
            assert e2 <= 1e-5, (i, name, e2)


def test_pipeline_with_kfkb_groups_and_grouped_weight_gradients():
    wl, parts, edges = _model(micro_batch=24, n_micro=7)
    b = wl.micro_batch
    print("[case] graph pipeline, 2F2B at the branch stages, grouped weight gradients", flush=True)
    caps, k = StagePipeline.in_flight_microbatches(4, edges, b, [[2], [2], [2], [2]])
    losses, grads, gin, caps2, _ = _run_pipeline(wl, parts, edges, [c * b for c in caps], k, flags=B.FLAG_GROUPED_DW, reps=2)
    assert caps2 == caps
    _check_against_oracle(wl, losses, grads, gin, wl.tol)


def test_pipeline_refuses_what_cannot_run():
    import torch
    wl, parts, edges = _model(micro_batch=8, n_micro=4)
    b = wl.micro_batch
    stages = [B.Stage(p.ops, b, p.params, slots=2) for p in parts]
    hs = [st.handle for st in stages]

    def status(fn, *a):
        with pytest.raises(B.GppError) as e:
            fn(*a)
        return e.value.status
    ok_i, ok_k = [2 * b, 2 * b, 2 * b, b], [1, 1, 1, 1]
    assert status(B.gpp_pipeline_workspace_bytes, hs, edges + [(3, -1, 0, -1)], ok_i, ok_k) == B.GPP_ERR_BAD_GRAPH
    assert status(B.gpp_pipeline_workspace_bytes, hs, edges, [3 * b, 2 * b, 2 * b, b], ok_k) == B.GPP_ERR_ORDER      # 3 in flight, 2 slots
    assert status(B.gpp_pipeline_workspace_bytes, hs, [(0, 0, 3, 3)], ok_i, ok_k) == B.GPP_ERR_SHAPE                 # a tower output into the target input
    assert status(B.gpp_pipeline_workspace_bytes, hs, edges + [(1, 0, 3, 0)], ok_i, ok_k) == B.GPP_ERR_UNSUPPORTED   # two producers for one input
    assert status(B.gpp_pipeline_workspace_bytes, hs, [(0, 5, 3, 0)], ok_i, ok_k) == B.GPP_ERR_INVALID_ARG
    # task lists that wait for each other: the merge stage runs 2F2B but a branch stage may hold one micro-batch
    pipe = StagePipeline(stages, edges, [b, 2 * b, 2 * b, 2 * b], [1, 1, 1, 2])
    io = []
    for s, (st, p) in enumerate(zip(stages, parts)):
        rows = []
        for j in range(wl.n_micro):
            dev = {i: st.to_device(i, a) for i, a in p.batches[j].items()}
            fed = {(e[2], e[3]) for e in edges}
            inputs = [None if (s, q) in fed else dev[i] for q, i in enumerate(st.input_ids)]
            rows.append((inputs, [None] * len(st.output_ids), torch.zeros(1, device=st.dev), None, [None] * len(inputs)))
        io.append(rows)
    with pytest.raises(B.GppError) as e:
        pipe.minibatch(io)
    assert e.value.status == B.GPP_ERR_ORDER
    pipe.close()
    # nothing was enqueued and no slot is held: the same stages run under a consistent configuration
    pipe = StagePipeline(stages, edges)
    pipe.minibatch(io)
    for st in stages:
        st.sync_status()
    pipe.close()
    for st in stages:
        st.close()
