"""kFkB schedules of one stage on the GPU: the library's executor (gpp_stage_run_schedule) under the task
lists of gpp_schedule_tasks, against the serial order and against the oracle.  Backward passes run in
micro-batch order under every schedule, so accumulated gradients must be bit-identical to the serial run."""
import numpy as np
import pytest

from oracle import schedule_oracle as S
from paper_2406_17145_amd import binding as B
from paper_2406_17145_amd import workloads as W
from paper_2406_17145_amd.schedule import TaskSchedule
from tests.parity_util import compare, run_gpu, run_oracle, t2n

pytestmark = pytest.mark.gpu


def _codes(tasks):
    return [(j + 1) if w == "F" else -(j + 1) for w, j in tasks]


def _run(wl, cap, k, two_streams, slots=None, gouts=None, reps=1, flags=0, lanes=(1, 1), shared_lanes=False, same_stream=False):
    import torch
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=slots or cap, flags=flags)
    n = len(wl.batches)
    dev_batches = [st.stage_inputs(mb) for mb in wl.batches]
    losses = [torch.zeros(1, dtype=torch.float32, device=st.dev) for _ in range(n)]
    outs = [st.alloc_outputs() for _ in range(n)]
    gins = [st.alloc_grad_inputs() for _ in range(n)]
    dg = None if gouts is None else [[st.to_device(i, g[i]) for i in st.output_ids] for g in gouts]
    sched = TaskSchedule(st, cap * wl.micro_batch, k, two_streams=two_streams, lanes=lanes, shared_lanes=shared_lanes, same_stream=same_stream)
    for _ in range(reps):
        tasks = sched.minibatch(dev_batches, outputs=outs, grad_outputs=dg, grad_inputs=gins, losses=losses)
    st.sync_status()
    res = [dict(loss=float(losses[j].cpu()[0]), outs={i: t2n(t) for i, t in zip(st.output_ids, outs[j])},
                gin={i: t2n(t) for i, t in zip(st.input_ids, gins[j]) if t is not None}) for j in range(n)]
    grads = st.grads_numpy()
    st.close()
    return tasks, res, grads


@pytest.mark.parametrize("two_streams", [False, True])
def test_kfkb_schedules_on_loss_stage_match_serial_and_oracle(two_streams):
    wl = W.candle_uno(micro_batch=48, n_micro=7, widths=(70, 131, 9, 33), hidden=160, act="gelu")
    _, g_serial = run_gpu(wl)
    ora_stage, ora_res = run_oracle(wl)
    for cap, k in [(1, 1), (2, 1), (3, 2), (4, 2), (4, 4), (7, 3)]:
        print(f"[case] {wl.name} kFkB cap={cap} k={k} two_streams={two_streams}", flush=True)
        tasks, res, grads = _run(wl, cap, k, two_streams, reps=2)
        assert tasks == _codes(S.schedule_task(wl.n_micro, cap * wl.micro_batch, k, wl.micro_batch))
        for i in g_serial:
            for kk in g_serial[i]:
                assert np.array_equal(g_serial[i][kk], grads[i][kk]), (cap, k, i, kk)
        compare(wl, res, grads, ora_stage, ora_res, label=f"kFkB cap={cap} k={k}")


def test_kfkb_schedule_on_mid_pipeline_stage_with_per_microbatch_gradients():
    # a stage with outputs: every micro-batch has its own output, output-gradient and input-gradient buffers
    wl = W.hetero(micro_batch=9, n_micro=5, base_width=16, out_width=24, dtype="f32", with_loss=False)
    out = len(wl.ops) - 1
    rng = np.random.default_rng(5)
    gouts = [{out: rng.standard_normal((9, 192)).astype(np.float32)} for _ in range(5)]
    ora_stage, ora_res = run_oracle(wl, gouts)
    res_serial, g_serial = run_gpu(wl, gouts=gouts)
    for cap, k, two in [(3, 1, True), (2, 2, False), (5, 2, True)]:
        print(f"[case] {wl.name} mid-pipeline kFkB cap={cap} k={k} two_streams={two}", flush=True)
        _, res, grads = _run(wl, cap, k, two, gouts=gouts)
        compare(wl, res, grads, ora_stage, ora_res, label=f"mid kFkB cap={cap} k={k}")
        for i in g_serial:
            for kk in g_serial[i]:
                assert np.array_equal(g_serial[i][kk], grads[i][kk]), (cap, k, i, kk)
        for a, b in zip(res_serial, res):
            for i in a["gin"]:
                assert np.array_equal(a["gin"][i], b["gin"][i])
            for i in a["outs"]:
                assert np.array_equal(a["outs"][i], b["outs"][i])


def test_kfkb_schedule_with_embedding_tables():
    # sparse path: sort buffers shared by the slots, touched-row log across five backward passes
    wl = W.dlrm(micro_batch=128, n_micro=5, n_tables=4, num_rows=3000, bottom=(64, 32, 128), top=(128, 64, 1))
    _, g_serial = run_gpu(wl)
    ora_stage, ora_res = run_oracle(wl)
    for cap, k, two in [(2, 1, True), (3, 2, True)]:
        print(f"[case] {wl.name} kFkB cap={cap} k={k} two_streams={two}", flush=True)
        _, res, grads = _run(wl, cap, k, two, reps=2)
        compare(wl, res, grads, ora_stage, ora_res, label=f"dlrm kFkB cap={cap} k={k}")
        for i in g_serial:
            for kk in g_serial[i]:
                assert np.array_equal(g_serial[i][kk], grads[i][kk]), (cap, k, i, kk)


def test_executor_refuses_invalid_task_lists_before_running_anything():
    import torch
    wl = W.tiny_mlp()
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=2)
    n = len(wl.batches)
    dev = [st.stage_inputs(mb) for mb in wl.batches]
    losses = [torch.zeros(1, dtype=torch.float32, device=st.dev) for _ in range(n)]
    io = [([t.data_ptr() for t in dev[j]], [], losses[j].data_ptr(), None, [None] * len(dev[j])) for j in range(n)]
    s = torch.cuda.current_stream().cuda_stream
    bad = {
        "backward before its forward": [-1, 1, 2, -2, 3, -3, 4, -4],
        "forward out of order": [2, 1, -1, -2, 3, -3, 4, -4],
        "backward out of order": [1, 2, -2, -1, 3, -3, 4, -4],
        "three in flight, two slots": [1, 2, 3, -1, -2, -3, 4, -4],
        "repeated forward": [1, 1, -1, -1, 2, -2, 3, -3],
    }
    for why, tasks in bad.items():
        with pytest.raises(B.GppError) as e:
            B.gpp_stage_run_schedule(st.handle, tasks, io, s, s)
        assert e.value.status == B.GPP_ERR_ORDER, why
    for tasks in ([1, 0, -1, 2, -2, 3, -3, 4], [1, -1, 2, -2]):      # a zero code; wrong length
        with pytest.raises(B.GppError) as e:
            B.gpp_stage_run_schedule(st.handle, tasks, io, s, s)
        assert e.value.status == B.GPP_ERR_INVALID_ARG
    # nothing ran and no slot is held: a valid list goes through and gives the serial result
    B.gpp_stage_run_schedule(st.handle, B.gpp_schedule_tasks(n, 2 * wl.micro_batch, 1, wl.micro_batch), io, s, s)
    st.sync_status()
    got = st.grads_numpy()
    st.close()
    _, ref = run_gpu(wl)
    for i in ref:
        for k in ref[i]:
            assert np.array_equal(ref[i][k], got[i][k])


def test_stage_memory_report():
    wl = W.candle_uno(micro_batch=64, n_micro=1, widths=(96, 200, 8, 64), hidden=128)
    seen = {}
    for slots in (1, 3):
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=slots)
        slot_b, shared_b, total_b = B.gpp_stage_memory(st.handle)
        assert total_b == st.ws_bytes == slots * slot_b + shared_b
        assert slot_b > 0 and slot_b % 256 == 0
        seen[slots] = (slot_b, shared_b)
        st.close()
    assert seen[1][0] == seen[3][0]            # one slot costs the same whatever their number


def test_config2_full_size_in_the_launch_configuration_the_benchmark_times():
    # the benchmark's default step: the full CANDLE-Uno-shaped stage, a stash slot per micro-batch, the scheduler's
    # task list for that many in-flight micro-batches run by the executor with micro-batch j on stream j mod 2
    # (forward and backward pass), one launch per step for the four micro-batches of a stream, weight gradients of
    # the whole run of backward passes in one grouped launch, everything captured once into a HIP graph and replayed.
    # Checked against the oracle in full (losses, input gradients, every accumulated gradient); every replay
    # (accumulators poisoned, eager work and synchronisations in between) must reproduce the eager run of the
    # same configuration bit for bit.
    import torch
    from paper_2406_17145_amd.schedule import GraphedMinibatch
    wl = W.candle_uno()
    n = wl.n_micro
    print(f"[case] {wl.name} full size, {n} in flight, grouped weight gradients, graph replay", flush=True)
    ora_stage, ora_res = run_oracle(wl)
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=n, flags=B.FLAG_GROUPED_DW | B.FLAG_SHARED_GPU | B.flag_group_launches(2))
    assert st.num_launches(2) == 1
    assert B.gpp_stage_lanes(st.handle) == (True, True)
    assert B.gpp_stage_group_launches(st.handle) == (2, n // 2)
    dev_batches = [st.stage_inputs(mb) for mb in wl.batches]
    losses = [torch.zeros(1, dtype=torch.float32, device=st.dev) for _ in range(n)]
    gins = [st.alloc_grad_inputs() for _ in range(n)]
    sched = TaskSchedule(st, n * wl.micro_batch, n, two_streams=True, lanes=(2, 2), shared_lanes=True)
    outs = [[] for _ in range(n)]
    sched.minibatch(dev_batches, outputs=outs, grad_inputs=gins, losses=losses)     # eager first
    st.sync_status()
    g_eager = st.grads_numpy()
    res = [dict(loss=float(losses[j].cpu()[0]), outs={},
                gin={i: t2n(t) for i, t in zip(st.input_ids, gins[j]) if t is not None}) for j in range(n)]
    compare(wl, res, g_eager, ora_stage, ora_res, label="full size, grouped, eager")
    graphed = GraphedMinibatch(sched, dev_batches, outputs=outs, grad_inputs=gins, losses=losses)
    scratch = torch.zeros(1 << 20, device=st.dev)
    for rep in range(3):
        for t in st.g_t.values():
            for g in t.values():
                g.fill_(float("nan"))
        for l in losses:
            l.fill_(-1.0)
        scratch.add_(1.0)
        torch.cuda.synchronize()
        graphed.replay()
        torch.cuda.synchronize()
        got = st.grads_numpy()
        for i in g_eager:
            for k in g_eager[i]:
                assert np.array_equal(g_eager[i][k], got[i][k]), (rep, i, k)
        for j in range(n):
            assert float(losses[j].cpu()[0]) == res[j]["loss"], (rep, j)
    st.sync_status()
    st.close()


# ---- grouped weight gradients: the weight-gradient GEMMs of a run of backward passes as one launch whose
# contraction runs over the stash slots of the whole run.  Sums are formed in another order than with one
# accumulation per micro-batch, so the comparison with the serial run is to rounding, not bit for bit.

def _close(a, b, tol):
    n = np.linalg.norm(b)
    return np.linalg.norm(a.astype(np.float64) - b) <= tol * max(n, 1e-30)


@pytest.mark.parametrize("two_streams", [False, True])
def test_grouped_weight_gradients_match_oracle_and_serial(two_streams):
    for mb, act in [(48, "gelu"), (37, "relu"), (64, "relu")]:      # rows per slot: less than, not a multiple of, exactly one k-step
        wl = W.candle_uno(micro_batch=mb, n_micro=7, widths=(70, 131, 9, 33), hidden=160, act=act)
        _, g_serial = run_gpu(wl)
        ora_stage, ora_res = run_oracle(wl)
        for cap, k in [(1, 1), (3, 2), (4, 4), (7, 7), (5, 3)]:
            print(f"[case] {wl.name} b={mb} grouped weight gradients cap={cap} k={k} two_streams={two_streams}", flush=True)
            _, res, grads = _run(wl, cap, k, two_streams, reps=2, flags=B.FLAG_GROUPED_DW)
            compare(wl, res, grads, ora_stage, ora_res, label=f"grouped cap={cap} k={k}")
            for i in g_serial:
                for kk in g_serial[i]:
                    assert _close(grads[i][kk], g_serial[i][kk], 1e-5), (cap, k, i, kk)


def test_grouped_weight_gradients_long_rows_per_slot():
    # several k-steps per slot with a ragged last one (300 = 4 * 64 + 44), wide layers (large tiles, ragged edges)
    wl = W.candle_uno(micro_batch=300, n_micro=4, widths=(264, 131, 520, 8), hidden=392, act="gelu")
    ora_stage, ora_res = run_oracle(wl)
    for cap, k in [(2, 2), (4, 4), (3, 2)]:
        print(f"[case] {wl.name} b=300 grouped weight gradients cap={cap} k={k}", flush=True)
        _, res, grads = _run(wl, cap, k, True, flags=B.FLAG_GROUPED_DW)
        compare(wl, res, grads, ora_stage, ora_res, label=f"grouped long cap={cap} k={k}")


def test_grouped_weight_gradients_transformer_stage():
    # per-slot gradient buffers: the cross-entropy kernels of the forward pass also write the loss gradient where a
    # row of logits fits their registers (50 and 1024 classes), and leave it to the backward pass where not (1500);
    # LayerNorm parameter gradients are folded once per backward pass
    for n_classes in (50, 1024, 1500):
        wl = W.mmt(micro_batch=2, n_micro=4, n_branches=2, n_layers=2, d_model=128, heads=2, d_ff=256, seq_len=48,
                   d_head_out=64, n_classes=n_classes)
        ora_stage, ora_res = run_oracle(wl)
        for cap, k in [(2, 2), (4, 4), (3, 1)]:
            print(f"[case] {wl.name} {n_classes} classes, grouped weight gradients cap={cap} k={k}", flush=True)
            _, res, grads = _run(wl, cap, k, True, reps=2, flags=B.FLAG_GROUPED_DW)
            compare(wl, res, grads, ora_stage, ora_res, label=f"mmt grouped {n_classes} cap={cap} k={k}")


def test_grouped_weight_gradients_with_embedding_tables_and_mid_pipeline_stage():
    wl = W.dlrm(micro_batch=128, n_micro=5, n_tables=4, num_rows=3000, bottom=(64, 32, 128), top=(128, 64, 1))
    ora_stage, ora_res = run_oracle(wl)
    for cap, k in [(3, 2), (5, 5)]:
        print(f"[case] {wl.name} grouped weight gradients cap={cap} k={k}", flush=True)
        _, res, grads = _run(wl, cap, k, True, reps=2, flags=B.FLAG_GROUPED_DW)
        compare(wl, res, grads, ora_stage, ora_res, label=f"dlrm grouped cap={cap} k={k}")
    # a stage with outputs, bf16 (grouped) and fp32 (the flag changes nothing: no layer is taken)
    for dtype in ("bf16", "f32"):
        wl = W.hetero(micro_batch=9, n_micro=5, base_width=16, out_width=24, dtype=dtype, with_loss=False)
        out = len(wl.ops) - 1
        rng = np.random.default_rng(5)
        gouts = [{out: rng.standard_normal((9, 192)).astype(np.float32)} for _ in range(5)]
        ora_stage, ora_res = run_oracle(wl, gouts)
        print(f"[case] {wl.name} {dtype} mid-pipeline grouped weight gradients", flush=True)
        _, res, grads = _run(wl, 3, 2, True, gouts=gouts, flags=B.FLAG_GROUPED_DW)
        compare(wl, res, grads, ora_stage, ora_res, label=f"mid grouped {dtype}")


def test_grouped_weight_gradients_state_machine():
    wl = W.candle_uno(micro_batch=16, n_micro=3, widths=(32, 40, 8, 24), hidden=64, act="gelu")
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=2, flags=B.FLAG_GROUPED_DW)
    assert st.num_launches(2) == 1                 # every LINEAR of the stage in one grouped launch
    st.grad_reset()
    st.forward(0, wl.batches[0])
    st.backward(0)
    with pytest.raises(B.GppError) as e:
        st.forward(0, wl.batches[1])               # the slot's operands still feed the weight gradients
    assert e.value.status == B.GPP_ERR_ORDER
    with pytest.raises(B.GppError) as e:
        st.grad_reset()
    assert e.value.status == B.GPP_ERR_ORDER
    st.forward(1, wl.batches[1])
    st.backward(1)
    st.backward_weights()                          # slots 0 and 1 in one launch
    st.forward(0, wl.batches[2])
    st.backward(0)
    st.backward_weights()
    st.backward_weights()                          # nothing pending: no-op
    st.sync_status()
    got = st.grads_numpy()
    st.close()
    ora_stage, _ = run_oracle(wl)
    for i, gr in ora_stage.grads.items():
        for k, ref in gr.items():
            assert _close(got[i][k], ref, wl.tol), (i, k)
    # without the flag the call does nothing
    st = B.Stage(wl.ops, wl.micro_batch, wl.params)
    assert st.num_launches(2) == 0
    st.backward_weights()
    st.close()


def test_grouped_weight_gradients_degenerate_sizes():
    # one and three rows per stash slot (a k-step of the grouped contraction is almost empty), one micro-batch
    # per mini-batch (a group of one), and more micro-batches than slots (several groups, the later ones add)
    for mb, n_micro, cap, k in [(1, 5, 5, 5), (3, 4, 2, 2), (5, 1, 1, 1), (2, 9, 3, 3)]:
        wl = W.candle_uno(micro_batch=mb, n_micro=n_micro, widths=(40, 72, 8, 24), hidden=64, act="gelu")
        ora_stage, ora_res = run_oracle(wl)
        print(f"[case] {wl.name} b={mb} x {n_micro}, grouped weight gradients cap={cap} k={k}", flush=True)
        _, res, grads = _run(wl, cap, k, True, flags=B.FLAG_GROUPED_DW)
        compare(wl, res, grads, ora_stage, ora_res, label=f"grouped degenerate b={mb}")


def test_executor_with_no_micro_batches_is_a_gradient_reset():
    import torch
    wl = W.tiny_mlp()
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=2)
    s = torch.cuda.current_stream().cuda_stream
    B.gpp_stage_run_schedule(st.handle, [], [], s, s)
    st.forward(0, wl.batches[0])          # the stage is usable afterwards
    st.backward(0)
    st.sync_status()
    st.close()


# ---- several streams per direction (gpp_stage_run_schedule_lanes) ------------------------------------

def _same(res_a, grads_a, res_b, grads_b, label):
    for j, (a, b) in enumerate(zip(res_a, res_b)):
        assert a["loss"] == b["loss"], (label, j)
        for kind in ("outs", "gin"):
            for i in a[kind]:
                assert np.array_equal(a[kind][i], b[kind][i]), (label, j, kind, i)
    for i in grads_a:
        for kk in grads_a[i]:
            assert np.array_equal(grads_a[i][kk], grads_b[i][kk]), (label, i, kk)


def test_lanes_give_the_one_stream_results_bit_for_bit():
    wl = W.candle_uno(micro_batch=48, n_micro=7, widths=(70, 131, 9, 33), hidden=160, act="gelu")
    ora_stage, ora_res = run_oracle(wl)
    for cap, k in [(7, 7), (4, 4), (5, 3), (3, 2)]:
        _, res1, grads1 = _run(wl, cap, k, False, reps=2, flags=B.FLAG_GROUPED_DW)
        compare(wl, res1, grads1, ora_stage, ora_res, label=f"one stream cap={cap} k={k}")
        for lanes in [(2, 1), (1, 2), (2, 2), (3, 2), (4, 4)]:
            print(f"[case] {wl.name} lanes={lanes} cap={cap} k={k}", flush=True)
            _, res, grads = _run(wl, cap, k, True, reps=2, flags=B.FLAG_GROUPED_DW, lanes=lanes)
            _same(res, grads, res1, grads1, f"lanes={lanes} cap={cap} k={k}")
        for n in (2, 4):       # the backward passes on the forward streams: one chain of launches per micro-batch
            print(f"[case] {wl.name} {n} shared lanes cap={cap} k={k}", flush=True)
            _, res, grads = _run(wl, cap, k, True, reps=2, flags=B.FLAG_GROUPED_DW, lanes=(n, n), shared_lanes=True)
            _same(res, grads, res1, grads1, f"shared lanes={n} cap={cap} k={k}")
        # with the workgroup sizes for a shared GPU (other kernels: compared with their own one-stream run)
        _, res4, grads4 = _run(wl, cap, k, False, reps=2, flags=B.FLAG_GROUPED_DW | B.FLAG_SHARED_GPU)
        compare(wl, res4, grads4, ora_stage, ora_res, label=f"four waves, one stream cap={cap} k={k}")
        print(f"[case] {wl.name} 4 shared lanes, four-wave workgroups cap={cap} k={k}", flush=True)
        _, res, grads = _run(wl, cap, k, True, reps=2, flags=B.FLAG_GROUPED_DW | B.FLAG_SHARED_GPU, lanes=(4, 4), shared_lanes=True)
        _same(res, grads, res4, grads4, f"four waves, shared lanes cap={cap} k={k}")


def test_lanes_on_a_mid_pipeline_stage():
    wl = W.hetero(micro_batch=9, n_micro=6, base_width=16, out_width=24, dtype="bf16", with_loss=False)
    out = len(wl.ops) - 1
    rng = np.random.default_rng(11)
    gouts = [{out: rng.standard_normal((9, 192)).astype(np.float32)} for _ in range(6)]
    ora_stage, ora_res = run_oracle(wl, gouts)
    _, res1, grads1 = _run(wl, 4, 2, False, gouts=gouts, flags=B.FLAG_GROUPED_DW)
    compare(wl, res1, grads1, ora_stage, ora_res, label="mid one stream")
    for lanes in [(2, 2), (3, 4)]:
        print(f"[case] {wl.name} mid-pipeline lanes={lanes}", flush=True)
        _, res, grads = _run(wl, 4, 2, True, gouts=gouts, flags=B.FLAG_GROUPED_DW, lanes=lanes)
        _same(res, grads, res1, grads1, f"mid lanes={lanes}")


def test_lanes_are_refused_where_passes_share_memory_or_accumulate():
    import torch
    cases = [
        (W.candle_uno(micro_batch=16, n_micro=3, widths=(32, 40, 8, 24), hidden=64, act="relu"), 0, (True, False)),
        (W.candle_uno(micro_batch=16, n_micro=3, widths=(32, 40, 8, 24), hidden=64, act="relu"), B.FLAG_GROUPED_DW, (True, True)),
        (W.dlrm(micro_batch=32, n_micro=3, n_tables=3, num_rows=500, bottom=(64, 32, 128), top=(128, 64, 1)), B.FLAG_GROUPED_DW, (None, False)),
        (W.mmt(micro_batch=2, n_micro=3, n_branches=2, seq_len=64, d_model=128, heads=2, n_layers=1, d_ff=256, d_head_out=128, n_classes=10), B.FLAG_GROUPED_DW, (None, False)),
    ]
    for wl, flags, (want_f, want_b) in cases:
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=3, flags=flags)
        ok_f, ok_b = B.gpp_stage_lanes(st.handle)
        print(f"[case] {wl.name} flags={flags}: lanes allowed forward={ok_f} backward={ok_b}", flush=True)
        assert ok_b == want_b and (want_f is None or ok_f == want_f)
        dev = [st.stage_inputs(mb) for mb in wl.batches]
        outs = [st.alloc_outputs() for _ in dev]
        gin = [st.alloc_grad_inputs() for _ in dev]
        loss = torch.zeros(1, dtype=torch.float32, device=st.dev)
        io = [([t.data_ptr() for t in mb], [t.data_ptr() for t in outs[j]], loss.data_ptr(), None,
               [t.data_ptr() if t is not None else None for t in gin[j]]) for j, mb in enumerate(dev)]
        tasks = B.gpp_schedule_tasks(3, 3 * wl.micro_batch, 3, wl.micro_batch)
        streams = [torch.cuda.Stream(device=st.dev) for _ in range(4)]
        sp = [s.cuda_stream for s in streams]
        for nf, nb, allowed in [(2, 1, ok_f), (1, 2, ok_b)]:
            if allowed:
                B.gpp_stage_run_schedule_lanes(st.handle, tasks, io, sp[:nf], sp[2:2 + nb])
                torch.cuda.synchronize()
            else:
                with pytest.raises(B.GppError) as e:
                    B.gpp_stage_run_schedule_lanes(st.handle, tasks, io, sp[:nf], sp[2:2 + nb])
                assert e.value.status == B.GPP_ERR_UNSUPPORTED
        with pytest.raises(B.GppError) as e:
            B.gpp_stage_run_schedule_lanes(st.handle, tasks, io, [], sp[:1])
        assert e.value.status == B.GPP_ERR_INVALID_ARG
        # the stage is untouched by a refusal: one more mini-batch on one stream
        main = torch.cuda.current_stream(st.dev).cuda_stream
        B.gpp_stage_run_schedule(st.handle, tasks, io, main, main)
        st.sync_status()
        st.close()


@pytest.mark.parametrize("lanes,shared", [((2, 3), False), ((4, 4), True)])
def test_lanes_in_a_captured_graph_replay_like_the_eager_run(lanes, shared):
    import torch
    from paper_2406_17145_amd.schedule import GraphedMinibatch
    wl = W.candle_uno(micro_batch=64, n_micro=6, widths=(70, 131, 9, 33), hidden=160, act="relu")
    _, res1, grads1 = _run(wl, 6, 6, False, flags=B.FLAG_GROUPED_DW)
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=6, flags=B.FLAG_GROUPED_DW)
    dev = [st.stage_inputs(mb) for mb in wl.batches]
    losses = [torch.zeros(1, dtype=torch.float32, device=st.dev) for _ in dev]
    outs = [st.alloc_outputs() for _ in dev]
    gins = [st.alloc_grad_inputs() for _ in dev]
    sched = TaskSchedule(st, 6 * wl.micro_batch, 6, two_streams=True, lanes=lanes, shared_lanes=shared)
    sched.minibatch(dev, outputs=outs, grad_inputs=gins, losses=losses)
    torch.cuda.synchronize()
    g = GraphedMinibatch(sched, dev, outputs=outs, grad_inputs=gins, losses=losses)
    for rep in range(3):
        for t in losses:
            t.zero_()                      # eager work between the replays
        for row in gins:
            for t in row:
                if t is not None:
                    t.zero_()
        torch.cuda.synchronize()
        print(f"[case] captured lanes {lanes} shared={shared}, replay {rep}", flush=True)
        g.replay()
        torch.cuda.synchronize()
        st.sync_status()
        res = [dict(loss=float(losses[j].cpu()[0]), outs={i: t2n(t) for i, t in zip(st.output_ids, outs[j])},
                    gin={i: t2n(t) for i, t in zip(st.input_ids, gins[j]) if t is not None}) for j in range(len(dev))]
        _same(res, st.grads_numpy(), res1, grads1, f"replay {rep}")
    st.close()


# ---- one-column head fused into its loss (stages with per-slot gradient buffers) -----------------------

def test_one_column_head_and_its_loss_in_one_launch():
    # Linear(K -> 1) + element-wise loss: with grouped weight gradients the loss's launch also computes the
    # Linear, the loss gradient and the gradient of the Linear's input.  Rows 1 ... 256 (one workgroup, four rows
    # of a wave in flight, ragged groups), every activation in front of the head, MSE and BCE, and sizes the
    # fusion does not take (a width that is not a multiple of 8); above 256 rows the head's workgroups leave partial
    # losses to the loss-sum launch
    for mb, hidden, act, fused in [(1, 160, "relu", True), (37, 160, "gelu", True), (64, 1000, "relu", True), (200, 72, "none", True),
                                   (8, 1536, "gelu", True), (40, 1536, "relu", True), (256, 160, "gelu", True), (300, 160, "relu", True), (701, 72, "gelu", True),
                                   (16, 100, "relu", False)]:
        wl = W.candle_uno(micro_batch=mb, n_micro=3, widths=(70, 131, 9, 33), hidden=hidden, act=act)
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=3, flags=B.FLAG_GROUPED_DW)
        launches = st.num_launches(False) + st.num_launches(True)
        st.close()
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=1)
        plain = st.num_launches(False) + st.num_launches(True)
        st.close()
        print(f"[case] {wl.name} b={mb} hidden={hidden} act={act}: {launches} launches per micro-batch (plain stage {plain})", flush=True)
        ora_stage, ora_res = run_oracle(wl)
        _, res, grads = _run(wl, 3, 3, False, reps=2, flags=B.FLAG_GROUPED_DW)
        compare(wl, res, grads, ora_stage, ora_res, label=f"head b={mb} hidden={hidden} act={act}")
        if fused:
            assert launches <= plain - 2, (launches, plain)
    wl = W.dlrm(micro_batch=128, n_micro=3, n_tables=4, num_rows=3000, bottom=(64, 32, 128), top=(128, 64, 1))
    ora_stage, ora_res = run_oracle(wl)
    print(f"[case] {wl.name} b=128 BCE head", flush=True)
    _, res, grads = _run(wl, 3, 3, True, reps=2, flags=B.FLAG_GROUPED_DW)
    compare(wl, res, grads, ora_stage, ora_res, label="dlrm BCE head")
    wl = W.dlrm(micro_batch=600, n_micro=2, n_tables=3, num_rows=2000, bottom=(64, 32, 128), top=(128, 64, 1))
    ora_stage, ora_res = run_oracle(wl)
    print(f"[case] {wl.name} b=600 tall BCE head", flush=True)
    _, res, grads = _run(wl, 2, 2, False, reps=2, flags=B.FLAG_GROUPED_DW)
    compare(wl, res, grads, ora_stage, ora_res, label="dlrm tall BCE head")


def test_forward_without_a_loss_pointer_still_seeds_the_backward_pass():
    # per-slot gradient buffers: the forward pass writes the loss gradient, also when the caller wants no loss value
    import torch
    for hidden in (160, 100):          # with and without the fused head
        wl = W.candle_uno(micro_batch=16, n_micro=2, widths=(32, 40, 8, 24), hidden=hidden, act="relu")
        ora_stage, ora_res = run_oracle(wl)
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=2, flags=B.FLAG_GROUPED_DW)
        dev = [st.stage_inputs(mb) for mb in wl.batches]
        gins = [st.alloc_grad_inputs() for _ in dev]
        io = [([t.data_ptr() for t in mb], [], None, None, [t.data_ptr() if t is not None else None for t in gins[j]])
              for j, mb in enumerate(dev)]
        main = torch.cuda.current_stream(st.dev).cuda_stream
        tasks = B.gpp_schedule_tasks(2, 2 * wl.micro_batch, 2, wl.micro_batch)
        print(f"[case] {wl.name} hidden={hidden} forward passes with loss_out = NULL", flush=True)
        B.gpp_stage_run_schedule(st.handle, tasks, io, main, main)
        st.sync_status()
        res = [dict(loss=ora_res[j][0].loss, outs={}, gin={i: t2n(t) for i, t in zip(st.input_ids, gins[j]) if t is not None})
               for j in range(2)]
        compare(wl, res, st.grads_numpy(), ora_stage, ora_res, label=f"no loss pointer hidden={hidden}")
        st.close()


def test_large_elementwise_loss_writes_its_gradient_in_the_forward_pass():
    # more loss elements than the one-workgroup loss kernel takes: the row-parallel loss kernel writes the
    # gradient as well (per-slot gradient buffers), so the backward pass has no loss launch
    for mb, dtype in [(40, "bf16"), (33, "f32")]:
        wl = W.hetero(micro_batch=mb, n_micro=3, base_width=32, out_width=64, dtype=dtype)
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=3, flags=B.FLAG_GROUPED_DW)
        bwd = st.num_launches(True)
        st.close()
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=1)
        bwd_plain = st.num_launches(True)
        st.close()
        print(f"[case] {wl.name} {dtype} b={mb}: backward launches {bwd} (plain stage {bwd_plain})", flush=True)
        ora_stage, ora_res = run_oracle(wl)
        _, res, grads = _run(wl, 3, 2, True, reps=2, flags=B.FLAG_GROUPED_DW)
        compare(wl, res, grads, ora_stage, ora_res, label=f"large loss {dtype}")


# ---- group launches: the micro-batches a run of tasks puts on one stream share one launch per step ------

def test_group_launches_give_the_one_stream_results_bit_for_bit():
    # (the last two have a head whose partial losses go through the loss-sum launch; 300 rows are five row blocks per member)
    for mb, hidden, act in [(48, 160, "gelu"), (64, 1000, "relu"), (200, 1000, "relu"), (300, 160, "relu")]:
        for n_micro, slots, lanes in ([(8, 8, 4), (7, 8, 4), (8, 8, 2), (12, 8, 4), (6, 6, 3), (5, 4, 2)] if mb != 200 else [(8, 8, 2), (7, 8, 4)]):
            wl = W.candle_uno(micro_batch=mb, n_micro=n_micro, widths=(70, 131, 9, 33), hidden=hidden, act=act)
            flags = B.FLAG_GROUPED_DW | B.FLAG_SHARED_GPU
            _, res1, grads1 = _run(wl, slots, slots, False, reps=2, flags=flags)
            st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=slots, flags=flags | B.flag_group_launches(lanes))
            assert B.gpp_stage_group_launches(st.handle) == (lanes, slots // lanes)
            st.close()
            for shared in (True, False):
                print(f"[case] {wl.name} b={mb} hidden={hidden} group launches: {n_micro} micro-batches, {slots} slots, {lanes} lanes, "
                      f"shared={shared}", flush=True)
                _, res, grads = _run(wl, slots, slots, True, reps=2, flags=flags | B.flag_group_launches(lanes), lanes=(lanes, lanes),
                                     shared_lanes=shared)
                _same(res, grads, res1, grads1, f"group launches n={n_micro} slots={slots} lanes={lanes} shared={shared}")
            # every lane on the caller's stream (no events at all), on a stage that has never seen two streams
            _, res, grads = _run(wl, slots, slots, False, reps=2, flags=flags | B.flag_group_launches(lanes), lanes=(lanes, lanes),
                                 same_stream=True)
            _same(res, grads, res1, grads1, f"group launches n={n_micro} slots={slots} lanes={lanes} on one stream")
        if hidden == 160:
            ora_stage, ora_res = run_oracle(wl)
            compare(wl, res, grads, ora_stage, ora_res, label="group launches vs oracle")


def test_group_launches_on_a_mid_pipeline_stage_and_where_they_do_not_apply():
    # a stage with outputs: the group launches carry the output, output-gradient and input-gradient pointers of all
    # their micro-batches
    wl = W.hetero(micro_batch=16, n_micro=8, base_width=64, out_width=64, dtype="bf16", with_loss=False)
    out = len(wl.ops) - 1
    rng = np.random.default_rng(12)
    gouts = [{out: rng.standard_normal((16, 512)).astype(np.float32)} for _ in range(8)]
    ora_stage, ora_res = run_oracle(wl, gouts)
    flags = B.FLAG_GROUPED_DW
    _, res1, grads1 = _run(wl, 8, 8, False, gouts=gouts, flags=flags)
    compare(wl, res1, grads1, ora_stage, ora_res, label="mid one stream")
    for lanes in (4, 2):
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=8, flags=flags | B.flag_group_launches(lanes))
        print(f"[case] {wl.name} mid-pipeline stage: group launches {B.gpp_stage_group_launches(st.handle)}", flush=True)
        assert B.gpp_stage_group_launches(st.handle) == (lanes, 8 // lanes)
        st.close()
        _, res, grads = _run(wl, 8, 8, True, gouts=gouts, flags=flags | B.flag_group_launches(lanes), lanes=(lanes, lanes), shared_lanes=True)
        _same(res, grads, res1, grads1, f"mid group launches, {lanes} lanes")
    # stages with steps that have no group form keep launching per micro-batch, whatever the flag asks for
    wl = W.dlrm(micro_batch=32, n_micro=4, n_tables=3, num_rows=500, bottom=(64, 32, 128), top=(128, 64, 1))
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=4, flags=flags | B.flag_group_launches(2))
    assert B.gpp_stage_group_launches(st.handle) == (0, 0)
    st.close()
    ora_stage, ora_res = run_oracle(wl)
    _, res, grads = _run(wl, 4, 4, True, flags=flags | B.flag_group_launches(2))
    compare(wl, res, grads, ora_stage, ora_res, label="dlrm with the group flag")


@pytest.mark.parametrize("make", [W.hetero, W.dlrm, W.mmt], ids=["hetero", "dlrm", "mmt"])
def test_full_size_single_micro_batch_workloads_as_the_benchmark_runs_them(make):
    # one micro-batch per step, serial order, the weight gradients of every layer in one launch after the backward
    # pass (stage flag bit 2) -- the configuration bench.py times for these workloads -- against the oracle in full
    wl = make()
    print(f"[case] {wl.name} full size, grouped weight gradients, serial", flush=True)
    ora_stage, ora_res = run_oracle(wl)
    _, res, grads = _run(wl, 1, 1, False, reps=2, flags=B.FLAG_GROUPED_DW)
    compare(wl, res, grads, ora_stage, ora_res, label=f"{wl.name} full size, grouped")


@pytest.mark.parametrize("make", [W.paper_candle, W.paper_mmt, W.paper_dlrm], ids=["paper_candle", "paper_mmt", "paper_dlrm"])
def test_paper_model_shapes_full_size_as_the_benchmark_runs_them(make):
    # the paper's own model shapes (appendix "DNN Model Configurations") at the sizes bench.py --config paper_* times
    # them: CANDLE-Uno 7 branches x 4 layers of 4096 at 64 rows, the multi-modal transformer 4 branches x 8 layers at
    # 2 x 256 tokens, DLRM 7 dense + 7 sparse branches (bags of 100 concatenated, 10^6-row tables) at 256 rows; one
    # micro-batch per step, serial, every weight gradient in one launch; the oracle runs once per case
    wl = make()
    print(f"[case] {wl.name} full size b={wl.micro_batch}, grouped weight gradients, serial", flush=True)
    ora_stage, ora_res = run_oracle(wl)
    _, res, grads = _run(wl, 1, 1, False, reps=2, flags=B.FLAG_GROUPED_DW)
    compare(wl, res, grads, ora_stage, ora_res, label=f"{wl.name} full size, grouped")
