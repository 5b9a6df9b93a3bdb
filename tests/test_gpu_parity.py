"""GPU parity: the HIP stage library against the CPU fp64 oracle, element by
element (norm-wise bar, see parity_util), on the same seeded inputs.  Every
call goes through the C ABI (ctypes binding)."""
import numpy as np
import pytest

from paper_2406_17145_amd import binding as B
from paper_2406_17145_amd import workloads as W
from tests.parity_util import compare, run_gpu, run_oracle

pytestmark = pytest.mark.gpu


def both(wl, gouts=None, **kw):
    print(f"[case] {wl.name} b={wl.micro_batch} Mb={wl.n_micro} ops={len(wl.ops)} kw={kw}", flush=True)
    gpu_res, gpu_grads = run_gpu(wl, gouts=gouts, **kw)
    ora_stage, ora_res = run_oracle(wl, gouts)
    worst = compare(wl, gpu_res, gpu_grads, ora_stage, ora_res, label=wl.name)
    w = max(worst.items(), key=lambda kv: kv[1][0])
    print(f"[ok] {wl.name}: worst l2-rel {w[1][0]:.2e} ({w[0]}) of {len(worst)} tensors, tol {wl.tol}", flush=True)
    return gpu_res, gpu_grads, ora_stage, ora_res


# ---- config 1 (exact) and fp32 variants of every graph family (1e-4) ----------------

def test_config1_tiny_mlp_fp32():
    both(W.tiny_mlp())


def test_config1_interleaved_schedule_two_slots():
    # 1F1B-like order over two stash slots: fw0 fw1 bw0 fw2 bw1 fw3 bw2 bw3 (satisfies C4)
    wl = W.tiny_mlp()
    sched = [("f", 0), ("f", 1), ("b", 0), ("f", 2), ("b", 1), ("f", 3), ("b", 2), ("b", 3)]
    both(wl, slots=2, schedule=sched)


def test_towers_fp32_ragged():
    both(W.candle_uno(micro_batch=37, n_micro=3, widths=(70, 131, 1, 33), hidden=100, dtype="f32"))


def test_transformer_fp32_small():
    both(W.mmt(micro_batch=3, n_micro=2, n_branches=2, n_layers=2, d_model=96, heads=4, d_ff=200,
               seq_len=70, d_head_out=50, n_classes=37, dtype="f32"))


@pytest.mark.parametrize("ragged", [False, True])
def test_dlrm_fp32_small(ragged):
    wl = W.dlrm(micro_batch=150, n_micro=2, n_dense=13, bottom=(40, 24), n_tables=5, num_rows=700,
                dim=24, bag=7, top=(60, 30, 1), dtype="f32", ragged=ragged)
    for p in wl.params.values():
        if "table" in p:
            p["table"] = p["table"] * 30
    both(wl)


def test_hetero_fp32_small_with_loss():
    both(W.hetero(micro_batch=19, n_micro=2, base_width=24, out_width=40, dtype="f32"))


def test_mid_pipeline_stage_without_loss_fp32():
    wl = W.hetero(micro_batch=9, n_micro=2, base_width=16, out_width=24, dtype="f32", with_loss=False)
    out = len(wl.ops) - 1
    rng = np.random.default_rng(5)
    gouts = [{out: rng.standard_normal((9, 192)).astype(np.float32)} for _ in range(2)]
    both(wl, gouts=gouts)


# ---- bf16 storage / fp32 accumulation (2e-2) -----------------------------------------

def test_towers_bf16_ragged():
    # smooth activation: every tile edge and ragged tail is checked with a wide margin
    both(W.candle_uno(micro_batch=37, n_micro=3, widths=(70, 131, 1, 33), hidden=100, act="gelu"))
    # ReLU masks at a size where one mask decision is a small part of a tensor
    both(W.candle_uno(micro_batch=300, n_micro=2, widths=(70, 131, 1, 33), hidden=250))


def test_transformer_bf16_small():
    both(W.mmt(micro_batch=2, n_micro=2, n_branches=2, n_layers=2, d_model=128, heads=2, d_ff=256,
               seq_len=96, d_head_out=64, n_classes=50))


def test_transformer_bf16_ragged_sequence():
    # head dimension 64 (matrix-core attention path), sequence length not a multiple of any tile
    both(W.mmt(micro_batch=3, n_micro=1, n_branches=2, n_layers=1, d_model=192, heads=3, d_ff=200,
               seq_len=83, d_head_out=40, n_classes=30))
    both(W.mmt(micro_batch=1, n_micro=1, n_branches=1, n_layers=1, d_model=64, heads=1, d_ff=64,
               seq_len=301, d_head_out=16, n_classes=5))
    # one key / query tile (the pipelined backward loop then prefetches only tiles that do not exist), one tile
    # exactly, and a second tile of a single row
    for seq_len in (20, 32, 33):
        both(W.mmt(micro_batch=2, n_micro=1, n_branches=1, n_layers=1, d_model=128, heads=2, d_ff=64,
                   seq_len=seq_len, d_head_out=16, n_classes=5))


def test_cross_entropy_row_paths():
    # the loss and its gradient keep a row of up to 1024 logits in registers, longer rows take the looping form;
    # above 16384 logits per micro-batch the loss comes from the kernel with a wave per row and partial sums
    kw = dict(n_micro=1, n_branches=1, n_layers=1, d_model=64, heads=1, d_ff=64, seq_len=8, d_head_out=32)
    both(W.mmt(micro_batch=20, n_classes=1000, **kw))
    both(W.mmt(micro_batch=12, n_classes=1500, **kw))
    both(W.mmt(micro_batch=2, n_classes=1500, **kw))
    both(W.mmt(micro_batch=3, n_classes=1024, **kw))


def test_dlrm_bf16_small():
    both(W.dlrm(micro_batch=256, n_micro=2, n_tables=6, num_rows=5000, bottom=(64, 32, 128),
                top=(128, 64, 1)))


def test_dlrm_embedding_bags_on_the_side_stream():
    # stage flag bit 3: gather and sort + segment sums on the stage's side stream next to the dense branches;
    # same kernels, same order per stream, so the results are those of the one-stream run bit for bit
    wl = W.dlrm(micro_batch=256, n_micro=3, n_tables=6, num_rows=5000, bottom=(64, 32, 128), top=(128, 64, 1))
    both(wl, flags=B.FLAG_SIDE_STREAM)
    res_a, g_a = run_gpu(wl)
    res_b, g_b = run_gpu(wl, flags=B.FLAG_SIDE_STREAM, slots=2)
    for i in g_a:
        for k in g_a[i]:
            assert np.array_equal(g_a[i][k], g_b[i][k]), (i, k)
    assert [r["loss"] for r in res_a] == [r["loss"] for r in res_b]


def test_dlrm_bf16_eleven_tables_ragged_bags():
    # eight or more tables: the gather's workgroups are laid out per table (eight tables bound to one XCD each,
    # three spread over all); 130 bags leave the last workgroup of every table half empty
    both(W.dlrm(micro_batch=130, n_micro=2, n_tables=11, num_rows=2000, bottom=(64, 32, 128), top=(128, 64, 1)))


def test_paper_dlrm_concatenated_bags():
    # the paper's DLRM shape in small: dense branches next to sparse branches whose bags are CONCATENATED
    # (ragged bags: empty, partial and full; unused slots must come out zero), bf16 and fp32 storage
    both(W.paper_dlrm(micro_batch=37, n_micro=2, n_dense=2, width=96, depth=2, n_tables=3, num_rows=700, dim=16, bag=8,
                      top=(64, 1), ragged=True))
    both(W.paper_dlrm(micro_batch=20, n_micro=2, n_dense=1, width=64, depth=1, n_tables=9, num_rows=3000, dim=64, bag=100,
                      top=(128, 1)))
    both(W.paper_dlrm(micro_batch=9, n_micro=2, n_dense=1, width=32, depth=1, n_tables=2, num_rows=300, dim=8, bag=24,
                      top=(32, 1), ragged=True, dtype="f32"))


def test_paper_model_shapes_small():
    both(W.paper_mmt(micro_batch=1, n_layers=3, d_model=128, heads=2, d_ff=256, seq_len=64, d_head_out=64, n_classes=20,
                     n_branches=2))
    both(W.paper_candle(micro_batch=33, n_micro=2, n_branches=7, width=96, depth=4))


def test_large_tile_gemm_ragged_edges():
    # many rows AND wide layers: the launches of the hidden layers go to the large-tile kernel
    # (forward, backward-data and backward-weight), with rows, columns and contraction lengths
    # that are multiples of no tile edge (1100 = 8*128 + 76, 1096 = 4*256 + 72, 264 = 4*64 + 8)
    both(W.candle_uno(micro_batch=1100, n_micro=2, widths=(512, 264, 1000, 8), hidden=1096, act="gelu"))


@pytest.mark.parametrize("act", ["gelu", "none"])
def test_direct_large_tile_loops_ragged(act):
    # launches of exactly one round of 256 x 256 tiles (4 branches x [1000 x 4000]: 4 x 16 tiles each), which
    # take the software-pipelined direct loops: forward with contraction lengths that end inside a k-step
    # (1000, 520, 264, 776) and a last row tile of 232 rows; with act "none" the backward-data launch of the
    # second level (contraction 4000 = 62 k-steps + 32) takes the direct loop too, with "gelu" its epilogue
    # multiplies by the stashed derivative and the forward epilogue writes that stash
    both(W.candle_uno(micro_batch=1000, n_micro=1, widths=(1000, 520, 264, 776), hidden=4000, depth=2, act=act))


def test_backward_weight_contraction_split_ragged():
    # many rows, small weight matrices: the backward-weight launches split the contraction over the
    # waves of a workgroup; 600 rows = 9 steps of 64 + 24, matrix edges 200 / 70 / 131 / 1 / 33
    both(W.candle_uno(micro_batch=600, n_micro=2, widths=(70, 131, 1, 33), hidden=200, act="gelu"))


@pytest.mark.parametrize("b", [1, 2, 4, 8, 16, 32, 64, 128])
def test_config5_hetero_sweep(b):
    both(W.hetero(micro_batch=b))


def test_config2_candle_uno_full():
    both(W.candle_uno())


def test_config2_overlapped_schedule_matches_serial_and_oracle():
    # the launch configuration bench.py times: forward calls on one stream, backward calls on another,
    # a stash slot per micro-batch, the whole mini-batch replayed from one HIP graph.  Backward calls stay in micro-batch order, so the accumulated gradients must be
    # bit-identical to the serial order, and they must match the oracle like the serial run does.
    import torch
    from paper_2406_17145_amd.schedule import OverlapSchedule
    wl = W.candle_uno()
    print(f"[case] {wl.name} overlapped schedule, two slots", flush=True)
    _, g_serial = run_gpu(wl)
    losses = None
    for slots in (2, wl.n_micro):      # fw_k waits for bw_{k-2}; then one slot per micro-batch (no such waits)
        if losses is not None:
            st.close()
        st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=slots)
        dev_batches = [st.stage_inputs(mb) for mb in wl.batches]
        losses = [torch.zeros(1, dtype=torch.float32, device=st.dev) for _ in wl.batches]
        gins = st.alloc_grad_inputs()
        sched = OverlapSchedule(st)
        for _ in range(3):             # repeated mini-batches: events and slots are reused
            sched.minibatch(dev_batches, outputs=[[] for _ in range(slots)], grad_inputs=gins, losses=losses)
        st.sync_status()
        g_overlap = st.grads_numpy()
        for i in g_serial:
            for k in g_serial[i]:
                assert np.array_equal(g_serial[i][k], g_overlap[i][k]), (slots, i, k)
    ora_stage, ora_res = run_oracle(wl)
    for j, (ost, _) in enumerate(ora_res):
        got = float(losses[j].cpu()[0])
        assert abs(got - ost.loss) <= wl.tol * abs(ost.loss), (j, got, ost.loss)
    # the same mini-batch as ONE captured HIP graph (what bench.py replays): every replay, with eager
    # work and synchronisations in between, must reproduce the eager gradients bit for bit
    from paper_2406_17145_amd.schedule import GraphedMinibatch
    graphed = GraphedMinibatch(sched, dev_batches, outputs=[[] for _ in range(wl.n_micro)], grad_inputs=gins, losses=losses)
    scratch = torch.zeros(1 << 20, device=st.dev)
    for rep in range(3):
        for t in st.g_t.values():              # poison the accumulators: a replay must overwrite them
            for g in t.values():
                g.fill_(float("nan"))
        for l in losses:
            l.fill_(-1.0)
        scratch.add_(1.0)                      # eager work between the replays
        torch.cuda.synchronize()
        graphed.replay()
        torch.cuda.synchronize()
        g_replay = st.grads_numpy()
        for i in g_serial:
            for k in g_serial[i]:
                assert np.array_equal(g_serial[i][k], g_replay[i][k]), (rep, i, k)
        for j, (ost, _) in enumerate(ora_res):
            got = float(losses[j].cpu()[0])
            assert abs(got - ost.loss) <= wl.tol * abs(ost.loss), (rep, j, got, ost.loss)
    st.sync_status()
    st.close()


def test_graph_replay_with_embedding_tables_matches_eager():
    # sparse path under graph replay: the gradient reset of a replay clears the rows the previous
    # replay touched (log slots), the sort buffers are reused, and the result must stay bit-identical
    import torch
    from paper_2406_17145_amd.schedule import GraphedMinibatch, SerialSchedule
    wl = W.dlrm(micro_batch=256, n_micro=2, n_tables=6, num_rows=5000, bottom=(64, 32, 128), top=(128, 64, 1))
    print(f"[case] {wl.name} graph replay, serial schedule", flush=True)
    _, g_eager = run_gpu(wl)
    st = B.Stage(wl.ops, wl.micro_batch, wl.params)
    dev_batches = [st.stage_inputs(mb) for mb in wl.batches]
    losses = [torch.zeros(1, dtype=torch.float32, device=st.dev)]
    gins = st.alloc_grad_inputs()
    sched = SerialSchedule(st)
    sched.minibatch(dev_batches, outputs=[], grad_inputs=gins, losses=losses)      # eager first
    graphed = GraphedMinibatch(sched, dev_batches, outputs=[], grad_inputs=gins, losses=losses)
    for rep in range(3):
        torch.cuda.synchronize()
        graphed.replay()
        torch.cuda.synchronize()
        g = st.grads_numpy()
        for i in g_eager:
            for k in g_eager[i]:
                assert np.array_equal(g_eager[i][k], g[i][k]), (rep, i, k)
    st.sync_status()
    st.close()


def test_config3_mmt_full():
    both(W.mmt())


def test_config4_dlrm_full():
    wl = W.dlrm()
    gpu_res, gpu_grads, st = run_gpu(wl, keep=True)
    ora_stage, ora_res = run_oracle(wl)
    compare(wl, gpu_res, gpu_grads, ora_stage, ora_res, label="dlrm")
    # integer artefacts of the sorted segment reduction: bit-exact
    for i, (sp, ur, so) in ora_res[-1][0].embedding_artefacts.items():
        g_sp, g_ur, g_so = st.embedding_sort_result(i)
        assert np.array_equal(g_sp, sp) and np.array_equal(g_ur, ur) and np.array_equal(g_so, so), i
    st.close()


# ---- embedding: integer artefacts, empty/ragged bags, determinism, index errors --------

def test_embedding_sort_artefacts_bit_exact_ragged():
    wl = W.dlrm(micro_batch=300, n_micro=1, n_tables=3, num_rows=1000, dim=16, bag=9, bottom=(8, 16),
                top=(16, 1), dtype="f32", ragged=True, seed=21)
    gpu_res, gpu_grads, st = run_gpu(wl, keep=True)
    ora_stage, ora_res = run_oracle(wl)
    compare(wl, gpu_res, gpu_grads, ora_stage, ora_res, label="dlrm-ragged")
    arte = ora_res[0][0].embedding_artefacts
    assert len(arte) == 3
    for i, (sp, ur, so) in arte.items():
        g_sp, g_ur, g_so = st.embedding_sort_result(i)
        assert np.array_equal(g_sp, sp), i
        assert np.array_equal(g_ur, ur), i
        assert np.array_equal(g_so, so), i
    st.close()


def test_embedding_all_bags_empty():
    wl = W.dlrm(micro_batch=40, n_micro=1, n_tables=2, num_rows=50, dim=8, bag=4, bottom=(8,), top=(8, 1),
                dtype="f32")
    for mb in wl.batches:
        for i, op in enumerate(wl.ops):
            if op.get("role") == "offsets":
                mb[i] = np.zeros_like(mb[i])
    both(wl)


def test_backward_is_bitwise_deterministic():
    wl = W.dlrm(micro_batch=512, n_micro=1, n_tables=4, num_rows=2000, bottom=(64, 128), top=(64, 1))
    _, g1 = run_gpu(wl)
    _, g2 = run_gpu(wl)
    for i in g1:
        for k in g1[i]:
            assert np.array_equal(g1[i][k], g2[i][k]), (i, k)


def test_out_of_range_index_is_reported_not_dereferenced():
    wl = W.dlrm(micro_batch=32, n_micro=1, n_tables=2, num_rows=64, dim=8, bag=4, bottom=(8,), top=(8, 1),
                dtype="f32")
    idx_id = next(i for i, op in enumerate(wl.ops) if op.get("role") == "indices")
    wl.batches[0][idx_id][3, 1] = 64            # == num_rows
    wl.batches[0][idx_id][5, 0] = -7
    st = B.Stage(wl.ops, wl.micro_batch, wl.params)
    st.grad_reset()
    st.forward(0, wl.batches[0])
    st.backward(0)
    with pytest.raises(B.GppError) as e:
        st.sync_status()
    assert e.value.status == B.GPP_ERR_INDEX
    st.sync_status()                            # flag is cleared by the report
    st.close()


def test_offsets_that_do_not_start_at_zero_and_labels_outside_the_classes_are_reported():
    # the bag offsets must start at 0: a first offset of 1 leaves position 0 in no bag.  The forward pass flags it; the
    # backward pass, which sorts every position below the last offset, must stay inside its buffers (the bag id it finds
    # for position 0 is whatever an earlier call left there: it is only used when it is a bag id)
    wl = W.dlrm(micro_batch=32, n_micro=1, n_tables=2, num_rows=64, dim=8, bag=4, bottom=(8,), top=(8, 1), dtype="f32")
    off_id = next(i for i, op in enumerate(wl.ops) if op.get("role") == "offsets")
    off = wl.batches[0][off_id]
    off.reshape(-1)[0] = 1
    st = B.Stage(wl.ops, wl.micro_batch, wl.params)
    st.grad_reset()
    st.forward(0, wl.batches[0])
    st.backward(0)
    with pytest.raises(B.GppError) as e:
        st.sync_status()
    assert e.value.status == B.GPP_ERR_INDEX
    st.close()
    # a class label beyond the classifier's width: no loss term for that sample, and the status says so
    wl = W.mmt(micro_batch=2, n_micro=1, n_branches=1, n_layers=1, d_model=64, heads=1, d_ff=64, seq_len=16, d_head_out=16, n_classes=5)
    lab_id = next(i for i, op in enumerate(wl.ops) if op["kind"] == "input" and op["dtype"] == "i32")
    wl.batches[0][lab_id].reshape(-1)[1] = 5
    st = B.Stage(wl.ops, wl.micro_batch, wl.params)
    st.grad_reset()
    st.forward(0, wl.batches[0])
    st.backward(0)
    with pytest.raises(B.GppError) as e:
        st.sync_status()
    assert e.value.status == B.GPP_ERR_INDEX
    st.close()


# ---- ordering condition C4 and the slot state machine ---------------------------------

def test_c4_order_violations_are_errors():
    wl = W.tiny_mlp()
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=2)
    with pytest.raises(B.GppError) as e:
        st.backward(0)                                   # bw_0 before fw_0
    assert e.value.status == B.GPP_ERR_ORDER
    st.forward(0, wl.batches[0])
    with pytest.raises(B.GppError) as e:
        st.forward(0, wl.batches[1])                     # slot still in flight
    assert e.value.status == B.GPP_ERR_ORDER
    st.forward(1, wl.batches[1])
    with pytest.raises(B.GppError) as e:
        st.backward(1)                                   # bw_1 before bw_0
    assert e.value.status == B.GPP_ERR_ORDER
    with pytest.raises(B.GppError) as e:
        st.grad_reset()                                  # micro-batches in flight
    assert e.value.status == B.GPP_ERR_ORDER
    st.backward(0)
    st.backward(1)
    st.grad_reset()
    st.sync_status()
    st.close()


def test_grad_reset_starts_new_sums():
    wl = W.tiny_mlp()
    st = B.Stage(wl.ops, wl.micro_batch, wl.params)
    for rep in range(2):
        st.grad_reset()
        for mb in wl.batches:
            st.forward(0, mb)
            st.backward(0)
        g = st.grads_numpy()
        if rep == 0:
            first = g
    for i in first:
        for k in first[i]:
            assert np.array_equal(first[i][k], g[i][k])
    st.close()


def test_generic_and_default_gemm_paths_agree_with_oracle():
    wl = W.candle_uno(micro_batch=64, n_micro=2, widths=(96, 200, 8, 64), hidden=128, act="gelu")
    both(wl, flags=B.FLAG_FORCE_GENERIC_GEMM)
    both(wl, flags=B.FLAG_SPLIT_K)
    both(wl)


def test_four_wave_few_row_kernels_agree_with_oracle():
    # stage flag bit 4 (launches that share the GPU): every tile shape of the few-row kernel, ragged K and N,
    # 1 to 256 rows, forward and backward-data, stand-alone and next to the merged backward launch
    for mb, widths, hidden, act in [(64, (96, 200, 8, 64), 128, "gelu"), (20, (942, 77, 2048, 1), 1000, "relu"),
                                    (200, (70, 131, 9, 33), 160, "gelu"), (1, (264, 131, 520, 8), 392, "relu")]:
        wl = W.candle_uno(micro_batch=mb, n_micro=2, widths=widths, hidden=hidden, act=act)
        both(wl, flags=B.FLAG_SHARED_GPU)
    both(W.hetero(micro_batch=33, n_micro=2, base_width=32, out_width=64), flags=B.FLAG_SHARED_GPU)
    both(W.hetero(micro_batch=128, n_micro=1, base_width=64, out_width=128), flags=B.FLAG_SHARED_GPU)


def test_split_k_is_deterministic_and_matches_unsplit():
    # long contraction, few output tiles: with the flag set the planner splits K across workgroups
    wl = W.candle_uno(micro_batch=48, n_micro=2, widths=(2048, 1500, 8, 64), hidden=96, act="gelu")
    _, g1 = run_gpu(wl, flags=B.FLAG_SPLIT_K)
    _, g2 = run_gpu(wl, flags=B.FLAG_SPLIT_K)
    _, g0 = run_gpu(wl)
    for i in g1:
        for k in g1[i]:
            assert np.array_equal(g1[i][k], g2[i][k]), (i, k)
            d = np.linalg.norm(g1[i][k] - g0[i][k]) / max(np.linalg.norm(g0[i][k]), 1e-30)
            assert d <= 2e-2, (i, k, d)
    both(wl, flags=B.FLAG_SPLIT_K)
