"""gpp_stage_create_static: a stage whose workspace is the library's static device array (no allocation in
the call) must compute what a stage on a caller-allocated workspace computes, bit for bit -- same kernels, same
launch tables, another address -- and the oracle's values within the stated bars.  Two static stages in a row on
one GPU, the second smaller than the first (it finds the first one's leftovers in the array)."""
import numpy as np
import pytest

from paper_2406_17145_amd import binding as B
from paper_2406_17145_amd import workloads as W
from tests.parity_util import compare, run_oracle, t2n

pytestmark = pytest.mark.gpu


def run(wl, static, slots=2):
    import torch
    st = B.Stage(wl.ops, wl.micro_batch, wl.params, slots=slots, static_workspace=static)
    assert (st.ws is None) == static
    st.grad_reset()
    res = []
    for j, mb in enumerate(wl.batches):
        loss = torch.zeros(1, dtype=torch.float32, device=st.dev)
        outs, _ = st.forward(j % slots, mb, loss=loss)
        gin = st.backward(j % slots)
        res.append(dict(loss=float(loss.cpu()[0]), outs={i: t2n(t) for i, t in zip(st.output_ids, outs)},
                        gin={i: t2n(t) for i, t in zip(st.input_ids, gin) if t is not None}))
    st.sync_status()
    grads = st.grads_numpy()
    st.close()
    return res, grads


def same(a, b):
    (res_a, g_a), (res_b, g_b) = a, b
    for ra, rb in zip(res_a, res_b):
        assert ra["loss"] == rb["loss"]
        for k in ("outs", "gin"):
            assert set(ra[k]) == set(rb[k])
            for i in ra[k]:
                assert np.array_equal(ra[k][i], rb[k][i]), (k, i)
    for i in g_a:
        for k in g_a[i]:
            assert np.array_equal(g_a[i][k], g_b[i][k]), (i, k)


def test_static_workspace_stage_matches_the_caller_workspace_stage_twice_in_a_row():
    first = W.candle_uno(micro_batch=96, n_micro=3, widths=(264, 131, 520, 8), hidden=392, act="gelu")
    second = W.dlrm(micro_batch=40, n_micro=2, n_tables=3, num_rows=500, bottom=(64, 32, 128), top=(128, 64, 1))
    for wl in (first, second):      # the second, smaller stage reuses the array the first one left behind
        print(f"[case] static workspace: {wl.name} b={wl.micro_batch} x{wl.n_micro}", flush=True)
        got = run(wl, static=True)
        same(got, run(wl, static=False))
        ora_stage, ora_res = run_oracle(wl)
        compare(wl, got[0], got[1], ora_stage, ora_res, label=f"static workspace {wl.name}")


def test_static_workspace_limits_and_ownership():
    wl = W.tiny_mlp()
    a = B.Stage(wl.ops, wl.micro_batch, wl.params, static_workspace=True)
    with pytest.raises(B.GppError) as e:        # one stage per GPU holds the array
        B.Stage(wl.ops, wl.micro_batch, wl.params, static_workspace=True)
    assert e.value.status == B.GPP_ERR_ORDER
    a.close()
    b = B.Stage(wl.ops, wl.micro_batch, wl.params, static_workspace=True)      # free again after destroy
    b.close()
    big = W.candle_uno(n_micro=1)               # 8 slots of the full-size tower stage: beyond the array
    with pytest.raises(B.GppError) as e:
        B.Stage(big.ops, big.micro_batch, big.params, slots=8, flags=B.FLAG_GROUPED_DW, static_workspace=True)
    assert e.value.status == B.GPP_ERR_WORKSPACE and "static workspace" in str(e.value)
    c = B.Stage(wl.ops, wl.micro_batch, wl.params, static_workspace=True)      # a refused create leaves the array free
    c.close()
