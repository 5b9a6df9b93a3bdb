"""Pins for the CPU oracle: things fixed by mathematics, not by the oracle itself.

  P1  central finite differences (every operator, and whole small stages)
  P2  sum of micro-batch gradients == gradient of the unpipelined full batch
      (synchronous schedule: paper section 6 default configuration, section 8)
  P3  computationally independent branches do not influence each other
      (paper section 2: independent operators may run concurrently)
  P4  closed-form special cases
  P5  dense one-hot brute force for the embedding backward
"""
import copy
import math

import numpy as np
import pytest

from oracle import gpp_oracle as O
from paper_2406_17145_amd import workloads as W


# --------------------------------------------------------------------------
# helpers
# --------------------------------------------------------------------------

def stage_loss(wl, params, batch, gout=None):
    st = O.OracleStage(wl.ops, wl.micro_batch, params).forward(batch)
    loss = st.loss
    if gout:
        for i, g in gout.items():
            loss += float((st.values[i] * g).sum())
    return loss


def analytic(wl, params, batch, gout=None):
    stage = O.OracleStage(wl.ops, wl.micro_batch, params)
    st = stage.forward(batch)
    gi = stage.backward(st, gout)
    return stage, st, gi


def fd_check(wl, batch, gout=None, h=1e-6, rtol=2e-6, n_single=3, seed=0):
    """Directional and single-element central differences against backward."""
    rng = np.random.default_rng(seed)
    params = {i: {k: v.astype(np.float64) for k, v in p.items()} for i, p in wl.params.items()}
    batch = {i: (a.astype(np.float64) if a.dtype != np.int32 else a) for i, a in batch.items()}
    stage, st, gi = analytic(wl, params, batch, gout)

    # keep away from ReLU kinks
    for i, op in enumerate(wl.ops):
        if op["kind"] == "linear" and op["act"] == "relu":
            z = st.saved[i][1]
            assert np.abs(z).min() > 10 * h, "pre-activation too close to the ReLU kink; reseed"

    def check(get, setv, grad, label):
        base = get()
        dirs = [rng.standard_normal(base.shape)]
        for _ in range(n_single):
            e = np.zeros(base.size)
            e[rng.integers(base.size)] = 1.0
            dirs.append(e.reshape(base.shape))
        for d in dirs:
            setv(base + h * d)
            lp = stage_loss(wl, params, batch, gout)
            setv(base - h * d)
            lm = stage_loss(wl, params, batch, gout)
            setv(base)
            num = (lp - lm) / (2 * h)
            ana = float((grad * d).sum())
            scale = max(abs(ana), np.abs(grad).max() * 1e-3, 1e-12)
            assert abs(num - ana) <= rtol * scale + 1e-9, (label, num, ana)

    for i, p in params.items():
        for k in p:
            check(lambda i=i, k=k: params[i][k].copy(),
                  lambda v, i=i, k=k: params[i].__setitem__(k, v),
                  stage.grads[i][k], f"op{i}.{k}")
    for i, g in gi.items():
        check(lambda i=i: batch[i].copy(), lambda v, i=i: batch.__setitem__(i, v), g, f"input{i}")
    return stage, gi


def widen_relu_margin(wl, margin=1e-4):
    """Reseed-free way to stay off ReLU kinks: nudge biases where needed."""
    for _ in range(20):
        st = O.OracleStage(wl.ops, wl.micro_batch, wl.params).forward(wl.batches[0])
        ok = True
        for i, op in enumerate(wl.ops):
            if op["kind"] == "linear" and op["act"] == "relu":
                z = st.saved[i][1]
                if np.abs(z).min() <= margin:
                    wl.params[i]["b"] = wl.params[i]["b"] + np.float32(3.3e-3)
                    ok = False
        if ok:
            return
    raise AssertionError("could not clear ReLU kinks")


# --------------------------------------------------------------------------
# P1 finite differences
# --------------------------------------------------------------------------

def test_fd_config1_whole():
    wl = W.tiny_mlp()           # config 1 exactly: seed 0, b=8, 4 micro-batches
    widen_relu_margin(wl)
    for mb in wl.batches[:2]:
        fd_check(wl, mb)


def test_fd_small_towers():
    wl = W.candle_uno(micro_batch=5, n_micro=1, widths=(7, 12, 3, 1), hidden=6, depth=3)
    widen_relu_margin(wl)
    fd_check(wl, wl.batches[0])


def test_fd_small_transformer():
    wl = W.mmt(micro_batch=2, n_micro=1, n_branches=2, n_layers=2, d_model=8, heads=2, d_ff=16,
               seq_len=5, d_head_out=6, n_classes=7)
    # make gamma/beta/biases non-trivial so their gradients are exercised
    rng = np.random.default_rng(1)
    for p in wl.params.values():
        for k in p:
            if k in ("b", "gamma", "beta"):
                p[k] = (p[k] + 0.3 * rng.standard_normal(p[k].shape)).astype(np.float32)
    fd_check(wl, wl.batches[0], rtol=5e-6)


@pytest.mark.parametrize("ragged", [False, True])
def test_fd_small_dlrm(ragged):
    wl = W.dlrm(micro_batch=6, n_micro=1, n_dense=5, bottom=(7, 4), n_tables=3, num_rows=11,
                dim=4, bag=3, top=(9, 5, 1), ragged=ragged, seed=11)
    for p in wl.params.values():            # larger table values -> non-negligible interaction
        if "table" in p:
            p["table"] = p["table"] * 50
    widen_relu_margin(wl)
    fd_check(wl, wl.batches[0], rtol=5e-6)


def test_fd_small_hetero_without_loss():
    wl = W.hetero(micro_batch=3, n_micro=1, n_branches=4, base_width=4, out_width=3,
                  with_loss=False)
    out_id = len(wl.ops) - 1
    gout = {out_id: np.random.default_rng(5).standard_normal((3, 12))}
    fd_check(wl, wl.batches[0], gout=gout, rtol=5e-6)


def test_fd_each_loss_head():
    rng = np.random.default_rng(0)
    y = rng.standard_normal((4, 5))
    h = 1e-6
    for kind, tgt in (("loss_mse", rng.standard_normal((4, 5))),
                      ("loss_ce", rng.integers(0, 5, (4, 1))),
                      ("loss_bce", (rng.random((4, 5)) < 0.5).astype(float))):
        _, dy = O.loss_fwd_bwd(kind, y, tgt, 0.37)
        for _ in range(5):
            d = rng.standard_normal(y.shape)
            lp, _ = O.loss_fwd_bwd(kind, y + h * d, tgt, 0.37)
            lm, _ = O.loss_fwd_bwd(kind, y - h * d, tgt, 0.37)
            assert abs((lp - lm) / (2 * h) - (dy * d).sum()) < 1e-8


def test_gelu_derivative_and_values():
    z = np.linspace(-4, 4, 41)
    h = 1e-6
    num = (O.act_fwd(z + h, "gelu") - O.act_fwd(z - h, "gelu")) / (2 * h)
    assert np.allclose(num, O.act_bwd(np.ones_like(z), z, "gelu"), atol=1e-8)
    # exact form: GELU(z) = z * Phi(z); Phi(1) = 0.841344746...
    assert abs(O.act_fwd(np.array([1.0]), "gelu")[0] - 0.8413447460685429) < 1e-12
    assert O.act_fwd(np.array([0.0]), "gelu")[0] == 0.0


# --------------------------------------------------------------------------
# P2 accumulation invariant
# --------------------------------------------------------------------------

def _full_batch(wl):
    ops = copy.deepcopy(wl.ops)
    merged = {}
    for i in wl.input_ids:
        merged[i] = np.concatenate([mb[i] for mb in wl.batches], axis=0)
    return ops, merged


@pytest.mark.parametrize("make", [
    lambda: W.tiny_mlp(),
    lambda: W.candle_uno(micro_batch=16, n_micro=4, widths=(30, 50, 20, 1), hidden=24),
    lambda: W.mmt(micro_batch=2, n_micro=3, n_branches=2, n_layers=1, d_model=16, heads=2,
                  d_ff=32, seq_len=6, d_head_out=8, n_classes=5),
    lambda: W.hetero(micro_batch=4, n_micro=2, n_branches=5, base_width=4, out_width=6),
])
def test_sum_of_microbatch_grads_equals_full_batch_grad(make):
    wl = make()
    stage, res = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches)
    ops, merged = _full_batch(wl)
    full = O.OracleStage(ops, wl.micro_batch * wl.n_micro, wl.params)
    st = full.forward(merged)
    gi_full = full.backward(st)
    assert abs(sum(r[0].loss for r in res) - st.loss) <= 1e-12 * max(1.0, abs(st.loss))
    for i, g in stage.grads.items():
        for k in g:
            ref = full.grads[i][k]
            assert np.abs(g[k] - ref).max() <= 1e-12 * max(np.abs(ref).max(), 1e-30), (i, k)
    for i in gi_full:
        stacked = np.concatenate([r[1][i] for r in res], axis=0)
        assert np.abs(stacked - gi_full[i]).max() <= 1e-12 * np.abs(gi_full[i]).max()


# --------------------------------------------------------------------------
# P3 branch independence
# --------------------------------------------------------------------------

def test_branches_are_independent():
    wl = W.hetero(micro_batch=4, n_micro=1, n_branches=4, base_width=4, out_width=3,
                  with_loss=False)
    out_id = len(wl.ops) - 1
    cat_id = out_id - 1
    # cut the tail off: look at the concat and at the branch weight gradients,
    # with an upstream gradient that is fixed
    ops = wl.ops[:cat_id + 1]
    params = {i: p for i, p in wl.params.items() if i <= cat_id}
    gout = {cat_id: np.random.default_rng(3).standard_normal((4, 12))}
    stage, st, gi = analytic(W.Workload("x", ops, 4, 1, params, wl.batches, 0), params,
                             wl.batches[0], gout)
    batch2 = dict(wl.batches[0])
    first_in = wl.input_ids[0]
    batch2[first_in] = batch2[first_in] + 1.0
    params2 = copy.deepcopy(params)
    first_lin = next(i for i, op in enumerate(ops) if op["kind"] == "linear" and op["branch"] == 0)
    params2[first_lin]["W"] = params2[first_lin]["W"] * 2
    stage2, st2, gi2 = analytic(W.Workload("x", ops, 4, 1, params2, wl.batches, 0), params2,
                                batch2, gout)
    changed = False
    for i, op in enumerate(ops):
        if op["kind"] != "linear":
            continue
        same = np.array_equal(stage.grads[i]["W"], stage2.grads[i]["W"])
        if op["branch"] == 0:
            changed |= not same
        else:
            assert same, f"branch {op['branch']} was influenced by branch 0"
            assert np.array_equal(st.values[i], st2.values[i])
    assert changed
    # one branch at a time == all together
    for br in range(4):
        keep = [i for i, op in enumerate(ops) if op["branch"] == br]
        remap = {old: new for new, old in enumerate(keep)}
        sub = []
        for i in keep:
            o = dict(ops[i])
            o["inputs"] = [remap[p] for p in o["inputs"]]
            sub.append(o)
        sp = {remap[i]: params[i] for i in keep if i in params}
        sb = {remap[i]: wl.batches[0][i] for i in keep if i in wl.batches[0]}
        s = O.OracleStage(sub, 4, sp)
        sst = s.forward(sb)
        last = len(sub) - 1
        s.backward(sst, {last: gout[cat_id][:, 3 * br:3 * br + 3]})
        assert np.array_equal(sst.values[last], st.values[cat_id][:, 3 * br:3 * br + 3])
        for i in keep:
            if i in params:
                assert np.array_equal(s.grads[remap[i]]["W"], stage.grads[i]["W"])


# --------------------------------------------------------------------------
# P4 closed forms
# --------------------------------------------------------------------------

def test_linear_identity_weight():
    x = np.random.default_rng(0).standard_normal((5, 4))
    op = dict(act="none")
    p = {"W": np.eye(4), "b": np.arange(4.0)}
    y, saved = O.linear_fwd(x, p, op)
    assert np.array_equal(y, x + np.arange(4.0))
    g = {"W": np.zeros((4, 4)), "b": np.zeros(4)}
    dy = np.ones((5, 4))
    (dx,) = O.linear_bwd(dy, saved, p, g, op)
    assert np.array_equal(dx, dy)
    assert np.allclose(g["W"], np.ones((4, 5)) @ x)     # dW[n,k] = sum_m dz[m,n] x[m,k]
    assert np.array_equal(g["b"], np.full(4, 5.0))


def test_linear_weight_is_out_by_in_not_transposed():
    # a non-square case where a transposed operand cannot go unnoticed
    x = np.array([[1.0, 2.0, 3.0]])
    p = {"W": np.array([[1.0, 0.0, 0.0], [0.0, 0.0, 2.0]])}
    y, _ = O.linear_fwd(x, p, dict(act="none"))
    assert np.array_equal(y, [[1.0, 6.0]])


def test_attention_equal_keys_gives_mean_of_values_and_zero_dq():
    rng = np.random.default_rng(0)
    b, s, h, dh = 2, 6, 2, 4
    d = h * dh
    qkv = rng.standard_normal((b * s, 3 * d))
    krow = rng.standard_normal(d)
    qkv[:, d:2 * d] = krow                   # all keys equal -> uniform probabilities
    op = dict(seq_len=s, heads=h)
    o, saved = O.attention_fwd(qkv, op, b)
    v = qkv[:, 2 * d:].reshape(b, s, d)
    assert np.allclose(o.reshape(b, s, d), np.repeat(v.mean(axis=1, keepdims=True), s, axis=1))
    (dqkv,) = O.attention_bwd(rng.standard_normal((b * s, d)), saved, op, b)
    assert np.abs(dqkv[:, :d]).max() < 1e-14          # dQ = 0
    # single-token sequences: P = 1, O = V, dV = dO
    qkv1 = rng.standard_normal((3, 3 * d))
    o1, sv1 = O.attention_fwd(qkv1, dict(seq_len=1, heads=h), 3)
    assert np.allclose(o1, qkv1[:, 2 * d:])
    do = rng.standard_normal((3, d))
    (dq1,) = O.attention_bwd(do, sv1, dict(seq_len=1, heads=h), 3)
    assert np.allclose(dq1[:, 2 * d:], do) and np.abs(dq1[:, :2 * d]).max() < 1e-14


def test_attention_heads_and_samples_do_not_mix():
    rng = np.random.default_rng(1)
    b, s, h, dh = 2, 3, 2, 2
    d = h * dh
    qkv = rng.standard_normal((b * s, 3 * d))
    op = dict(seq_len=s, heads=h)
    o, _ = O.attention_fwd(qkv, op, b)
    # by hand for sample 1, head 1
    rows = slice(s, 2 * s)
    q = qkv[rows, 0 * d + dh:0 * d + 2 * dh]
    k = qkv[rows, 1 * d + dh:1 * d + 2 * dh]
    v = qkv[rows, 2 * d + dh:2 * d + 2 * dh]
    sc = q @ k.T / math.sqrt(dh)
    p = np.exp(sc) / np.exp(sc).sum(axis=1, keepdims=True)
    assert np.allclose(o[rows, dh:2 * dh], p @ v)


def test_softmax_ce_gradient_rows_sum_to_zero_and_uniform_logits():
    rng = np.random.default_rng(0)
    z = rng.standard_normal((6, 9))
    lab = rng.integers(0, 9, (6, 1))
    loss, dz = O.loss_fwd_bwd("loss_ce", z, lab, 1.0 / 6)
    assert np.abs(dz.sum(axis=1)).max() < 1e-15
    loss0, _ = O.loss_fwd_bwd("loss_ce", np.zeros((6, 9)), lab, 1.0 / 6)
    assert abs(loss0 - math.log(9)) < 1e-14


def test_bce_at_zero_logit_and_mse_at_target():
    y = np.zeros((4, 1))
    t = np.array([[0.0], [1.0], [1.0], [0.0]])
    loss, dy = O.loss_fwd_bwd("loss_bce", y, t, 0.25)
    assert abs(loss - math.log(2.0)) < 1e-15
    assert np.allclose(dy, 0.25 * (0.5 - t))
    # large |logit| stays finite and matches the asymptote
    big, dbig = O.loss_fwd_bwd("loss_bce", np.array([[800.0], [-800.0]]), np.array([[1.0], [0.0]]), 1.0)
    assert big == 0.0 and np.abs(dbig).max() == 0.0
    l2, d2 = O.loss_fwd_bwd("loss_mse", t, t, 3.0)
    assert l2 == 0.0 and not d2.any()
    wl = W.tiny_mlp()
    st = O.OracleStage(wl.ops, 8, wl.params).forward(wl.batches[0])
    tid = next(i for i, op in enumerate(wl.ops) if op.get("role") == "target")
    cat = next(i for i, op in enumerate(wl.ops) if op["kind"] == "concat")
    mb = dict(wl.batches[0])
    mb[tid] = st.values[cat]
    stage, st2, gi = analytic(wl, wl.params, mb)
    assert st2.loss == 0.0
    assert all(not g[k].any() for g in stage.grads.values() for k in g)


def test_layernorm_properties():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((7, 16)) * 3 + 1
    op = dict(eps=1e-5)
    p = {"gamma": np.ones(16), "beta": np.zeros(16)}
    y, saved = O.layernorm_fwd(x, p, op)
    var = x.var(axis=1)
    assert np.abs(y.mean(axis=1)).max() < 1e-14
    assert np.allclose(y.var(axis=1), var / (var + 1e-5), rtol=1e-12)
    g = {"gamma": np.zeros(16), "beta": np.zeros(16)}
    dy = rng.standard_normal((7, 16))
    (dx,) = O.layernorm_bwd(dy, saved, p, g, op)
    assert np.abs(dx.sum(axis=1)).max() < 1e-13
    assert np.allclose(g["beta"], dy.sum(axis=0))
    # a constant shift of the input changes nothing
    y2, _ = O.layernorm_fwd(x + 5.0, p, op)
    assert np.allclose(y, y2, atol=1e-12)


def test_meanpool_and_concat_and_add():
    x = np.arange(24.0).reshape(6, 4)
    y, _ = O.meanpool_fwd(x, dict(seq_len=3), 2)
    assert np.array_equal(y, np.stack([x[:3].mean(0), x[3:].mean(0)]))
    (dx,) = O.meanpool_bwd(np.ones((2, 4)), dict(seq_len=3), 2)
    assert np.allclose(dx, np.full((6, 4), 1 / 3))


def test_interaction_orthonormal_vectors_give_zero_terms_and_term_order():
    d, f = 8, 5
    t = np.eye(d)[:f]                      # f orthonormal vectors
    x = np.tile(t.reshape(1, -1), (3, 1))
    y, _ = O.dot_interact_fwd(x, dict(in_features=d))
    assert y.shape == (3, d + f * (f - 1) // 2)
    assert np.array_equal(y[:, :d], x[:, :d])
    assert not y[:, d:].any()
    # order (1,0),(2,0),(2,1),(3,0)...
    assert O.interact_terms(4) == [(1, 0), (2, 0), (2, 1), (3, 0), (3, 1), (3, 2)]
    v = np.arange(1.0, 7.0).reshape(1, 6)            # three vectors of width 2
    y2, _ = O.dot_interact_fwd(v, dict(in_features=2))
    assert np.array_equal(y2[0], [1, 2, 1 * 3 + 2 * 4, 1 * 5 + 2 * 6, 3 * 5 + 4 * 6])
    assert 27 * 26 // 2 == 351 and 128 + 351 == 479      # the DLRM-shaped config's counts


def test_embedding_distinct_indices_is_a_scatter_and_column_sum_identity():
    rng = np.random.default_rng(0)
    rows, dim, nb, bag = 40, 5, 6, 3
    table = rng.standard_normal((rows, dim))
    idx = rng.permutation(rows)[:nb * bag].astype(np.int32)
    off = np.arange(0, nb * bag + 1, bag, dtype=np.int32)
    out, saved = O.embedding_bag_fwd(idx, off, {"table": table}, {})
    assert np.allclose(out, table[idx].reshape(nb, bag, dim).sum(axis=1))
    dout = rng.standard_normal((nb, dim))
    g = {"table": np.zeros_like(table)}
    O.embedding_bag_bwd(dout, saved, g)
    for j, r in enumerate(idx):
        assert np.array_equal(g["table"][r], dout[j // bag])
    assert np.count_nonzero(g["table"].any(axis=1)) == nb * bag
    # with repeats: column sums of dTable == sum_j dout[bag(j)]
    idx2 = rng.integers(0, 4, nb * bag).astype(np.int32)
    out2, saved2 = O.embedding_bag_fwd(idx2, off, {"table": table}, {})
    g2 = {"table": np.zeros_like(table)}
    O.embedding_bag_bwd(dout, saved2, g2)
    assert np.allclose(g2["table"].sum(axis=0), bag * dout.sum(axis=0))


# --------------------------------------------------------------------------
# P5 brute force for the embedding path
# --------------------------------------------------------------------------

@pytest.mark.parametrize("seed", [0, 1, 2])
def test_embedding_backward_matches_one_hot_brute_force(seed):
    rng = np.random.default_rng(seed)
    rows, dim, nb = 9, 3, 7
    lens = rng.integers(0, 5, nb)                   # includes empty bags
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    cap = int(off[-1]) + 4                          # unused tail capacity
    idx = rng.integers(0, rows, cap).astype(np.int32)
    table = rng.standard_normal((rows, dim))
    out, saved = O.embedding_bag_fwd(idx, off, {"table": table}, {})
    # forward by explicit loops
    ref = np.zeros((nb, dim))
    for s in range(nb):
        for j in range(off[s], off[s + 1]):
            ref[s] += table[idx[j]]
    assert np.allclose(out, ref, atol=1e-15)
    dout = rng.standard_normal((nb, dim))
    g = {"table": np.zeros_like(table)}
    sorted_pos, unique_rows, seg_offsets = O.embedding_bag_bwd(dout, saved, g)
    n = int(off[-1])
    onehot = np.zeros((n, rows))
    onehot[np.arange(n), idx[:n]] = 1.0
    bag = np.repeat(np.arange(nb), lens)
    assert np.allclose(g["table"], onehot.T @ dout[bag], atol=1e-14)
    # integer artefacts by brute force
    pairs = sorted((int(idx[j]), j) for j in range(n))
    assert [p[1] for p in pairs] == sorted_pos.tolist()
    assert sorted(set(idx[:n].tolist())) == unique_rows.tolist()
    counts = [sum(1 for r, _ in pairs if r == u) for u in unique_rows]
    assert np.array_equal(seg_offsets, np.concatenate([[0], np.cumsum(counts)]))


@pytest.mark.parametrize("seed", [0, 1, 2])
def test_concatenated_embedding_bag_matches_loops_and_one_hot_brute_force(seed):
    # the paper's DLRM concatenates the rows of a bag: slot j of sample s holds the row of its j-th index
    rng = np.random.default_rng(seed)
    rows, dim, nb, cap = 11, 3, 6, 4
    lens = rng.integers(0, cap + 1, nb)             # empty, partial and full bags
    off = np.concatenate([[0], np.cumsum(lens)]).astype(np.int32)
    idx = rng.integers(0, rows, nb * cap).astype(np.int32)
    table = rng.standard_normal((rows, dim))
    out, saved = O.embedding_bag_concat_fwd(idx, off, {"table": table}, {"bag_size": cap})
    ref = np.zeros((nb, cap * dim))
    for s in range(nb):
        for j in range(off[s], off[s + 1]):
            ref[s, (j - off[s]) * dim:(j - off[s] + 1) * dim] = table[idx[j]]
    assert np.array_equal(out, ref)
    # summing the slots of the concatenated bag gives the sum-pooled bag
    pooled, _ = O.embedding_bag_fwd(idx, off, {"table": table}, {})
    assert np.allclose(out.reshape(nb, cap, dim).sum(axis=1), pooled, atol=1e-15)
    dout = rng.standard_normal((nb, cap * dim))
    g = {"table": np.zeros_like(table)}
    sorted_pos, unique_rows, seg_offsets = O.embedding_bag_concat_bwd(dout, saved, g)
    n = int(off[-1])
    onehot = np.zeros((n, rows))
    onehot[np.arange(n), idx[:n]] = 1.0
    piece = np.stack([dout[s, (j - off[s]) * dim:(j - off[s] + 1) * dim] for s in range(nb) for j in range(off[s], off[s + 1])]) \
        if n else np.zeros((0, dim))
    assert np.allclose(g["table"], onehot.T @ piece, atol=1e-14)
    # the gradient is linear in dout: <dTable, dT> == <dout, d out / d table [dT]> for a random direction
    dT = rng.standard_normal(table.shape)
    out_dir, _ = O.embedding_bag_concat_fwd(idx, off, {"table": dT}, {"bag_size": cap})
    assert np.isclose((g["table"] * dT).sum(), (dout * out_dir).sum(), atol=1e-12)
    assert [p[1] for p in sorted((int(idx[j]), j) for j in range(n))] == sorted_pos.tolist()


def test_concatenated_embedding_bag_rejects_a_bag_longer_than_its_capacity():
    with pytest.raises(IndexError):
        O.embedding_bag_concat_fwd(np.zeros(6, np.int32), np.array([0, 3], np.int32), {"table": np.zeros((4, 2))}, {"bag_size": 2})


def test_embedding_rejects_out_of_range_index():
    with pytest.raises(IndexError):
        O.embedding_bag_fwd(np.array([0, 9], np.int32), np.array([0, 2], np.int32),
                            {"table": np.zeros((9, 2))}, {})


def test_graph_validation():
    with pytest.raises(ValueError):
        O.topological_order([dict(kind="add", inputs=[1, 1]), dict(kind="add", inputs=[0, 0])])
    with pytest.raises(ValueError):
        O.topological_order([dict(kind="add", inputs=[5, 5])])


# --------------------------------------------------------------------------
# storage model
# --------------------------------------------------------------------------

def test_store_as_bf16_rounds_to_nearest_even_on_8_bit_significands():
    x = np.array([1.0, 1.0 + 2.0 ** -7, 1.0 + 2.0 ** -8, 1.0 + 3 * 2.0 ** -8, 1.0 + 2.0 ** -8 + 2.0 ** -20,
                  -3.1415926, 0.0, 2.0 ** -100, 65504.0])
    r = O.store_as(x, "bf16")
    assert r[0] == 1.0 and r[1] == 1.0 + 2.0 ** -7
    assert r[2] == 1.0                      # tie -> even significand
    assert r[3] == 1.0 + 2.0 ** -6          # tie -> even significand (1.0000010b)
    assert r[4] == 1.0 + 2.0 ** -7          # just above the tie
    assert r[5] == -3.140625 and r[6] == 0.0 and r[7] == 2.0 ** -100
    assert r[8] == 65536.0
    # agrees with the float32-bit-pattern formulation used for input generation
    v = np.random.default_rng(0).standard_normal(10000).astype(np.float32)
    assert np.array_equal(O.store_as(v.astype(np.float64), "bf16"), W.round_to_bf16(v).astype(np.float64))
    assert O.store_as(x, "f32") is x
    # idempotent, and inert for fp32 workloads
    assert np.array_equal(O.store_as(r, "bf16"), r)
    wl = W.tiny_mlp()
    a, _ = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches, model_storage=True)
    b, _ = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches)
    assert all(np.array_equal(a.grads[i][k], b.grads[i][k]) for i in a.grads for k in a.grads[i])


@pytest.mark.parametrize("which", ["candle_uno", "dlrm"])
def test_relu_mask_noise_floor(which):
    """Input gradients of a bf16-storage ReLU stack are decided by a few mask bits
    (tests/relu_noise.py).  The oracle with its Linear products re-ordered in float32 (nothing
    else changed) is measured against itself on ALL micro-batches of the two full-size workloads
    that have ReLU layers; the figures the GPU parity bars are derived from
    (tests/parity_bars.py) must bracket that measurement from both sides.  Weight gradients,
    summed over the mini-batch, stay far inside the stated bar."""
    from tests import parity_bars as PB
    from tests.relu_noise import measure
    wl = W.candle_uno() if which == "candle_uno" else W.dlrm()
    # the recommendation model's oracle run takes half a minute: two of the four orders there
    m = measure(wl) if which == "candle_uno" else measure(wl, ("blas", "blk64g"))
    pinned = PB.RELU_SPREAD_PINNED[PB.workload_key(wl)]
    print(f"[relu noise] {which}: l2 {m['l2']:.3e} max-norm {m['max']:.3e} rows over 2e-2 {m['rows_over']:.4f} "
          f"weight gradients {m['dw']:.3e}; opposite decisions at most {m['flips']} of {m['decisions']}, "
          f"{m['near_zero']} pre-activations within one bf16 step of zero")
    for k in ("l2", "max", "rows_over", "dw") + (("dt",) if which == "dlrm" else ()):
        assert pinned[k] / PB.BAND <= m[k] <= pinned[k] * PB.BAND, (k, m[k], pinned[k])
    assert 0 < m["flips"] < 1e-4 * m["decisions"] and m["flips"] < m["near_zero"]
    assert m["dw"] < 0.5 * PB.STATED_L2["bf16"] and PB.relu_dw_bar(pinned) == PB.STATED_L2["bf16"]   # weight gradients: stated bar
    # what follows for the GPU bars: the recommendation model needs no exception at all
    b2, bm, _ = PB.relu_gin_bars(pinned, wl.micro_batch)
    if which == "dlrm":
        assert b2 == PB.STATED_L2["bf16"] and bm == PB.STATED_MAX["bf16"]
    else:
        assert PB.STATED_L2["bf16"] < b2 < 3.3e-2
