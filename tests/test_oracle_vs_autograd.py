"""Third opinion for the oracle: the same operator DAG evaluated with library
routines (torch.nn.functional, float64, CPU) and differentiated by autograd.

Every operator of the oracle reduces here to a library routine (F.linear,
F.layer_norm, F.scaled_dot_product_attention, F.embedding_bag, F.gelu,
F.cross_entropy, ...), so a dropped term, a wrong sign or a transposed operand
in the oracle's hand-written backward fails this test.  Test-only: neither the
oracle nor the product uses autograd.
"""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

from oracle import gpp_oracle as O
from paper_2406_17145_amd import workloads as W


def torch_stage(wl, batch, gout=None):
    ops, b = wl.ops, wl.micro_batch
    P = {i: {k: torch.tensor(v, dtype=torch.float64, requires_grad=True) for k, v in p.items()}
         for i, p in wl.params.items()}
    val, leaves = {}, {}
    loss = torch.zeros((), dtype=torch.float64)
    for i, op in enumerate(ops):
        k = op["kind"]
        src = [val[p] for p in op["inputs"]]
        if k == "input":
            if op["dtype"] == "i32":
                val[i] = torch.tensor(batch[i], dtype=torch.int64)
            else:
                val[i] = torch.tensor(batch[i], dtype=torch.float64,
                                      requires_grad=op.get("role") == "data")
                leaves[i] = val[i]
        elif k == "linear":
            z = F.linear(src[0], P[i]["W"], P[i].get("b"))
            val[i] = {"none": lambda t: t, "relu": F.relu, "gelu": F.gelu}[op["act"]](z)
        elif k == "layernorm":
            val[i] = F.layer_norm(src[0], (op["out_features"],), P[i]["gamma"], P[i]["beta"],
                                  op["eps"])
        elif k == "attention":
            s, h = op["seq_len"], op["heads"]
            d = op["out_features"]
            q, kk, v = (t.reshape(b, s, h, d // h).transpose(1, 2) for t in src[0].split(d, dim=1))
            o = F.scaled_dot_product_attention(q, kk, v)
            val[i] = o.transpose(1, 2).reshape(b * s, d)
        elif k == "add":
            val[i] = src[0] + src[1]
        elif k == "meanpool":
            val[i] = src[0].reshape(b, op["seq_len"], -1).mean(dim=1)
        elif k == "concat":
            val[i] = torch.cat(src, dim=1)
        elif k == "embedding_bag_sum":
            off = src[1].reshape(-1)
            val[i] = F.embedding_bag(src[0].reshape(-1)[: int(off[-1])], P[i]["table"], off[:-1],
                                     mode="sum")
        elif k == "dot_interact":
            d = op["in_features"]
            t = src[0].reshape(b, -1, d)
            gm = torch.bmm(t, t.transpose(1, 2))
            li, lj = torch.tril_indices(t.shape[1], t.shape[1], offset=-1)
            val[i] = torch.cat([t[:, 0, :], gm[:, li, lj]], dim=1)
        elif k == "loss_mse":
            loss = loss + op["loss_scale"] * F.mse_loss(src[0], src[1], reduction="sum")
        elif k == "loss_ce":
            loss = loss + op["loss_scale"] * F.cross_entropy(src[0], src[1].reshape(-1),
                                                             reduction="sum")
        elif k == "loss_bce":
            loss = loss + op["loss_scale"] * F.binary_cross_entropy_with_logits(
                src[0], src[1], reduction="sum")
        else:
            raise ValueError(k)
    total = loss
    for i, g in (gout or {}).items():
        total = total + (val[i] * torch.tensor(g)).sum()
    total.backward()
    return val, float(loss.detach()), P, leaves


def compare(wl, gout=None, rtol=1e-10):
    for mb in wl.batches:
        stage = O.OracleStage(wl.ops, wl.micro_batch, wl.params)
        st = stage.forward(mb)
        gi = stage.backward(st, gout)
        val, loss, P, leaves = torch_stage(wl, mb, gout)
        assert abs(loss - st.loss) <= rtol * max(1.0, abs(loss))
        for i in stage.output_ids:
            assert np.allclose(st.values[i], val[i].detach().numpy(), rtol=rtol, atol=1e-12)
        for i, g in stage.grads.items():
            for k in g:
                ref = P[i][k].grad
                ref = np.zeros_like(g[k]) if ref is None else ref.numpy()
                err = np.abs(g[k] - ref).max()
                assert err <= rtol * max(np.abs(ref).max(), 1e-300) + 1e-18, (i, k, err)
        assert set(gi) == {i for i in leaves if leaves[i].requires_grad}
        for i, g in gi.items():
            ref = leaves[i].grad.numpy()
            assert np.abs(g - ref).max() <= rtol * np.abs(ref).max() + 1e-18, i


def _randomise_small_params(wl, seed):
    rng = np.random.default_rng(seed)
    for p in wl.params.values():
        for k in p:
            if k in ("b", "gamma", "beta"):
                p[k] = (p[k] + 0.5 * rng.standard_normal(p[k].shape)).astype(np.float32)


def test_config1_exact():
    compare(W.tiny_mlp())


def test_towers_small_and_ragged_widths():
    wl = W.candle_uno(micro_batch=9, n_micro=2, widths=(13, 38, 20, 1), hidden=10)
    _randomise_small_params(wl, 0)
    compare(wl)


def test_transformer_small():
    wl = W.mmt(micro_batch=3, n_micro=2, n_branches=2, n_layers=2, d_model=24, heads=3, d_ff=40,
               seq_len=7, d_head_out=10, n_classes=11)
    _randomise_small_params(wl, 1)
    compare(wl, rtol=1e-9)


@pytest.mark.parametrize("ragged", [False, True])
def test_dlrm_small(ragged):
    wl = W.dlrm(micro_batch=16, n_micro=2, n_dense=13, bottom=(12, 8), n_tables=5, num_rows=30,
                dim=8, bag=6, top=(20, 10, 1), ragged=ragged)
    _randomise_small_params(wl, 2)
    for p in wl.params.values():
        if "table" in p:
            p["table"] = p["table"] * 30
    compare(wl, rtol=1e-9)


def test_hetero_small_mid_pipeline_stage():
    wl = W.hetero(micro_batch=5, n_micro=1, n_branches=8, base_width=4, out_width=6,
                  with_loss=False)
    _randomise_small_params(wl, 3)
    out = len(wl.ops) - 1
    gout = {out: np.random.default_rng(0).standard_normal((5, 48))}
    compare(wl, gout)


def test_hetero_small_with_loss():
    wl = W.hetero(micro_batch=4, n_micro=2, n_branches=8, base_width=4, out_width=6)
    compare(wl)
