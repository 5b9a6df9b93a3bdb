"""Seeded synthetic stage workloads (graph descriptors + tensors).

This module only *describes* stages and draws their data.  It holds none of the
method's arithmetic: no forward pass, no gradient, no sort.  Both the HIP path
(through the binding) and the CPU oracle (through the tests) consume what it
produces, so the two are compared on identical inputs.

A stage is the sub-graph G_i of the operator DAG together with its micro-batch
size b_i (paper section 3, the stage tuple); the five builders below are shaped
like the paper's evaluation models (appendix "DNN Model Configurations":
multi-branch transformer, DLRM, CANDLE-Uno feature towers) but use synthetic
data throughout -- they stand in for those models, no dataset is involved.

Graph vocabulary (one dict per operator, `inputs` are producer op ids):

  input      rows = micro_batch*seq_len + rows_extra, features = out_features
  linear     y = act(x W^T + b), W is [out_features, in_features]
  layernorm  over the feature dimension, affine (gamma, beta), eps
  attention  input [b*S, 3d] = (Q|K|V) column blocks, `heads` heads, softmax(QK^T/sqrt(dh))V
  add        elementwise sum of two producers
  meanpool   mean over the seq_len rows of each sample
  concat     feature-wise concatenation
  embedding_bag_sum   inputs (indices, offsets); sums table rows per bag
  embedding_bag_concat  same inputs; concatenates the rows of a bag (in_features = row width)
  dot_interact        input [b, F*d] viewed as F vectors of d; out = [vec0 | lower-triangle dots]
  loss_mse / loss_ce / loss_bce   inputs (prediction, target)

Draw order (fixed): for each op in id order its parameters (weights, then
bias); then for each micro-batch every input op in id order.
"""
from __future__ import annotations

import math
from dataclasses import dataclass, field

import numpy as np

F32, BF16, I32 = "f32", "bf16", "i32"


def round_to_bf16(x: np.ndarray) -> np.ndarray:
    """Round float32 values to the nearest bf16-representable value (ties to even).

    The result is still float32; it is data preparation so that values handed
    to both implementations are exactly representable in bf16 storage.
    """
    x = np.ascontiguousarray(x, dtype=np.float32)
    u = x.view(np.uint32).astype(np.uint64)
    lsb = (u >> 16) & 1
    u = (u + 0x7FFF + lsb) & 0xFFFF0000
    return u.astype(np.uint32).view(np.float32).reshape(x.shape)


@dataclass
class Workload:
    name: str
    ops: list            # list of op dicts (see module docstring)
    micro_batch: int     # b_i
    n_micro: int         # micro-batches accumulated per mini-batch
    params: dict         # op id -> {"W":..,"b":..} / {"gamma","beta"} / {"table"} (float32 arrays)
    batches: list        # per micro-batch: {input op id -> array}
    tol: float           # relative tolerance of the parity bar for this numeric mode
    notes: dict = field(default_factory=dict)

    @property
    def input_ids(self):
        return [i for i, op in enumerate(self.ops) if op["kind"] == "input"]


class _Graph:
    def __init__(self):
        self.ops = []

    def add(self, kind, inputs=(), **kw):
        op = dict(kind=kind, inputs=list(inputs), branch=kw.pop("branch", -1))
        op.update(kw)
        self.ops.append(op)
        return len(self.ops) - 1

    def input(self, features, dtype, branch=-1, seq_len=1, rows_extra=0, role="data"):
        return self.add("input", (), out_features=features, dtype=dtype, branch=branch,
                        seq_len=seq_len, rows_extra=rows_extra, role=role)

    def linear(self, x, n_in, n_out, act, dtype, branch=-1, bias=True, out_dtype=None):
        return self.add("linear", (x,), in_features=n_in, out_features=n_out, act=act,
                        bias=bias, dtype=dtype, out_dtype=out_dtype or dtype, branch=branch)


def _draw_params(ops, rng, table_init=0.01):
    """Weights ~ N(0, 1/fan_in) (variance 1/fan_in), biases 0, gamma 1, beta 0,
    embedding rows ~ U(-table_init, table_init)."""
    params = {}
    for i, op in enumerate(ops):
        k = op["kind"]
        if k == "linear":
            n_in, n_out = op["in_features"], op["out_features"]
            w = rng.standard_normal((n_out, n_in)).astype(np.float32) / np.float32(math.sqrt(n_in))
            if op["dtype"] == BF16:
                w = round_to_bf16(w)
            p = {"W": w}
            if op["bias"]:
                p["b"] = np.zeros(n_out, np.float32)
            params[i] = p
        elif k == "layernorm":
            d = op["out_features"]
            params[i] = {"gamma": np.ones(d, np.float32), "beta": np.zeros(d, np.float32)}
        elif k in ("embedding_bag_sum", "embedding_bag_concat"):
            t = rng.uniform(-table_init, table_init,
                            (op["num_rows"], op["in_features"] if k == "embedding_bag_concat" else op["out_features"]))
            params[i] = {"table": t.astype(np.float32)}
    return params


def bounded_zipf_cdf(num_rows, alpha):
    r = np.arange(1, num_rows + 1, dtype=np.float64)
    p = r ** (-alpha)
    c = np.cumsum(p)
    return c / c[-1]


def _draw_batches(ops, micro_batch, n_micro, rng, samplers):
    """samplers: op id -> callable(rng, shape) -> array; default N(0,1)."""
    batches = []
    for _ in range(n_micro):
        mb = {}
        for i, op in enumerate(ops):
            if op["kind"] != "input":
                continue
            rows = micro_batch * op["seq_len"] + op["rows_extra"]
            shape = (rows, op["out_features"])
            if i in samplers:
                a = samplers[i](rng, shape)
            else:
                a = rng.standard_normal(shape).astype(np.float32)
            if op["dtype"] == BF16:
                a = round_to_bf16(a)
            elif op["dtype"] == I32:
                a = np.ascontiguousarray(a, dtype=np.int32)
            else:
                a = np.ascontiguousarray(a, dtype=np.float32)
            mb[i] = a
        batches.append(mb)
    return batches


# --------------------------------------------------------------------------
# config 1: tiny two-branch MLP, fp32
# --------------------------------------------------------------------------
def tiny_mlp(micro_batch=8, n_micro=4, seed=0, d_in=64, d_hid=128, d_out=64, n_branches=2,
             with_loss=True, dtype=F32):
    g = _Graph()
    outs = []
    for br in range(n_branches):
        x = g.input(d_in, dtype, branch=br)
        h = g.linear(x, d_in, d_hid, "relu", dtype, branch=br)
        outs.append(g.linear(h, d_hid, d_out, "none", dtype, branch=br))
    cat = g.add("concat", outs, out_features=d_out * n_branches, dtype=dtype)
    samplers = {}
    if with_loss:
        t = g.input(d_out * n_branches, F32, role="target")
        b_tot = micro_batch * n_micro
        g.add("loss_mse", (cat, t), loss_scale=0.5 / (b_tot * d_out * n_branches))
    rng = np.random.Generator(np.random.PCG64(seed))
    params = _draw_params(g.ops, rng)
    batches = _draw_batches(g.ops, micro_batch, n_micro, rng, samplers)
    return Workload("tiny_mlp", g.ops, micro_batch, n_micro, params, batches,
                    1e-4 if dtype == F32 else 2e-2)


# --------------------------------------------------------------------------
# config 2: CANDLE-Uno-shaped feature towers, bf16 storage / fp32 accumulate
# --------------------------------------------------------------------------
def candle_uno(micro_batch=64, n_micro=8, seed=2, widths=(942, 3820, 2048, 1), hidden=1000,
               depth=3, dtype=BF16, act="relu"):
    g = _Graph()
    outs = []
    for br, w in enumerate(widths):
        x = g.input(w, dtype, branch=br)
        k = w
        for _ in range(depth):
            x = g.linear(x, k, hidden, act, dtype, branch=br)
            k = hidden
        outs.append(x)
    cat_w = hidden * len(widths)
    cat = g.add("concat", outs, out_features=cat_w, dtype=dtype)
    h = g.linear(cat, cat_w, hidden, act, dtype)
    y = g.linear(h, hidden, 1, "none", dtype, out_dtype=F32)
    t = g.input(1, F32, role="target")
    g.add("loss_mse", (y, t), loss_scale=1.0 / (micro_batch * n_micro * 1))
    rng = np.random.Generator(np.random.PCG64(seed))
    params = _draw_params(g.ops, rng)
    samplers = {t: lambda r, s: r.uniform(0.0, 1.0, s).astype(np.float32)}
    batches = _draw_batches(g.ops, micro_batch, n_micro, rng, samplers)
    return Workload("candle_uno", g.ops, micro_batch, n_micro, params, batches,
                    2e-2 if dtype == BF16 else 1e-4)


# --------------------------------------------------------------------------
# config 3: multi-modal-transformer-shaped stage
# --------------------------------------------------------------------------
def mmt(micro_batch=4, n_micro=1, seed=3, n_branches=4, n_layers=2, d_model=1024, heads=16,
        d_ff=4096, seq_len=512, d_head_out=1024, n_classes=1000, dtype=BF16):
    g = _Graph()
    pooled = []
    for br in range(n_branches):
        x = g.input(d_model, dtype, branch=br, seq_len=seq_len)
        for _ in range(n_layers):
            a = g.add("layernorm", (x,), out_features=d_model, eps=1e-5, dtype=dtype, branch=br,
                      seq_len=seq_len)
            qkv = g.linear(a, d_model, 3 * d_model, "none", dtype, branch=br)
            o = g.add("attention", (qkv,), out_features=d_model, heads=heads, seq_len=seq_len,
                      dtype=dtype, branch=br)
            p = g.linear(o, d_model, d_model, "none", dtype, branch=br)
            h = g.add("add", (x, p), out_features=d_model, dtype=dtype, branch=br)
            c = g.add("layernorm", (h,), out_features=d_model, eps=1e-5, dtype=dtype, branch=br,
                      seq_len=seq_len)
            f = g.linear(c, d_model, d_ff, "gelu", dtype, branch=br)
            f2 = g.linear(f, d_ff, d_model, "none", dtype, branch=br)
            x = g.add("add", (h, f2), out_features=d_model, dtype=dtype, branch=br)
        pooled.append(g.add("meanpool", (x,), out_features=d_model, seq_len=seq_len, dtype=dtype,
                            branch=br))
    cat = g.add("concat", pooled, out_features=d_model * n_branches, dtype=dtype)
    h = g.linear(cat, d_model * n_branches, d_head_out, "none", dtype)
    z = g.linear(h, d_head_out, n_classes, "none", dtype, out_dtype=F32)
    lab = g.input(1, I32, role="target")
    g.add("loss_ce", (z, lab), loss_scale=1.0 / (micro_batch * n_micro))
    rng = np.random.Generator(np.random.PCG64(seed))
    params = _draw_params(g.ops, rng)
    samplers = {lab: lambda r, s: r.integers(0, n_classes, s)}
    batches = _draw_batches(g.ops, micro_batch, n_micro, rng, samplers)
    return Workload("mmt", g.ops, micro_batch, n_micro, params, batches,
                    2e-2 if dtype == BF16 else 1e-4)


# --------------------------------------------------------------------------
# config 4: DLRM-shaped stage
# --------------------------------------------------------------------------
def dlrm(micro_batch=2048, n_micro=1, seed=4, n_dense=13, bottom=(512, 256, 128), n_tables=26,
         num_rows=100_000, dim=128, bag=20, top=(1024, 1024, 512, 256, 1), alpha=1.05,
         pos_rate=0.03, dtype=BF16, ragged=False):
    """`ragged=True` draws a random bag length in [0, bag] per sample (empty bags
    included) instead of the fixed length; indices beyond offsets[-1] are unused."""
    g = _Graph()
    assert bottom[-1] == dim
    x = g.input(n_dense, dtype, branch=0)
    k = n_dense
    for j, w in enumerate(bottom):
        x = g.linear(x, k, w, "relu", dtype, branch=0)
        k = w
    vecs = [x]
    idx_ids, off_ids = [], []
    for t in range(n_tables):
        idx = g.input(bag, I32, branch=1 + t, role="indices")
        off = g.input(1, I32, branch=1 + t, rows_extra=1, role="offsets")
        idx_ids.append(idx)
        off_ids.append(off)
        vecs.append(g.add("embedding_bag_sum", (idx, off), out_features=dim, num_rows=num_rows,
                          bag_size=bag, dtype=dtype, branch=1 + t))
    n_vec = n_tables + 1
    cat = g.add("concat", vecs, out_features=dim * n_vec, dtype=dtype)
    n_terms = n_vec * (n_vec - 1) // 2
    z = g.add("dot_interact", (cat,), in_features=dim, out_features=dim + n_terms, dtype=dtype)
    k = dim + n_terms
    for j, w in enumerate(top):
        last = j == len(top) - 1
        z = g.linear(z, k, w, "none" if last else "relu", dtype,
                     out_dtype=F32 if last else dtype)
        k = w
    lab = g.input(1, F32, role="target")
    g.add("loss_bce", (z, lab), loss_scale=1.0 / (micro_batch * n_micro))

    rng = np.random.Generator(np.random.PCG64(seed))
    params = _draw_params(g.ops, rng)
    cdf = bounded_zipf_cdf(num_rows, alpha)
    perms = [rng.permutation(num_rows).astype(np.int32) for _ in range(n_tables)]
    state = {"lens": None}

    def make_idx(t):
        def f(r, s):
            u = r.random(s)
            rank = np.minimum(np.searchsorted(cdf, u, side="left"), num_rows - 1)
            return perms[t][rank]
        return f

    def make_off(t):
        def f(r, s):
            if ragged:
                lens = r.integers(0, bag + 1, micro_batch)
            else:
                lens = np.full(micro_batch, bag)
            return np.concatenate([[0], np.cumsum(lens)]).reshape(s)
        return f

    samplers = {x_id: make_idx(t) for t, x_id in enumerate(idx_ids)}
    samplers.update({o_id: make_off(t) for t, o_id in enumerate(off_ids)})
    samplers[0] = lambda r, s: r.lognormal(0.0, 1.0, s).astype(np.float32)
    samplers[lab] = lambda r, s: (r.random(s) < pos_rate).astype(np.float32)
    batches = _draw_batches(g.ops, micro_batch, n_micro, rng, samplers)
    return Workload("dlrm", g.ops, micro_batch, n_micro, params, batches,
                    2e-2 if dtype == BF16 else 1e-4)


# --------------------------------------------------------------------------
# config 5: heterogeneous 8-branch stage
# --------------------------------------------------------------------------
def hetero(micro_batch=128, n_micro=1, seed=7, n_branches=8, base_width=256, out_width=512,
           dtype=BF16, with_loss=True):
    """Branch i: width w_i = base_width * 2^(i mod 5); 2 + (i mod 3) layers
    Linear(w_i -> w_i) + GELU; then Linear(w_i -> out_width) without activation
    into concat slice i; tail Linear(n_branches*out_width -> same)."""
    g = _Graph()
    outs = []
    for i in range(n_branches):
        w = base_width * 2 ** (i % 5)
        x = g.input(w, dtype, branch=i)
        for _ in range(2 + (i % 3)):
            x = g.linear(x, w, w, "gelu", dtype, branch=i)
        outs.append(g.linear(x, w, out_width, "none", dtype, branch=i))
    cw = out_width * n_branches
    cat = g.add("concat", outs, out_features=cw, dtype=dtype)
    y = g.linear(cat, cw, cw, "none", dtype, out_dtype=F32 if with_loss else dtype)
    if with_loss:
        t = g.input(cw, F32, role="target")
        g.add("loss_mse", (y, t), loss_scale=1.0 / (micro_batch * n_micro * cw))
    rng = np.random.Generator(np.random.PCG64(seed))
    params = _draw_params(g.ops, rng)
    batches = _draw_batches(g.ops, micro_batch, n_micro, rng, {})
    return Workload("hetero", g.ops, micro_batch, n_micro, params, batches,
                    2e-2 if dtype == BF16 else 1e-4)


# --------------------------------------------------------------------------
# the paper's own model shapes (appendix "DNN Model Configurations"), as a second set of workloads
# --------------------------------------------------------------------------
def paper_mmt(micro_batch=2, n_micro=1, seed=13, **kw):
    """Four parallel branches of EIGHT transformer layers, sequence length 256, hidden 1024, 16 heads, FFN 4096."""
    args = dict(n_branches=4, n_layers=8, d_model=1024, heads=16, d_ff=4096, seq_len=256)
    args.update(kw)
    wl = mmt(micro_batch=micro_batch, n_micro=n_micro, seed=seed, **args)
    wl.name = "paper_mmt"
    return wl


def paper_candle(micro_batch=64, n_micro=1, seed=12, n_branches=7, width=4096, depth=4, **kw):
    """Seven branches of four feed-forward layers, hidden size 4096 (the paper names no input widths: 4096 too)."""
    wl = candle_uno(micro_batch=micro_batch, n_micro=n_micro, seed=seed, widths=(width,) * n_branches, hidden=width,
                    depth=depth, **kw)
    wl.name = "paper_candle"
    return wl


def paper_dlrm(micro_batch=256, n_micro=1, seed=14, n_dense=7, width=4096, depth=4, n_tables=7, num_rows=1_000_000,
               dim=64, bag=100, top=(4096, 4096, 1), alpha=1.05, pos_rate=0.03, dtype=BF16, ragged=False):
    """Seven dense branches (a 4096-wide feature through four feed-forward layers of 4096) and seven sparse
    branches (a table of one million rows of 64, a bag of 100 whose rows are CONCATENATED), all concatenated,
    then feed-forward layers of 4096 and a logit."""
    g = _Graph()
    outs = []
    for br in range(n_dense):
        x = g.input(width, dtype, branch=br)
        for _ in range(depth):
            x = g.linear(x, width, width, "relu", dtype, branch=br)
        outs.append(x)
    idx_ids, off_ids = [], []
    for t in range(n_tables):
        idx = g.input(bag, I32, branch=n_dense + t, role="indices")
        off = g.input(1, I32, branch=n_dense + t, rows_extra=1, role="offsets")
        idx_ids.append(idx)
        off_ids.append(off)
        outs.append(g.add("embedding_bag_concat", (idx, off), in_features=dim, out_features=bag * dim,
                          num_rows=num_rows, bag_size=bag, dtype=dtype, branch=n_dense + t))
    k = n_dense * width + n_tables * bag * dim
    z = g.add("concat", outs, out_features=k, dtype=dtype)
    for j, w in enumerate(top):
        last = j == len(top) - 1
        z = g.linear(z, k, w, "none" if last else "relu", dtype, out_dtype=F32 if last else dtype)
        k = w
    lab = g.input(1, F32, role="target")
    g.add("loss_bce", (z, lab), loss_scale=1.0 / (micro_batch * n_micro))
    rng = np.random.Generator(np.random.PCG64(seed))
    params = _draw_params(g.ops, rng)
    cdf = bounded_zipf_cdf(num_rows, alpha)
    perms = [rng.permutation(num_rows).astype(np.int32) for _ in range(n_tables)]

    def make_idx(t):
        def f(r, s):
            rank = np.minimum(np.searchsorted(cdf, r.random(s), side="left"), num_rows - 1)
            return perms[t][rank]
        return f

    def make_off(t):
        def f(r, s):
            lens = r.integers(0, bag + 1, micro_batch) if ragged else np.full(micro_batch, bag)
            return np.concatenate([[0], np.cumsum(lens)]).reshape(s)
        return f
    samplers = {x_id: make_idx(t) for t, x_id in enumerate(idx_ids)}
    samplers.update({o_id: make_off(t) for t, o_id in enumerate(off_ids)})
    samplers[lab] = lambda r, s: (r.random(s) < pos_rate).astype(np.float32)
    batches = _draw_batches(g.ops, micro_batch, n_micro, rng, samplers)
    return Workload("paper_dlrm", g.ops, micro_batch, n_micro, params, batches, 2e-2 if dtype == BF16 else 1e-4)


CONFIGS = {
    "tiny_mlp": tiny_mlp,
    "candle_uno": candle_uno,
    "mmt": mmt,
    "dlrm": dlrm,
    "hetero": hetero,
    "paper_mmt": paper_mmt,
    "paper_candle": paper_candle,
    "paper_dlrm": paper_dlrm,
}


# --------------------------------------------------------------------------
# cutting a workload's operator graph G_C into stages (paper section 3: the G_i partition G_C, C1;
# an edge of G_C between two stages becomes an edge of the stage graph, C2).  Graph surgery only.
# --------------------------------------------------------------------------
@dataclass
class StagePart:
    ops: list              # the stage's operator list (local ids)
    params: dict           # local op id -> parameter arrays
    batches: list          # per micro-batch: {local input op id -> array} (the caller's inputs only)
    global_of: list        # local op id -> op id in the whole graph (-1 for an input that an edge feeds)
    output_global: list    # global ids of the stage's outputs, in the stage's output order


def partition(wl: Workload, stage_of: dict, n_stages: int):
    """stage_of: op id -> stage, for every non-input operator; an input goes where its consumers are.
    A tensor that crosses a cut must have all its consumers in ONE other stage and none in its own (fan-out
    lives inside a stage).  Returns (parts, edges): edges are (from_stage, from_output, to_stage, to_input)."""
    ops = wl.ops
    users = {i: [] for i in range(len(ops))}
    for i, op in enumerate(ops):
        for p in op["inputs"]:
            users[p].append(i)
    st = dict(stage_of)
    for i, op in enumerate(ops):
        if op["kind"] == "input":
            homes = {st[u] for u in users[i]}
            assert len(homes) == 1, f"input {i} feeds several stages"
            st[i] = homes.pop()
    seq = {}                                   # rows per sample of every tensor
    for i, op in enumerate(ops):
        if op["kind"] == "input":
            seq[i] = op.get("seq_len", 1)
        elif op["kind"] in ("meanpool", "embedding_bag_sum", "embedding_bag_concat"):
            seq[i] = 1
        elif op["inputs"]:
            seq[i] = seq[op["inputs"][0]]
    cuts = []                                  # (producer id, consumer stage)
    for i, op in enumerate(ops):
        away = {st[u] for u in users[i]} - {st[i]}
        if away:
            assert len(away) == 1 and all(st[u] != st[i] for u in users[i]), f"tensor {i} fans out across a cut"
            cuts.append((i, away.pop()))
    parts, local = [], [dict() for _ in range(n_stages)]
    for s in range(n_stages):
        new_ops, global_of = [], []
        for (prod, cs) in cuts:                # inputs that edges feed come first, in producer order
            if cs != s:
                continue
            p = ops[prod]
            new_ops.append(dict(kind="input", inputs=[], branch=p.get("branch", -1), out_features=p["out_features"],
                                dtype=p.get("out_dtype", p["dtype"]), seq_len=seq[prod], rows_extra=0, role="data"))
            local[s][("cut", prod)] = len(new_ops) - 1
            global_of.append(-1)
        for i, op in enumerate(ops):
            if st[i] != s:
                continue
            o = dict(op)
            o["inputs"] = [local[s][p] if p in local[s] else local[s][("cut", p)] for p in op["inputs"]]
            new_ops.append(o)
            local[s][i] = len(new_ops) - 1
            global_of.append(i)
        params = {local[s][i]: p for i, p in wl.params.items() if st[i] == s}
        batches = [{local[s][i]: a for i, a in mb.items() if st[i] == s} for mb in wl.batches]
        used = {p for o in new_ops for p in o["inputs"]}
        outs = [global_of[l] for l, o in enumerate(new_ops)
                if l not in used and o["kind"] != "input" and not o["kind"].startswith("loss")]
        parts.append(StagePart(new_ops, params, batches, global_of, outs))
    edges = []
    for (prod, cs) in cuts:
        ps = st[prod]
        to_inputs = [l for l, o in enumerate(parts[cs].ops) if o["kind"] == "input"]
        edges.append((ps, parts[ps].output_global.index(prod), cs, to_inputs.index(local[cs][("cut", prod)])))
    return parts, edges
