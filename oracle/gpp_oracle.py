"""CPU fp64 oracle for one graph-pipeline-parallel stage.  TEST INFRASTRUCTURE ONLY.

Only tests, the smoke check and the benchmark's cpu_baseline leg may import
this file; the product (the HIP library and its binding) never does, and this
file imports nothing from the product.

What it computes.  A GPP stage S_i = <G_i, b_i, D_i, Pi_i> (paper section 3)
executes, per micro-batch j, a forward pass fw_j over its operator sub-graph
G_i and later the matching backward pass bw_j; intermediate activations are
kept from fw_j until bw_j (paper section 1, "in-flight" micro-batches), and,
the schedule being synchronous (paper section 6, default configuration;
section 8, synchronous pipeline parallelism keeps training semantics), weight
gradients are summed over the micro-batches of a mini-batch and weights do
not change in between.  The method approximates nothing on this path, so the
oracle is the plain definition: evaluate the operator DAG in topological
order in float64, then differentiate in reverse order, operator by operator,
with the textbook formula for each operator.  The paper names operator types
only (appendix "DNN Model Configurations": feed-forward layers, transformer
layers with multi-head attention, embedding bags, concatenation of branches,
an interaction); it states no activation, normalisation, loss or constant, so
every formula below is the textbook one and the constants are this build's
readings (listed in the design notes).

Precision: float64 throughout.  For the "bf16 storage, fp32 accumulation" mode
the stage can additionally round operator outputs to bf16 where the workload
declares bf16 storage (store_as); this is a model of storage, not of the
kernels.

Pins (tests/test_oracle_*.py): central finite differences on every operator
and on whole small stages; sum of micro-batch gradients == full-batch
gradient; branch independence; closed-form special cases; dense one-hot brute
force for the embedding backward; an independent autograd cross-check.
No function here is "parity unpinned".
"""
from __future__ import annotations

import math

import numpy as np

try:  # erf for the exact GELU; scipy is a library primitive here
    from scipy.special import erf as _erf
except Exception:  # pragma: no cover
    _erf = np.vectorize(math.erf)


# ---------------------------------------------------------------------------
# operator definitions: forward returns (output, saved); backward returns
# input gradients and adds parameter gradients into `g`
# ---------------------------------------------------------------------------

def act_fwd(z, act):
    """Activation of a feed-forward layer: identity, ReLU max(z,0), or GELU in
    its exact (erf) form z*Phi(z)."""
    if act == "none":
        return z
    if act == "relu":
        return np.maximum(z, 0.0)
    if act == "gelu":
        return 0.5 * z * (1.0 + _erf(z / math.sqrt(2.0)))
    raise ValueError(act)


def act_bwd(dy, z, act):
    """dz = dy * act'(z); ReLU' is 1 for z > 0 and 0 otherwise (0 at z == 0);
    GELU'(z) = Phi(z) + z*phi(z)."""
    if act == "none":
        return dy
    if act == "relu":
        return dy * (z > 0.0)
    if act == "gelu":
        cdf = 0.5 * (1.0 + _erf(z / math.sqrt(2.0)))
        pdf = np.exp(-0.5 * z * z) / math.sqrt(2.0 * math.pi)
        return dy * (cdf + z * pdf)
    raise ValueError(act)


def linear_fwd(x, p, op):
    """Feed-forward layer (paper appendix, model configurations): z = x W^T + b,
    y = act(z), with W stored [out_features, in_features]."""
    z = x @ p["W"].T
    if "b" in p:
        z = z + p["b"]
    return act_fwd(z, op["act"]), (x, z)


def linear_bwd(dy, saved, p, g, op):
    """dz = dy*act'(z); dx = dz W; dW += dz^T x; db += column sums of dz."""
    x, z = saved
    dz = act_bwd(dy, z, op["act"])
    g["W"] += dz.T @ x
    if "b" in p:
        g["b"] += dz.sum(axis=0)
    return [dz @ p["W"]]


def layernorm_fwd(x, p, op):
    """Normalisation over the feature dimension inside a transformer layer:
    mu = mean, var = biased variance, xhat = (x-mu)/sqrt(var+eps),
    y = gamma*xhat + beta."""
    mu = x.mean(axis=1, keepdims=True)
    var = ((x - mu) ** 2).mean(axis=1, keepdims=True)
    rstd = 1.0 / np.sqrt(var + op["eps"])
    xhat = (x - mu) * rstd
    return xhat * p["gamma"] + p["beta"], (xhat, rstd)


def layernorm_bwd(dy, saved, p, g, op):
    """dgamma += sum dy*xhat; dbeta += sum dy;
    dx = rstd*(gh - mean(gh) - xhat*mean(gh*xhat)) with gh = dy*gamma."""
    xhat, rstd = saved
    g["gamma"] += (dy * xhat).sum(axis=0)
    g["beta"] += dy.sum(axis=0)
    gh = dy * p["gamma"]
    m1 = gh.mean(axis=1, keepdims=True)
    m2 = (gh * xhat).mean(axis=1, keepdims=True)
    return [rstd * (gh - m1 - xhat * m2)]


def _split_heads(qkv, b, s, h):
    d = qkv.shape[1] // 3
    dh = d // h
    q, k, v = (qkv[:, i * d:(i + 1) * d].reshape(b, s, h, dh).transpose(0, 2, 1, 3)
               for i in range(3))
    return q, k, v, d, dh


def attention_fwd(qkv, op, b):
    """Multi-head softmax attention (paper appendix: hidden 1024, 16 heads),
    non-causal, no mask, no dropout: per sample and head
    P = softmax_rows(Q K^T / sqrt(dh)), O = P V.  The input holds Q, K, V as
    three column blocks of width d; head i owns columns [i*dh, (i+1)*dh) of each."""
    s, h = op["seq_len"], op["heads"]
    q, k, v, d, dh = _split_heads(qkv, b, s, h)
    sc = np.einsum("bhid,bhjd->bhij", q, k) / math.sqrt(dh)
    sc = sc - sc.max(axis=-1, keepdims=True)
    e = np.exp(sc)
    pr = e / e.sum(axis=-1, keepdims=True)
    o = np.einsum("bhij,bhjd->bhid", pr, v)
    return o.transpose(0, 2, 1, 3).reshape(b * s, d), (q, k, v, pr)


def attention_bwd(do, saved, op, b):
    """dV = P^T dO; dP = dO V^T; dS = P*(dP - rowsum(dP*P));
    dQ = dS K / sqrt(dh); dK = dS^T Q / sqrt(dh)."""
    s, h = op["seq_len"], op["heads"]
    q, k, v, pr = saved
    dh = q.shape[-1]
    d = h * dh
    do = do.reshape(b, s, h, dh).transpose(0, 2, 1, 3)
    dv = np.einsum("bhij,bhid->bhjd", pr, do)
    dp = np.einsum("bhid,bhjd->bhij", do, v)
    ds = pr * (dp - (dp * pr).sum(axis=-1, keepdims=True))
    dq = np.einsum("bhij,bhjd->bhid", ds, k) / math.sqrt(dh)
    dk = np.einsum("bhij,bhid->bhjd", ds, q) / math.sqrt(dh)
    out = np.empty((b * s, 3 * d))
    for i, t in enumerate((dq, dk, dv)):
        out[:, i * d:(i + 1) * d] = t.transpose(0, 2, 1, 3).reshape(b * s, d)
    return [out]


def meanpool_fwd(x, op, b):
    """Mean over the sequence positions of each sample: [b*S, d] -> [b, d]."""
    s = op["seq_len"]
    return x.reshape(b, s, -1).mean(axis=1), None


def meanpool_bwd(dy, op, b):
    s = op["seq_len"]
    return [np.repeat(dy / s, s, axis=0)]


def bag_of_position(offsets, n_used):
    """bag id of each index position j: the s with offsets[s] <= j < offsets[s+1]."""
    return (np.searchsorted(offsets, np.arange(n_used), side="right") - 1).astype(np.int64)


def embedding_bag_fwd(indices, offsets, p, op):
    """Embedding bag with sum pooling (paper appendix, DLRM sparse branches; sum
    pooling is the workload's reading): out[s,:] = sum over j in
    [offsets[s], offsets[s+1]) of table[indices[j],:], added in ascending j."""
    table = p["table"]
    idx = indices.reshape(-1)
    off = offsets.reshape(-1).astype(np.int64)
    n_bags = off.shape[0] - 1
    n_used = int(off[-1])
    if n_used and (idx[:n_used].min() < 0 or idx[:n_used].max() >= table.shape[0]):
        raise IndexError("embedding index out of range")
    bag = bag_of_position(off, n_used)
    out = np.zeros((n_bags, table.shape[1]))
    np.add.at(out, bag, table[idx[:n_used]])       # unbuffered, in order of j
    return out, (idx[:n_used].copy(), bag)


def embedding_sort(idx_used):
    """Integer artefacts of the deterministic backward: positions stably sorted
    by row (ties keep ascending original position), the distinct rows in
    ascending order, and the start of each row's segment in the sorted list."""
    sorted_pos = np.argsort(idx_used, kind="stable").astype(np.int32)
    sorted_rows = idx_used[sorted_pos]
    if sorted_rows.size == 0:
        return sorted_pos, np.zeros(0, np.int32), np.zeros(1, np.int32)
    head = np.ones(sorted_rows.shape[0], bool)
    head[1:] = sorted_rows[1:] != sorted_rows[:-1]
    starts = np.flatnonzero(head)
    unique_rows = sorted_rows[starts].astype(np.int32)
    seg_offsets = np.concatenate([starts, [sorted_rows.shape[0]]]).astype(np.int32)
    return sorted_pos, unique_rows, seg_offsets


def embedding_bag_bwd(dout, saved, g):
    """Sorted segment-sum: dTable[r,:] += sum over the positions p of row r's
    segment, in sorted (= ascending original position) order, of dout[bag(p),:]."""
    idx_used, bag = saved
    sorted_pos, unique_rows, seg_offsets = embedding_sort(idx_used)
    rows_sorted = idx_used[sorted_pos]
    np.add.at(g["table"], rows_sorted, dout[bag[sorted_pos]])
    return (sorted_pos, unique_rows, seg_offsets)


def embedding_bag_concat_fwd(indices, offsets, p, op):
    """Embedding bag whose rows are CONCATENATED (paper appendix, DLRM: the embeddings of a bag are
    concatenated): out[s, j*d:(j+1)*d] = table[indices[offsets[s] + j], :] for the j-th index of bag s;
    slots beyond the bag's length (bags may be shorter than bag_size) are zero."""
    table = p["table"]
    d, cap = table.shape[1], op["bag_size"]
    idx = indices.reshape(-1)
    off = offsets.reshape(-1).astype(np.int64)
    n_bags = off.shape[0] - 1
    n_used = int(off[-1])
    if n_used and (idx[:n_used].min() < 0 or idx[:n_used].max() >= table.shape[0]):
        raise IndexError("embedding index out of range")
    bag = bag_of_position(off, n_used)
    slot = np.arange(n_used) - off[bag]
    if n_used and slot.max() >= cap:
        raise IndexError("a bag is longer than bag_size")
    out = np.zeros((n_bags, cap, d))
    out[bag, slot] = table[idx[:n_used]]
    return out.reshape(n_bags, cap * d), (idx[:n_used].copy(), bag, slot)


def embedding_bag_concat_bwd(dout, saved, g):
    """dTable[r,:] += sum over the positions p that hold row r, in sorted (= ascending original
    position) order, of dout[bag(p), slot(p)*d:(slot(p)+1)*d]."""
    idx_used, bag, slot = saved
    d = g["table"].shape[1]
    sorted_pos, unique_rows, seg_offsets = embedding_sort(idx_used)
    pieces = dout.reshape(dout.shape[0], -1, d)[bag[sorted_pos], slot[sorted_pos]]
    np.add.at(g["table"], idx_used[sorted_pos], pieces)
    return (sorted_pos, unique_rows, seg_offsets)


def interact_terms(n_vec):
    """Strictly-lower-triangular pairs (i, j), i > j, enumerated row by row."""
    return [(i, j) for i in range(n_vec) for j in range(i)]


def dot_interact_fwd(x, op):
    """Pairwise-dot feature interaction (paper appendix: DLRM "interaction"):
    view x as F vectors of width d per sample; output = [vector 0 | <v_i, v_j>
    for i > j]."""
    d = op["in_features"]
    f = x.shape[1] // d
    t = x.reshape(-1, f, d)
    gm = np.einsum("sid,sjd->sij", t, t)
    ii = np.array([i for i, _ in interact_terms(f)], dtype=np.int64)
    jj = np.array([j for _, j in interact_terms(f)], dtype=np.int64)
    return np.concatenate([t[:, 0, :], gm[:, ii, jj]], axis=1), (t, ii, jj)


def dot_interact_bwd(dy, saved, op):
    t, ii, jj = saved
    d = op["in_features"]
    dt = np.zeros_like(t)
    dt[:, 0, :] += dy[:, :d]
    dterms = dy[:, d:]
    for n in range(ii.shape[0]):               # each term feeds both of its vectors
        i, j = ii[n], jj[n]
        dt[:, i, :] += dterms[:, n:n + 1] * t[:, j, :]
        dt[:, j, :] += dterms[:, n:n + 1] * t[:, i, :]
    return [dt.reshape(dy.shape[0], -1)]


def loss_fwd_bwd(kind, y, target, scale):
    """Loss heads with the mini-batch normalisation folded into `scale`, so that
    micro-batch gradients add up to the full-batch gradient:
      mse: L = scale * sum (y-t)^2                 dy = 2*scale*(y-t)
      ce : L = -scale * sum_s log softmax(y_s)[t_s] dy = scale*(softmax(y) - onehot)
      bce: L = scale * sum softplus(y) - t*y        dy = scale*(sigmoid(y) - t)"""
    if kind == "loss_mse":
        diff = y - target
        return scale * float((diff * diff).sum()), 2.0 * scale * diff
    if kind == "loss_ce":
        lab = target.reshape(-1).astype(np.int64)
        zs = y - y.max(axis=1, keepdims=True)
        lse = np.log(np.exp(zs).sum(axis=1, keepdims=True))
        logp = zs - lse
        rows = np.arange(y.shape[0])
        loss = -scale * float(logp[rows, lab].sum())
        dy = np.exp(logp)
        dy[rows, lab] -= 1.0
        return loss, scale * dy
    if kind == "loss_bce":
        softplus = np.maximum(y, 0.0) + np.log1p(np.exp(-np.abs(y)))
        sig = np.where(y >= 0, 1.0 / (1.0 + np.exp(-np.abs(y))),
                       np.exp(-np.abs(y)) / (1.0 + np.exp(-np.abs(y))))
        return scale * float((softplus - target * y).sum()), scale * (sig - target)
    raise ValueError(kind)


# ---------------------------------------------------------------------------
# storage precision
# ---------------------------------------------------------------------------

def store_as(x, dtype):
    """Value of x after being stored in `dtype`.  "bf16": nearest number with an
    8-bit significand, ties to even (1 sign, 8 exponent, 7 explicit fraction
    bits); anything else: unchanged.  The numeric mode "bf16 storage with fp32
    accumulation" keeps tensors between operators in bf16; the oracle models
    that storage step, and nothing else of the kernels' arithmetic, so that
    the 0/1 decisions taken from stored values (which side of a ReLU kink an
    element is on) are taken from the same numbers on both sides."""
    if dtype != "bf16":
        return x
    m, e = np.frexp(x)                       # x = m * 2^e, 0.5 <= |m| < 1
    return np.ldexp(np.rint(m * 256.0) / 256.0, e)


# ---------------------------------------------------------------------------
# the stage
# ---------------------------------------------------------------------------

def topological_order(ops):
    """Order of G_i's vertices with every producer before its consumers; raises
    on a cycle or a dangling edge (a stage's sub-graph must be a DAG)."""
    n = len(ops)
    indeg = [0] * n
    users = [[] for _ in range(n)]
    for i, op in enumerate(ops):
        for p in op["inputs"]:
            if not 0 <= p < n:
                raise ValueError("dangling edge")
            indeg[i] += 1
            users[p].append(i)
    ready = [i for i in range(n) if indeg[i] == 0]
    order = []
    while ready:
        i = ready.pop(0)
        order.append(i)
        for u in users[i]:
            indeg[u] -= 1
            if indeg[u] == 0:
                ready.append(u)
    if len(order) != n:
        raise ValueError("operator graph has a cycle")
    return order, users


class Stash:
    """Everything fw_j keeps for bw_j."""

    def __init__(self):
        self.values = {}
        self.saved = {}
        self.loss = 0.0
        self.loss_grads = {}
        self.embedding_artefacts = {}


class OracleStage:
    def __init__(self, ops, micro_batch, params, model_storage=False):
        """model_storage: round every operator output whose declared dtype is
        bf16 to bf16 (see store_as); all arithmetic stays float64."""
        self.ops = ops
        self.b = int(micro_batch)
        self.model_storage = bool(model_storage)
        self.order, self.users = topological_order(ops)
        self.params = {i: {k: np.asarray(v, dtype=np.float64) for k, v in p.items()}
                       for i, p in params.items()}
        self.grads = {}
        self.grad_reset()
        self.output_ids = [i for i, op in enumerate(ops)
                           if not self.users[i] and not op["kind"].startswith("loss")
                           and op["kind"] != "input"]

    def grad_reset(self):
        """Start of a mini-batch: weight-gradient accumulators back to zero."""
        self.grads = {i: {k: np.zeros_like(v) for k, v in p.items()}
                      for i, p in self.params.items()}

    # -- fw_j ---------------------------------------------------------------
    def forward(self, inputs):
        st = Stash()
        val = st.values
        for i in self.order:
            op = self.ops[i]
            k = op["kind"]
            src = [val[p] for p in op["inputs"]]
            if k == "input":
                a = np.asarray(inputs[i])
                val[i] = a.astype(np.float64) if op["dtype"] != "i32" else a.astype(np.int64)
            elif k == "linear":
                val[i], st.saved[i] = linear_fwd(src[0], self.params[i], op)
            elif k == "layernorm":
                val[i], st.saved[i] = layernorm_fwd(src[0], self.params[i], op)
            elif k == "attention":
                val[i], st.saved[i] = attention_fwd(src[0], op, self.b)
            elif k == "add":
                val[i] = src[0] + src[1]
            elif k == "meanpool":
                val[i], _ = meanpool_fwd(src[0], op, self.b)
            elif k == "concat":
                val[i] = np.concatenate(src, axis=1)
            elif k == "embedding_bag_sum":
                val[i], st.saved[i] = embedding_bag_fwd(src[0], src[1], self.params[i], op)
            elif k == "embedding_bag_concat":
                val[i], st.saved[i] = embedding_bag_concat_fwd(src[0], src[1], self.params[i], op)
            elif k == "dot_interact":
                val[i], st.saved[i] = dot_interact_fwd(src[0], op)
            elif k.startswith("loss"):
                loss, dy = loss_fwd_bwd(k, src[0], src[1], op["loss_scale"])
                st.loss += loss
                st.loss_grads[i] = dy
                val[i] = None
            else:
                raise ValueError(k)
            if self.model_storage and val[i] is not None and k != "input":
                val[i] = store_as(val[i], op.get("out_dtype", op.get("dtype")))
        return st

    # -- bw_j ---------------------------------------------------------------
    def backward(self, st, grad_outputs=None):
        """grad_outputs: {output op id: dL/d(output)} for outputs that leave the
        stage; returns {float input op id: dL/d(input)}."""
        grad_outputs = grad_outputs or {}
        gval = {}

        def give(p, g):
            gval[p] = g if p not in gval else gval[p] + g

        for i in self.output_ids:
            give(i, np.asarray(grad_outputs[i], dtype=np.float64))
        for i in reversed(self.order):
            op = self.ops[i]
            k = op["kind"]
            ins = op["inputs"]
            if k.startswith("loss"):
                give(ins[0], st.loss_grads[i])
                continue
            if i not in gval:
                continue
            dy = gval[i]
            if k == "input":
                continue
            if k == "linear":
                dxs = linear_bwd(dy, st.saved[i], self.params[i], self.grads[i], op)
            elif k == "layernorm":
                dxs = layernorm_bwd(dy, st.saved[i], self.params[i], self.grads[i], op)
            elif k == "attention":
                dxs = attention_bwd(dy, st.saved[i], op, self.b)
            elif k == "add":
                dxs = [dy, dy]
            elif k == "meanpool":
                dxs = meanpool_bwd(dy, op, self.b)
            elif k == "concat":
                dxs, c = [], 0
                for p in ins:
                    w = st.values[p].shape[1]
                    dxs.append(dy[:, c:c + w])
                    c += w
            elif k == "embedding_bag_sum":
                st.embedding_artefacts[i] = embedding_bag_bwd(dy, st.saved[i], self.grads[i])
                continue
            elif k == "embedding_bag_concat":
                st.embedding_artefacts[i] = embedding_bag_concat_bwd(dy, st.saved[i], self.grads[i])
                continue
            elif k == "dot_interact":
                dxs = dot_interact_bwd(dy, st.saved[i], op)
            else:
                raise ValueError(k)
            for p, dx in zip(ins, dxs):
                give(p, dx)
        return {i: gval[i] for i, op in enumerate(self.ops)
                if op["kind"] == "input" and op["dtype"] != "i32"
                and op.get("role", "data") == "data" and i in gval}


def run_minibatch(ops, micro_batch, params, batches, grad_outputs=None, model_storage=False):
    """Convenience for tests: fw_j then bw_j for j = 0..Mb-1 (a schedule that
    satisfies ordering condition C4), gradients accumulated.  Returns the
    stage and per-micro-batch (stash, input gradients)."""
    stage = OracleStage(ops, micro_batch, params, model_storage)
    results = []
    for j, mb in enumerate(batches):
        st = stage.forward(mb)
        gi = stage.backward(st, None if grad_outputs is None else grad_outputs[j])
        results.append((st, gi))
    return stage, results
