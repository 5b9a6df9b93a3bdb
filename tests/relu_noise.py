"""How far the INPUT gradients of a bf16-storage ReLU graph move when nothing but the
floating-point order of the matrix products changes.  CPU only, oracle only.

Why this exists.  With bf16 storage a ReLU mask is decided from a rounded value: the
float32 sum of a layer lands on one or the other side of a bf16 rounding boundary of
the stored activation depending on the ORDER of the sum, the next layer's
pre-activations then differ by a few 1e-4, and the few of them that sit that close to
zero get opposite masks.  One opposite decision changes one sample's whole gradient
row by the weight of that unit (several percent of the row).  No kernel can avoid
this, and the fp64 oracle takes just one of the possible decisions.  The parity bar of
those tensors is therefore derived from the spread that the oracle itself shows under
re-ordered float32 sums (`measure`), not from a chosen number.

The variants change ONLY the arithmetic of Linear (paper appendix: feed-forward
layers); everything else of the oracle runs as it is:

  blas     float32 product by the BLAS (its own blocking)
  blk64    float32, contraction in steps of 64 added one after the other
  split8   float32, contraction cut into 8 parts, each summed in steps of 32, parts
           combined pairwise
  blk64g   blk64, and the gradient handed to the producer rounded to bf16 (gradients
           stored in the storage type, like the activations)
"""
import numpy as np

from oracle import gpp_oracle as O

VARIANTS = ("blas", "blk64", "split8", "blk64g")
ROW_BAR = 2e-2      # the stated bf16 tolerance, applied per sample row


def _product_f32(x32, w32, kind):
    K = x32.shape[1]
    if kind == "blas":
        return x32 @ w32
    if kind in ("blk64", "blk64g"):
        z = np.zeros((x32.shape[0], w32.shape[1]), np.float32)
        for k in range(0, K, 64):
            z = z + x32[:, k:k + 64] @ w32[k:k + 64]
        return z
    if kind == "split8":
        step = -(-K // 8)
        parts = []
        for s in range(8):
            a, b = s * step, min(K, (s + 1) * step)
            acc = np.zeros((x32.shape[0], w32.shape[1]), np.float32)
            for k in range(a, b, 32):
                acc = acc + x32[:, k:min(b, k + 32)] @ w32[k:min(b, k + 32)]
            parts.append(acc)
        while len(parts) > 1:
            parts = [parts[i] + parts[i + 1] for i in range(0, len(parts), 2)]
        return parts[0]
    raise ValueError(kind)


def _run(wl, kind):
    fwd, bwd = O.linear_fwd, O.linear_bwd

    def linear_fwd(x, p, op):
        z = _product_f32(x.astype(np.float32), p["W"].T.astype(np.float32), kind).astype(np.float64)
        if "b" in p:
            z = z + p["b"]
        return O.act_fwd(z, op["act"]), (x, z)

    def linear_bwd(dy, saved, p, g, op):
        dx = bwd(dy, saved, p, g, op)
        return [O.store_as(d, op.get("dtype")) for d in dx]

    if kind is not None:
        O.linear_fwd = linear_fwd
        if kind.endswith("g"):
            O.linear_bwd = linear_bwd
    try:
        stage, res = O.run_minibatch(wl.ops, wl.micro_batch, wl.params, wl.batches, model_storage=True)
    finally:
        O.linear_fwd, O.linear_bwd = fwd, bwd
    # only gradients, input gradients and pre-activations are compared: the stage's float64 copy of the
    # parameters (10 GB for the largest workload) is not kept while the next order runs
    stage.params = None
    return stage, res


def row_errors(got, ref):
    """l2-relative error of every row (sample) of a gradient matrix; rows whose
    reference is zero count as exact when the other side is zero too."""
    got = np.asarray(got, np.float64).reshape(ref.shape[0], -1)
    ref = np.asarray(ref, np.float64).reshape(ref.shape[0], -1)
    n = np.linalg.norm(ref, axis=1)
    d = np.linalg.norm(got - ref, axis=1)
    return np.where(n > 0, d / np.where(n > 0, n, 1.0), (d > 0) * 1.0)


def measure(wl, variants=VARIANTS):
    """Returns a dict: worst l2-relative and max-relative difference of an input-gradient
    tensor between the fp64 oracle and any variant, the largest fraction of sample rows
    that differ by more than ROW_BAR, the worst weight-gradient and table-gradient difference, and how many
    ReLU decisions were opposite / how many pre-activations lie within one bf16 step
    (2^-8 of the layer's r.m.s.) of zero."""
    ref, res = _run(wl, None)
    relu = [i for i, op in enumerate(wl.ops) if op["kind"] == "linear" and op.get("act") == "relu"]
    out = dict(l2=0.0, max=0.0, rows_over=0.0, dw=0.0, dt=0.0, flips=0, decisions=0, near_zero=0, per_variant={})
    for (st, _) in res:
        for i in relu:
            z = st.saved[i][1]
            out["decisions"] += z.size
            out["near_zero"] += int((np.abs(z) <= 2.0 ** -8 * np.sqrt((z * z).mean())).sum())
    for kind in variants:
        r2, res2 = _run(wl, kind)
        l2 = mx = rows = 0.0
        flips = 0
        for (sa, ga), (sb, gb) in zip(res, res2):
            for i in ga:
                a, b = ga[i], gb[i]
                l2 = max(l2, np.linalg.norm(a - b) / np.linalg.norm(a))
                mx = max(mx, np.abs(a - b).max() / np.abs(a).max())
                rows = max(rows, float((row_errors(b, a) > ROW_BAR).mean()))
            for i in relu:
                flips += int(((sa.saved[i][1] > 0) != (sb.saved[i][1] > 0)).sum())
        dw = max(np.linalg.norm(ref.grads[i][k] - r2.grads[i][k]) / max(np.linalg.norm(ref.grads[i][k]), 1e-300)
                 for i in ref.grads for k in ref.grads[i] if k != "table")
        # embedding tables sit in front of the ReLU stack like inputs: their gradients are the (scattered)
        # gradients of the pooled vectors and carry the same opposite decisions
        dt = max([np.linalg.norm(ref.grads[i][k] - r2.grads[i][k]) / max(np.linalg.norm(ref.grads[i][k]), 1e-300)
                  for i in ref.grads for k in ref.grads[i] if k == "table"] or [0.0])
        out["per_variant"][kind] = dict(l2=l2, max=mx, rows_over=rows, dw=dw, dt=dt, flips=flips)
        out["dt"] = max(out["dt"], dt)
        out["l2"], out["max"] = max(out["l2"], l2), max(out["max"], mx)
        out["rows_over"], out["dw"] = max(out["rows_over"], rows), max(out["dw"], dw)
        out["flips"] = max(out["flips"], flips)
    return out
