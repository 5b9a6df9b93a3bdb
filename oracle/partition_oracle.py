"""CPU oracle for the pipeline stage partitioner.  TEST INFRASTRUCTURE ONLY.

Only tests may import this file; the product never does, and this file imports nothing from the
product (it uses the scheduler oracle next to it for in-flight counts).

What it follows (paper section 5, Alg. 1, and the problem statement of section 3): given the
operator graph G_C with a cost per operator, a number of devices and a memory budget per device,
find the stage graph G_S -- a partition of the operators into stages (C1), each with a set of
devices (C3: the device sets partition the devices) -- whose bottleneck stage has the smallest
time per sample, subject to every stage fitting its devices' memory with the in-flight
micro-batches its schedule needs (section 6).  The paper reaches it by series-parallel
decomposition + dynamic programming + binary search on the target time; that is a search METHOD.
The RESULT it is after has a plain definition, so the oracle is that definition written out:

    enumerate EVERY stage graph the decomposition can express, evaluate each one from the
    definitions (time per sample of a stage = sum of its operators' times / its devices; in-flight
    samples by the scheduler's reverse traversal of the stage graph; memory = weights + in-flight
    samples per device x activation bytes per sample), and take the feasible one with the smallest
    bottleneck time.

No memoisation, no binary search, no incremental in-flight bookkeeping.

Readings (the paper leaves them open; the product takes the same ones and the design notes list them):
* default schedule configuration of section 6 throughout: 1F1B, one micro-batch size b for all stages;
* a stage on d devices is data-parallel: time per sample = (sum of operator times) / d, plus, for d > 1,
  the gradient all-reduce of its parameters once per mini-batch as a ring: 2 (d - 1) / d x parameter
  bytes x seconds per byte / mini-batch samples (the paper extrapolates communication from profiles
  that do not exist here; tensors between stages are not charged);
* memory of a stage per device = sum of its operators' parameter bytes (replicated) + (in-flight
  samples / d) x sum of its operators' stashed bytes per sample;
* series-parallel structure of an operator graph (operators are NODES here): a set of operators that
  falls into several weakly connected parts is their PARALLEL composition; a connected set is split in
  SERIES at every operator that all other operators of the set are ancestors or descendants of; a
  connected set without such an operator is one indivisible block;
* a stage is a whole node of that tree or a run of consecutive children of one of its nodes;
* every device is used (C3) and a stage has at least one device;
* among stage graphs with the same bottleneck time the one whose first stages hold the fewest
  in-flight samples is preferred (the paper's PickBetter: less memory).

Pins (tests/test_partition_oracle.py): a chain of n equal operators on n devices gives n stages of
one operator with (n + 1 - x) b in-flight samples at stage x (section 6); independent branches become
parallel stages with the depth-2 in-flight counts of section 2 when devices allow, and the memory
budget decides between the deep and the shallow stage graph; conditions C1-C3 on every returned
stage graph; one device gives one stage; an impossible budget gives nothing.
"""

from oracle import schedule_oracle as S


# ---- series-parallel structure of an operator DAG -------------------------------------------------

def _closure(n, edges):
    succ = [set() for _ in range(n)]
    for u, v in edges:
        succ[u].add(v)
    order, seen = [], [False] * n

    def visit(u):
        seen[u] = True
        for v in succ[u]:
            if not seen[v]:
                visit(v)
        order.append(u)
    for u in range(n):
        if not seen[u]:
            visit(u)
    desc = [set() for _ in range(n)]
    for u in order:                       # children before parents
        for v in succ[u]:
            desc[u] |= {v} | desc[v]
    return desc


def sp_tree(n, edges):
    """("leaf", op) | ("block", [ops]) | ("series", [children]) | ("parallel", [children])."""
    desc = _closure(n, edges)
    anc = [set() for _ in range(n)]
    for u in range(n):
        for v in desc[u]:
            anc[v].add(u)
    nbr = [set() for _ in range(n)]
    for u, v in edges:
        nbr[u].add(v)
        nbr[v].add(u)

    def parts(ops):
        left, out = set(ops), []
        while left:
            start = min(left)
            comp, todo = {start}, [start]
            while todo:
                u = todo.pop()
                for v in nbr[u]:
                    if v in left and v not in comp:
                        comp.add(v)
                        todo.append(v)
            left -= comp
            out.append(sorted(comp))
        return out

    def build(ops):
        if len(ops) == 1:
            return ("leaf", ops[0])
        comps = parts(ops)
        if len(comps) > 1:
            return ("parallel", [build(c) for c in comps])
        s = set(ops)
        cuts = [v for v in ops if (anc[v] & s) | (desc[v] & s) | {v} == s]
        if not cuts:
            return ("block", list(ops))
        cuts.sort(key=lambda v: len(anc[v] & s))          # along the graph
        children, before = [], set()
        for v in cuts:
            seg = (anc[v] & s) - before
            if seg:
                children.append(build(sorted(seg)))
            children.append(("leaf", v))
            before |= seg | {v}
        rest = s - before
        if rest:
            children.append(build(sorted(rest)))
        return ("series", children) if len(children) > 1 else children[0]
    return build(list(range(n)))


def ops_of(node):
    kind, body = node
    if kind == "leaf":
        return [body]
    if kind == "block":
        return list(body)
    return [o for c in body for o in ops_of(c)]


# ---- every stage graph the tree can express ---------------------------------------------------------

def _plans(node, d):
    """All ways to cover the operators of `node` with stages using exactly d devices: lists of
    (frozenset of operators, devices)."""
    kind, body = node
    out = {((frozenset(ops_of(node)), d),)}
    if kind in ("series", "parallel") and d >= 2:
        for s in range(1, len(body)):
            left = body[0] if s == 1 else (kind, body[:s])
            right = body[s] if s == len(body) - 1 else (kind, body[s:])
            for d2 in range(1, d):
                for p1 in _plans(left, d - d2):
                    for p2 in _plans(right, d2):
                        out.add(tuple(sorted(p1 + p2, key=lambda st: min(st[0]))))
    return out


def stage_time(ops, d, t, w, sync_per_byte, mini_batch):
    compute = sum(t[o] for o in ops) / d
    if d == 1:
        return compute
    return compute + 2.0 * (d - 1) / d * sum(w[o] for o in ops) * sync_per_byte / mini_batch


def evaluate(plan, n, edges, t, w, a, b, memory, sync_per_byte=0.0, mini_batch=1):
    """Bottleneck time per sample, per-stage in-flight samples and memory of one stage graph, from the
    definitions; None if it violates C1 (stage graph with a cycle) or the memory budget."""
    stage_of = {}
    for s, (ops, _) in enumerate(plan):
        for o in ops:
            stage_of[o] = s
    s_edges = sorted({(stage_of[u], stage_of[v]) for u, v in edges if stage_of[u] != stage_of[v]})
    try:
        inflight, _ = S.assign_schedules(len(plan), s_edges, [b] * len(plan), [[1]] * len(plan))
    except ValueError:
        return None
    tps, mem = [], []
    for s, (ops, d) in enumerate(plan):
        tps.append(stage_time(ops, d, t, w, sync_per_byte, mini_batch))
        mem.append(sum(w[o] for o in ops) + inflight[s] / d * sum(a[o] for o in ops))
        if mem[-1] > memory:
            return None
    sources = [s for s in range(len(plan)) if all(y != s for _, y in s_edges)]
    return dict(tps=max(tps), in_flight=inflight, memory=mem, edges=s_edges,
                source_in_flight=max(inflight[s] for s in sources))


def best_stage_graph(n, edges, t, w, a, n_devices, b, memory, sync_per_byte=0.0, mini_batch=1):
    """The definition: the feasible stage graph with the smallest bottleneck time per sample (then the
    fewest in-flight samples at its first stages).  Returns (plan, evaluation) or None."""
    tree = sp_tree(n, edges)
    best = None
    for plan in _plans(tree, n_devices):
        ev = evaluate(plan, n, edges, t, w, a, b, memory, sync_per_byte, mini_batch)
        if ev is None:
            continue
        key = (ev["tps"], ev["source_in_flight"], len(plan))
        if best is None or key < best[0]:
            best = (key, plan, ev)
    return None if best is None else (best[1], best[2])


# ---- per-stage schedule configurations (paper section 5: the configuration loop of Alg. 1) -----------
#
# Alg. 1 does not only cut the graph: SearchStageGraph and the series case of DP enumerate schedule
# configurations c = (i, b, k) -- micro-batch size b and group size k of a stage's kFkB schedule, with the
# in-flight samples i that follow from them (section 6, appendix table) -- so that stages may run at
# different micro-batch sizes.  The definition of the result stays the same (smallest bottleneck time per
# sample among the stage graphs that fit), the search space grows: every stage of every stage graph takes
# one (b, k) out of the candidate lists.
#
# Readings, beyond those at the top of this file:
# * the time per sample of an operator depends on the micro-batch size of its stage (the paper profiles
#   every operator; compute efficiency rises with the micro-batch size, section 2): t[o][j] is the time at
#   micro-batch size b_values[j];
# * tensors between stages cost time, affine per message as in the paper's "extrapolating communication
#   latency by affine functions": a stage pays, per micro-batch, link_latency + bytes * link_seconds_per_byte
#   for every operator edge with exactly one end inside it (activations in, gradients back), i.e. per sample
#   cut_edges * link_latency / b + cut_bytes_per_sample * link_seconds_per_byte;
# * k and b enter the memory side only through the in-flight samples (scheduler oracle, reverse traversal);
# * Alg. 1 hands both halves of a PARALLEL decomposition the same c_f (they share the source in the paper's
#   picture): the stages that come first inside a parallel composition all carry one configuration.  The
#   enumeration below applies the same rule, so that it spans the space the method is defined over;
# * SearchStageGraph's loop: the enumerated c is the configuration of the FIRST stage(s) of the whole graph,
#   the dummy c_0 stands for the successor that the last stage does not have.

def cut_of(ops, edges, x):
    """(number, bytes per sample) of the operator edges with exactly one end in `ops`."""
    n = 0
    by = 0.0
    for e, (u, v) in enumerate(edges):
        if (u in ops) != (v in ops):
            n += 1
            by += x[e] if x is not None else 0.0
    return n, by


def stage_time_cfg(ops, d, j, tb, w, b_values, edges, x, sync_per_byte, mini_batch, link_latency, link_spb):
    compute = sum(tb[o][j] for o in ops) / d
    if d > 1:
        compute += 2.0 * (d - 1) / d * sum(w[o] for o in ops) * sync_per_byte / mini_batch
    n_cut, by = cut_of(ops, edges, x)
    return compute + n_cut * link_latency / b_values[j] + by * link_spb


def _parallel_sets(node, out):
    kind, body = node
    if kind in ("series", "parallel"):
        if kind == "parallel":
            out.append(frozenset(ops_of(node)))
        for c in body:
            _parallel_sets(c, out)
    return out


def evaluate_cfg(plan, cfg, n, edges, tb, w, a, b_values, k_values, memory, par_sets, x=None, sync_per_byte=0.0,
                 mini_batch=1, link_latency=0.0, link_spb=0.0):
    """One stage graph with one (index into b_values, index into k_values) per stage, from the definitions; None
    if it breaks C1, the memory budget or the shared configuration inside a parallel composition."""
    stage_of = {}
    for s, (ops, _) in enumerate(plan):
        for o in ops:
            stage_of[o] = s
    s_edges = sorted({(stage_of[u], stage_of[v]) for u, v in edges if stage_of[u] != stage_of[v]})
    for pset in par_sets:
        inside = [s for s, (ops, _) in enumerate(plan) if ops < pset]           # stages strictly inside the composition
        first = [s for s in inside if not any(y == s and xx in inside for xx, y in s_edges)]
        if len({cfg[s] for s in first}) > 1:
            return None
    try:
        inflight, _ = S.assign_schedules(len(plan), s_edges, [b_values[cfg[s][0]] for s in range(len(plan))],
                                         [[k_values[cfg[s][1]]] for s in range(len(plan))])
    except ValueError:
        return None
    tps, mem = [], []
    for s, (ops, d) in enumerate(plan):
        tps.append(stage_time_cfg(ops, d, cfg[s][0], tb, w, b_values, edges, x, sync_per_byte, mini_batch, link_latency, link_spb))
        mem.append(sum(w[o] for o in ops) + inflight[s] / d * sum(a[o] for o in ops))
        if mem[-1] > memory:
            return None
    sources = [s for s in range(len(plan)) if all(y != s for _, y in s_edges)]
    return dict(tps=max(tps), in_flight=inflight, memory=mem, edges=s_edges,
                source_in_flight=max(inflight[s] for s in sources))


def best_stage_graph_cfg(n, edges, tb, w, a, n_devices, b_values, k_values, memory, x=None, sync_per_byte=0.0,
                         mini_batch=1, link_latency=0.0, link_spb=0.0):
    """The definition with per-stage configurations: the feasible (stage graph, configuration per stage) with the
    smallest bottleneck time per sample, then the fewest in-flight samples at the first stages.  Exhaustive:
    every plan times every assignment of configurations.  Returns (plan, configurations, evaluation) or None."""
    import itertools
    tree = sp_tree(n, edges)
    par_sets = _parallel_sets(tree, [])
    cands = [(j, q) for j in range(len(b_values)) for q in range(len(k_values))]
    best = None
    for plan in _plans(tree, n_devices):
        for cfg in itertools.product(cands, repeat=len(plan)):
            ev = evaluate_cfg(plan, cfg, n, edges, tb, w, a, b_values, k_values, memory, par_sets, x, sync_per_byte,
                              mini_batch, link_latency, link_spb)
            if ev is None:
                continue
            key = (ev["tps"], ev["source_in_flight"], len(plan))
            if best is None or key < best[0]:
                best = (key, plan, cfg, ev)
    return None if best is None else (best[1], best[2], best[3])
