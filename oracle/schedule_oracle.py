"""CPU oracle for the static micro-batch scheduler of one stage.  TEST INFRASTRUCTURE ONLY.

Only tests may import this file; the product (the HIP library and its binding) never does, and
this file imports nothing from the product.  Pure integer logic in plain Python.

What it follows (paper section 6 and appendix "Generalized Per-stage kFkB Schedule"):

* compute_in_flight  -- the appendix table: the number of in-flight SAMPLES i_x of a stage S_x
  that runs k_x F k_x B with micro-batch size b_x, in front of a stage S_y that runs k_y F k_y B
  with micro-batch size b_y and holds i_y in-flight samples.  The table's conditions are tried in
  the printed order and the first one that holds gives the result.
* assign_schedules   -- section 6: the last stage is scheduled first, then the stage graph's edges
  are followed in reverse; a stage takes, over its candidate k, the k that minimises the largest
  table value over its successors (the appendix's argmin-max formula).
* kfkb_tasks         -- the footnote of section 6: l forward passes, then k backward and k forward
  passes in turn, then l backward passes.
* schedule_task      -- ScheduleTask of Alg. 2: given c = (i, k, b), issue forward passes until the
  stage holds i samples, and from then on resolve in-flight micro-batches as early as the kFkB
  grouping allows (k backward passes as soon as the stage is full, k forward passes to fill it
  again), greedily, one decision per task.

Readings (the paper does not state them):
* a stage without successor holds the k micro-batches of one forward group: i = k * b;
* several candidate k with the same in-flight count: the smallest k wins;
* i_x not a multiple of b_x: the stage may hold floor(i_x / b_x) micro-batches (at least one);
* a mini-batch with fewer micro-batches than the warm-up needs: all forwards, then all backwards;
* a last alternation group that the number of micro-batches cuts short is simply shorter;
* k larger than the number of micro-batches the stage may hold acts as that number.

Pins (tests/test_schedule_oracle.py): the sequential-pipeline rule (stage x of n under 1F1B with
one micro-batch size b holds (n + 1 - x) * b samples, section 6), the worked example of section 6
(sizes 1, 2, 4: 12 in-flight with one size, 10 with per-stage sizes and schedules), the depth-2
versus depth-4 example of section 2 (first stages store 2 and 4 micro-batches), overlap-consistency
and completeness of the table over all small integers, order condition C4 (section 3), the
footnote's shape of every generated task list, and the peak number of in-flight micro-batches.
"""


def compute_in_flight(kx, bx, ky, by, iy):
    """Appendix table.  All arguments are positive integers; returns in-flight samples of S_x."""
    for v in (kx, bx, ky, by, iy):
        if int(v) != v or v <= 0:
            raise ValueError("compute_in_flight: arguments must be positive integers")
    X, Y, m = kx * bx, ky * by, max(bx, by)
    if m < X < Y:
        return iy + 2 * m
    if m == X < Y:
        return iy + m
    if bx <= by < Y < X:
        return iy + X - Y + 2 * by
    if bx <= by == Y < X:
        return iy + X
    if by <= bx < Y < X:
        return iy + X - Y + 2 * bx
    if by <= bx == Y < X:
        return iy + X
    if m == Y == X:
        return iy + Y
    if m < Y == X:
        return iy + 2 * m
    if bx <= X < by <= Y:
        return iy + by
    if by <= Y < bx <= X:
        return iy + X - Y + bx
    raise ArithmeticError("compute_in_flight: no row of the table applies")


def assign_schedules(n_stages, edges, b, k_candidates):
    """Reverse traversal of the stage graph.  edges: (x, y) pairs, S_x feeds S_y; b[x]: micro-batch
    size of S_x; k_candidates[x]: the k values S_x may use.  Returns (i, k): in-flight samples and
    chosen k per stage."""
    succ = [[] for _ in range(n_stages)]
    for x, y in edges:
        succ[x].append(y)
    # reverse topological order by repeated removal of stages whose successors are all done
    done, order = [False] * n_stages, []
    while len(order) < n_stages:
        ready = [x for x in range(n_stages) if not done[x] and all(done[y] for y in succ[x])]
        if not ready:
            raise ValueError("assign_schedules: the stage graph has a cycle")
        for x in ready:
            done[x] = True
            order.append(x)
    i, k = [0] * n_stages, [0] * n_stages
    for x in order:
        best = None
        for kx in sorted(k_candidates[x]):
            if succ[x]:
                val = max(compute_in_flight(kx, b[x], k[y], b[y], i[y]) for y in succ[x])
            else:
                val = kx * b[x]
            if best is None or val < best[0]:
                best = (val, kx)
        i[x], k[x] = best
    return i, k


def kfkb_tasks(n_micro, l, k):
    """Footnote of section 6, written out: ("F", j) / ("B", j) in issue order."""
    l = min(l, n_micro)
    k = min(k, l)                 # a group cannot be larger than what the stage holds
    tasks = [("F", j) for j in range(l)]
    f, bwd = l, 0
    while f < n_micro:
        for _ in range(min(k, f - bwd)):
            tasks.append(("B", bwd))
            bwd += 1
        for _ in range(min(k, n_micro - f)):
            tasks.append(("F", f))
            f += 1
    tasks += [("B", j) for j in range(bwd, n_micro)]
    return tasks


def schedule_task(n_micro, i, k, b):
    """ScheduleTask for c = (i, k, b): one greedy decision at a time.  While micro-batches remain to
    be injected and the stage has room, a forward pass is issued; once the stage holds its i samples
    the k oldest in-flight micro-batches are resolved (backward passes, oldest first); when nothing is
    left to inject, every remaining backward pass runs."""
    cap = max(1, i // b)          # micro-batches the stage may hold
    tasks, f, bwd = [], 0, 0      # forward / backward passes issued so far
    while bwd < n_micro:
        held = f - bwd
        if f == n_micro:
            group = held
        elif held >= cap:
            group = min(k, held)
        else:
            group = 0
        if group:
            for _ in range(group):
                tasks.append(("B", bwd))
                bwd += 1
        else:
            tasks.append(("F", f))
            f += 1
    return tasks


def peak_in_flight(tasks):
    held = peak = 0
    for what, _ in tasks:
        held += 1 if what == "F" else -1
        peak = max(peak, held)
    return peak
