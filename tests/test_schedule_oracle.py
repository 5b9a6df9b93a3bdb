"""Pins of the scheduler oracle against what the paper and plain counting fix (no GPU, no product code)."""
import itertools

import pytest

from oracle import schedule_oracle as S


# ---- the appendix table

def _all_rows(kx, bx, ky, by, iy):
    """Every row of the appendix table whose condition holds, retyped from the table as
    (condition, result) pairs so that overlap and completeness can be examined row by row."""
    X, Y, m = kx * bx, ky * by, max(bx, by)
    rows = [
        (m < X < Y, iy + 2 * m),
        (m == X and X < Y, iy + m),
        (bx <= by < Y < X, iy + X - Y + 2 * by),
        (bx <= by and by == Y and Y < X, iy + X),
        (by <= bx < Y < X, iy + X - Y + 2 * bx),
        (by <= bx and bx == Y and Y < X, iy + X),
        (m == Y and Y == X, iy + Y),
        (m < Y and Y == X, iy + 2 * m),
        (bx <= X < by <= Y, iy + by),
        (by <= Y < bx <= X, iy + X - Y + bx),
    ]
    return [r for c, r in rows if c]


def test_table_rows_cover_every_case_and_overlaps_agree():
    rng = range(1, 9)
    for kx, bx, ky, by in itertools.product(rng, rng, rng, rng):
        hits = _all_rows(kx, bx, ky, by, 5)
        assert hits, (kx, bx, ky, by)
        assert len(set(hits)) == 1, (kx, bx, ky, by, hits)
        assert S.compute_in_flight(kx, bx, ky, by, 5) == hits[0]


def test_table_is_affine_in_the_successor_count():
    for args in [(1, 4, 1, 4), (2, 1, 2, 2), (4, 1, 2, 2), (1, 8, 2, 1), (3, 2, 1, 2)]:
        base = S.compute_in_flight(*args, 7)
        assert S.compute_in_flight(*args, 107) == base + 100


def test_table_rejects_non_positive_arguments():
    for bad in [(0, 1, 1, 1, 1), (1, -2, 1, 1, 1), (1, 1, 1, 1, 0)]:
        with pytest.raises(ValueError):
            S.compute_in_flight(*bad)


# ---- section 6: sequential pipelines under 1F1B hold (n + 1 - x) * b samples at stage x

@pytest.mark.parametrize("n,b", [(1, 3), (2, 1), (4, 4), (7, 2)])
def test_sequential_pipeline_rule(n, b):
    edges = [(x, x + 1) for x in range(n - 1)]
    i, k = S.assign_schedules(n, edges, [b] * n, [[1]] * n)
    assert k == [1] * n
    assert i == [(n - x) * b for x in range(n)]          # x counted from 0: (n + 1 - (x + 1)) * b


# ---- section 6, worked example: three stages whose best micro-batch sizes are 1, 2 and 4

def test_worked_example_uniform_size_gives_12():
    i, k = S.assign_schedules(3, [(0, 1), (1, 2)], [4, 4, 4], [[1]] * 3)
    assert i == [12, 8, 4]


def test_worked_example_per_stage_sizes_give_10():
    # k * b = 4 samples per group at the last two stages, any k at the first
    i, k = S.assign_schedules(3, [(0, 1), (1, 2)], [1, 2, 4], [[1, 2, 4], [2], [1]])
    assert i[2] == 4 and i[1] == 8
    assert i[0] == 10
    # both shorter groupings reach it, the full group of four does not
    assert S.compute_in_flight(1, 1, 2, 2, 8) == 10
    assert S.compute_in_flight(2, 1, 2, 2, 8) == 10
    assert S.compute_in_flight(4, 1, 2, 2, 8) == 12


# ---- section 2, example: three independent stages in front of one (depth 2) against a chain of four

def test_depth_two_graph_against_depth_four_chain():
    b = 2
    gi, _ = S.assign_schedules(4, [(0, 3), (1, 3), (2, 3)], [b] * 4, [[1]] * 4)
    si, _ = S.assign_schedules(4, [(0, 1), (1, 2), (2, 3)], [b] * 4, [[1]] * 4)
    assert [v // b for v in gi] == [2, 2, 2, 1]
    assert [v // b for v in si] == [4, 3, 2, 1]


def test_several_successors_take_the_largest_and_order_of_edges_is_irrelevant():
    # S0 feeds a chain of two (S1 -> S2) and, directly, the sink S3 that S2 also feeds
    edges = [(0, 1), (1, 2), (2, 3), (0, 3)]
    a, _ = S.assign_schedules(4, edges, [1] * 4, [[1]] * 4)
    b, _ = S.assign_schedules(4, edges[::-1], [1] * 4, [[1]] * 4)
    assert a == b == [4, 3, 2, 1]


def test_cycle_is_refused():
    with pytest.raises(ValueError):
        S.assign_schedules(2, [(0, 1), (1, 0)], [1, 1], [[1], [1]])


# ---- task lists: order condition C4 (section 3) and the footnote's shape

def _check_c4(tasks, n):
    pos_f = {j: t for t, (w, j) in enumerate(tasks) if w == "F"}
    pos_b = {j: t for t, (w, j) in enumerate(tasks) if w == "B"}
    assert len(tasks) == 2 * n and sorted(pos_f) == sorted(pos_b) == list(range(n))
    for j in range(n):
        assert pos_f[j] < pos_b[j]
        if j + 1 < n:
            assert pos_f[j] < pos_f[j + 1] and pos_b[j] < pos_b[j + 1]


def _runs(tasks):
    return [(w, len(list(g))) for w, g in itertools.groupby(w for w, _ in tasks)]


@pytest.mark.parametrize("n", [1, 2, 5, 8, 13])
@pytest.mark.parametrize("cap", [1, 2, 3, 4, 8])
@pytest.mark.parametrize("k", [1, 2, 3, 4])
def test_greedy_task_list_is_valid_and_is_the_footnote_pattern(n, cap, k):
    b = 3
    tasks = S.schedule_task(n, cap * b, k, b)
    _check_c4(tasks, n)
    assert S.peak_in_flight(tasks) == min(cap, n)
    assert tasks == S.kfkb_tasks(n, cap, k)
    runs = _runs(tasks)
    l = min(cap, n)
    assert runs[0] == ("F", l)                                   # warm-up
    assert runs[-1][0] == "B"
    if n > cap and k <= cap:
        # the alternation: groups of k, except where the mini-batch ends
        inner = runs[1:-1]
        assert all(c <= k for _, c in inner)
        assert all(c == k for _, c in inner[:-2])
        held_before_cooldown = l - sum(c for w, c in inner if w == "B") + sum(c for w, c in inner if w == "F")
        assert runs[-1][1] == held_before_cooldown


def test_1f1b_at_stage_x_of_n_runs_n_plus_1_minus_x_forwards_before_its_first_backward():
    n_stages, b, n_micro = 4, 2, 9
    i, k = S.assign_schedules(n_stages, [(x, x + 1) for x in range(n_stages - 1)], [b] * n_stages, [[1]] * n_stages)
    for x in range(n_stages):
        tasks = S.schedule_task(n_micro, i[x], k[x], b)
        first_b = next(t for t, (w, _) in enumerate(tasks) if w == "B")
        assert first_b == n_stages + 1 - (x + 1)
        # and strictly alternating afterwards until the injections end
        mid = tasks[first_b:first_b + 2 * (n_micro - first_b)]
        assert [w for w, _ in mid] == ["B", "F"] * (n_micro - first_b)


def test_fewer_micro_batches_than_warm_up():
    assert S.schedule_task(2, 12, 1, 2) == [("F", 0), ("F", 1), ("B", 0), ("B", 1)]


def test_fractional_capacity_rounds_down_but_never_to_zero():
    assert S.peak_in_flight(S.schedule_task(6, 10, 1, 4)) == 2
    assert S.peak_in_flight(S.schedule_task(6, 3, 1, 4)) == 1
