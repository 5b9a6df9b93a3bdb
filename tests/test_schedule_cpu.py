"""The library's host-side scheduler routines (C ABI, no GPU needed) against the scheduler oracle: integer
work, so every comparison is exact."""
import itertools
import random

import pytest

from oracle import schedule_oracle as S
from paper_2406_17145_amd import binding as B


def _codes(tasks):
    return [(j + 1) if w == "F" else -(j + 1) for w, j in tasks]


def test_in_flight_table_matches_oracle_on_all_small_arguments():
    rng = range(1, 11)
    for kx, bx, ky, by in itertools.product(rng, rng, rng, rng):
        for iy in (1, ky * by, 37):
            assert B.gpp_compute_in_flight(kx, bx, ky, by, iy) == S.compute_in_flight(kx, bx, ky, by, iy), (kx, bx, ky, by, iy)


def test_in_flight_table_matches_oracle_on_large_arguments():
    r = random.Random(5)
    for _ in range(20000):
        bx, by = (1 << r.randrange(0, 12)) * r.choice((1, 1, 3)), (1 << r.randrange(0, 12)) * r.choice((1, 1, 5))
        kx, ky = r.choice((1, 2, 3, 4, 8, 16, 1000)), r.choice((1, 2, 3, 4, 8, 16, 1000))
        iy = r.randrange(1, 1 << 40)
        assert B.gpp_compute_in_flight(kx, bx, ky, by, iy) == S.compute_in_flight(kx, bx, ky, by, iy), (kx, bx, ky, by, iy)


@pytest.mark.parametrize("bad", [(0, 1, 1, 1, 1), (1, 0, 1, 1, 1), (1, 1, -1, 1, 1), (1, 1, 1, 0, 1), (1, 1, 1, 1, 0),
                                 (1 << 31, 1, 1, 1, 1)])
def test_in_flight_table_rejects_bad_arguments(bad):
    with pytest.raises(B.GppError) as e:
        B.gpp_compute_in_flight(*bad)
    assert e.value.status == B.GPP_ERR_INVALID_ARG


def _random_stage_graph(r, n):
    """A DAG over a random permutation of the stage ids (edges go forward in that hidden order), every stage but
    the hidden last one with at least one successor: the shape of a stage graph with branches and joins."""
    order = list(range(n))
    r.shuffle(order)
    edges = set()
    for a in range(n - 1):
        for c in r.sample(range(a + 1, n), k=min(n - 1 - a, r.choice((1, 1, 2, 3)))):
            edges.add((order[a], order[c]))
    edges = list(edges)
    r.shuffle(edges)
    return edges


def test_stage_graph_schedules_match_oracle_on_random_graphs():
    r = random.Random(11)
    for trial in range(300):
        n = r.randrange(1, 12)
        edges = _random_stage_graph(r, n)
        b = [1 << r.randrange(0, 5) if r.random() < 0.8 else r.randrange(1, 20) for _ in range(n)]
        ks = [sorted(r.sample([1, 2, 3, 4, 6, 8], k=r.randrange(1, 4)), reverse=r.random() < 0.5) for _ in range(n)]
        assert B.gpp_assign_schedules(n, edges, b, ks) == tuple(S.assign_schedules(n, edges, b, ks)), (trial, n, edges, b, ks)


def test_stage_graph_schedules_of_the_papers_examples():
    # section 6: sizes 1, 2, 4; section 2: depth 2 against depth 4
    assert B.gpp_assign_schedules(3, [(0, 1), (1, 2)], [4, 4, 4], [[1]] * 3)[0] == [12, 8, 4]
    assert B.gpp_assign_schedules(3, [(0, 1), (1, 2)], [1, 2, 4], [[1, 2, 4], [2], [1]])[0] == [10, 8, 4]
    assert B.gpp_assign_schedules(4, [(0, 3), (1, 3), (2, 3)], [1] * 4, [[1]] * 4)[0] == [2, 2, 2, 1]
    assert B.gpp_assign_schedules(4, [(0, 1), (1, 2), (2, 3)], [1] * 4, [[1]] * 4)[0] == [4, 3, 2, 1]


def test_stage_graph_errors():
    with pytest.raises(B.GppError) as e:
        B.gpp_assign_schedules(3, [(0, 1), (1, 2), (2, 1)], [1, 1, 1], [[1]] * 3)
    assert e.value.status == B.GPP_ERR_BAD_GRAPH
    for args in [(2, [(0, 2)], [1, 1], [[1], [1]]), (2, [(0, 1)], [1, 0], [[1], [1]]), (2, [(0, 1)], [1, 1], [[1], []]),
                 (2, [(0, 1)], [1, 1], [[0], [1]])]:
        with pytest.raises(B.GppError) as e:
            B.gpp_assign_schedules(*args)
        assert e.value.status == B.GPP_ERR_INVALID_ARG


def test_task_lists_match_oracle():
    for n in list(range(0, 14)) + [33, 64]:
        for cap, k, b in itertools.product((1, 2, 3, 4, 5, 8, 70), (1, 2, 3, 4, 9), (1, 2, 4)):
            for extra in (0, b - 1):          # in-flight counts that are not a multiple of b round down
                i = cap * b + extra
                assert B.gpp_schedule_tasks(n, i, k, b) == _codes(S.schedule_task(n, i, k, b)), (n, i, k, b)
    assert B.gpp_schedule_tasks(6, 3, 1, 4) == _codes(S.schedule_task(6, 3, 1, 4))     # capacity never below one


def test_task_list_errors():
    for args in [(-1, 1, 1, 1), (4, 0, 1, 1), (4, 1, 0, 1), (4, 1, 1, 0)]:
        with pytest.raises(B.GppError) as e:
            B.gpp_schedule_tasks(*args)
        assert e.value.status == B.GPP_ERR_INVALID_ARG


# ---- cutting an operator graph into stages (graph surgery of the workload module) and the stage graph's counts

def test_partition_of_a_branchy_model_gives_its_stage_graph():
    from paper_2406_17145_amd import workloads as W
    from paper_2406_17145_amd.schedule import StagePipeline
    wl = W.candle_uno(micro_batch=8, n_micro=2, widths=(70, 131, 33), hidden=96, act="gelu")
    stage_of = {i: (op["branch"] if op["branch"] >= 0 else 3) for i, op in enumerate(wl.ops) if op["kind"] != "input"}
    parts, edges = W.partition(wl, stage_of, 4)
    assert edges == [(0, 0, 3, 0), (1, 0, 3, 1), (2, 0, 3, 2)]
    assert [len(p.output_global) for p in parts] == [1, 1, 1, 0]
    # every operator and parameter of the model is in exactly one stage (C1: the G_i partition G_C)
    owned = sorted(g for p in parts for g in p.global_of if g >= 0)
    assert owned == list(range(len(wl.ops)))
    assert sorted(p.global_of[l] for p in parts for l in p.params) == sorted(wl.params)
    # edge-fed inputs of the merge stage have the producers' widths and storage type
    merge = parts[3].ops
    assert [(o["kind"], o["out_features"], o["dtype"]) for o in merge[:3]] == [("input", 96, "bf16")] * 3
    # the stage graph's in-flight micro-batches: side by side (depth 2) against chained (depth 4), section 2
    assert StagePipeline.in_flight_microbatches(4, edges, 8)[0] == [2, 2, 2, 1]
    assert StagePipeline.in_flight_microbatches(4, edges + [(0, -1, 1, -1), (1, -1, 2, -1)], 8)[0] == [4, 3, 2, 1]


def test_partition_refuses_fan_out_across_a_cut():
    from paper_2406_17145_amd import workloads as W
    wl = W.tiny_mlp()
    # the first layer of branch 0 alone in a stage is fine; cutting between an input and two stages is not
    stage_of = {i: 0 for i, op in enumerate(wl.ops) if op["kind"] != "input"}
    parts, edges = W.partition(wl, stage_of, 1)
    assert edges == [] and len(parts[0].ops) == len(wl.ops)


def test_capture_of_slot_reuse_waits_is_refused_on_the_host():
    """GraphedMinibatch / StagePipeline refuse, before any GPU call, the one form whose capture has crashed:
    several streams and fewer stash slots than micro-batches."""
    from types import SimpleNamespace
    from paper_2406_17145_amd import schedule as S

    def fake(cls, slots, **attrs):
        obj = object.__new__(cls)
        obj.st = SimpleNamespace(slots=slots)
        for k, v in attrs.items():
            setattr(obj, k, v)
        return obj

    batches = [None] * 3
    with pytest.raises(ValueError, match="capture refused"):
        S.GraphedMinibatch(fake(S.OverlapSchedule, 2), batches)
    with pytest.raises(ValueError, match="capture refused"):
        S.GraphedMinibatch(fake(S.TaskSchedule, 2, two=True), batches)
    S.GraphedMinibatch.check_capturable(fake(S.OverlapSchedule, 3), 3)            # a slot per micro-batch: allowed
    S.GraphedMinibatch.check_capturable(fake(S.TaskSchedule, 1, two=False), 3)    # one stream: no event waits
    S.GraphedMinibatch.check_capturable(fake(S.SerialSchedule, 1), 3)
    pipe = object.__new__(S.StagePipeline)
    pipe.stages = [SimpleNamespace(slots=2), SimpleNamespace(slots=4)]
    io = [[None] * 4, [None] * 4]
    with pytest.raises(ValueError, match="capture refused"):
        pipe.check_not_capturing_slot_reuse(io, capturing=True)
    pipe.check_not_capturing_slot_reuse(io, capturing=False)
    pipe.stages[0].slots = 4
    pipe.check_not_capturing_slot_reuse(io, capturing=True)
