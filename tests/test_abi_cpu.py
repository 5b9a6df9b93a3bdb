"""Host-side checks that need no GPU: the library loads, exports every symbol
the header declares, and validates stage descriptors (condition C1: a stage's
sub-graph must be a DAG; shapes of connected operators must agree)."""
import copy
import os
import re

import pytest

from paper_2406_17145_amd import binding as B
from paper_2406_17145_amd import workloads as W

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


@pytest.fixture(scope="module")
def lib():
    if not os.path.exists(B.LIB_PATH):
        from paper_2406_17145_amd.build import build_library
        build_library(verbose=False)
    return B.load()


def test_every_declared_symbol_is_exported(lib):
    hdr = open(os.path.join(ROOT, "include", "gpp.h")).read()
    declared = set(re.findall(r"\b(gpp_[a-z_]+)\s*\(", hdr))
    assert declared == set(B.EXPORTS), declared ^ set(B.EXPORTS)
    for name in declared:
        assert hasattr(lib, name), name


def test_ld_rule(lib):
    assert [B.gpp_ld(x) for x in (1, 8, 64, 65, 479, 942, 1000, 3820)] == [64, 64, 64, 128, 512, 960, 1024, 3840]


def ws(ops, b=4, slots=1):
    d, keep = B.build_desc(ops, b, slots)
    return B.gpp_stage_workspace_bytes(d)


@pytest.mark.parametrize("make", [W.tiny_mlp, lambda: W.candle_uno(n_micro=1),
                                  lambda: W.mmt(micro_batch=1, seq_len=16, d_model=64, heads=4, d_ff=128),
                                  lambda: W.dlrm(micro_batch=8, num_rows=100), lambda: W.hetero(micro_batch=2)])
def test_all_config_graphs_plan_on_the_host(lib, make):
    wl = make()
    n1 = ws(wl.ops, wl.micro_batch, 1)
    n3 = ws(wl.ops, wl.micro_batch, 3)
    assert 0 < n1 < n3          # more in-flight slots need a larger activation stash


def expect(ops, status, b=4):
    with pytest.raises(B.GppError) as e:
        ws(ops, b)
    assert e.value.status == status, str(e.value)


def test_cycle_is_rejected(lib):
    ops = copy.deepcopy(W.tiny_mlp().ops)
    ops[1]["inputs"] = [2]          # linear 1 <- linear 2 <- linear 1
    expect(ops, B.GPP_ERR_BAD_GRAPH, 8)


def test_dangling_edge_and_arity(lib):
    ops = copy.deepcopy(W.tiny_mlp().ops)
    ops[1]["inputs"] = [99]
    expect(ops, B.GPP_ERR_BAD_GRAPH, 8)
    ops = copy.deepcopy(W.tiny_mlp().ops)
    ops[1]["inputs"] = [0, 0]
    expect(ops, B.GPP_ERR_BAD_GRAPH, 8)


def test_shape_mismatch(lib):
    ops = copy.deepcopy(W.tiny_mlp().ops)
    ops[1]["in_features"] = 65
    expect(ops, B.GPP_ERR_SHAPE, 8)
    ops = copy.deepcopy(W.tiny_mlp().ops)
    cat = next(i for i, o in enumerate(ops) if o["kind"] == "concat")
    ops[cat]["out_features"] = 127
    expect(ops, B.GPP_ERR_SHAPE, 8)


def test_dtype_mix_is_unsupported(lib):
    ops = copy.deepcopy(W.tiny_mlp().ops)
    ops[1]["dtype"] = "bf16"        # bf16 weights on an f32 producer
    expect(ops, B.GPP_ERR_UNSUPPORTED, 8)


def test_bad_sizes(lib):
    ops = W.tiny_mlp().ops
    d, keep = B.build_desc(ops, 0)
    with pytest.raises(B.GppError) as e:
        B.gpp_stage_workspace_bytes(d)
    assert e.value.status == B.GPP_ERR_INVALID_ARG
    d, keep = B.build_desc(ops, 8, slots=0)
    with pytest.raises(B.GppError) as e:
        B.gpp_stage_workspace_bytes(d)
    assert e.value.status == B.GPP_ERR_INVALID_ARG


def test_embedding_needs_integer_inputs(lib):
    wl = W.dlrm(micro_batch=8, num_rows=100, n_tables=2)
    ops = copy.deepcopy(wl.ops)
    emb = next(i for i, o in enumerate(ops) if o["kind"] == "embedding_bag_sum")
    ops[ops[emb]["inputs"][0]]["dtype"] = "f32"
    expect(ops, B.GPP_ERR_BAD_GRAPH, 8)


def test_create_rejects_missing_workspace_before_touching_the_gpu(lib):
    wl = W.tiny_mlp()
    fake = {i: [4096, 4096] for i in wl.params}     # non-null, aligned, never dereferenced here
    d, keep = B.build_desc(wl.ops, 8, 1, 0, fake, fake)
    with pytest.raises(B.GppError) as e:
        B.gpp_stage_create(d, None, 0)
    assert e.value.status == B.GPP_ERR_WORKSPACE
    d2, keep2 = B.build_desc(wl.ops, 8)             # null parameter pointers
    with pytest.raises(B.GppError) as e:
        B.gpp_stage_create(d2, 256, 1 << 30)
    assert e.value.status == B.GPP_ERR_INVALID_ARG


def test_stage_flags_in_the_workspace_size(lib):
    # per-slot gradient buffers (flag bit 2) and the second copy of the launch tables for group launches (bits 8-11)
    # both show in the workspace; a lane count the slots cannot be split into, or group launches without per-slot
    # gradient buffers, are ignored
    wl = W.candle_uno(micro_batch=16, n_micro=1, widths=(32, 40, 8, 24), hidden=64)

    def size(slots, flags):
        d, keep = B.build_desc(wl.ops, wl.micro_batch, slots, flags=flags)
        return B.gpp_stage_workspace_bytes(d)
    plain, grouped = size(8, 0), size(8, B.FLAG_GROUPED_DW)
    assert grouped > plain
    with_tables = size(8, B.FLAG_GROUPED_DW | B.flag_group_launches(2))
    assert with_tables > grouped
    assert size(8, B.FLAG_GROUPED_DW | B.flag_group_launches(4)) == with_tables      # the same number of table copies
    assert size(8, B.FLAG_GROUPED_DW | B.flag_group_launches(3)) == grouped          # 8 slots do not split into 3 lanes
    assert size(8, B.FLAG_GROUPED_DW | B.flag_group_launches(8)) == grouped          # one micro-batch per lane: nothing to group
    assert size(8, B.flag_group_launches(2)) == plain                                # needs per-slot gradient buffers
    assert size(8, B.FLAG_GROUPED_DW | B.FLAG_SHARED_GPU) == grouped                 # workgroup sizes only
