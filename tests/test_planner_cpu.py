"""Host logic of the library without a GPU: the C-ABI library loads and exports
every declared symbol, the planner's type checker agrees with the oracle's on
the rule-by-rule corpus and on a seeded random corpus, plans can be created and
inspected, and every error path that is decided on the host returns a status
code and leaves the context usable."""
import ctypes
import os
import re

import pytest

from oracle import graph as OG
from paper_1810_00952_amd import binding as B
import workloads as W
from typing_corpus import CASES, random_graphs

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def test_library_exports_every_declared_symbol():
    header = open(os.path.join(ROOT, "include", "relayhip.h")).read()
    declared = set(re.findall(r"^(?:rl_status|void|const char \*)\s*(rl_[a-z_0-9]+)\(", header, flags=re.M))
    assert declared == set(B.SYMBOLS), declared ^ set(B.SYMBOLS)
    L = ctypes.CDLL(B.LIB_PATH)
    for s in declared:
        assert hasattr(L, s), s


@pytest.mark.parametrize("name,builder,expected", CASES, ids=[c[0] for c in CASES])
def test_planner_typing_corpus(name, builder, expected):
    ctx = B.Context()
    try:
        B.Plan(B.graph_from_spec(ctx, builder()))
        got = None
    except B.RelayError as e:
        got = e.category
        assert ctx.last_error()
    assert got == expected, ctx.last_error()
    # the context stays usable after a rejection
    B.Plan(B.graph_from_spec(ctx, CASES[0][1]()))


def test_planner_agrees_with_oracle_on_random_graphs():
    ctx = B.Context()
    n_rej = 0
    for spec, _ in random_graphs(200):
        try:
            OG.check(spec)
            oracle_ok = True
        except OG.IllTyped:
            oracle_ok = False
        try:
            B.Plan(B.graph_from_spec(ctx, spec))
            lib_ok = True
        except B.RelayError as e:
            assert e.category in ("kind", "shape", "type", "group")
            lib_ok = False
        assert oracle_ok == lib_ok, (spec.name, ctx.last_error())
        n_rej += not lib_ok
    assert 20 < n_rej < 180


def test_failed_op_leaves_graph_unchanged():
    ctx = B.Context()
    g = B.Graph(ctx)
    a = g.input("f32", (2, 3))
    b = g.input("f32", (3,))
    with pytest.raises(B.RelayError) as ei:
        g.op("add", [a, b], [("f32", (2, 3))])
    assert ei.value.category == "type" and "broadcast" in str(ei.value)
    o, (y,) = g.op("relu", [a], [("f32", (2, 3))])
    assert (o, y) == (0, 2)          # ids continue as if the failed call never happened


def test_resnet18_plan_structure():
    spec, raw, bn = W.resnet18(batch=64, dtype="bf16")
    ctx = B.Context()
    plan = B.Plan(B.graph_from_spec(ctx, spec))
    d = plan.describe()
    kernels = [s["kernel"] for s in d["steps"]]
    assert sum(k.startswith("igemm_conv2d") for k in kernels) == 20
    assert sum(k.startswith("igemm_dense") for k in kernels) == 1
    assert kernels.count("maxpool_nhwc") == 1 and kernels.count("gavgpool_nhwc") == 1
    flops = sum(s["flops"] for s in d["steps"] if s["kernel"].startswith("igemm"))
    assert flops == 2 * 64 * (1813561344 + 512000)
    # every conv weight wants a kernel-native copy except the 1x1 projections
    packed = {p["value"] for p in d["packed_params"]}
    names = {spec.values[v].name for v in packed}
    assert "conv1.wf" in names and "l2.b0.ds.wf" not in names and len(names) == 17
    assert 0 < plan.workspace_bytes() < 2 * 64 * 64 * 112 * 112 * 2 * 2


def test_workspace_reuse_is_liveness_safe():
    # two buffers alive at the same step never overlap (checked from the description)
    spec, raw, bn = W.resnet18(batch=2, dtype="f32", image=64)
    plan = B.Plan(B.graph_from_spec(B.Context(), spec))
    total = sum(v.type.shape[0] * v.type.shape[1] * v.type.shape[2] * v.type.shape[3] * 4
                for v in spec.values if v.role == "op" and len(v.type.shape) == 4)
    assert plan.workspace_bytes() < total        # reuse happened


def test_host_side_error_paths_without_gpu():
    spec, data = W.mlp(batch=4, d_in=16, d_hidden=8, d_out=4)
    ctx = B.Context()
    plan = B.Plan(B.graph_from_spec(ctx, spec))
    fake = 0x1000
    with pytest.raises(B.RelayError) as ei:      # missing bindings
        plan.run({0: fake}, fake, 1 << 20)
    assert ei.value.category == "binding"
    with pytest.raises(B.RelayError) as ei:      # unknown id
        plan.run({999: fake}, fake, 1 << 20)
    assert ei.value.category == "binding"
    with pytest.raises(B.RelayError) as ei:      # intermediate is not bindable
        plan.run({5: fake}, fake, 1 << 20)
    assert ei.value.category == "binding"
    with pytest.raises(B.RelayError) as ei:      # misaligned pointer
        plan.run({0: fake + 4}, fake, 1 << 20)
    assert ei.value.category == "align"
    ids = {i: fake for i, v in enumerate(spec.values) if v.role != "op"}
    ids[spec.outputs[0]] = fake
    with pytest.raises(B.RelayError) as ei:      # workspace too small
        plan.run(ids, fake, 16)
    assert ei.value.category == "workspace"
    with pytest.raises(B.RelayError) as ei:      # not a param
        plan.packed_bytes(0)
    assert ei.value.category == "binding"
    assert plan.packed_bytes(1) == 0             # dense weight with K % 4 == 0 is used as is
    # null handles
    assert B.lib().rl_plan_run(None, None, 0, None, 0, None) == -1
    assert B.lib().rl_graph_create(None, None) == -1


def test_cyclic_group_dependency_is_rejected():
    g = W.GraphSpec("cyc")
    a = g.input("a", "f32", (2, 4))
    o0, (y0,) = g.op("relu", [a], [("f32", (2, 4))])
    o1, (y1,) = g.op("neg", [y0], [("f32", (2, 4))])
    o2, (y2,) = g.op("add", [y1, y0], [("f32", (2, 4))])
    g.group([o0, o2])       # o2 needs o1, o1 needs o0: group {o0,o2} and {o1} depend on each other
    g.output(y2)
    with pytest.raises(B.RelayError) as ei:
        B.Plan(B.graph_from_spec(B.Context(), g))
    assert ei.value.category == "group"
