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


def test_degenerate_tensor_types():
    """A dimension is a positive constant (an empty tensor has no type here), a scalar is a rank-0 tensor, the rank and
    the base type are bounded: the degenerate declarations are errors of their own category, and leave the graph as it was."""
    ctx = B.Context()
    g = B.Graph(ctx)
    for shape in [(0, 3), (2, 0), (-1, 3)]:
        with pytest.raises(B.RelayError) as ei:
            g.input("f32", shape)
        assert ei.value.category == "shape" and "positive" in str(ei.value)
    with pytest.raises(B.RelayError) as ei:
        g.input("f32", (1,) * 9)
    assert ei.value.category == "kind" and "rank" in str(ei.value)
    with pytest.raises(B.RelayError) as ei:
        g.input("f16", (2, 2))
    assert ei.value.category == "kind"
    a = g.input("f32", ())                       # rank 0
    assert a == 0                                # none of the failed declarations took an id
    o, (y,) = g.op("tanh", [a], [("f32", ())])
    with pytest.raises(B.RelayError) as ei:      # a scalar is not a rank-1 tensor of one element
        g.op("relu", [y], [("f32", (1,))])
    assert ei.value.category == "type"
    g.group([o]); g.output(y)
    d = B.Plan(g).describe()
    assert [s["kernel"] for s in d["steps"]] == ["eltwise_chain"]


def test_resnet18_plan_structure():
    spec, raw, bn = W.resnet18(batch=64, dtype="bf16")
    ctx = B.Context()
    plan = B.Plan(B.graph_from_spec(ctx, spec))
    d = plan.describe()
    kernels = [s["kernel"] for s in d["steps"]]
    # 20 convolutions; each of the three stride-2 convolutions shares its launch with the 1x1 projection next to it
    assert sum(k.startswith("igemm_conv2d") for k in kernels) == 17
    assert kernels.count("(launched with the step before)") == 3
    assert sum(" | " in s["name"] for s in d["steps"]) == 3
    assert sum(k.startswith("igemm_dense") for k in kernels) == 1
    # the stem group and the max-pool group behind it run as one kernel; the pool kernel is gone from the plan
    # (and it reads the channel-first input itself: no frame copy in front of it)
    assert kernels.count("igemm_conv2d_bf16_stem_maxpool_direct") == 1 and kernels.count("maxpool_nhwc") == 0 and kernels.count("stem_pad_nhwc4") == 0
    k2 = [s["kernel"] for s in B.Plan(B.graph_from_spec(ctx, spec), {"no_stem_direct": 1}).describe()["steps"]]
    assert k2.count("igemm_conv2d_bf16_stem_maxpool") == 1 and k2.count("stem_pad_nhwc4") == 1 and len(k2) == len(kernels) + 1
    assert kernels.count("gavgpool_nhwc") == 1
    flops = sum(s["flops"] for s in d["steps"] if s["kernel"].startswith("igemm"))
    assert flops == 2 * 64 * (1813561344 + 512000)
    # every conv weight wants a kernel-native copy except the 1x1 projections
    packed = {p["value"] for p in d["packed_params"]}
    names = {spec.values[v].name for v in packed}
    assert "conv1.wf" in names and "l2.b0.ds.wf" not in names and len(names) == 17
    assert 0 < plan.workspace_bytes() < 2 * 64 * 64 * 112 * 112 * 2 * 2


def test_workspace_reuse_is_liveness_safe():
    # two workspace buffers that hold live data at the same step never overlap, and all lie inside the workspace
    for spec in (W.resnet18(batch=2, dtype="f32", image=64)[0], W.resnet18(batch=64, dtype="bf16")[0], W.resnet18(batch=1, dtype="f32")[0],
                 W.lenet(5, "bf16")[0], W.mlp()[0], W.lstm_unrolled_graph(4, 8, 64, 64, "bf16", fused=False),
                 W.grad_case("conv2d_grad_w", (64, 128, 28, 28, 128, 3), "bf16", 1, 1, second_is_param=False)[0],
                 W.grad_case("conv2d_grad_x", (64, 64, 56, 56, 128, 3), "bf16", 2, 1)[0], W.grad_chain(8, 128, 28, 3, "bf16")[0]):
        plan = B.Plan(B.graph_from_spec(B.Context(), spec))
        d = plan.describe()
        bufs = d["buffers"]
        ws = plan.workspace_bytes()
        assert d["workspace_bytes"] == ws
        n_steps = len(d["steps"])
        for b in bufs:
            assert b["offset"] % 256 == 0 and b["bytes"] > 0 and b["offset"] + b["bytes"] <= ws
            assert 0 <= b["first"] <= b["last"] < n_steps
        n_shared = 0
        for i, a in enumerate(bufs):
            for b in bufs[i + 1:]:
                live_together = a["first"] <= b["last"] and b["first"] <= a["last"]
                overlap = a["offset"] < b["offset"] + b["bytes"] and b["offset"] < a["offset"] + a["bytes"]
                assert not (live_together and overlap), (spec.name, a, b)
                n_shared += overlap
        if len(bufs) > 3:
            assert n_shared > 0 and ws < sum(b["bytes"] for b in bufs), spec.name        # reuse happened


def test_gradient_operators_plan_onto_the_fast_kernels():
    ctx = B.Context()
    k = lambda spec, opts=None: [s["kernel"] for s in B.Plan(B.graph_from_spec(ctx, spec), opts).describe()["steps"]]
    # with respect to the input, through a param: the forward operator on re-ordered weights ...
    spec = W.grad_case("conv2d_grad_x", (64, 128, 28, 28, 128, 3), "bf16", 1, 1)[0]
    # (its result, a graph output in Shape order, written channel-last by the nine-taps-from-one-copy kernel and transposed)
    assert k(spec) == ["nchw_to_nhwc", "igemm_conv2d_grad_x_bf16_256x128_run", "nhwc_to_nchw"]
    assert k(spec, {"no_out_transpose": 1}) == ["nchw_to_nhwc", "igemm_conv2d_grad_x_bf16_128x128_dma"]
    assert k(spec, {"no_grad_fwd": 1}) == ["igemm_conv2d_grad_x_bf16_64x64_gather"]
    # ... inside a chain on the nine-taps-from-one-copy kernel, like the forward pass
    assert k(W.grad_chain(64, 128, 28, 3, "bf16")[0]) == ["nchw_to_nhwc", "igemm_conv2d_grad_x_bf16_256x128_run", "igemm_conv2d_grad_x_bf16_256x128_run",
                                                         "igemm_conv2d_grad_x_bf16_256x128_run", "nhwc_to_nchw"]
    # ... at a stride on dy spread out with zeros
    spec = W.grad_case("conv2d_grad_x", (64, 64, 56, 56, 128, 3), "bf16", 2, 1)[0]
    assert k(spec) == ["nchw_to_nhwc", "dilate_nhwc", "igemm_conv2d_grad_x_bf16_128x64_lp", "nhwc_to_nchw"]
    assert k(spec, {"no_out_transpose": 1}) == ["nchw_to_nhwc", "dilate_nhwc", "igemm_conv2d_grad_x_bf16_128x64_dma"]
    # through weights that are an activation: the element gather, its operand gathered by a step of the plan
    spec = W.grad_case("conv2d_grad_x", (64, 64, 56, 56, 128, 3), "bf16", 2, 1, second_is_param=False)[0]
    assert k(spec) == ["pack_gather", "igemm_conv2d_grad_x_bf16_64x64_gather"]
    # with respect to the weights, bf16 batches of 64: images-last operands, contraction, ordered reduction
    spec = W.grad_case("conv2d_grad_w", (64, 128, 28, 28, 128, 3), "bf16", 1, 1, second_is_param=False)[0]
    assert k(spec) == ["transpose_images_last", "transpose_images_last", "conv2d_grad_w_bf16_128x64_images_last", "wgrad_reduce"]
    assert k(spec, {"no_wgrad": 1}) == ["pack_gather", "igemm_conv2d_grad_w_bf16_64x64_gather_splitk"]
    for dims, dtype in (((32, 128, 28, 28, 128, 3), "bf16"), ((64, 128, 28, 28, 128, 3), "f32"), ((64, 96, 28, 28, 128, 3), "bf16"), ((64, 128, 28, 28, 128, 5), "bf16")):
        pad = dims[5] // 2
        assert "wgrad_reduce" not in k(W.grad_case("conv2d_grad_w", dims, dtype, 1, pad, second_is_param=False)[0])     # other batches, dtypes, channel counts, filters


def test_plan_options_are_fixed_in_the_plan():
    # the switches travel in the options struct and stay with the plan; a struct larger than the library's is refused
    spec = W.conv_group(16, 64, 64, 56, 56, 3, 1, 1, "bf16", residual=True, relu=True, tail=True)[0]
    ctx = B.Context()
    g = B.graph_from_spec(ctx, spec)
    k = lambda opts: [s["kernel"] for s in B.Plan(g, opts).describe()["steps"] if s["kernel"].startswith("igemm")]
    assert k(None) == ["igemm_conv2d_bf16_3x3_c64"] == k({})
    assert k({"no_c64": 1}) == ["igemm_conv2d_bf16_128x64_lp"]
    assert k({"no_c64": 1, "ws_all": 1}) == ["igemm_conv2d_bf16_128x64_ws"]
    assert k({"no_c64": 1, "no_lp": 1}) == ["igemm_conv2d_bf16_128x64_dma"]
    assert k(None) == ["igemm_conv2d_bf16_3x3_c64"]
    o = B.make_opts({})
    o.struct_size = ctypes.sizeof(B.rl_plan_opts) + 4
    h = ctypes.c_void_p()
    assert B.lib().rl_plan_create(g._h, ctypes.byref(o), ctypes.byref(h)) == -2 and "struct_size" in ctx.last_error()
    o.struct_size = 8                              # an older caller that only knows the first switch
    o.no_lp = 1; o.no_c64 = 1                      # the second lies beyond its struct and must be ignored
    assert B.lib().rl_plan_create(g._h, ctypes.byref(o), ctypes.byref(h)) == 0
    B.lib().rl_plan_destroy(h)
    with pytest.raises(KeyError):
        B.make_opts({"no_such_switch": 1})


def test_static_entry_point_refuses_plans_beyond_its_workspace():
    # decided on the host before anything touches a GPU
    spec = W.resnet18(batch=64, dtype="bf16")[0]
    ctx = B.Context()
    plan = B.Plan(B.graph_from_spec(ctx, spec))
    assert plan.workspace_bytes() > B.STATIC_WORKSPACE_BYTES
    header = open(os.path.join(ROOT, "include", "relayhip.h")).read()
    assert re.search(r"#define RL_STATIC_WORKSPACE_BYTES \((\d+)u << 20\)", header).group(1) == str(B.STATIC_WORKSPACE_BYTES >> 20)
    with pytest.raises(B.RelayError) as ei:
        plan.run_static({0: 0x1000}, 0)
    assert ei.value.category == "workspace" and str(B.STATIC_WORKSPACE_BYTES) in str(ei.value)
    assert B.lib().rl_plan_run_static(None, None, 0, None) == -1


def test_recurrent_call_rejects_mismatched_roles_on_the_host():
    fake = 0x10000
    ctx = B.Context()
    # h' declared f32 while the cell's h operand is bf16: feeding h' back as h would reinterpret the bytes
    g = W.GraphSpec("cell")
    Bt, I, H = 4, 32, 32
    x = g.input("x", "bf16", (Bt, I)); h = g.input("h", "bf16", (Bt, H)); c = g.input("c", "f32", (Bt, H))
    w = g.param("w", "bf16", (4 * H, I + H)); b = g.param("b", "f32", (4 * H,))
    o0, (xh,) = g.op("concat", [x, h], [("bf16", (Bt, I + H))], axis=1)
    o1, (z,) = g.op("dense", [xh, w], [("f32", (Bt, 4 * H))], out_dtype="f32")
    o2, (z,) = g.op("bias_add", [z, b], [("f32", (Bt, 4 * H))], axis=1)
    o3, (c2, h2) = g.op("lstm_gates", [z, c], [("f32", (Bt, H)), ("f32", (Bt, H))])
    g.group([o0, o1, o2, o3]); g.output(c2); g.output(h2)
    plan = B.Plan(B.graph_from_spec(ctx, g))
    roles = {"x": x, "h_in": h, "c_in": c, "c_out": c2, "h_out": h2}
    with pytest.raises(B.RelayError) as ei:
        plan.run_recurrent(3, roles, fake, Bt * I * 2, fake, fake, fake, Bt * H * 4, {w: fake, b: fake}, fake, 1 << 20)
    assert ei.value.category == "binding" and "h input" in str(ei.value)
    # well-typed cell: strides smaller than a step's tensors would make the steps overlap
    spec = W.lstm_cell_graph(Bt, I, H, "bf16", True)
    n = {v.name: i for i, v in enumerate(spec.values)}
    plan = B.Plan(B.graph_from_spec(ctx, spec))
    roles = {"x": n["x"], "h_in": n["h"], "c_in": n["c"], "c_out": spec.outputs[0], "h_out": spec.outputs[1]}
    params = {n["w"]: fake, n["b"]: fake}
    for xs, hs, what in ((Bt * I * 2 - 16, Bt * H * 2, "x_step_bytes"), (Bt * I * 2, Bt * H * 2 - 16, "h_step_bytes")):
        with pytest.raises(B.RelayError) as ei:
            plan.run_recurrent(3, roles, fake, xs, fake, fake, fake, hs, params, fake, 1 << 20)
        assert ei.value.category == "binding" and what in str(ei.value)
    # c' played by a value of another type than c
    with pytest.raises(B.RelayError) as ei:
        plan.run_recurrent(3, dict(roles, c_out=spec.outputs[1], h_out=spec.outputs[0]), fake, Bt * I * 2, fake, fake, fake, Bt * H * 4, params,
                           fake, 1 << 20)
    assert ei.value.category == "binding"
    # zero steps of a well-formed call launch nothing and succeed without a GPU
    plan.run_recurrent(0, roles, fake, Bt * I * 2, fake, fake, fake, Bt * H * 2, params, fake, 1 << 20)


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


# ---------------------------------------------------------------- automatic fusion (host logic only)
def _auto(spec):
    g = B.graph_from_spec(B.Context(), spec, auto_groups=True)
    return g, g.groups(len(spec.ops))


@pytest.mark.parametrize("name,build", [
    ("mlp", lambda: W.mlp()[0]),
    ("conv group", lambda: W.conv_group()[0]),
    ("resnet18 f32 b1", lambda: W.resnet18(1, "f32")[0]),
    ("resnet18 bf16 b64", lambda: W.resnet18(64, "bf16")[0]),
    ("lstm cell", lambda: W.lstm_cell_graph(64, 1024, 1024, "bf16", True)),
    ("lstm unrolled", lambda: W.lstm_unrolled_graph(3, 16, 32, 32, "bf16", True)),
    ("lenet", lambda: W.lenet()[0]),
    ("eltwise", lambda: W.eltwise_bias_res_relu((4, 8, 6, 6))[0]),
    ("eltwise chain", lambda: W.eltwise_chain()[0]),
    ("channel-last block", lambda: W.channel_last_block()[0]),
])
def test_autogroup_reproduces_the_declared_groups(name, build):
    # the pass, run on the bare calls, must arrive at the grouping every workload declares by hand,
    # and the result must plan
    spec = build()
    g, got = _auto(spec)
    assert got == [sorted(x) for x in spec.groups]
    B.Plan(g)


def test_autogroup_rules():
    # y = relu(conv(x) + b); z = neg(y); outputs y and z: y is an output, so neg must not be absorbed
    g = W.GraphSpec("t")
    x = g.input("x", "f32", (1, 8, 6, 6)); w = g.param("w", "f32", (8, 8, 3, 3)); b = g.param("b", "f32", (8,))
    t = ("f32", (1, 8, 6, 6))
    o0, (y,) = g.op("conv2d", [x, w], [t], stride=(1, 1), pad=(1, 1))
    o1, (y,) = g.op("bias_add", [y, b], [t], axis=1)
    o2, (y,) = g.op("relu", [y], [t])
    o3, (z,) = g.op("neg", [y], [t])
    g.output(y); g.output(z)
    assert _auto(g)[1] == [[o0, o1, o2], [o3]]

    # a result with two uses ends its group.  Of its users, relu cannot take the add: the add's other operand (tanh's
    # result) is defined after relu's group opened; tanh cannot either, because the add does not take tanh's result
    # first.  With the operands the other way round tanh's group absorbs the add.
    for swap, want in ((False, lambda o: [[o[0]], [o[1]], [o[2]], [o[3]]]), (True, lambda o: [[o[0]], [o[1]], [o[2], o[3]]])):
        g = W.GraphSpec("t")
        x = g.input("x", "f32", (4, 16)); w = g.param("w", "f32", (16, 16))
        t = ("f32", (4, 16))
        o0, (y,) = g.op("dense", [x, w], [t])
        o1, (a,) = g.op("relu", [y], [t])
        o2, (c,) = g.op("tanh", [y], [t])
        o3, (d,) = g.op("add", [c, a] if swap else [a, c], [t])
        g.output(d)
        lib, got = _auto(g)
        assert got == want([o0, o1, o2, o3])
        B.Plan(lib)

    # the gate operator joins a dense contraction's group (through its bias), but behind a bare injective chain it stays
    # a group of its own -- and either graph plans
    g = W.lstm_cell_graph(2, 64, 64, "bf16", True); g.groups.clear()
    lib, got = _auto(g)
    assert got == [[0, 1, 2, 3]]
    B.Plan(lib)
    g = W.GraphSpec("t")
    z = g.input("z", "f32", (2, 64)); b = g.param("b", "f32", (64,)); c = g.input("c", "f32", (2, 16))
    o0, (zb,) = g.op("bias_add", [z, b], [("f32", (2, 64))], axis=1)
    o1, (c2, h2) = g.op("lstm_gates", [zb, c], [("f32", (2, 16)), ("f32", (2, 16))])
    g.output(c2); g.output(h2)
    lib, got = _auto(g)
    assert got == [[o0], [o1]]
    assert [s["kernel"] for s in B.Plan(lib).describe()["steps"]] == ["eltwise_chain", "lstm_gates"]

    # a second contraction never joins; pools stay alone; hand-declared groups are kept
    g = W.GraphSpec("t")
    x = g.input("x", "f32", (2, 8, 8, 8)); w1 = g.param("w1", "f32", (8, 8, 1, 1)); w2 = g.param("w2", "f32", (8, 8, 1, 1))
    t = ("f32", (2, 8, 8, 8))
    o0, (y,) = g.op("conv2d", [x, w1], [t], stride=(1, 1), pad=(0, 0))
    o1, (y,) = g.op("relu", [y], [t])
    o2, (y,) = g.op("conv2d", [y, w2], [t], stride=(1, 1), pad=(0, 0))
    o3, (y,) = g.op("maxpool2d", [y], [("f32", (2, 8, 4, 4))], kernel=(2, 2), stride=(2, 2), pad=(0, 0))
    o4, (y,) = g.op("relu", [y], [("f32", (2, 8, 4, 4))])
    g.output(y)
    assert _auto(g)[1] == [[o0, o1], [o2], [o3], [o4]]
    g.groups = [[o0]]                                     # the caller fixes conv alone: relu must then stand alone too
    lib = B.graph_from_spec(B.Context(), g)               # declares [o0], then outputs
    lib.autogroup()
    assert lib.groups(len(g.ops)) == [[o0], [o1], [o2], [o3], [o4]]
    assert lib.autogroup() == 0                           # nothing left to group


# ---------------------------------------------------------------- typed changes of layout (host logic only)
def _plan_steps(spec):
    plan = B.Plan(B.graph_from_spec(B.Context(), spec))
    return [(s["name"], s["kernel"]) for s in plan.describe()["steps"]]


def test_channel_last_views_cost_no_kernel():
    # channel-last input and output around two convolution groups: the planner runs those channel-last anyway, so
    # the two layout_transform calls alias storage: two launches, no transposition, no copy
    steps = _plan_steps(W.channel_last_block(3, 64, 14, 14, "bf16")[0])
    assert len(steps) == 2 and all(k.startswith("igemm_conv2d") for _, k in steps), steps
    # without the typed view a channel-first input is transposed first (and the last group writes channel-first)
    g, _ = W.conv_group(batch=3, cin=64, cout=64, h=14, w=14, dtype="bf16")
    assert [k for _, k in _plan_steps(g)][0] == "nchw_to_nhwc"


def test_layout_transform_kernel_choice():
    kern = lambda shape, perm: [k for _, k in _plan_steps(W.layout_case(shape, perm, "f32")[0])]
    assert kern((3, 5, 7, 4), (0, 2, 3, 1)) == ["transpose_tiled"]          # batched transposition
    assert kern((3, 5, 7, 4), (0, 3, 1, 2)) == ["nhwc_to_nchw"]             # the result is wanted in Shape order: one transposition
    assert kern((6, 10), (1, 0)) == ["transpose_tiled"]
    assert kern((2, 3, 4, 5, 6), (0, 1, 4, 2, 3)) == ["transpose_tiled"]
    assert kern((2, 3, 4, 5), (2, 0, 3, 1)) == ["permute_gather"]
    assert kern((2, 3, 4), (0, 1, 2)) == ["eltwise_chain"]                  # identity: the copy into the output buffer
    assert kern((2, 1, 4, 5), (0, 2, 3, 1)) == ["eltwise_chain"]            # one channel: same order in memory


# ---------------------------------------------------------------- K split over workgroups (host logic only)
def test_split_k_is_planned_for_few_tiles_and_long_k():
    def kernels(spec, opts=None):
        d = B.Plan(B.graph_from_spec(B.Context(), spec), opts).describe()
        return [s["kernel"] for s in d["steps"] if s["kernel"].startswith("igemm")], d["workspace_bytes"]
    # batch 1, 512 -> 512 channels on 7x7: 8 tiles of 64x64, 144 K tiles of 32: split, and the scratch tensor
    # [16 slices][49][512] f32 is part of the workspace
    spec = W.conv_group(1, 512, 512, 7, 7, 3, 1, 1, "f32")[0]
    k, ws = kernels(spec)
    assert k == ["igemm_conv2d_f32_64x64_dma_splitk"] and ws >= 16 * 49 * 512 * 4
    k1, ws1 = kernels(spec, {"no_splitk": 1})
    assert k1 == ["igemm_conv2d_f32_64x64_dma"] and ws1 < ws
    # many tiles: no split; the benchmark graph (batch 64, bf16) has none either
    assert not any(x.endswith("_splitk") for x in kernels(W.conv_group(16, 64, 64, 56, 56, 3, 1, 1, "f32")[0])[0])
    assert not any(x.endswith("_splitk") for x in kernels(W.resnet18(64, "bf16")[0])[0])
    # a dense contraction with a partial last K tile (784 = 24.5 x 32) takes the direct-load kernel
    assert kernels(W.mlp(32, 784, 128, 10, "f32")[0], {"no_dense_chain": 1})[0] == ["igemm_dense_f32_64x64_dma_splitk", "igemm_dense_f32_64x64_dma"]
    # ... and, by default, its adding launch also runs the 128 -> 10 layer behind it
    d = B.Plan(B.graph_from_spec(B.Context(), W.mlp(32, 784, 128, 10, "f32")[0])).describe()
    assert [s["kernel"] for s in d["steps"]] == ["igemm_dense_f32_64x64_dma_splitk+dense", "(launched with the step before)"]
    assert d["steps"][1]["flops"] == 0 and d["steps"][0]["flops"] == 2.0 * 32 * (784 * 128 + 128 * 10)
