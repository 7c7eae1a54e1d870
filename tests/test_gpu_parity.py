"""Parity of the HIP library against the CPU oracle, element by element, on
seeded synthetic inputs -- needs an MI355X.  Every call goes through the C ABI."""
import numpy as np
import pytest

import oracle as O
from oracle import graph as OG
import workloads as W
from helpers import assert_close, error_budget, extract_group, extract_groups_channel_last, fold_resnet_hip, fold_resnet_oracle, run_hip, store_as

pytestmark = pytest.mark.gpu


def check_graph(spec, data, what, opts=None, rms_scaled=False):
    # fp32: the stated gate; an element outside it must lie within the first-order fp32 error budget of the graph
    # (computed only when needed); rms_scaled is for deep graphs, where that budget is vacuous
    ref = OG.run(spec, data)
    got, _ = run_hip(spec, data, opts=opts)
    for vid in spec.outputs:
        dt = spec.values[vid].type.dtype
        budget = None if (dt == "bf16" or rms_scaled) else (lambda vid=vid: error_budget(spec, data)[vid])
        assert_close(got[vid], ref[vid], dt, f"{what} value {vid}", budget=budget, rms_scaled=rms_scaled)
    return got, ref


# ------------------------------------------------------------------ dense / MLP
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("batch,d_in,d_hidden,d_out", [(32, 784, 128, 10), (1, 8, 8, 8), (70, 200, 136, 24), (5, 30, 7, 3), (300, 512, 256, 72)])
def test_mlp(dtype, batch, d_in, d_hidden, d_out):
    if dtype == "bf16" and d_hidden % 8:
        d_hidden += 8 - d_hidden % 8
    spec, data = W.mlp(batch, d_in, d_hidden, d_out, dtype)
    check_graph(spec, data, f"mlp {dtype} {batch}x{d_in}x{d_hidden}x{d_out}")


DENSE_CHAIN_CASES = [(32, 784, 128, 10, "f32"), (32, 784, 128, 10, "bf16"), (1, 800, 500, 10, "f32"), (64, 800, 500, 10, "f32"), (7, 2048, 2048, 64, "f32"),
                     (130, 1024, 136, 3, "f32"), (5, 516, 100, 1, "f32"), (33, 1000, 72, 24, "bf16")]


@pytest.mark.parametrize("case", DENSE_CHAIN_CASES, ids=[f"b{c[0]}-{c[1]}-{c[2]}-{c[3]}-{c[4]}" for c in DENSE_CHAIN_CASES])
def test_small_dense_layer_behind_a_split_contraction_rides_on_its_adding_launch(case):
    # two launches (split contraction; its slices added, epilogue, the small layer) against three or four, the tensor
    # between the groups never stored: against the oracle like every other plan, and the same plan without the chain
    # beside it (the small layer's sums run in another order there, so the two agree to rounding, not to the bit)
    b, d_in, d_h, d_out, dtype = case
    spec, data = W.mlp(b, d_in, d_h, d_out, dtype)
    ks = [st["kernel"] for st in s_plan_steps(spec)]
    assert ks[-2].endswith("_splitk+dense") and ks[-1] == "(launched with the step before)", ks
    assert not any(k.endswith("+dense") for k in [st["kernel"] for st in s_plan_steps(spec, {"no_dense_chain": 1})])
    got, ref = check_graph(spec, data, f"dense chain {case}")
    got2, _ = check_graph(spec, data, f"dense chain {case} as separate steps", opts={"no_dense_chain": 1})
    for vid in spec.outputs:
        assert_close(got[vid], got2[vid], dtype, f"dense chain {case}: chained against separate")


def test_dense_chain_is_not_planned_where_the_tensor_between_is_needed():
    # the hidden tensor as a graph output, or read by a third group: the plan keeps the steps apart
    spec, data = W.mlp(32, 784, 128, 10, "f32")
    spec.output(spec.ops[2].outputs[0])             # the first group's result is an output too
    assert not any(st["kernel"].endswith("+dense") for st in s_plan_steps(spec))
    check_graph(spec, data, "mlp with its hidden layer as an output")
    spec, data = W.mlp(32, 784, 128, 100, "f32")    # a second layer wider than the chain takes
    assert not any(st["kernel"].endswith("+dense") for st in s_plan_steps(spec))


def test_dense_gather_path_odd_k():
    # K not a multiple of the 16-byte vector: weights are re-laid-out with zero padding, A rows are gathered
    for dtype, k in (("f32", 30), ("bf16", 30), ("f32", 5), ("bf16", 77)):
        spec, data = W.mlp(9, k, 16, 6, dtype)
        check_graph(spec, data, f"mlp odd K {dtype} {k}")


def test_dense_with_a_partial_last_k_tile():
    # K a multiple of the 16-byte vector but not of the K tile: direct-load kernel on zero-padded weight rows, the
    # activation chunks past K requested out of range
    from paper_1810_00952_amd import binding
    for dtype, batch, k, hidden in (("f32", 5, 100, 36), ("bf16", 70, 200, 136), ("f32", 3, 68, 8), ("bf16", 33, 456, 72)):
        spec, data = W.mlp(batch, k, hidden, 8, dtype)
        desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
        assert "_dma" in desc["steps"][0]["kernel"], desc["steps"][0]["kernel"]
        got, _ = check_graph(spec, data, f"mlp partial K tile {dtype} {k}")
        # what lies behind a row's K elements (the next row) must not leak into it, whatever it is
        x = data["x"].copy()
        if dtype == "bf16":
            x[1:, :16] = 0x7F80                        # +inf in bf16
        else:
            x[1:, :16] = np.inf
        poisoned, _ = run_hip(spec, dict(data, x=x))
        v = spec.outputs[0]
        np.testing.assert_array_equal(poisoned[v][0], got[v][0])


# ------------------------------------------------------------------ conv groups
CONV_CASES = [
    # batch cin cout h  w  k s p residual relu
    (1, 64, 64, 56, 56, 3, 1, 1, False, True),      # the single-group configuration
    (2, 8, 24, 13, 11, 3, 1, 1, True, True),        # ragged M and N tails
    (3, 16, 40, 15, 15, 3, 2, 1, False, True),      # stride 2
    (2, 32, 64, 14, 14, 1, 2, 0, False, False),     # 1x1 stride-2 projection, no ReLU
    (1, 3, 16, 33, 33, 7, 2, 3, False, True),       # 3 input channels: gather path straight from NCHW
    (2, 5, 7, 9, 10, 3, 1, 0, True, False),         # odd everything
    (1, 128, 128, 28, 28, 3, 1, 1, True, True),     # 128-wide tiles
    (2, 64, 130, 20, 20, 3, 1, 1, False, True),     # N tail on a 128 tile
    (1, 8, 8, 3, 3, 3, 1, 1, False, False),         # input as small as the kernel
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", CONV_CASES, ids=[f"c{i}" for i in range(len(CONV_CASES))])
def test_conv_group(dtype, case):
    b, ci, co, h, w, k, s, p, res, relu = case
    spec, data = W.conv_group(b, ci, co, h, w, k, s, p, dtype, residual=res, relu=relu)
    check_graph(spec, data, f"conv {dtype} {case}")


# The conv group's result stays an intermediate (channel-last inside the plan), which is what selects the
# pixel-on-lane bf16 kernel: every tile shape, stride-2 and 1x1 taps, K tiles spanning several taps,
# ragged M tails inside and across tiles, N tails on 8-channel granularity, and epilogues with and
# without residual / ReLU.
LP_CASES = [
    # batch cin cout h  w  k s p residual relu
    (2, 64, 64, 14, 14, 3, 1, 1, True, True),        # 64x64 tile, M = 392
    (3, 64, 128, 29, 29, 3, 1, 1, True, True),       # M = 2523: ragged last tile
    (16, 64, 64, 56, 56, 3, 1, 1, True, True),       # 128x64 tile, two workgroups per CU
    (16, 128, 128, 28, 28, 3, 1, 1, False, True),    # 128x128 tile, 18 K tiles
    (4, 64, 128, 57, 57, 3, 2, 1, False, True),      # stride 2, odd image
    (4, 64, 136, 28, 28, 1, 2, 0, False, False),     # 1x1 stride-2 projection: a single K tile, N tail of 8
    (2, 128, 72, 9, 7, 3, 1, 1, True, False),        # N = 72, no ReLU
    (1, 192, 64, 5, 5, 5, 1, 2, False, True),        # 25 taps, 3 K tiles per tap
    (2, 256, 512, 7, 7, 3, 1, 1, True, True),        # image smaller than a tile row block
    (40, 64, 64, 30, 30, 1, 1, 0, True, True),       # 1x1, M = 36000: many tiles, K = one tile
    (17, 64, 136, 55, 55, 3, 1, 1, True, True),      # 256x128 tile (eight waves), ragged M tail, N tail of 8
]


@pytest.mark.parametrize("case", LP_CASES, ids=[f"lp{i}" for i in range(len(LP_CASES))])
def test_conv_group_internal_layout_bf16(case):
    opts = {"no_c64": 1, "no_run": 1}                # the general kernel also on the shapes that have one of their own
    b, ci, co, h, w, k, s, p, res, relu = case
    spec, data = W.conv_group(b, ci, co, h, w, k, s, p, "bf16", residual=res, relu=relu, tail=True)
    from paper_1810_00952_amd import binding
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec), opts).describe()
    assert any(st["kernel"].endswith(("_lp", "_ws")) for st in desc["steps"]), [st["kernel"] for st in desc["steps"]]
    check_graph(spec, data, f"conv lp {case}", opts=opts)


def test_conv_weights_stationary_shallow_ring():
    # K = 576 (9 weight tiles, 5-stage ring, residual through the ring): opt-in, the planner prefers the per-tile kernel there
    opts = {"ws_all": 1, "no_c64": 1}
    for case in [(16, 64, 64, 56, 56, 3, 1, 1, True, True), (3, 64, 48, 29, 31, 3, 1, 1, False, True)]:
        b, ci, co, h, w, k, s, p, res, relu = case
        spec, data = W.conv_group(b, ci, co, h, w, k, s, p, "bf16", residual=res, relu=relu, tail=True)
        from paper_1810_00952_amd import binding
        desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec), opts).describe()
        assert any(st["kernel"].endswith("_ws") for st in desc["steps"]), [st["kernel"] for st in desc["steps"]]
        check_graph(spec, data, f"conv ws {case}", opts=opts)


STEM_CASES = [
    # batch cin cout h   w   k s p relu
    (2, 3, 64, 224, 224, 7, 2, 3, True),     # the ResNet stem
    (3, 3, 16, 33, 35, 7, 2, 3, True),       # odd sizes, ragged M
    (2, 1, 8, 20, 20, 5, 2, 2, False),       # one channel, 5x5
    (2, 4, 32, 17, 18, 3, 2, 1, True),       # four channels, 3x3
    (1, 2, 24, 12, 40, 8, 4, 0, True),       # 8-wide filter, stride 4
]


@pytest.mark.parametrize("case", STEM_CASES, ids=[f"stem{i}" for i in range(len(STEM_CASES))])
def test_conv_stem_few_channels_bf16(case):
    b, ci, co, h, w, k, s, p, relu = case
    spec, data = W.conv_group(b, ci, co, h, w, k, s, p, "bf16", relu=relu, tail=True)
    from paper_1810_00952_amd import binding
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
    assert any(st["kernel"] == "stem_pad_nhwc4" for st in desc["steps"]), [st["kernel"] for st in desc["steps"]]
    check_graph(spec, data, f"conv stem {case}")


# Stem convolution + max-pool 3x3/2/1 as one kernel: regions at every image border, images smaller than a region,
# fewer and more regions than workgroups (so workgroups stream on from one region into the next), one, three and
# four input channels, 7- and 8-wide filters, with and without ReLU, pooled tensor as output and as intermediate.
STEM_POOL_CASES = [
    # batch cin h    w   k s p relu  tail
    (2, 3, 224, 224, 7, 2, 3, True, False),
    (3, 3, 33, 35, 7, 2, 3, True, True),
    (5, 1, 12, 12, 7, 2, 3, False, False),
    (70, 3, 64, 64, 7, 2, 3, True, False),
    (9, 4, 61, 127, 8, 2, 3, True, True),
    (1, 3, 7, 250, 7, 2, 3, False, True),
    (64, 3, 224, 224, 7, 2, 3, True, True),          # the benchmark's stem at full size: 12 544 regions streaming through 512 workgroups
    (4, 2, 30, 46, 5, 2, 2, False, True),            # two planes, 5x5 with even padding (the window starts at the filter)
    (3, 3, 40, 38, 8, 2, 4, True, False),            # 8x8 filter, even padding: every window column and both rows of the last pair used
    (2, 3, 9, 12, 3, 2, 1, True, True),              # 3x3: two row pairs per plane, half of the second one zero weights
]


@pytest.mark.parametrize("case", STEM_POOL_CASES, ids=[f"sp{i}" for i in range(len(STEM_POOL_CASES))])
def test_stem_conv_with_maxpool_in_one_kernel(case):
    b, ci, h, w, k, s_, p, relu, tail = case
    spec, data = W.conv_pool(b, ci, 64, h, w, k, s_, p, "bf16", relu=relu, tail=tail)
    from paper_1810_00952_amd import binding
    kernels = [st["kernel"] for st in binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()["steps"]]
    # up to three planes of even width, and a filter that fits the 8-pixel window: patches fetched from the channel-first
    # input itself, no frame copy; everything else through the padded 4-channel frame
    direct = ci <= 3 and w % 2 == 0 and k + (p & 1) <= 8
    assert ("igemm_conv2d_bf16_stem_maxpool_direct" in kernels) == direct and ("stem_pad_nhwc4" in kernels) == (not direct), kernels
    assert any(kn.startswith("igemm_conv2d_bf16_stem_maxpool") for kn in kernels), kernels
    print(f"stem+pool case {case}", flush=True)
    check_graph(spec, data, f"stem+pool {case}")
    # the frame form of the fused kernel (filters 7 or 8 rows high; its own contraction order) ...
    kernels = [st["kernel"] for st in binding.Plan(binding.graph_from_spec(binding.Context(), spec), {"no_stem_direct": 1}).describe()["steps"]]
    assert ("igemm_conv2d_bf16_stem_maxpool" in kernels) == (k >= 7) and "stem_pad_nhwc4" in kernels, kernels
    got, _ = check_graph(spec, data, f"stem+pool {case} from the frame", opts={"no_stem_direct": 1})
    # ... gives the same bits as the two-kernel form of the same plan: max commutes with bias, ReLU and the rounding
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec), {"no_stem_pool": 1}).describe()
    assert any(st["kernel"] == "maxpool_nhwc" for st in desc["steps"])
    two, _ = run_hip(spec, data, opts={"no_stem_pool": 1})
    for vid in spec.outputs:
        np.testing.assert_array_equal(got[vid], two[vid])


# 3x3 / stride 1 / pad 1 convolution from 64 to 64 channels with weights in registers: images smaller than a region,
# exactly one region, regions that end inside an image row, rows of 1 and of 63 pixels (the widest it takes), one
# image row, fewer and more regions than workgroups, every epilogue form it accepts.
C64_CASES = [
    # batch h   w  bias  residual relu
    (2, 56, 56, True, True, True),
    (1, 5, 7, True, False, True),
    (5, 16, 16, True, True, False),
    (3, 9, 63, False, True, True),
    (2, 40, 1, True, False, False),
    (2, 1, 40, False, False, False),
    (1, 33, 31, False, False, True),
    (70, 28, 30, True, True, True),
]


@pytest.mark.parametrize("case", C64_CASES, ids=[f"c64_{i}" for i in range(len(C64_CASES))])
def test_conv3x3_c64_weights_in_registers(case):
    b, h, w, bias, res, relu = case
    spec, data = W.conv_group(b, 64, 64, h, w, 3, 1, 1, "bf16", residual=res, relu=relu, tail=True, bias=bias)
    from paper_1810_00952_amd import binding
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
    assert any(st["kernel"] == "igemm_conv2d_bf16_3x3_c64" for st in desc["steps"]), [st["kernel"] for st in desc["steps"]]
    print(f"conv3x3_c64 case {case}", flush=True)
    got, _ = check_graph(spec, data, f"conv3x3_c64 {case}")
    # the general kernel accumulates the same 16-element slices of K in the same order: same bits
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec), {"no_c64": 1}).describe()
    assert not any(st["kernel"] == "igemm_conv2d_bf16_3x3_c64" for st in desc["steps"])
    gen, _ = run_hip(spec, data, opts={"no_c64": 1})
    for vid in spec.outputs:
        np.testing.assert_array_equal(got[vid], gen[vid])


# 3x3 / stride 1 / pad 1 convolutions on short image rows, nine taps read from one copy of the input rows: each of
# its three tiles, one, two, three and four 64-channel slices, rows of 7 to 30 pixels, images smaller than a tile
# (so that a tile spans several), ragged M and N tails, every epilogue form.
RUN_CASES = [
    # batch cin cout h   w  bias  residual relu   tile
    (16, 128, 128, 28, 28, True, True, True, "128x64"),
    (196, 192, 72, 7, 9, True, False, False, "128x64"),
    (140, 64, 128, 3, 30, False, True, True, "128x64"),
    (196, 256, 72, 7, 9, False, True, True, "128x64"),      # even slice count: K split over the waves; N tail
    (16, 128, 256, 28, 28, True, True, True, "128x128"),
    (64, 256, 256, 14, 14, False, False, True, "128x128"),
    (16, 192, 264, 28, 28, True, False, True, "128x128"),    # odd slice count: eight waves with 64x32 tiles; N tail
    (63, 128, 128, 28, 28, True, True, True, "256x128"),
    (64, 512, 512, 7, 7, True, True, True, "128x64"),       # the benchmark's last stage: K split over the waves, tiles numbered channel-tile-major
]


@pytest.mark.parametrize("case", RUN_CASES, ids=[f"run{i}" for i in range(len(RUN_CASES))])
def test_conv3x3_taps_from_one_copy_of_the_rows(case):
    b, ci, co, h, w, bias, res, relu, tile = case
    spec, data = W.conv_group(b, ci, co, h, w, 3, 1, 1, "bf16", residual=res, relu=relu, tail=True, bias=bias)
    from paper_1810_00952_amd import binding
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
    assert any(st["kernel"] == f"igemm_conv2d_bf16_{tile}_run" for st in desc["steps"]), [st["kernel"] for st in desc["steps"]]
    if ci == 512:
        st = [st for st in desc["steps"] if st["kernel"].endswith("_run")][0]
        assert st["k_split_waves"] == 1 and st["channel_tile_major"] == 1, st
    print(f"conv3x3 run case {case}", flush=True)
    got, _ = check_graph(spec, data, f"conv3x3 run {case}")
    # against the general kernel: same products, another summation order
    gen, _ = run_hip(spec, data, opts={"no_run": 1})
    for vid in spec.outputs:
        assert_close(got[vid], gen[vid], "bf16", f"run vs general {case}")


# A stage's stride-2 convolution and its 1x1 projection go out as one grid: every kernel variant that can be
# shared (64x64, 128x64 in both depths, 128x128, 256x128), and the same bits as two launches.
PAIR_CASES = [
    # batch cin cout h   w
    (4, 64, 128, 32, 32),        # 64x64 tiles
    (27, 64, 128, 56, 56),       # 128x64, three stages (two workgroups per CU)
    (16, 64, 128, 56, 56),       # 128x64, four stages
    (17, 64, 136, 55, 57),       # 128x128, odd image, N tail
    (64, 64, 128, 56, 56),       # 256x128
    (8, 128, 256, 28, 28),       # the projection reads 128 channels: two K tiles
    (64, 128, 256, 28, 28),      # the benchmark's second pair
    (3, 128, 384, 9, 11),        # six channel chunks, ragged pixel tiles
    (2, 64, 256, 5, 7),          # fewer pixel tiles than waves
    (9, 256, 512, 14, 14),       # 256 input channels: four K tiles
]


@pytest.mark.parametrize("case", PAIR_CASES, ids=[f"pair{i}" for i in range(len(PAIR_CASES))])
def test_independent_contractions_in_one_launch(case):
    b, ci, co, h, w = case
    spec, data = W.downsample_block(b, ci, co, h, w, "bf16")
    from paper_1810_00952_amd import binding
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
    assert sum(st["kernel"] == "(launched with the step before)" for st in desc["steps"]) == 1, [st["kernel"] for st in desc["steps"]]
    assert not any(st["kernel"].endswith("3x3s2_pair") for st in desc["steps"])
    print(f"paired launch case {case}: {[st['kernel'] for st in desc['steps']]}", flush=True)
    got, _ = check_graph(spec, data, f"paired launch {case}")
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec), {"no_pair": 1}).describe()
    assert not any(st["kernel"] == "(launched with the step before)" for st in desc["steps"])
    two, _ = run_hip(spec, data, opts={"no_pair": 1})
    for vid in spec.outputs:
        np.testing.assert_array_equal(got[vid], two[vid])


# The same pair as ONE contraction (the projection's K tile rides on the 3x3 window's centre tap, second accumulators):
# one, two, three and four 64-channel slices, rows of 3 to 28 output pixels (both run-buffer sizes), images smaller than
# a tile (so that a tile spans several) and tiles that end inside an image row, ragged M and N tails, a single tile.
# Both convolutions' own results are compared (tapped as channel-last views), then the block's.
S2_PAIR_CASES = [
    # batch cin cout h   w
    (4, 64, 128, 32, 32),
    (16, 64, 128, 56, 56),       # the benchmark's first pair at a quarter of its batch: rows of 28, the larger run buffer
    (8, 128, 256, 28, 28),       # two slices
    (9, 256, 512, 14, 14),       # four slices, rows of 7: nine images under a tile
    (3, 192, 72, 12, 20),        # three slices, N tail inside the only channel tile
    (5, 64, 136, 6, 10),         # N tail in a second channel tile, tiny images
    (1, 64, 128, 2, 2),          # a single output pixel
    (7, 128, 264, 10, 38),       # rows of 19, ragged last tile
]


@pytest.mark.parametrize("case", S2_PAIR_CASES, ids=[f"s2pair{i}" for i in range(len(S2_PAIR_CASES))])
def test_stride2_convolution_and_projection_as_one_contraction(case):
    b, ci, co, h, w = case
    spec, data = W.downsample_block(b, ci, co, h, w, "bf16", taps=True)
    from paper_1810_00952_amd import binding
    opts = {"s2_pair": 1}                           # opt-in: the planner's own choice is two contractions in one grid
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec), opts).describe()
    assert sum(st["kernel"] == "igemm_conv2d_bf16_3x3s2_pair" for st in desc["steps"]) == 1, [st["kernel"] for st in desc["steps"]]
    print(f"stride-2 pair case {case}: {[st['kernel'] for st in desc['steps']]}", flush=True)
    ref = OG.run(spec, data)
    got, _ = run_hip(spec, data, opts=opts)
    y, c1, d = spec.outputs
    for vid, what in ((c1, "3x3/2"), (d, "1x1/2 projection"), (y, "block")):
        assert_close(got[vid], ref[vid], "bf16", f"stride-2 pair {case} {what}")
    # against the two contractions launched as one grid: same products, another summation order
    lp, s = run_hip(spec, data)
    assert not any(st["kernel"].endswith("3x3s2_pair") for st in s.plan.describe()["steps"])
    for vid, what in ((c1, "3x3/2"), (d, "1x1/2 projection")):
        assert_close(got[vid], lp[vid], "bf16", f"stride-2 pair {case} {what} against the general kernel")
    again, _ = run_hip(spec, data, opts=opts)
    for vid in spec.outputs:
        np.testing.assert_array_equal(got[vid], again[vid])


def test_conv_large_tiles_many_blocks():
    # enough rows that the planner picks its largest tile (several tiles + ragged tail)
    for dtype in ("f32", "bf16"):
        spec, data = W.conv_group(8, 64, 128, 57, 57, 3, 1, 1, dtype, residual=True)
        check_graph(spec, data, f"conv big {dtype}")


def test_fused_equals_unfused_on_device():
    spec, data = W.conv_group(2, 16, 32, 12, 12, 3, 1, 1, "f32", residual=True)
    fused, _ = run_hip(spec, data)
    unf, _ = run_hip(spec.ungrouped(), data)
    assert_close(fused[spec.outputs[0]], unf[spec.outputs[0]], "f32", "fused vs unfused", budget=lambda: 2 * error_budget(spec, data)[spec.outputs[0]])
    # and the unfused plan itself matches the oracle's unfused run
    check_graph(spec.ungrouped(), data, "unfused conv group")


def test_conv1x1_equals_dense_on_device():
    b, c, o, h, w = 2, 32, 48, 6, 5
    spec, data = W.conv_group(b, c, o, h, w, 1, 1, 0, "f32", relu=False)
    y, _ = run_hip(spec, data)
    y = y[spec.outputs[0]]
    g = W.GraphSpec("dense_view")
    x2 = g.input("x", "f32", (b * h * w, c)); w2 = g.param("w", "f32", (o, c)); b2 = g.param("b", "f32", (o,))
    o0, (t,) = g.op("dense", [x2, w2], [("f32", (b * h * w, o))])
    o1, (t,) = g.op("bias_add", [t, b2], [("f32", (b * h * w, o))], axis=1)
    g.group([o0, o1]); g.output(t)
    d2 = {"x": np.ascontiguousarray(data["x"].transpose(0, 2, 3, 1).reshape(-1, c)), "w": data["w"].reshape(o, c), "b": data["b"]}
    z, _ = run_hip(g, d2)
    z = z[g.outputs[0]].reshape(b, h, w, o).transpose(0, 3, 1, 2)
    assert_close(y, z, "f32", "1x1 conv vs dense", budget=lambda: 2 * error_budget(spec, data)[spec.outputs[0]])


def test_run_twice_is_bitwise_identical():
    spec, data = W.conv_group(4, 64, 64, 28, 28, 3, 1, 1, "bf16", residual=True)
    a, s = run_hip(spec, data)
    first = a[spec.outputs[0]].copy()
    s.run()
    import torch
    from paper_1810_00952_amd import harness
    torch.cuda.synchronize()
    second = O.widen(harness.to_host(s.output()), "bf16")
    np.testing.assert_array_equal(first, second)


# ------------------------------------------------------------------ elementwise groups
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(7, 5, 33), (4096,), (3, 1000, 9), (1,), (2, 3, 4, 5, 6), ()])
def test_eltwise_chain_all_ops(dtype, shape):
    spec, data = W.eltwise_chain(shape, dtype)
    check_graph(spec, data, f"eltwise chain {dtype} {shape}")


UNARY_CHAINS = [("neg",), ("sq",), ("relu",), ("sigmoid",), ("tanh",), ("tanh", "neg", "sq"), ("sigmoid", "tanh", "relu", "neg", "sq", "tanh", "neg", "relu"),
                ("relu", "relu"), ("neg", "relu")]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(4096,), (3, 5, 7), (2, 24, 10, 10), (1,), (37, 8)])
def test_groups_of_unary_operators(dtype, shape):
    # operand-free chains of every length up to eight behind nothing, behind a bias, behind one tensor operand (added,
    # multiplied, subtracted, divided) and behind both: whole 16-byte units take the kernels compiled per form, ragged
    # sizes the interpreting kernel; same values either way
    for chain in UNARY_CHAINS:
        for lead in ("", "bias", "bias+add", "add", "mul", "bias+sub", "div"):
            if lead.startswith("bias") and len(shape) < 2:
                continue
            rng = W.rng_for(9, salt=len(chain) * 7 + len(lead))
            g = W.GraphSpec("unary")
            t = (dtype, shape)
            x = g.input("x", dtype, shape)
            data = {"x": W.as_dtype(W.normal(rng, shape), dtype)}
            ops, y = [], x
            if lead.startswith("bias"):
                b = g.param("b", "f32", (shape[1],)); data["b"] = W.as_dtype(W.normal(rng, (shape[1],)), "f32")
                o, (y,) = g.op("bias_add", [y, b], [t], axis=1); ops.append(o)
            if lead.endswith(("add", "mul", "sub", "div")):
                r = g.input("r", dtype, shape)
                data["r"] = W.as_dtype(W.uniform(rng, shape, 1.0, 2.0) if lead.endswith("div") else W.normal(rng, shape), dtype)
                o, (y,) = g.op(lead[-3:], [y, r], [t]); ops.append(o)
            for k in chain:
                o, (y,) = g.op(k, [y], [t]); ops.append(o)
            g.group(ops); g.output(y)
            check_graph(g, data, f"unary chain {lead} {chain} {dtype} {shape}")


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape", [(2, 16, 8, 8), (3, 5, 7, 9), (1, 64, 56, 56), (2, 3, 1, 1), (4, 8, 2, 4)])
def test_eltwise_bias_residual_relu(dtype, shape):
    spec, make = W.eltwise_bias_res_relu(shape, dtype)
    check_graph(spec, make(), f"bias+res+relu {dtype} {shape}")


def test_eltwise_more_than_2_pow_31_elements():
    # 72 x 8 x 2048 x 2048 bf16: 2.4e9 elements, 4.8 GB per tensor -- past 32-bit element and byte offsets.
    # Inputs are drawn on the device (seeded); the oracle checks whole (image, channel) planes, among them the
    # first and the last of the tensor, each as a 1 x 1 x H x W problem with that channel's bias.
    import torch
    from paper_1810_00952_amd import harness
    shape = (72, 8, 2048, 2048)
    spec, _ = W.eltwise_bias_res_relu(shape, "bf16")
    s = harness.Session(spec)
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(11)
    n = s.by_name
    for name in ("x", "r"):
        t = torch.empty(shape, dtype=torch.bfloat16, device="cuda:0")
        for i in range(shape[0]):                     # image by image: no fp32 copy of the whole tensor
            t[i] = torch.randn(shape[1:], generator=gen, device="cuda:0", dtype=torch.float32).to(torch.bfloat16)
        s.tensors[n[name]] = t
    b = np.linspace(-0.5, 0.5, shape[1]).astype(np.float32)
    s.load({"b": b})
    s.alloc(); s.run(); torch.cuda.synchronize()
    y = s.output()
    sub, _ = W.eltwise_bias_res_relu((1, 1) + shape[2:], "bf16")
    for (i, c) in [(0, 0), (0, 7), (35, 3), (44, 5), (71, 0), (71, 7)]:
        d = {"x": harness.to_host(s.tensors[n["x"]][i, c])[None, None], "r": harness.to_host(s.tensors[n["r"]][i, c])[None, None],
             "b": b[c:c + 1]}
        ref = OG.run(sub, d)[sub.outputs[0]]
        got = O.widen(harness.to_host(y[i, c])[None, None], "bf16")
        assert_close(got, ref, "bf16", f"large eltwise plane ({i},{c})")
    # the planes on either side of flat element 2^31 (image 64, channel 0 starts exactly there)
    assert 64 * 8 * 2048 * 2048 == 2 ** 31
    for (i, c) in [(63, 7), (64, 0)]:
        d = {"x": harness.to_host(s.tensors[n["x"]][i, c])[None, None], "r": harness.to_host(s.tensors[n["r"]][i, c])[None, None],
             "b": b[c:c + 1]}
        ref = OG.run(sub, d)[sub.outputs[0]]
        assert_close(O.widen(harness.to_host(y[i, c])[None, None], "bf16"), ref, "bf16", f"large eltwise plane ({i},{c})")


def test_conv_activations_beyond_2_gib():
    # 66 x 8 x 1024 x 1024 f32 (2.2 GB in, 2.2 GB out): past the 32-bit byte offsets the vector-load kernels use, so
    # the planner must fall back to the 64-bit gather kernel.  The oracle computes the first and the last image.
    import torch
    from paper_1810_00952_amd import harness
    B_, C, H = 66, 8, 1024
    spec, data1 = W.conv_group(1, C, C, H, H, 3, 1, 1, "f32", residual=False, relu=True, make_x=False)
    big, _ = W.conv_group(B_, C, C, H, H, 3, 1, 1, "f32", residual=False, relu=True, make_x=False)
    s = harness.Session(big)
    n = s.by_name
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(12)
    x = torch.randn((B_, C, H, H), generator=gen, device="cuda:0", dtype=torch.float32)
    s.tensors[n["x"]] = x
    s.load(data1)
    s.alloc(); s.run(); torch.cuda.synchronize()
    assert any(st["kernel"].endswith("_gather") for st in s.plan.describe()["steps"])
    y = s.output()
    for i in (0, B_ - 1):
        d = dict(data1); d["x"] = harness.to_host(x[i:i + 1])
        ref = OG.run(spec, d)[spec.outputs[0]]
        assert_close(O.widen(harness.to_host(y[i:i + 1]), "f32"), ref, "f32", f"large conv image {i}", budget=lambda: error_budget(spec, d)[spec.outputs[0]])
    assert float((y[0] - y[B_ - 1]).abs().max()) > 1e-3


def test_eltwise_operand_order_and_self_operands():
    for dtype in ("f32", "bf16"):
        g = W.GraphSpec("order")
        t = (dtype, (5, 13))
        a = g.input("a", dtype, t[1]); b = g.input("b", dtype, t[1]); c = g.input("c", dtype, t[1])
        ops = []
        o, (y,) = g.op("sub", [b, a], [t]); ops.append(o)       # start value is b
        o, (y,) = g.op("sub", [c, y], [t]); ops.append(o)       # running value on the right
        o, (y,) = g.op("div", [a, y], [t]); ops.append(o)
        o, (y,) = g.op("add", [y, y], [t]); ops.append(o)       # both operands the running value
        o, (y,) = g.op("mul", [y, y], [t]); ops.append(o)
        g.group(ops); g.output(y)
        rng = W.rng_for(8)
        data = {"a": W.as_dtype(rng.uniform(1, 2, t[1]), dtype), "b": W.as_dtype(rng.uniform(3, 4, t[1]), dtype),
                "c": W.as_dtype(rng.uniform(-1, 0, t[1]), dtype)}
        check_graph(g, data, f"operand order {dtype}")


def test_cast_group():
    g = W.GraphSpec("cast")
    x = g.input("x", "f32", (3, 50))
    o0, (y,) = g.op("cast", [x], [("bf16", (3, 50))], to="bf16")
    o1, (y,) = g.op("tanh", [y], [("bf16", (3, 50))])
    o2, (y,) = g.op("cast", [y], [("f32", (3, 50))], to="f32")
    g.group([o0, o1, o2]); g.output(y)
    data = {"x": W.as_dtype(W.rng_for(9).standard_normal((3, 50)), "f32")}
    got, ref = check_graph(g, data, "cast chain")


# ------------------------------------------------------------------ window reductions
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("shape,k,s,p", [((2, 16, 15, 14), 3, 2, 1), ((1, 5, 9, 9), 3, 2, 1), ((2, 8, 8, 8), 2, 2, 0), ((1, 64, 112, 112), 3, 2, 1)])
def test_maxpool_signed_inputs(dtype, shape, k, s, p):
    g = W.GraphSpec("pool")
    x = g.input("x", dtype, shape)
    oh, ow = W.conv_out(shape[2], k, s, p), W.conv_out(shape[3], k, s, p)
    o, (y,) = g.op("maxpool2d", [x], [(dtype, (shape[0], shape[1], oh, ow))], kernel=(k, k), stride=(s, s), pad=(p, p))
    g.output(y)
    data = {"x": W.as_dtype(W.rng_for(10).standard_normal(shape) - 2.0, dtype)}      # mostly negative: padding must not win
    got, ref = check_graph(g, data, f"maxpool {dtype} {shape}")
    np.testing.assert_array_equal(got[y], ref[y])                                      # selection is exact


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_global_avgpool_flatten_dense(dtype):
    g = W.GraphSpec("head")
    x = g.input("x", dtype, (3, 24, 7, 7))
    w = g.param("w", dtype, (10, 24)); b = g.param("b", "f32", (10,))
    o, (y,) = g.op("global_avgpool", [x], [(dtype, (3, 24, 1, 1))])
    o, (y,) = g.op("flatten", [y], [(dtype, (3, 24))])
    o0, (y,) = g.op("dense", [y, w], [(dtype, (3, 10))])
    o1, (y,) = g.op("bias_add", [y, b], [(dtype, (3, 10))], axis=1)
    g.group([o0, o1]); g.output(y)
    rng = W.rng_for(11)
    data = {"x": W.as_dtype(rng.standard_normal((3, 24, 7, 7)), dtype), "w": W.as_dtype(rng.standard_normal((10, 24)) * 0.2, dtype),
            "b": W.as_dtype(rng.uniform(-.1, .1, 10), "f32")}
    check_graph(g, data, f"head {dtype}")


# ------------------------------------------------------------------ weight preparation
def test_fold_batchnorm_matches_oracle_bitwise():
    import torch
    from paper_1810_00952_amd import harness, binding
    rng = W.rng_for(12)
    O_, per = 37, 3 * 7 * 7
    w = W.as_dtype(rng.standard_normal((O_, per)), "f32")
    st = [W.as_dtype(a, "f32") for a in (rng.uniform(.5, 1.5, O_), rng.uniform(-.1, .1, O_), rng.standard_normal(O_) * .1, rng.uniform(.5, 1.5, O_))]
    wf64, bf64 = O.fold_batchnorm(w, *st, W.BN_EPS)
    ctx = binding.Context()
    dw = harness.to_device(w, "f32"); ds = [harness.to_device(a, "f32") for a in st]
    for dtype in ("f32", "bf16"):
        out = torch.empty((O_, per), dtype=torch.bfloat16 if dtype == "bf16" else torch.float32, device="cuda:0")
        bo = torch.empty(O_, dtype=torch.float32, device="cuda:0")
        ctx.fold_batchnorm(dw.data_ptr(), *[d.data_ptr() for d in ds], W.BN_EPS, out.data_ptr(), dtype, bo.data_ptr(), O_, per)
        torch.cuda.synchronize()
        np.testing.assert_array_equal(harness.to_host(out), store_as(O.round_to(wf64, "f32"), dtype))
        np.testing.assert_array_equal(harness.to_host(bo), bf64.astype(np.float32))


# ------------------------------------------------------------------ ResNet-18-shaped graphs
def _resnet_hip(spec, raw, bn, dtype):
    import torch
    from paper_1810_00952_amd import harness
    s = harness.Session(spec)
    fold_resnet_hip(s, raw, bn, dtype)
    s.alloc(); s.run(); torch.cuda.synchronize()
    return O.widen(harness.to_host(s.output()), dtype), s


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_resnet_small_end_to_end_and_per_group(dtype):
    spec, raw, bn = W.resnet18(batch=2, dtype=dtype, image=64, width=16, classes=24)
    data = fold_resnet_oracle(raw, bn, dtype)
    allv = OG.run(spec, data, keep_all=True)
    got, _ = _resnet_hip(spec, raw, bn, dtype)
    assert_close(got, allv[spec.outputs[0]], dtype, f"resnet small {dtype} end to end", rms_scaled=True)      # 20 contractions deep
    # every group on its own, fed the oracle's values at its boundary
    for gi in range(len(spec.groups)):
        sub, vmap = extract_group(spec, gi)
        if not sub.outputs:
            continue
        sd = {}
        for old, new in vmap.items():
            if sub.values[new].role in ("input", "param"):
                sd[sub.values[new].name] = store_as(allv[old], sub.values[new].type.dtype)
        out, _ = run_hip(sub, sd)
        inv = {n: o for o, n in vmap.items()}
        for vid in sub.outputs:
            assert_close(out[vid], allv[inv[vid]], sub.values[vid].type.dtype, f"resnet small {dtype} group {gi} ({spec.ops[spec.groups[gi][0]].kind})",
                         budget=None if dtype == "bf16" else (lambda: error_budget(sub, sd)[vid]))


@pytest.mark.parametrize("which", ["resnet_small_f32", "resnet_small_bf16", "conv_bf16", "mlp_f32", "splitk_f32", "channel_last_bf16", "grad_w_bf16", "grad_x_stride2_bf16",
                                   "stem_pool_bf16"])
def test_plan_replays_from_a_hip_graph(which):
    # one rl_plan_run captured into a HIP graph, then replayed with fresh inputs, with eager work and
    # synchronisation between the replays; every replay must reproduce the eager run bit for bit
    import torch
    from paper_1810_00952_amd import harness
    if which.startswith("resnet"):
        dtype = which.rsplit("_", 1)[1]
        spec, raw, bn = W.resnet18(batch=2, dtype=dtype, image=64, width=16, classes=24)
        s = harness.Session(spec)
        fold_resnet_hip(s, raw, bn, dtype)
    elif which == "conv_bf16":
        spec, data = W.conv_group(3, 64, 128, 29, 29, 3, 1, 1, "bf16", residual=True, relu=True, tail=True)
        s = harness.Session(spec); s.load(data)
    elif which == "splitk_f32":                     # two kernels per step and a scratch tensor in the workspace
        spec, data = W.conv_group(1, 256, 256, 14, 14, 3, 1, 1, "f32", residual=True, relu=True)
        s = harness.Session(spec); s.load(data)
        assert any(st["kernel"].endswith("_splitk") for st in s.plan.describe()["steps"])
    elif which == "grad_w_bf16":                    # two transpositions, the contraction, the ordered reduction of its row segments
        spec, data = W.grad_case("conv2d_grad_w", (64, 64, 9, 8, 128, 3), "bf16", 2, 1, second_is_param=False)
        s = harness.Session(spec); s.load(data)
        assert any(st["kernel"] == "wgrad_reduce" for st in s.plan.describe()["steps"])
    elif which == "grad_x_stride2_bf16":            # dy spread out with zeros by a step of its own, then the forward kernels
        spec, data = W.grad_case("conv2d_grad_x", (3, 8, 15, 14, 16, 3), "bf16", 2, 1)
        s = harness.Session(spec); s.load(data)
        assert any(st["kernel"] == "dilate_nhwc" for st in s.plan.describe()["steps"])
    elif which == "stem_pool_bf16":                 # the fused stem + pool kernel reading the channel-first input
        spec, data = W.conv_pool(3, 3, 64, 40, 48, 7, 2, 3, "bf16", relu=True, tail=True)
        s = harness.Session(spec); s.load(data)
        assert any(st["kernel"].endswith("stem_maxpool_direct") for st in s.plan.describe()["steps"])
    elif which == "channel_last_bf16":              # typed views: the first group reads the caller's buffer, the last writes the output
        spec, data = W.channel_last_block(3, 64, 14, 14, "bf16")
        s = harness.Session(spec); s.load(data)
    else:
        spec, data = W.mlp()
        s = harness.Session(spec); s.load(data)
    s.alloc()
    g = s.capture()
    xin = [vid for vid, v in enumerate(spec.values) if v.role == "input"]
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(7)
    for rep in range(3):
        for vid in xin:
            t = s.tensors[vid]
            t.copy_(torch.randn(t.shape, generator=gen, device="cuda:0", dtype=torch.float32).to(t.dtype))
        for vid in spec.outputs:
            s.tensors[vid].zero_()
        torch.cuda.synchronize()
        g.replay()
        torch.cuda.synchronize()
        got = [s.tensors[vid].clone() for vid in spec.outputs]
        for vid in spec.outputs:
            s.tensors[vid].zero_()
        s.run()
        torch.cuda.synchronize()
        for a, vid in zip(got, spec.outputs):
            assert torch.equal(a.view(torch.uint8), s.tensors[vid].view(torch.uint8)), f"{which}: replay {rep} differs from the eager run"
        assert all(bool(torch.isfinite(a.float()).all()) for a in got)


@pytest.mark.parametrize("which", ["resnet_bf16", "resnet_f32", "grad_w_bf16"])
def test_two_sessions_on_two_streams_do_not_disturb_each_other(which):
    # Independent steps may overlap on the GPU (a caller's second stream, or the two-stream figure of the benchmark):
    # two sessions with buffers of their own and different inputs, launched alternately on two streams without any
    # synchronisation in between, must each give the bits they give when run alone.
    import torch
    from paper_1810_00952_amd import harness
    sess = []
    for k in range(2):
        if which.startswith("resnet"):
            dtype = which.split("_")[1]
            spec, raw, bn = W.resnet18(batch=4, dtype=dtype, image=96, width=64, classes=40)
            s = harness.Session(spec)
            fold_resnet_hip(s, raw, bn, dtype)
        else:                                       # a plan with scratch tensors in its workspace
            spec, data = W.grad_case("conv2d_grad_w", (64, 64, 9, 8, 128, 3), "bf16", 2, 1, second_is_param=False)
            s = harness.Session(spec); s.load(data)
        s.alloc()
        sess.append(s)
    gen = torch.Generator(device="cuda:0"); gen.manual_seed(11)
    xin = [vid for vid, v in enumerate(spec.values) if v.role == "input"]
    for s in sess:                                  # different inputs in the two sessions
        for vid in xin:
            t = s.tensors[vid]
            t.copy_(torch.randn(t.shape, generator=gen, device="cuda:0", dtype=torch.float32).to(t.dtype))
    alone = []
    for s in sess:
        s.run()
        torch.cuda.synchronize()
        alone.append([s.tensors[vid].clone() for vid in spec.outputs])
        for vid in spec.outputs:
            s.tensors[vid].zero_()
    assert not torch.equal(alone[0][0], alone[1][0])
    torch.cuda.synchronize()
    streams = [torch.cuda.Stream(), torch.cuda.Stream()]
    for rep in range(6):
        for k in (0, 1):
            with torch.cuda.stream(streams[k]):
                sess[k].run()
    torch.cuda.synchronize()
    for k in (0, 1):
        for a, vid in zip(alone[k], spec.outputs):
            assert torch.equal(a.view(torch.uint8), sess[k].tensors[vid].view(torch.uint8)), f"{which}: session {k} differs when overlapped with the other"


def test_resnet18_f32_batch1():
    spec, raw, bn = W.resnet18(batch=1, dtype="f32")
    ref = OG.run(spec, fold_resnet_oracle(raw, bn, "f32"))[spec.outputs[0]]
    got, _ = _resnet_hip(spec, raw, bn, "f32")
    assert_close(got, ref, "f32", "resnet18 f32 b1", rms_scaled=True)          # 21 contractions deep: the worst-case budget is vacuous


def test_resnet18_bf16_batch64_every_image_and_every_group():
    # The benchmark configuration at full size.
    # (1) The plan bench.py times: all 64 images' logits against the oracle, over the batch and image by image.
    # (2) Every fusion group at full size on the oracle's values at its boundary (so that nothing but the group's own
    #     arithmetic separates the two sides), in the kernel and launch shape it has inside the whole plan (asserted):
    #     groups are cut out with channel-last inputs and results behind views, the stem with the max-pool behind it and
    #     each stride-2 convolution with the 1x1 projection beside it, as the plan launches them.  Every element of
    #     every group's result, all 64 images.
    from paper_1810_00952_amd import binding
    spec, raw, bn = W.resnet18(batch=64, dtype="bf16")
    data = fold_resnet_oracle(raw, bn, "bf16")
    gout = {gi: spec.ops[sorted(g)[-1]].outputs[0] for gi, g in enumerate(spec.groups)}
    print("oracle: 64 images, every group's result", flush=True)
    ref = OG.run(spec, data, keep=list(gout.values()) + [i for i, v in enumerate(spec.values) if v.role == "input"])
    print("device: whole plan", flush=True)
    got, s = _resnet_hip(spec, raw, bn, "bf16")
    assert got.shape == (64, 1000)
    assert_close(got, ref[spec.outputs[0]], "bf16", "resnet18 bf16 b64 logits, 64 images")
    for n in range(64):                           # image by image, so that one bad image cannot hide in the batch's RMS
        assert_close(got[n], ref[spec.outputs[0]][n], "bf16", f"resnet18 bf16 b64 logits of image {n}")
    # images differ, so must the logits (guards against a batch-index bug that repeats one image)
    assert np.abs(got[0] - got[63]).max() > 1e-3
    whole = {st["name"]: (st["kernel"], st.get("M"), st.get("N"), st.get("K")) for st in s.plan.describe()["steps"]}
    del s
    # launches of the whole plan -> the groups each one covers
    def name_of(gi):                              # a convolution group goes by its weight's name
        op = spec.ops[sorted(spec.groups[gi])[0]]
        return spec.values[op.inputs[1]].name[:-len(".wf")] if op.kind == "conv2d" else op.kind
    gi_of = {name_of(gi): gi for gi in range(len(spec.groups))}
    units = [[gi_of["conv1"], gi_of["maxpool2d"]]]
    for st in range(1, 5):
        for b in range(2):
            pre = f"l{st}.b{b}"
            units.append([gi_of[pre + ".c1"]] + ([gi_of[pre + ".ds"]] if pre + ".ds" in gi_of else []))
            units.append([gi_of[pre + ".c2"]])
    units.append([gi_of["global_avgpool"], gi_of["flatten"], gi_of["dense"]])
    xid = [i for i, v in enumerate(spec.values) if v.role == "input"][0]
    seen_kernels = set()
    for gis in units:
        sub, feeds, results = extract_groups_channel_last(spec, gis, native_inputs=(xid,))
        sd = {}
        for old, (name, cl) in feeds.items():
            a = ref[old]
            sd[name] = store_as(np.ascontiguousarray(np.transpose(a, (0, 2, 3, 1))) if cl else a, spec.values[old].type.dtype)
        for v in sub.values:
            if v.role == "param":
                sd[v.name] = data[v.name]
        label = "+".join(name_of(g) for g in gis)
        print(f"device: {label}", flush=True)
        out, ss = run_hip(sub, sd)
        for st in ss.plan.describe()["steps"]:
            k = (st["kernel"], st.get("M"), st.get("N"), st.get("K"))
            assert k in whole.values(), (label, k)           # the kernel and shape this group has inside the whole plan
            seen_kernels.add(k)
        for old, new in results.items():
            r = ref[old]
            r = np.ascontiguousarray(np.transpose(r, (0, 2, 3, 1))) if r.ndim == 4 else r
            assert_close(out[new], r, "bf16", f"resnet18 bf16 b64 group {label}, 64 images")
            for n in (0, 21, 42, 63):
                assert_close(out[new][n], r[n], "bf16", f"resnet18 bf16 b64 group {label}, image {n}")
    assert seen_kernels == set(whole.values()), set(whole.values()) - seen_kernels


# ------------------------------------------------------------------ automatic fusion
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_automatically_fused_graphs(dtype):
    # groups formed by the library from the bare calls: where they differ from the declared ones (the trailing neg
    # joins the conv group; the gate op joins its contraction) and where they coincide (a small ResNet)
    spec, data = W.conv_group(3, 64, 72, 13, 11, 3, 1, 1, dtype, residual=True, relu=True, tail=True)
    ref = OG.run(spec, data)
    got, s = run_hip(spec, data, auto_groups=True)
    assert len(s.plan.describe()["steps"]) < len(run_hip(spec, data)[1].plan.describe()["steps"])
    for vid in spec.outputs:
        assert_close(got[vid], ref[vid], dtype, f"auto-fused conv tail {dtype}", budget=None if dtype == "bf16" else (lambda: error_budget(spec, data)[vid]))
    spec, raw, bn = W.resnet18(batch=2, dtype=dtype, image=64, width=16, classes=24)
    from paper_1810_00952_amd import harness
    import torch
    outs = []
    for auto in (False, True):
        s = harness.Session(spec, auto_groups=auto)
        fold_resnet_hip(s, raw, bn, dtype)
        s.alloc(); s.run(); torch.cuda.synchronize()
        outs.append(harness.to_host(s.output()))
    np.testing.assert_array_equal(outs[0], outs[1])


# ------------------------------------------------------------------ the paper's LeNet-shaped example
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("batch", [1, 5, 64])
def test_lenet_shaped_graph(dtype, batch):
    # tanh epilogues on conv and dense anchors, unpadded 5x5 convolutions from one and from 20 channels,
    # non-overlapping 2x2 pooling, flatten of a channel-last intermediate back to (N, C*H*W) order
    spec, data = W.lenet(batch, dtype)
    check_graph(spec, data, f"lenet {dtype} b{batch}")
    # every op in a group of its own gives the same values up to the rounding of the stored intermediates
    check_graph(spec.ungrouped(), data, f"lenet ungrouped {dtype} b{batch}")


# ------------------------------------------------------------------ LSTM
def _lstm_hip(T, B, I, H, dtype, fused, d, hoist_steps=0):
    # hoist_steps: room in the workspace for that many steps' input projections (0: only the cell plan's own)
    import torch
    from paper_1810_00952_amd import harness
    spec = W.lstm_cell_graph(B, I, H, dtype, fused)
    s = harness.Session(spec)
    s.load({"w": d["w"], "b": d["b"]})
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    x = harness.to_device(d["x"], dtype)
    h0 = torch.zeros((B, H), dtype=tdt, device="cuda:0")
    c = torch.zeros((B, H), dtype=torch.float32, device="cuda:0")
    hs = torch.empty((T, B, H), dtype=tdt, device="cuda:0")
    nws = s.plan.workspace_bytes()
    if hoist_steps:
        assert s.plan.recurrent_workspace_bytes(0) == (nws + 255) // 256 * 256
        nws = s.plan.recurrent_workspace_bytes(hoist_steps)
        assert nws == s.plan.recurrent_workspace_bytes(0) + hoist_steps * B * 4 * H * 4, "cell not recognised as hoistable"
    ws = torch.empty(max(256, nws), dtype=torch.uint8, device="cuda:0")
    n = s.by_name
    roles = {"x": n["x"], "h_in": n["h"], "c_in": n["c"], "c_out": spec.outputs[0], "h_out": spec.outputs[1]}
    esz = 2 if dtype == "bf16" else 4
    s.plan.run_recurrent(T, roles, x.data_ptr(), B * I * esz, h0.data_ptr(), c.data_ptr(), hs.data_ptr(), B * H * esz,
                         {n["w"]: s.tensors[n["w"]].data_ptr(), n["b"]: s.tensors[n["b"]].data_ptr()}, ws.data_ptr(), ws.numel(),
                         harness.stream_handle())
    torch.cuda.synchronize()
    return O.widen(harness.to_host(hs), dtype), O.widen(harness.to_host(c), "f32")


@pytest.mark.parametrize("fused", [True, False])
@pytest.mark.parametrize("dtype,T,B,I,H", [("bf16", 6, 8, 32, 32), ("f32", 5, 3, 24, 16), ("bf16", 4, 70, 64, 48), ("bf16", 3, 64, 256, 128)])
def test_lstm_recurrent(fused, dtype, T, B, I, H):
    d = W.lstm_data(T, B, I, H, dtype)
    hs_ref, c_ref = O.lstm_sequence(O.widen(d["x"], dtype), O.widen(d["w"], dtype), O.widen(d["b"], "f32"),
                                    np.zeros((B, H)), np.zeros((B, H)), h_dtype=dtype)
    hs, c = _lstm_hip(T, B, I, H, dtype, fused, d)
    assert_close(hs, hs_ref, dtype, f"lstm h {dtype} fused={fused}", rms_scaled=True)
    assert_close(c, c_ref, dtype if dtype == "bf16" else "f32", f"lstm c {dtype} fused={fused}", rms_scaled=True)


# Hoisted form (input projection of many steps in one contraction, then one recurrent kernel per step):
# batch tails inside and across 64-row blocks, hidden sizes that give the four waves 1, 2 or no K tiles each,
# the whole sequence in one chunk and chunks of 8 and 9 steps with a ragged last chunk.
@pytest.mark.parametrize("T,B,I,H,room", [(3, 64, 256, 128, 3), (5, 70, 128, 192, 5), (20, 8, 128, 64, 8), (19, 33, 192, 320, 9),
                                          (4, 130, 128, 512, 4)])
def test_lstm_recurrent_hoisted_projection(T, B, I, H, room):
    d = W.lstm_data(T, B, I, H, "bf16")
    hs_ref, c_ref = O.lstm_sequence(O.widen(d["x"], "bf16"), O.widen(d["w"], "bf16"), O.widen(d["b"], "f32"),
                                    np.zeros((B, H)), np.zeros((B, H)), h_dtype="bf16")
    hs, c = _lstm_hip(T, B, I, H, "bf16", True, d, hoist_steps=room)
    assert_close(hs, hs_ref, "bf16", f"lstm hoisted h T={T} B={B} I={I} H={H}")
    assert_close(c, c_ref, "bf16", f"lstm hoisted c T={T} B={B} I={I} H={H}")
    # and against the per-step replay of the same cell on the same data: the two forms differ by summation order only
    hs2, c2 = _lstm_hip(T, B, I, H, "bf16", True, d, hoist_steps=0)
    assert np.abs(hs - hs2).max() <= 2e-2 and np.abs(c - c2).max() <= 2e-2 * max(1.0, np.abs(c2).max())


def test_lstm_unrolled_graph_equals_recurrent_call():
    T, B, I, H = 3, 16, 32, 32
    d = W.lstm_data(T, B, I, H, "bf16")
    hs, c = _lstm_hip(T, B, I, H, "bf16", True, d)
    spec = W.lstm_unrolled_graph(T, B, I, H, "bf16", fused=True)
    data = {f"x{t}": d["x"][t] for t in range(T)}
    data.update(h0=np.zeros((B, H), np.uint16), c0=np.zeros((B, H), np.float32), w=d["w"], b=d["b"])
    out, _ = run_hip(spec, data)
    for t in range(T):
        np.testing.assert_array_equal(out[spec.outputs[t]], hs[t])
    np.testing.assert_array_equal(out[spec.outputs[T]], c)


def test_lstm_full_configuration():
    T, B, I, H = 128, 64, 1024, 1024
    d = W.lstm_data(T, B, I, H, "bf16")
    hs, c = _lstm_hip(T, B, I, H, "bf16", True, d, hoist_steps=T)
    hs_ref, c_ref = O.lstm_sequence(O.widen(d["x"], "bf16"), O.widen(d["w"], "bf16"), O.widen(d["b"], "f32"),
                                    np.zeros((B, H)), np.zeros((B, H)), h_dtype="bf16")
    assert_close(hs, hs_ref, "bf16", "lstm full h")
    assert_close(c, c_ref, "bf16", "lstm full c")


# ---- a convolution group whose result is a graph output in Shape order (channel-first) ------------------
OUT_ORDER_CASES = [
    # batch cin cout h  w  k s p residual relu
    (16, 128, 128, 28, 28, 3, 1, 1, True, True),       # nine-taps-from-one-copy kernel, channel-first residual transposed too
    (16, 128, 128, 28, 28, 3, 1, 1, False, True),
    (9, 64, 64, 56, 56, 3, 1, 1, True, True),          # weights-in-registers kernel
    (24, 64, 128, 30, 26, 3, 2, 1, False, True),       # stride 2: the general pixel-on-lane kernel
    (33, 256, 136, 14, 14, 1, 1, 0, True, False),      # 1x1, ragged channel tile, no ReLU
]


@pytest.mark.parametrize("case", OUT_ORDER_CASES, ids=[f"oo{i}" for i in range(len(OUT_ORDER_CASES))])
def test_convolution_result_as_channel_first_output(case):
    # the fast kernels write channel-last into the workspace and a transposition fills the output; the plan option
    # keeps the kernel that stores channel-first itself.  Both against the oracle.
    b, ci, co, h, w, k, s, p, res, relu = case
    spec, data = W.conv_group(b, ci, co, h, w, k, s, p, "bf16", residual=res, relu=relu)
    ks = [st["kernel"] for st in s_plan_steps(spec)]
    assert ks[-1] == "nhwc_to_nchw" and not ks[-2].endswith("_dma") and ks.count("nchw_to_nhwc") == (2 if res else 1), ks
    ks1 = [st["kernel"] for st in s_plan_steps(spec, {"no_out_transpose": 1})]
    assert "_dma" in ks1[-1] and "nhwc_to_nchw" not in ks1, ks1
    check_graph(spec, data, f"conv to channel-first output {case}")
    check_graph(spec, data, f"conv storing channel-first itself {case}", opts={"no_out_transpose": 1})


# ---- bf16 contractions with operand-free steps other than one ReLU in their group -----------------------
ANYACT_CASES = [
    # batch cin cout h  w  k s p residual relu acts
    (16, 128, 128, 28, 28, 3, 1, 1, False, False, ("tanh",)),
    (5, 64, 64, 56, 56, 3, 1, 1, True, False, ("sigmoid", "sq")),          # shapes the register-weight kernel would take with a ReLU
    (9, 128, 136, 14, 15, 3, 2, 1, True, True, ("tanh", "neg")),            # ReLU first, then more; stride 2, ragged channel tile
    (70, 256, 72, 7, 7, 1, 1, 0, False, False, ("neg",)),
    (3, 64, 64, 28, 28, 3, 1, 1, False, False, ("sigmoid", "tanh", "relu", "neg", "sq", "tanh", "neg", "relu")),   # eight steps
]


@pytest.mark.parametrize("case", ANYACT_CASES, ids=[f"aa{i}" for i in range(len(ANYACT_CASES))])
def test_bf16_contraction_with_any_operand_free_steps(case):
    # the general pixel-on-lane kernel interprets the steps behind bias and residual in its epilogue; without it
    # (plan option no_lp) the direct-load kernel does.  Both against the oracle.
    b, ci, co, h, w, k, s, p, res, relu, acts = case
    spec, data = W.conv_group(b, ci, co, h, w, k, s, p, "bf16", residual=res, relu=relu, acts=acts, tail=True)
    ks = [st["kernel"] for st in s_plan_steps(spec)]
    assert any(x.endswith("_lp") for x in ks) and not any(x.endswith(("_run", "_c64", "_ws")) for x in ks), ks
    check_graph(spec, data, f"any activation {case}")
    check_graph(spec, data, f"any activation {case} without the pixel-on-lane kernels", opts={"no_lp": 1})
    # a dense layer with tanh, as the LeNet shape has them
    spec, data = W.mlp(70, 512, 256, 72, "bf16")
    g = W.GraphSpec("dense_tanh")
    x = g.input("x", "bf16", (70, 512)); wv = g.param("w1", "bf16", (256, 512)); bv = g.param("b1", "f32", (256,))
    o0, (y,) = g.op("dense", [x, wv], [("bf16", (70, 256))])
    o1, (y,) = g.op("bias_add", [y, bv], [("bf16", (70, 256))], axis=1)
    o2, (y,) = g.op("tanh", [y], [("bf16", (70, 256))])
    g.group([o0, o1, o2]); g.output(y)
    assert [st["kernel"] for st in s_plan_steps(g)] == ["igemm_dense_bf16_64x64_lp"]
    check_graph(g, {k_: data[k_] for k_ in ("x", "w1", "b1")}, "dense + bias + tanh bf16")


# ---- K split over several workgroups per tile (few tiles, long K) --------------------------------------
SPLITK_CASES = [
    # batch cin cout h  w  k s p residual relu dtype tail
    (1, 256, 256, 14, 14, 3, 1, 1, False, True, "f32", False),     # 16 tiles, 72 K tiles: 16 slices
    (1, 512, 512, 7, 7, 3, 1, 1, True, True, "f32", False),        # 8 tiles, 144 K tiles, residual
    (1, 256, 512, 14, 14, 3, 2, 1, False, True, "f32", True),      # stride 2, result kept channel-last
    (2, 64, 72, 9, 11, 3, 1, 1, True, False, "f32", False),        # ragged M and N, 18 K tiles: 4 slices of 5, 5, 5, 3
    (1, 512, 40, 5, 5, 1, 1, 0, False, False, "f32", False),       # 1x1: one tap, 16 K tiles
    (3, 128, 136, 7, 7, 3, 1, 1, True, True, "bf16", False),       # bf16 through the same kernel (result in Shape order)
    # channel counts that are no multiple of the K tile: the kernel that fetches through registers, K tiles across taps
    (64, 20, 50, 12, 12, 5, 1, 0, False, False, "f32", False),     # the LeNet shape's second convolution: 64 tiles, 16 K tiles
    (1, 20, 50, 12, 12, 5, 1, 0, False, True, "f32", True),        # one tile, 8 slices of 2
    (3, 36, 24, 9, 7, 3, 2, 1, True, True, "f32", False),          # stride 2, ragged last K tile (324 = 10.1 x 32), residual
    (2, 40, 40, 8, 8, 5, 1, 2, False, True, "bf16", True),         # bf16: 1000 = 15.6 K tiles of 64, result kept channel-last
]


@pytest.mark.parametrize("case", SPLITK_CASES, ids=[f"sk{i}" for i in range(len(SPLITK_CASES))])
def test_contraction_with_k_split_over_workgroups(case):
    from paper_1810_00952_amd import binding
    b, ci, co, h, w, k, s, p, res, relu, dtype, tail = case
    spec, data = W.conv_group(b, ci, co, h, w, k, s, p, dtype, residual=res, relu=relu, tail=tail)
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
    assert any(st["kernel"].endswith("_splitk") for st in desc["steps"]), [st["kernel"] for st in desc["steps"]]
    got, _ = run_hip(spec, data)
    ref = OG.run(spec, data)
    v = spec.outputs[0]
    bud = None if dtype == "bf16" else (lambda: error_budget(spec, data)[v])
    assert_close(got[v], ref[v], dtype, f"split-K {case}", budget=bud)
    again, _ = run_hip(spec, data)
    np.testing.assert_array_equal(got[v], again[v])               # slices are added in a fixed order
    whole, s1 = run_hip(spec, data, opts={"no_splitk": 1})
    assert not any(st["kernel"].endswith("_splitk") for st in s1.plan.describe()["steps"])
    assert_close(whole[v], ref[v], dtype, f"unsplit {case}", budget=bud)


# ---- partial derivatives of the contractions ---------------------------------------------------------------
GRAD_CASES = [
    # kind             dims                      stride pad  second operand a param?
    ("dense_grad_x", (32, 10, 128), 1, 0, True),          # the MLP's second layer
    ("dense_grad_x", (70, 136, 200), 1, 0, False),
    ("dense_grad_x", (5, 7, 30), 1, 0, True),             # nothing a multiple of anything
    ("dense_grad_w", (32, 128, 784), 1, 0, False),        # the MLP's first layer
    ("dense_grad_w", (9, 6, 16), 1, 0, False),
    ("dense_grad_w", (300, 72, 40), 1, 0, False),
    ("conv2d_grad_x", (2, 16, 12, 12, 24, 3), 1, 1, True),
    ("conv2d_grad_x", (3, 8, 15, 14, 16, 3), 2, 1, True),     # stride 2: (H + 2p - K) % s = 0 for H and 1 for W
    ("conv2d_grad_x", (2, 32, 14, 14, 64, 1), 2, 0, True),    # the 1x1 / stride 2 projection: three of four pixels get no gradient
    ("conv2d_grad_x", (1, 3, 33, 33, 16, 7), 2, 3, False),    # the stem's geometry, small; weights as an activation
    ("conv2d_grad_x", (2, 5, 9, 10, 7, 3), 1, 0, True),
    ("conv2d_grad_w", (2, 16, 12, 12, 24, 3), 1, 1, False),
    ("conv2d_grad_w", (3, 8, 15, 14, 16, 3), 2, 1, False),
    ("conv2d_grad_w", (2, 32, 14, 14, 64, 1), 2, 0, False),
    ("conv2d_grad_w", (1, 3, 33, 33, 16, 7), 2, 3, False),
    ("conv2d_grad_w", (4, 64, 14, 14, 64, 3), 1, 1, False),   # a ResNet block's shape, small batch
    # through a param at stride 1: planned as the forward operator on re-ordered weights (its fast kernels in bf16)
    ("conv2d_grad_x", (4, 64, 28, 28, 128, 3), 1, 1, True),
    ("conv2d_grad_x", (2, 256, 14, 14, 256, 3), 1, 1, True),
    ("conv2d_grad_x", (3, 64, 20, 20, 64, 3), 1, 1, True),
    ("conv2d_grad_x", (2, 128, 14, 14, 256, 1), 1, 0, True),
    ("dense_grad_x", (64, 1000, 512), 1, 0, True),        # ResNet-18's logits layer
]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
@pytest.mark.parametrize("case", GRAD_CASES, ids=[f"{c[0]}-{i}" for i, c in enumerate(GRAD_CASES)])
def test_gradient_operators(dtype, case):
    kind, dims, stride, pad, is_param = case
    spec, data = W.grad_case(kind, dims, dtype, stride, pad, second_is_param=is_param)
    print(f"gradient case {dtype} {case}", flush=True)
    check_graph(spec, data, f"{kind} {dtype} {dims} s{stride} p{pad}")
    kernels = [st["kernel"] for st in s_plan_steps(spec)]
    assert any(k.startswith(f"igemm_{kind}_") for k in kernels), kernels
    assert ("pack_gather" in kernels) == (not is_param), kernels          # a param's operand form is made at prepack time
    # through a param, the gradient with respect to the first operand is planned as the forward operator (at a stride: on
    # dy spread out with zeros by a step of its own)
    as_forward = is_param and kind in ("dense_grad_x", "conv2d_grad_x")
    assert ("dilate_nhwc" in kernels) == (as_forward and kind == "conv2d_grad_x" and stride > 1), kernels
    if as_forward:
        # the same operator on the element-gather kernel, as the other gradients run
        check_graph(spec, data, f"{kind} {dtype} {dims} s{stride} p{pad} gather", opts={"no_grad_fwd": 1})
        kernels = [st["kernel"] for st in s_plan_steps(spec, {"no_grad_fwd": 1})]
        assert any(k.startswith(f"igemm_{kind}_") and "_gather" in k for k in kernels), kernels
    if dtype == "bf16":
        # fp32 results from bf16 operands (what an optimizer would accumulate into): no rounding of the sum at all
        spec32, _ = W.grad_case(kind, dims, dtype, stride, pad, second_is_param=is_param, out_dtype="f32")
        ref = OG.run(spec32, data)
        out, _ = run_hip(spec32, data)
        v = spec32.outputs[0]
        assert_close(out[v], ref[v], "f32", f"{kind} bf16->f32 {dims}", budget=lambda: error_budget(spec32, data)[v])


def s_plan_steps(spec, opts=None):
    from paper_1810_00952_amd import binding
    return binding.Plan(binding.graph_from_spec(binding.Context(), spec), opts).describe()["steps"]


# A seeded sweep over conv groups nobody picked by hand: whatever kernel the planner chooses for the shape, the result
# must match the oracle (shapes small enough for the oracle, wide enough to reach the gather, vector, direct-load,
# pixel-on-lane, weights-stationary, stem and split-K forms and every epilogue).
def _random_conv_cases(n, seed=1810):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        k = int(rng.choice([1, 1, 2, 3, 3, 3, 5, 7]))
        stride = int(rng.choice([1, 1, 1, 2, 2, 3]))
        pad = int(rng.integers(0, k))
        h, w = int(rng.integers(1, 24)), int(rng.integers(1, 24))
        if h + 2 * pad < k or w + 2 * pad < k:
            continue
        cases.append((int(rng.integers(1, 6)), int(rng.choice([1, 3, 4, 8, 16, 24, 64, 72, 128, 192])), int(rng.choice([3, 8, 16, 24, 64, 72, 128, 200])), h, w, k, stride, pad,
                      str(rng.choice(["f32", "bf16", "bf16"])), bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2)), bool(rng.integers(0, 2))))
    return cases


RANDOM_CONV_CASES = _random_conv_cases(60)


@pytest.mark.parametrize("case", RANDOM_CONV_CASES, ids=[f"rc{i}" for i in range(len(RANDOM_CONV_CASES))])
def test_random_conv_groups(case):
    b, ci, co, h, w, k, stride, pad, dtype, bias, res, relu, tail = case
    spec, data = W.conv_group(b, ci, co, h, w, k, stride, pad, dtype, residual=res, relu=relu, tail=tail, bias=bias)
    print(f"random conv case {case}: {[st['kernel'] for st in s_plan_steps(spec)]}", flush=True)
    check_graph(spec, data, f"random conv {case}")


def _random_mlp_cases(n, seed=952):
    rng = np.random.default_rng(seed)
    dims = [1, 2, 7, 8, 10, 16, 31, 32, 64, 65, 100, 128, 200, 256, 513, 784, 1000, 1024]
    return [(int(rng.integers(1, 140)), int(rng.choice(dims)), int(rng.choice(dims)), int(rng.choice(dims)), str(rng.choice(["f32", "bf16"]))) for _ in range(n)]


RANDOM_MLP_CASES = _random_mlp_cases(30)


@pytest.mark.parametrize("case", RANDOM_MLP_CASES, ids=[f"rm{i}" for i in range(len(RANDOM_MLP_CASES))])
def test_random_dense_groups(case):
    # two dense groups in a row (bias + ReLU fused into the first, bias into the second) on sizes nobody picked by hand:
    # odd and partial K tiles, single rows, K split over workgroups, element gather
    b, d_in, d_h, d_out, dtype = case
    spec, data = W.mlp(b, d_in, d_h, d_out, dtype)
    print(f"random dense case {case}: {[st['kernel'] for st in s_plan_steps(spec)]}", flush=True)
    check_graph(spec, data, f"random dense {case}")


BENCH_GRAD_CASES = [("conv2d_grad_x", (64, 128, 28, 28, 128, 3), 1, 1, True), ("conv2d_grad_w", (64, 128, 28, 28, 128, 3), 1, 1, False),
                    ("conv2d_grad_x", (64, 64, 56, 56, 128, 3), 2, 1, True), ("conv2d_grad_w", (64, 64, 56, 56, 128, 3), 2, 1, False),
                    ("dense_grad_x", (64, 1000, 512), 1, 0, True), ("dense_grad_w", (64, 1000, 512), 1, 0, False)]


@pytest.mark.parametrize("case", BENCH_GRAD_CASES, ids=[f"{c[0]}-s{c[2]}" for c in BENCH_GRAD_CASES])
def test_gradient_operators_at_the_sizes_the_bench_times(case):
    # every element, at full size, in the plans `bench.py --workload grads` times
    kind, dims, stride, pad, is_param = case
    spec, data = W.grad_case(kind, dims, "bf16", stride, pad, second_is_param=is_param)
    print(f"bench-size gradient case {case}: {[st['kernel'] for st in s_plan_steps(spec)]}", flush=True)
    check_graph(spec, data, f"bench-size {kind} {dims} s{stride}")


def test_gradient_chain_at_the_size_the_bench_times():
    spec, data = W.grad_chain(64, 128, 28, 3, "bf16")
    check_graph(spec, data, "bench-size chain of three conv2d_grad_x")


def _random_grad_cases(n, seed=4952):
    rng = np.random.default_rng(seed)
    cases = []
    while len(cases) < n:
        kind = str(rng.choice(["dense_grad_x", "dense_grad_w", "conv2d_grad_x", "conv2d_grad_x", "conv2d_grad_w", "conv2d_grad_w"]))
        dtype, is_param = str(rng.choice(["f32", "bf16"])), bool(rng.integers(0, 2))
        if kind.startswith("dense"):
            cases.append((kind, (int(rng.integers(1, 100)), int(rng.choice([1, 5, 8, 16, 40, 64, 100, 128])), int(rng.choice([1, 7, 8, 16, 30, 64, 128, 200]))), 1, 0, dtype, is_param))
            continue
        k = int(rng.choice([1, 2, 3, 3, 5])); stride = int(rng.choice([1, 1, 2, 2, 3])); pad = int(rng.integers(0, k))
        h, w = int(rng.integers(1, 18)), int(rng.integers(1, 18))
        if h + 2 * pad < k or w + 2 * pad < k:
            continue
        nb = int(rng.choice([1, 2, 3, 5, 64]))
        c, o = int(rng.choice([1, 3, 8, 16, 24, 64])), int(rng.choice([4, 8, 16, 24, 64, 128]))
        if nb == 64:
            h, w = min(h, 7), min(w, 7)
            if h + 2 * pad < k or w + 2 * pad < k:
                continue
        cases.append((kind, (nb, c, h, w, o, k), stride, pad, dtype, is_param))
    return cases


RANDOM_GRAD_CASES = _random_grad_cases(60)


@pytest.mark.parametrize("case", RANDOM_GRAD_CASES, ids=[f"rg{i}" for i in range(len(RANDOM_GRAD_CASES))])
def test_random_gradient_operators(case):
    kind, dims, stride, pad, dtype, is_param = case
    spec, data = W.grad_case(kind, dims, dtype, stride, pad, second_is_param=is_param)
    print(f"random gradient case {case}: {[st['kernel'] for st in s_plan_steps(spec)]}", flush=True)
    check_graph(spec, data, f"random gradient {case}")


# conv2d_grad_w on bf16 batches that are multiples of 64: both operands transposed to images-last, one contraction per output
# pixel, filter tap and group of 64 images.
WGRAD_CASES = [
    # n   c    h   w   o   k  s  p
    (64, 64, 6, 6, 64, 3, 1, 1),          # 64-channel blocks (four waves), one segment per row
    (64, 128, 7, 9, 128, 3, 1, 1),        # 128 output channels (eight waves), two blocks of input channels, ragged segments
    (64, 64, 9, 8, 128, 3, 2, 1),         # stride 2: two new window columns per pixel; (H + 2p - K) % s = 0 for H and 1 for W
    (64, 64, 8, 8, 128, 1, 2, 0),         # the 1x1 / stride 2 projection
    (64, 64, 5, 5, 64, 3, 1, 0),          # no padding: every tap inside the image
    (64, 128, 10, 6, 64, 3, 2, 1),
    (64, 64, 30, 3, 64, 3, 1, 1),         # more rows than columns: one pixel per segment
    (64, 192, 4, 33, 192, 3, 1, 1),       # 192 = 3 x 64 channels on both sides (64-wide output blocks), long rows
    (64, 128, 9, 9, 64, 1, 1, 0),         # 1x1 at stride 1: one tap, one new column per pixel
    (64, 64, 6, 7, 64, 3, 1, 2),          # padding 2: the result is larger than the input, whole windows outside it
    (64, 64, 11, 11, 64, 3, 2, 0),        # stride 2 without padding
    (128, 64, 5, 6, 64, 3, 1, 1),         # two groups of 64 images: the segment is walked twice
    (192, 64, 4, 4, 128, 3, 2, 1),        # three groups, stride 2
]


@pytest.mark.parametrize("case", WGRAD_CASES, ids=[f"wgrad{i}" for i in range(len(WGRAD_CASES))])
def test_conv2d_grad_w_images_last(case):
    n, c, h, w, o, k, stride, pad = case
    for out_dtype in (None, "f32"):
        spec, data = W.grad_case("conv2d_grad_w", (n, c, h, w, o, k), "bf16", stride, pad, second_is_param=False, out_dtype=out_dtype)
        kernels = [st["kernel"] for st in s_plan_steps(spec)]
        assert kernels.count("transpose_images_last") == 2 and "wgrad_reduce" in kernels and any(kn.startswith("conv2d_grad_w_bf16_") for kn in kernels), kernels
        print(f"wgrad case {case} {out_dtype}", flush=True)
        v = spec.outputs[0]
        if out_dtype == "f32":
            ref = OG.run(spec, data)
            out, _ = run_hip(spec, data)
            assert_close(out[v], ref[v], "f32", f"conv2d_grad_w images-last bf16->f32 {case}", budget=lambda: error_budget(spec, data)[v])
        else:
            check_graph(spec, data, f"conv2d_grad_w images-last {case}")
    # the element-gather form of the same operator
    spec, data = W.grad_case("conv2d_grad_w", (n, c, h, w, o, k), "bf16", stride, pad, second_is_param=False)
    kernels = [st["kernel"] for st in s_plan_steps(spec, {"no_wgrad": 1})]
    assert any(kn.startswith("igemm_conv2d_grad_w_") for kn in kernels), kernels
    check_graph(spec, data, f"conv2d_grad_w gather {case}", opts={"no_wgrad": 1})


def test_gradient_chain_through_two_convolutions():
    # dy pushed back through two stacked 3x3 convolutions: the first gradient's result stays channel-last inside the
    # plan, so it runs on the forward operator's bf16 kernels (nine taps from one copy of the rows)
    for dtype, N, C, H in (("bf16", 32, 128, 28), ("bf16", 4, 256, 14), ("f32", 2, 64, 12)):
        g, data = W.grad_chain(N, C, H, 2, dtype)
        check_graph(g, data, f"two conv2d_grad_x in a row {dtype} {N}x{C}x{H}x{H}")
        kernels = [st["kernel"] for st in s_plan_steps(g)]
        print("gradient chain kernels", kernels, flush=True)
        if dtype == "bf16":
            assert any(k.startswith("igemm_conv2d_grad_x_bf16") and k.endswith("_run" if N == 32 else "_lp") for k in kernels), kernels


def test_gradients_inside_a_graph():
    # forward dense + bias + relu, then the two gradients of the dense for a given dy: the weight is read by the forward
    # contraction in its own layout and by dense_grad_x through a gather step; x feeds dense_grad_w
    for dtype in ("f32", "bf16"):
        g = W.GraphSpec("train_step")
        M, K, N = 24, 40, 16
        x = g.input("x", dtype, (M, K)); w = g.param("w", dtype, (N, K)); b = g.param("b", "f32", (N,)); dy = g.input("dy", dtype, (M, N))
        o0, (y,) = g.op("dense", [x, w], [(dtype, (M, N))])
        o1, (y,) = g.op("bias_add", [y, b], [(dtype, (M, N))], axis=1)
        g.group([o0, o1])
        o2, (dx,) = g.op("dense_grad_x", [dy, w], [(dtype, (M, K))]); g.group([o2])
        o3, (dw,) = g.op("dense_grad_w", [dy, x], [(dtype, (N, K))]); g.group([o3])
        g.output(y); g.output(dx); g.output(dw)
        rng = W.rng_for(16)
        data = {"x": W.as_dtype(W.normal(rng, (M, K)), dtype), "w": W.as_dtype(W.normal(rng, (N, K)) * 0.2, dtype),
                "b": W.as_dtype(W.uniform(rng, (N,), -0.1, 0.1), "f32"), "dy": W.as_dtype(W.normal(rng, (M, N)), dtype)}
        check_graph(g, data, f"forward and gradients in one graph {dtype}")


# ---- typed changes of layout -----------------------------------------------------------------------------
LAYOUT_CASES = [
    ((3, 5, 7, 4), (0, 2, 3, 1), "f32"), ((3, 5, 7, 4), (0, 3, 1, 2), "bf16"), ((37, 70), (1, 0), "bf16"), ((2, 3, 33, 65), (0, 1, 3, 2), "f32"),
    ((2, 3, 4, 5, 6), (0, 1, 4, 2, 3), "bf16"), ((5, 3, 9, 4), (2, 0, 3, 1), "f32"), ((2, 3, 2, 3, 2, 5), (5, 0, 4, 1, 3, 2), "bf16"),
    ((2, 3, 4), (0, 1, 2), "f32"), ((2, 1, 4, 5), (0, 2, 3, 1), "bf16"), ((1,), (0,), "f32"), ((4, 64, 56, 56), (0, 2, 3, 1), "bf16"),
    ((70000, 3), (1, 0), "f32"),
]


@pytest.mark.parametrize("shape,perm,dtype", LAYOUT_CASES, ids=[f"{'x'.join(map(str, c[0]))}-{''.join(map(str, c[1]))}-{c[2]}" for c in LAYOUT_CASES])
def test_layout_transform_moves_every_element(shape, perm, dtype):
    # data movement only: every element, bit for bit (tiled transposition, element gather, aliases and the copy-out)
    spec, data = W.layout_case(shape, perm, dtype)
    got, _ = run_hip(spec, data)
    ref = OG.run(spec, data)
    v = spec.outputs[0]
    np.testing.assert_array_equal(got[v], ref[v])


@pytest.mark.parametrize("batch,c,h,w,dtype", [(3, 64, 14, 14, "bf16"), (2, 128, 14, 14, "bf16"), (2, 24, 9, 7, "f32"), (1, 256, 7, 7, "bf16")])
def test_block_between_channel_last_tensors(batch, c, h, w, dtype):
    # channel-last input -> to_first -> two convolution groups (the second adds the input) -> to_last -> output:
    # the two changes of layout are views of the storage the groups use anyway
    from paper_1810_00952_amd import binding
    spec, data = W.channel_last_block(batch, c, h, w, dtype)
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
    assert [st["kernel"].split("_")[0] for st in desc["steps"]] == ["igemm", "igemm"], [st["kernel"] for st in desc["steps"]]
    got, _ = run_hip(spec, data)
    ref = OG.run(spec, data)
    v = spec.outputs[0]
    assert_close(got[v], ref[v], dtype, "channel-last block", budget=None if dtype == "bf16" else (lambda: error_budget(spec, data)[v]))


@pytest.mark.parametrize("batch,c,h,w,k,s,p,dtype", [(2, 16, 33, 31, 3, 2, 1, "bf16"), (1, 8, 40, 17, 3, 2, 0, "f32"), (2, 64, 112, 112, 3, 2, 1, "bf16"),
                                                   (3, 24, 16, 16, 3, 2, 1, "f32"), (1, 8, 9, 9, 2, 2, 0, "bf16")])
def test_maxpool_between_channel_last_tensors(batch, c, h, w, k, s, p, dtype):
    # signed inputs: taps outside the image must be ignored, not read as zeros; bit-exact (a selection)
    from paper_1810_00952_amd import binding
    spec, data = W.channel_last_maxpool(batch, c, h, w, k, s, p, dtype)
    desc = binding.Plan(binding.graph_from_spec(binding.Context(), spec)).describe()
    assert [st["kernel"] for st in desc["steps"]] == ["maxpool_nhwc"]
    got, _ = run_hip(spec, data)
    ref = OG.run(spec, data)
    v = spec.outputs[0]
    np.testing.assert_array_equal(got[v], ref[v])


def test_layout_views_inside_a_graph():
    # the same value wanted channel-last (an output) and channel-first (another output), and a channel-last view
    # feeding an elementwise group declared on the permuted Shape
    g = W.GraphSpec("views")
    rng = W.rng_for(13)
    dt = "bf16"
    x = g.input("x", dt, (2, 16, 6, 5)); w = g.param("w", dt, (16, 16, 3, 3)); b = g.param("b", "f32", (16,))
    data = {"x": W.as_dtype(W.normal(rng, (2, 16, 6, 5)), dt), "w": W.as_dtype(W.kaiming_normal(rng, (16, 16, 3, 3), 144), dt),
            "b": W.as_dtype(W.uniform(rng, (16,), -0.1, 0.1), "f32")}
    t = (dt, (2, 16, 6, 5)); tl = (dt, (2, 6, 5, 16))
    o0, (y,) = g.op("conv2d", [x, w], [t], stride=(1, 1), pad=(1, 1))
    o1, (y,) = g.op("bias_add", [y, b], [t], axis=1)
    g.group([o0, o1])
    o2, (yl,) = g.op("layout_transform", [y], [tl], perm=(0, 2, 3, 1)); g.group([o2])
    o3, (z,) = g.op("tanh", [yl], [tl])
    o4, (z,) = g.op("mul", [z, yl], [tl])
    g.group([o3, o4])
    o5, (zf,) = g.op("layout_transform", [z], [t], perm=(0, 3, 1, 2)); g.group([o5])
    g.output(y); g.output(yl); g.output(zf)
    got, _ = run_hip(g, data)
    ref = OG.run(g, data)
    np.testing.assert_array_equal(got[yl], np.transpose(got[y], (0, 2, 3, 1)))
    for v in (y, yl, zf):
        assert_close(got[v], ref[v], dt, f"views value {v}")


def test_library_loaded_before_torch_shares_one_hip_runtime():
    # Planning needs no GPU, so a caller may well load the library (and build plans) before anything imports
    # torch.  Both must then end up on one HIP runtime: with two copies in a process the second to
    # initialise finds no device.  Fresh interpreter, library first, then a small group run through torch.
    import os, subprocess, sys
    root = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
    code = (
        "import sys; sys.path.insert(0, %r); sys.path.insert(0, %r)\n"
        "from paper_1810_00952_amd import binding\n"
        "binding.lib()\n"
        "import workloads as W\n"
        "spec, data = W.conv_group(2, 64, 64, 14, 14, 3, 1, 1, 'bf16', residual=True, relu=True, tail=True)\n"
        "plan = binding.Plan(binding.graph_from_spec(binding.Context(), spec))\n"
        "from helpers import run_hip\n"
        "out = run_hip(spec, data)\n"
        "print('ok', len(out))\n"
    ) % (root, os.path.join(root, "tests"))
    r = subprocess.run([sys.executable, "-c", code], capture_output=True, text=True, timeout=300)
    assert r.returncode == 0 and "ok" in r.stdout, r.stdout + r.stderr
