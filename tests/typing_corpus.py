"""Well- and ill-typed graph descriptions, one per typing rule.

Each case: (name, builder, expected) with expected None for "accepted" or the
rejection class ("kind" | "shape" | "type" | "group" | "unsupported").  Both
the oracle's checker and the library's planner are run over this corpus and
must agree with `expected` (and so with each other).  Rule names refer to the
paper's figure of expression typing rules.
"""
import numpy as np

from workloads import GraphSpec
import workloads as W


def _unary_ok():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3))
    o, (y,) = g.op("sq", [x], [("f32", (2, 3))]); g.group([o]); g.output(y); return g


def _unary_changes_shape():          # Type-UnaryOp keeps Tensor(b, s)
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3))
    o, (y,) = g.op("neg", [x], [("f32", (3, 2))]); g.output(y); return g


def _unary_changes_dtype():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3))
    o, (y,) = g.op("relu", [x], [("bf16", (2, 3))]); g.output(y); return g


def _binary_ok():
    g = GraphSpec("t"); a = g.input("a", "bf16", (4, 5)); b = g.input("b", "bf16", (4, 5))
    o, (y,) = g.op("mul", [a, b], [("bf16", (4, 5))]); g.output(y); return g


def _binary_broadcast():             # Type-Noncomp-BinaryOp: same s -- no implicit broadcast
    g = GraphSpec("t"); a = g.input("a", "f32", (2, 3, 4, 4)); b = g.input("b", "f32", (3,))
    o, (y,) = g.op("add", [a, b], [("f32", (2, 3, 4, 4))]); g.output(y); return g


def _binary_broadcast_ones():
    g = GraphSpec("t"); a = g.input("a", "f32", (2, 3)); b = g.input("b", "f32", (1, 3))
    o, (y,) = g.op("add", [a, b], [("f32", (2, 3))]); g.output(y); return g


def _binary_mixed_dtype():           # same b -- no implicit promotion
    g = GraphSpec("t"); a = g.input("a", "f32", (2, 3)); b = g.input("b", "bf16", (2, 3))
    o, (y,) = g.op("sub", [a, b], [("f32", (2, 3))]); g.output(y); return g


def _binary_arity():                 # Type-Call: argument count
    g = GraphSpec("t"); a = g.input("a", "f32", (2, 3))
    o, (y,) = g.op("div", [a], [("f32", (2, 3))]); g.output(y); return g


def _dense_ok():
    g, _ = W.mlp(batch=3, d_in=8, d_hidden=4, d_out=2); return g


def _dense_inner_mismatch():         # Type-Call: argument types must match the arrow type
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8)); w = g.param("w", "f32", (4, 7))
    o, (y,) = g.op("dense", [x, w], [("f32", (2, 4))]); g.output(y); return g


def _dense_wrong_declared():         # declared result type != inferred
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8)); w = g.param("w", "f32", (4, 8))
    o, (y,) = g.op("dense", [x, w], [("f32", (2, 8))]); g.output(y); return g


def _dense_transposed_weight():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8)); w = g.param("w", "f32", (8, 4))
    o, (y,) = g.op("dense", [x, w], [("f32", (2, 4))]); g.output(y); return g


def _dense_mixed():
    g = GraphSpec("t"); x = g.input("x", "bf16", (2, 8)); w = g.param("w", "f32", (4, 8))
    o, (y,) = g.op("dense", [x, w], [("f32", (2, 4))], out_dtype="f32"); g.output(y); return g


def _dense_bf16_to_f32_ok():
    g = GraphSpec("t"); x = g.input("x", "bf16", (2, 8)); w = g.param("w", "bf16", (4, 8))
    o, (y,) = g.op("dense", [x, w], [("f32", (2, 4))], out_dtype="f32"); g.output(y); return g


def _dense_f32_to_bf16():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8)); w = g.param("w", "f32", (4, 8))
    o, (y,) = g.op("dense", [x, w], [("bf16", (2, 4))], out_dtype="bf16"); g.output(y); return g


def _conv_ok():
    g, _ = W.conv_group(batch=1, cin=4, cout=4, h=6, w=6); return g


def _conv_ok_stride2():
    g, _ = W.conv_group(batch=2, cin=4, cout=8, h=9, w=9, k=3, stride=2, pad=1, residual=True); return g


def _conv_channel_mismatch():
    g = GraphSpec("t"); x = g.input("x", "f32", (1, 3, 8, 8)); w = g.param("w", "f32", (4, 2, 3, 3))
    o, (y,) = g.op("conv2d", [x, w], [("f32", (1, 4, 6, 6))], stride=(1, 1), pad=(0, 0)); g.output(y); return g


def _conv_wrong_out_hw():            # ceil instead of floor
    g = GraphSpec("t"); x = g.input("x", "f32", (1, 2, 8, 8)); w = g.param("w", "f32", (4, 2, 3, 3))
    o, (y,) = g.op("conv2d", [x, w], [("f32", (1, 4, 4, 4))], stride=(2, 2), pad=(0, 0)); g.output(y); return g


def _conv_rank3():
    g = GraphSpec("t"); x = g.input("x", "f32", (3, 8, 8)); w = g.param("w", "f32", (4, 3, 3, 3))
    o, (y,) = g.op("conv2d", [x, w], [("f32", (4, 6, 6))], stride=(1, 1), pad=(0, 0)); g.output(y); return g


def _conv_kernel_too_big():
    g = GraphSpec("t"); x = g.input("x", "f32", (1, 2, 2, 2)); w = g.param("w", "f32", (4, 2, 5, 5))
    o, (y,) = g.op("conv2d", [x, w], [("f32", (1, 4, 1, 1))], stride=(1, 1), pad=(0, 0)); g.output(y); return g


def _conv_dilated():
    g = GraphSpec("t"); x = g.input("x", "f32", (1, 2, 8, 8)); w = g.param("w", "f32", (4, 2, 3, 3))
    o, (y,) = g.op("conv2d", [x, w], [("f32", (1, 4, 4, 4))], stride=(1, 1), pad=(0, 0), dilation=(2, 2)); g.output(y); return g


def _bias_ok_bf16_f32():
    g = GraphSpec("t"); x = g.input("x", "bf16", (2, 3, 4, 4)); b = g.param("b", "f32", (3,))
    o, (y,) = g.op("bias_add", [x, b], [("bf16", (2, 3, 4, 4))], axis=1); g.output(y); return g


def _bias_wrong_len():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3, 4, 4)); b = g.param("b", "f32", (4,))
    o, (y,) = g.op("bias_add", [x, b], [("f32", (2, 3, 4, 4))], axis=1); g.output(y); return g


def _bias_f32_with_bf16_bias():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3)); b = g.param("b", "bf16", (3,))
    o, (y,) = g.op("bias_add", [x, b], [("f32", (2, 3))], axis=1); g.output(y); return g


def _zero_dim():                     # Shape-T: dims are constants; here >= 1
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 0))
    o, (y,) = g.op("neg", [x], [("f32", (2, 0))]); g.output(y); return g


def _negative_dim():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, -1))
    o, (y,) = g.op("neg", [x], [("f32", (2, -1))]); g.output(y); return g


def _rank7():
    g = GraphSpec("t"); x = g.input("x", "f32", (1,) * 7)
    o, (y,) = g.op("neg", [x], [("f32", (1,) * 7)]); g.output(y); return g


def _rank0_ok():                     # Type-Float-Literal: a scalar is a rank-0 tensor
    g = GraphSpec("t"); x = g.input("x", "f32", ())
    o, (y,) = g.op("sq", [x], [("f32", ())]); g.output(y); return g


def _bad_dtype():                    # BaseType-T
    g = GraphSpec("t"); x = g.input("x", "f16", (2, 2))
    o, (y,) = g.op("neg", [x], [("f16", (2, 2))]); g.output(y); return g


def _unknown_op():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 2))
    o, (y,) = g.op("softmax", [x], [("f32", (2, 2))]); g.output(y); return g


def _pool_ok():
    g = GraphSpec("t"); x = g.input("x", "f32", (1, 2, 7, 7))
    o, (y,) = g.op("maxpool2d", [x], [("f32", (1, 2, 4, 4))], kernel=(3, 3), stride=(2, 2), pad=(1, 1)); g.output(y); return g


def _pool_wrong_out():
    g = GraphSpec("t"); x = g.input("x", "f32", (1, 2, 7, 7))
    o, (y,) = g.op("maxpool2d", [x], [("f32", (1, 2, 3, 3))], kernel=(3, 3), stride=(2, 2), pad=(1, 1)); g.output(y); return g


def _gavg_flatten_ok():
    g = GraphSpec("t"); x = g.input("x", "bf16", (2, 8, 3, 3))
    o, (y,) = g.op("global_avgpool", [x], [("bf16", (2, 8, 1, 1))])
    o, (y,) = g.op("flatten", [y], [("bf16", (2, 8))]); g.output(y); return g


def _flatten_wrong():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8, 3, 3))
    o, (y,) = g.op("flatten", [x], [("f32", (2, 8))]); g.output(y); return g


def _lstm_ok():
    return W.lstm_cell_graph(batch=2, d_in=8, hidden=16, dtype="bf16", fused=True)


def _lstm_unfused_ok():
    return W.lstm_cell_graph(batch=2, d_in=8, hidden=8, dtype="bf16", fused=False)


def _lstm_gates_wrong_width():
    g = GraphSpec("t"); z = g.input("z", "f32", (2, 12)); c = g.input("c", "f32", (2, 4))
    o, (c2, h2) = g.op("lstm_gates", [z, c], [("f32", (2, 4)), ("bf16", (2, 4))]); g.output(h2); return g


def _lstm_gates_bf16_z():
    g = GraphSpec("t"); z = g.input("z", "bf16", (2, 16)); c = g.input("c", "f32", (2, 4))
    o, (c2, h2) = g.op("lstm_gates", [z, c], [("f32", (2, 4)), ("bf16", (2, 4))]); g.output(h2); return g


def _group_gates_behind_injective_chain():      # the gate operator is a contraction's epilogue or a group of its own
    g = GraphSpec("t"); z = g.input("z", "f32", (2, 16)); b = g.param("b", "f32", (16,)); c = g.input("c", "f32", (2, 4))
    o0, (zb,) = g.op("bias_add", [z, b], [("f32", (2, 16))], axis=1)
    o1, (c2, h2) = g.op("lstm_gates", [zb, c], [("f32", (2, 4)), ("f32", (2, 4))])
    g.group([o0, o1]); g.output(c2); g.output(h2); return g


def _gates_behind_injective_chain_ungrouped_ok():
    g = _group_gates_behind_injective_chain(); g.groups.clear(); return g


def _group_gates_skip_the_bias():               # the gate operator reads the contraction's bare result, not the chain's last one
    g = GraphSpec("t"); x = g.input("x", "bf16", (2, 8)); w = g.param("w", "bf16", (16, 8)); b = g.param("b", "f32", (16,))
    c = g.input("c", "f32", (2, 4))
    o0, (z,) = g.op("dense", [x, w], [("f32", (2, 16))], out_dtype="f32")
    o1, (zb,) = g.op("bias_add", [z, b], [("f32", (2, 16))], axis=1)
    o2, (c2, h2) = g.op("lstm_gates", [z, c], [("f32", (2, 4)), ("bf16", (2, 4))])
    g.group([o0, o1, o2]); g.output(c2); g.output(h2); return g


def _dense_grad_ok():
    return W.grad_case("dense_grad_x", (4, 6, 8))[0]


def _dense_grad_w_ok_f32_from_bf16():
    return W.grad_case("dense_grad_w", (4, 6, 8), "bf16", out_dtype="f32")[0]


def _dense_grad_x_inner_mismatch():          # dy's columns are W's rows
    g = GraphSpec("t"); dy = g.input("dy", "f32", (4, 6)); w = g.param("w", "f32", (5, 8))
    o, (y,) = g.op("dense_grad_x", [dy, w], [("f32", (4, 8))]); g.output(y); return g


def _dense_grad_w_wrong_declared():          # the gradient has the weight's Shape [N, K], not its transpose
    g = GraphSpec("t"); dy = g.input("dy", "f32", (4, 6)); x = g.input("x", "f32", (4, 8))
    o, (y,) = g.op("dense_grad_w", [dy, x], [("f32", (8, 6))]); g.output(y); return g


def _conv_grad_x_ok_stride2():                # 7 -> floor((7 + 2 - 3)/2) + 1 = 4; and so does 8: the declaration decides
    return W.grad_case("conv2d_grad_x", (2, 3, 8, 7, 4, 3), stride=2, pad=1)[0]


def _conv_grad_x_declared_size_not_a_preimage():
    g = GraphSpec("t"); dy = g.input("dy", "f32", (1, 4, 4, 4)); w = g.param("w", "f32", (4, 3, 3, 3))
    o, (y,) = g.op("conv2d_grad_x", [dy, w], [("f32", (1, 3, 9, 8))], stride=(2, 2), pad=(1, 1)); g.output(y); return g


def _conv_grad_w_ok():
    return W.grad_case("conv2d_grad_w", (2, 3, 6, 6, 4, 3), stride=1, pad=1, second_is_param=False)[0]


def _conv_grad_w_channel_mismatch():
    g = GraphSpec("t"); dy = g.input("dy", "f32", (2, 4, 6, 6)); x = g.input("x", "f32", (2, 3, 6, 6))
    o, (y,) = g.op("conv2d_grad_w", [dy, x], [("f32", (4, 5, 3, 3))], stride=(1, 1), pad=(1, 1)); g.output(y); return g


def _group_grad_fused():                      # a gradient operator is neither a contraction that opens a group nor injective
    g = GraphSpec("t"); dy = g.input("dy", "f32", (4, 6)); w = g.param("w", "f32", (6, 8))
    o0, (y,) = g.op("dense_grad_x", [dy, w], [("f32", (4, 8))])
    o1, (y,) = g.op("relu", [y], [("f32", (4, 8))])
    g.group([o0, o1]); g.output(y); return g


def _cast_ok():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 4))
    o, (y,) = g.op("cast", [x], [("bf16", (2, 4))], to="bf16"); g.output(y); return g


def _cast_wrong_declared():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 4))
    o, (y,) = g.op("cast", [x], [("f32", (2, 4))], to="bf16"); g.output(y); return g


# ---- change of layout: an operator whose arrow type permutes the Shape
def _layout_ok():
    g = GraphSpec("t"); x = g.input("x", "bf16", (2, 3, 4, 5))
    o, (y,) = g.op("layout_transform", [x], [("bf16", (2, 4, 5, 3))], perm=(0, 2, 3, 1)); g.output(y); return g


def _layout_wrong_declared():        # the inverse permutation's Shape
    g = GraphSpec("t"); x = g.input("x", "bf16", (2, 3, 4, 5))
    o, (y,) = g.op("layout_transform", [x], [("bf16", (2, 5, 3, 4))], perm=(0, 2, 3, 1)); g.output(y); return g


def _layout_not_a_permutation():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3, 4))
    o, (y,) = g.op("layout_transform", [x], [("f32", (2, 4, 4))], perm=(0, 2, 2)); g.output(y); return g


def _layout_perm_too_short():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3, 4))
    o, (y,) = g.op("layout_transform", [x], [("f32", (3, 2))], perm=(1, 0)); g.output(y); return g


def _layout_changes_dtype():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3))
    o, (y,) = g.op("layout_transform", [x], [("bf16", (3, 2))], perm=(1, 0)); g.output(y); return g


def _group_layout_fused():           # a change of layout is not injective on the group's output shape
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 3))
    o0, (y,) = g.op("relu", [x], [("f32", (2, 3))])
    o1, (y,) = g.op("layout_transform", [y], [("f32", (3, 2))], perm=(1, 0))
    g.group([o0, o1]); g.output(y); return g


# ---- fusion-group legality
def _group_two_anchors():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8)); w1 = g.param("w1", "f32", (8, 8)); w2 = g.param("w2", "f32", (4, 8))
    o0, (y,) = g.op("dense", [x, w1], [("f32", (2, 8))])
    o1, (y,) = g.op("dense", [y, w2], [("f32", (2, 4))])
    g.group([o0, o1]); g.output(y); return g


def _group_anchor_not_first():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8)); w = g.param("w", "f32", (4, 8))
    o0, (y,) = g.op("relu", [x], [("f32", (2, 8))])
    o1, (y,) = g.op("dense", [y, w], [("f32", (2, 4))])
    g.group([o0, o1]); g.output(y); return g


def _group_intermediate_escapes():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 8)); w = g.param("w", "f32", (4, 8))
    o0, (y0,) = g.op("dense", [x, w], [("f32", (2, 4))])
    o1, (y1,) = g.op("relu", [y0], [("f32", (2, 4))])
    g.group([o0, o1]); g.output(y0); g.output(y1); return g


def _group_disconnected():
    g = GraphSpec("t"); a = g.input("a", "f32", (2, 4)); b = g.input("b", "f32", (2, 4))
    o0, (y0,) = g.op("relu", [a], [("f32", (2, 4))])
    o1, (y1,) = g.op("neg", [b], [("f32", (2, 4))])
    g.group([o0, o1]); g.output(y1); return g


def _group_pool_fused():
    g = GraphSpec("t"); x = g.input("x", "f32", (1, 2, 7, 7))
    o0, (y,) = g.op("relu", [x], [("f32", (1, 2, 7, 7))])
    o1, (y,) = g.op("maxpool2d", [y], [("f32", (1, 2, 4, 4))], kernel=(3, 3), stride=(2, 2), pad=(1, 1))
    g.group([o0, o1]); g.output(y); return g


def _group_op_twice():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 4))
    o0, (y,) = g.op("relu", [x], [("f32", (2, 4))])
    g.group([o0]); g.group([o0]); g.output(y); return g


def _group_elementwise_ok():
    g, _ = W.eltwise_chain(); return g


def _use_before_def():
    g = GraphSpec("t"); x = g.input("x", "f32", (2, 4))
    o0, (y,) = g.op("relu", [x], [("f32", (2, 4))])
    g.ops[0].inputs[0] = y      # consumes its own result
    g.output(y); return g


CASES = [
    ("unary_ok", _unary_ok, None),
    ("unary_changes_shape", _unary_changes_shape, "type"),
    ("unary_changes_dtype", _unary_changes_dtype, "type"),
    ("binary_ok", _binary_ok, None),
    ("binary_broadcast", _binary_broadcast, "type"),
    ("binary_broadcast_ones", _binary_broadcast_ones, "type"),
    ("binary_mixed_dtype", _binary_mixed_dtype, "type"),
    ("binary_arity", _binary_arity, "type"),
    ("dense_ok", _dense_ok, None),
    ("dense_inner_mismatch", _dense_inner_mismatch, "type"),
    ("dense_wrong_declared", _dense_wrong_declared, "type"),
    ("dense_transposed_weight", _dense_transposed_weight, "type"),
    ("dense_mixed", _dense_mixed, "type"),
    ("dense_bf16_to_f32_ok", _dense_bf16_to_f32_ok, None),
    ("dense_f32_to_bf16", _dense_f32_to_bf16, "type"),
    ("conv_ok", _conv_ok, None),
    ("conv_ok_stride2", _conv_ok_stride2, None),
    ("conv_channel_mismatch", _conv_channel_mismatch, "type"),
    ("conv_wrong_out_hw", _conv_wrong_out_hw, "type"),
    ("conv_rank3", _conv_rank3, "type"),
    ("conv_kernel_too_big", _conv_kernel_too_big, "shape"),
    ("conv_dilated", _conv_dilated, "unsupported"),
    ("bias_ok_bf16_f32", _bias_ok_bf16_f32, None),
    ("bias_wrong_len", _bias_wrong_len, "type"),
    ("bias_f32_with_bf16_bias", _bias_f32_with_bf16_bias, "type"),
    ("zero_dim", _zero_dim, "shape"),
    ("negative_dim", _negative_dim, "shape"),
    ("rank7", _rank7, "kind"),
    ("rank0_ok", _rank0_ok, None),
    ("bad_dtype", _bad_dtype, "kind"),
    ("unknown_op", _unknown_op, "kind"),
    ("pool_ok", _pool_ok, None),
    ("pool_wrong_out", _pool_wrong_out, "type"),
    ("gavg_flatten_ok", _gavg_flatten_ok, None),
    ("flatten_wrong", _flatten_wrong, "type"),
    ("lstm_ok", _lstm_ok, None),
    ("lstm_unfused_ok", _lstm_unfused_ok, None),
    ("lstm_gates_wrong_width", _lstm_gates_wrong_width, "type"),
    ("lstm_gates_bf16_z", _lstm_gates_bf16_z, "type"),
    ("group_gates_behind_injective_chain", _group_gates_behind_injective_chain, "group"),
    ("gates_behind_injective_chain_ungrouped_ok", _gates_behind_injective_chain_ungrouped_ok, None),
    ("group_gates_skip_the_bias", _group_gates_skip_the_bias, "group"),
    ("dense_grad_ok", _dense_grad_ok, None),
    ("dense_grad_w_ok_f32_from_bf16", _dense_grad_w_ok_f32_from_bf16, None),
    ("dense_grad_x_inner_mismatch", _dense_grad_x_inner_mismatch, "type"),
    ("dense_grad_w_wrong_declared", _dense_grad_w_wrong_declared, "type"),
    ("conv_grad_x_ok_stride2", _conv_grad_x_ok_stride2, None),
    ("conv_grad_x_declared_size_not_a_preimage", _conv_grad_x_declared_size_not_a_preimage, "type"),
    ("conv_grad_w_ok", _conv_grad_w_ok, None),
    ("conv_grad_w_channel_mismatch", _conv_grad_w_channel_mismatch, "type"),
    ("group_grad_fused", _group_grad_fused, "group"),
    ("cast_ok", _cast_ok, None),
    ("cast_wrong_declared", _cast_wrong_declared, "type"),
    ("layout_ok", _layout_ok, None),
    ("layout_wrong_declared", _layout_wrong_declared, "type"),
    ("layout_not_a_permutation", _layout_not_a_permutation, "kind"),
    ("layout_perm_too_short", _layout_perm_too_short, "kind"),
    ("layout_changes_dtype", _layout_changes_dtype, "type"),
    ("group_layout_fused", _group_layout_fused, "group"),
    ("group_two_anchors", _group_two_anchors, "group"),
    ("group_anchor_not_first", _group_anchor_not_first, "group"),
    ("group_intermediate_escapes", _group_intermediate_escapes, "group"),
    ("group_disconnected", _group_disconnected, "group"),
    ("group_pool_fused", _group_pool_fused, "group"),
    ("group_op_twice", _group_op_twice, "group"),
    ("group_elementwise_ok", _group_elementwise_ok, None),
    ("use_before_def", _use_before_def, "type"),
]


def random_graphs(n, seed=7):
    """Seeded corpus of small random elementwise/dense graphs, about half of
    them broken by one mutation (a dim changed, a dtype flipped, a declared
    type altered).  Yields (spec, mutated: bool); `mutated` graphs may still be
    well typed (the checkers only have to agree)."""
    rng = np.random.default_rng(seed)
    for i in range(n):
        g = GraphSpec(f"rand{i}")
        m, k, nn = (int(v) for v in rng.integers(1, 6, 3))
        dt = "f32" if rng.random() < 0.6 else "bf16"
        x = g.input("x", dt, (m, k)); w = g.param("w", dt, (nn, k)); b = g.param("b", "f32", (nn,))
        r = g.input("r", dt, (m, nn))
        t = (dt, (m, nn))
        ops = []
        o, (y,) = g.op("dense", [x, w], [t]); ops.append(o)
        o, (y,) = g.op("bias_add", [y, b], [t], axis=1); ops.append(o)
        for _ in range(int(rng.integers(0, 4))):
            kind = ["add", "mul", "relu", "tanh", "sq", "sub"][int(rng.integers(0, 6))]
            if kind in ("add", "mul", "sub"):
                o, (y,) = g.op(kind, [y, r], [t])
            else:
                o, (y,) = g.op(kind, [y], [t])
            ops.append(o)
        g.group(ops); g.output(y)
        mutated = rng.random() < 0.5
        if mutated:
            vid = int(rng.integers(0, len(g.values)))
            v = g.values[vid]
            shape = list(v.type.shape)
            choice = int(rng.integers(0, 3))
            if choice == 0 and shape:
                shape[int(rng.integers(0, len(shape)))] += int(rng.integers(1, 3))
                g.values[vid] = W.Value(v.name, v.role, W.TType(v.type.dtype, tuple(shape)))
            elif choice == 1:
                g.values[vid] = W.Value(v.name, v.role, W.TType("bf16" if v.type.dtype == "f32" else "f32", v.type.shape))
            else:
                g.values[vid] = W.Value(v.name, v.role, W.TType(v.type.dtype, tuple(reversed(shape))))
        yield g, mutated
