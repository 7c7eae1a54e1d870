"""Seeded synthetic workloads: graph descriptions and input tensors.

This module is the only thing the CPU oracle and the HIP library have in
common.  It holds no operator arithmetic: it draws random tensors from a
seeded generator and writes down *descriptions* of typed operator graphs
(operator kind, operand ids, attributes, declared result types, caller's
fusion groups) as plain data.  Each side type-checks and executes those
descriptions with code of its own.

Graph vocabulary follows the paper's grammar: a program is a list of operator
calls over values whose types are Tensor(BaseType, Shape) with constant
shapes (grammar figure, productions Operator, Type, BaseType, Shape).  The
caller declares every result type; the consumer re-derives it (rule
Type-Call).

Tensors are numpy arrays: float32 for dtype "f32"; uint16 bit patterns for
dtype "bf16" (the upper half of the float32 encoding, rounded to nearest
even when produced from float32 data here).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Sequence, Tuple

import numpy as np

BASE_SEED = 181000952  # + config index 1..5


# --------------------------------------------------------------------------
# plain-data graph description
# --------------------------------------------------------------------------
@dataclasses.dataclass(frozen=True)
class TType:
    """Tensor(dtype, Shape(dims...)) with every dim a positive constant."""
    dtype: str            # "f32" | "bf16"
    shape: Tuple[int, ...]


@dataclasses.dataclass
class Value:
    name: str
    role: str             # "input" | "param" | "op"
    type: TType


@dataclasses.dataclass
class Op:
    kind: str             # "dense", "conv2d", "bias_add", "add", ... (lower-case op names)
    inputs: List[int]
    attrs: Dict[str, object]
    outputs: List[int]    # value ids, each with its *declared* type


class GraphSpec:
    """Append-only list of typed values, operator calls, groups and outputs."""

    def __init__(self, name: str):
        self.name = name
        self.values: List[Value] = []
        self.ops: List[Op] = []
        self.groups: List[List[int]] = []
        self.outputs: List[int] = []

    def _val(self, name, role, dtype, shape) -> int:
        self.values.append(Value(name, role, TType(dtype, tuple(int(d) for d in shape))))
        return len(self.values) - 1

    def input(self, name, dtype, shape) -> int:
        return self._val(name, "input", dtype, shape)

    def param(self, name, dtype, shape) -> int:
        return self._val(name, "param", dtype, shape)

    def op(self, kind: str, inputs: Sequence[int], out_types: Sequence[Tuple[str, Sequence[int]]],
           name: str | None = None, **attrs) -> Tuple[int, List[int]]:
        outs = [self._val(f"{name or kind}{len(self.ops)}.{i}", "op", dt, sh)
                for i, (dt, sh) in enumerate(out_types)]
        self.ops.append(Op(kind, list(inputs), dict(attrs), outs))
        return len(self.ops) - 1, outs

    def group(self, op_ids: Sequence[int]) -> int:
        self.groups.append(list(op_ids))
        return len(self.groups) - 1

    def output(self, vid: int) -> None:
        self.outputs.append(vid)

    def type_of(self, vid: int) -> TType:
        return self.values[vid].type

    def ungrouped(self) -> "GraphSpec":
        """Same operator calls, every op a fusion group of its own."""
        g = GraphSpec(self.name + ".unfused")
        g.values = list(self.values)
        g.ops = list(self.ops)
        g.groups = [[i] for i in range(len(self.ops))]
        g.outputs = list(self.outputs)
        return g


# --------------------------------------------------------------------------
# random tensors
# --------------------------------------------------------------------------
def rng_for(config: int, salt: int = 0) -> np.random.Generator:
    return np.random.Generator(np.random.PCG64(BASE_SEED + config + 1000003 * salt))


def f32_to_bf16_bits(a: np.ndarray) -> np.ndarray:
    """float32 -> bf16 bit patterns (uint16), round to nearest, ties to even."""
    shape = np.shape(a)
    u = np.ascontiguousarray(a, dtype=np.float32).view(np.uint32)
    lsb = (u >> np.uint32(16)) & np.uint32(1)
    r = u + np.uint32(0x7FFF) + lsb
    return (r >> np.uint32(16)).astype(np.uint16).reshape(shape)          # (a rank-0 array stays rank 0)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (np.ascontiguousarray(b, dtype=np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32).reshape(np.shape(b))


def as_dtype(a: np.ndarray, dtype: str) -> np.ndarray:
    a = np.asarray(a, dtype=np.float64).astype(np.float32)
    return f32_to_bf16_bits(a) if dtype == "bf16" else a


def normal(rng, shape, std=1.0):
    return rng.standard_normal(size=shape) * std


def uniform(rng, shape, lo, hi):
    return rng.uniform(lo, hi, size=shape)


def kaiming_uniform(rng, shape, fan_in):
    b = np.sqrt(6.0 / fan_in)
    return rng.uniform(-b, b, size=shape)


def kaiming_normal(rng, shape, fan_in):
    return rng.standard_normal(size=shape) * np.sqrt(2.0 / fan_in)


def conv_out(h: int, k: int, s: int, p: int) -> int:
    return (h + 2 * p - k) // s + 1


# --------------------------------------------------------------------------
# config 1: MLP
# --------------------------------------------------------------------------
def mlp(batch=32, d_in=784, d_hidden=128, d_out=10, dtype="f32", config=1):
    """dense+bias+ReLU (one group), dense+bias (one group)."""
    rng = rng_for(config)
    g = GraphSpec("mlp")
    data = {}
    x = g.input("x", dtype, (batch, d_in))
    data["x"] = as_dtype(normal(rng, (batch, d_in)), dtype)
    w1 = g.param("w1", dtype, (d_hidden, d_in))
    data["w1"] = as_dtype(kaiming_uniform(rng, (d_hidden, d_in), d_in), dtype)
    b1 = g.param("b1", "f32", (d_hidden,))
    data["b1"] = as_dtype(uniform(rng, (d_hidden,), -0.1, 0.1), "f32")
    w2 = g.param("w2", dtype, (d_out, d_hidden))
    data["w2"] = as_dtype(kaiming_uniform(rng, (d_out, d_hidden), d_hidden), dtype)
    b2 = g.param("b2", "f32", (d_out,))
    data["b2"] = as_dtype(uniform(rng, (d_out,), -0.1, 0.1), "f32")

    o0, (h,) = g.op("dense", [x, w1], [(dtype, (batch, d_hidden))])
    o1, (h,) = g.op("bias_add", [h, b1], [(dtype, (batch, d_hidden))], axis=1)
    o2, (h,) = g.op("relu", [h], [(dtype, (batch, d_hidden))])
    g.group([o0, o1, o2])
    o3, (y,) = g.op("dense", [h, w2], [(dtype, (batch, d_out))])
    o4, (y,) = g.op("bias_add", [y, b2], [(dtype, (batch, d_out))], axis=1)
    g.group([o3, o4])
    g.output(y)
    return g, data


# --------------------------------------------------------------------------
# config 2: one fused conv2d group
# --------------------------------------------------------------------------
def conv_group(batch=1, cin=64, cout=64, h=56, w=56, k=3, stride=1, pad=1, dtype="f32",
               residual=False, relu=True, config=2, tail=False, make_x=True, bias=True, acts=()):
    """One fused conv2d group.  tail=True appends a second group (neg) so that the
    conv group's result is an intermediate the plan keeps in its private layout.
    make_x=False leaves x out of the data (the caller supplies it); weights and bias then
    do not depend on the batch.  acts: unary operators appended to the group (after the ReLU, if any)."""
    rng = rng_for(config)
    g = GraphSpec("conv_group")
    data = {}
    oh, ow = conv_out(h, k, stride, pad), conv_out(w, k, stride, pad)
    x = g.input("x", dtype, (batch, cin, h, w))
    if make_x:
        data["x"] = as_dtype(normal(rng, (batch, cin, h, w)), dtype)
    wt = g.param("w", dtype, (cout, cin, k, k))
    data["w"] = as_dtype(kaiming_normal(rng, (cout, cin, k, k), cin * k * k), dtype)
    if bias:
        b = g.param("b", "f32", (cout,))
        data["b"] = as_dtype(uniform(rng, (cout,), -0.1, 0.1), "f32")
    ot = (dtype, (batch, cout, oh, ow))
    ids = []
    o, (y,) = g.op("conv2d", [x, wt], [ot], stride=(stride, stride), pad=(pad, pad)); ids.append(o)
    if bias:
        o, (y,) = g.op("bias_add", [y, b], [ot], axis=1); ids.append(o)
    if residual:
        r = g.input("r", dtype, ot[1])
        data["r"] = as_dtype(normal(rng, ot[1]), dtype)
        o, (y,) = g.op("add", [y, r], [ot]); ids.append(o)
    if relu:
        o, (y,) = g.op("relu", [y], [ot]); ids.append(o)
    for kind in acts:
        o, (y,) = g.op(kind, [y], [ot]); ids.append(o)
    g.group(ids)
    if tail:
        o, (y,) = g.op("neg", [y], [ot])
        g.group([o])
    g.output(y)
    return g, data


def downsample_block(batch=4, cin=64, cout=128, h=32, w=32, dtype="bf16", config=10, taps=False):
    """The first block of a ResNet stage on its own: y = relu(conv3x3(relu(conv3x3/2(x) + b1)) + b3 + (conv1x1/2(x) + b2)).
    The stride-2 convolution and the 1x1 projection both read x and neither needs the other.
    taps=True: their two results are graph outputs as well (behind y), as channel-last views."""
    rng = rng_for(config)
    g = GraphSpec("downsample_block")
    data = {}
    oh, ow = conv_out(h, 3, 2, 1), conv_out(w, 3, 2, 1)
    x = g.input("x", dtype, (batch, cin, h, w))
    data["x"] = as_dtype(normal(rng, (batch, cin, h, w)), dtype)
    ot = (dtype, (batch, cout, oh, ow))

    def conv(name, xin, ci, k, stride, pad, extra=None, relu=True):
        wt = g.param(name + ".w", dtype, (cout, ci, k, k))
        data[name + ".w"] = as_dtype(kaiming_normal(rng, (cout, ci, k, k), ci * k * k), dtype)
        b = g.param(name + ".b", "f32", (cout,))
        data[name + ".b"] = as_dtype(uniform(rng, (cout,), -0.1, 0.1), "f32")
        ids = []
        o, (y,) = g.op("conv2d", [xin, wt], [ot], stride=(stride, stride), pad=(pad, pad)); ids.append(o)
        o, (y,) = g.op("bias_add", [y, b], [ot], axis=1); ids.append(o)
        if extra is not None:
            o, (y,) = g.op("add", [y, extra], [ot]); ids.append(o)
        if relu:
            o, (y,) = g.op("relu", [y], [ot]); ids.append(o)
        g.group(ids)
        return y

    c1 = conv("c1", x, cin, 3, 2, 1)
    d = conv("ds", x, cin, 1, 2, 0, relu=False)
    y = conv("c2", c1, cout, 3, 1, 1, extra=d)
    g.output(y)
    if taps:
        for v in (c1, d):
            o, (t,) = g.op("layout_transform", [v], [(dtype, (batch, oh, ow, cout))], perm=(0, 2, 3, 1))
            g.group([o])
            g.output(t)
    return g, data


def grad_case(kind, dims, dtype="f32", stride=1, pad=0, second_is_param=True, out_dtype=None, config=15):
    """One partial-derivative operator on its own.  dims: dense kinds (M, N, K); conv kinds (n, c, h, w, o, k).
    dy ~ N(0,1); the second operand (W or x) is a param or an input as asked."""
    rng = rng_for(config, salt=sum((i + 1) * int(d) for i, d in enumerate(dims)) + 7 * stride + pad)
    g = GraphSpec(kind)
    od = out_dtype or dtype
    attrs = {"out_dtype": out_dtype} if out_dtype else {}
    second = g.param if second_is_param else g.input
    if kind in ("dense_grad_x", "dense_grad_w"):
        M, N, K = dims
        dy = g.input("dy", dtype, (M, N))
        b_shape, out_shape = ((N, K), (M, K)) if kind == "dense_grad_x" else ((M, K), (N, K))
        scale = 1.0 / np.sqrt(N if kind == "dense_grad_x" else M)
    else:
        n, c, h, w, o, k = dims
        oh, ow = conv_out(h, k, stride, pad), conv_out(w, k, stride, pad)
        dy = g.input("dy", dtype, (n, o, oh, ow))
        b_shape, out_shape = (((o, c, k, k), (n, c, h, w)) if kind == "conv2d_grad_x" else ((n, c, h, w), (o, c, k, k)))
        attrs.update(stride=(stride, stride), pad=(pad, pad))
        scale = 1.0 / np.sqrt(o * k * k if kind == "conv2d_grad_x" else n * oh * ow)
    b = second("b", dtype, b_shape)
    o_, (y,) = g.op(kind, [dy, b], [(od, out_shape)], **attrs)
    g.group([o_])
    g.output(y)
    data = {"dy": as_dtype(normal(rng, g.values[dy].type.shape), dtype), "b": as_dtype(normal(rng, b_shape) * scale, dtype)}
    return g, data


def grad_chain(n, c, h, depth=2, dtype="bf16", config=23):
    """dy pushed back through `depth` stacked 3x3 / stride 1 / pad 1 convolutions of c channels: conv2d_grad_x applied
    `depth` times, each through a param of its own (He-scaled), each a group of its own."""
    g = GraphSpec("conv_backward_chain")
    d = g.input("dy", dtype, (n, c, h, h))
    rng = rng_for(config, salt=n + 3 * c + 5 * h + 7 * depth)
    data = {"dy": as_dtype(normal(rng, (n, c, h, h)), dtype)}
    sc = (2.0 / (9 * c)) ** 0.5
    for i in reversed(range(depth)):
        w = g.param(f"w{i}", dtype, (c, c, 3, 3))
        data[f"w{i}"] = as_dtype(normal(rng, (c, c, 3, 3)) * sc, dtype)
        o, (d,) = g.op("conv2d_grad_x", [d, w], [(dtype, (n, c, h, h))], stride=(1, 1), pad=(1, 1))
        g.group([o])
    g.output(d)
    return g, data


def layout_case(shape=(3, 5, 7, 4), perm=(0, 2, 3, 1), dtype="f32", config=11):
    """One change of layout on its own: y = layout_transform(x; perm), y's Shape is x's Shape permuted."""
    rng = rng_for(config, salt=len(shape) * 100 + sum((i + 1) * p for i, p in enumerate(perm)))
    g = GraphSpec("layout_case")
    x = g.input("x", dtype, shape)
    data = {"x": as_dtype(normal(rng, shape), dtype)}
    o, (y,) = g.op("layout_transform", [x], [(dtype, tuple(shape[p] for p in perm))], perm=tuple(perm))
    g.group([o])
    g.output(y)
    return g, data


def channel_last_maxpool(batch=64, c=64, h=112, w=112, k=3, stride=2, pad=1, dtype="bf16", config=14):
    """A max-pool between channel-last tensors (typed views around it): y = to_last(maxpool(to_first(x)))."""
    rng = rng_for(config)
    g = GraphSpec("channel_last_maxpool")
    xl = g.input("x", dtype, (batch, h, w, c))
    data = {"x": as_dtype(normal(rng, (batch, h, w, c)), dtype)}
    oh, ow = conv_out(h, k, stride, pad), conv_out(w, k, stride, pad)
    o, (x,) = g.op("layout_transform", [xl], [(dtype, (batch, c, h, w))], perm=(0, 3, 1, 2)); g.group([o])
    o, (y,) = g.op("maxpool2d", [x], [(dtype, (batch, c, oh, ow))], kernel=(k, k), stride=(stride, stride), pad=(pad, pad)); g.group([o])
    o, (yl,) = g.op("layout_transform", [y], [(dtype, (batch, oh, ow, c))], perm=(0, 2, 3, 1)); g.group([o])
    g.output(yl)
    return g, data


def channel_last_block(batch=3, c=64, h=14, w=14, dtype="bf16", config=12):
    """A residual block between channel-last tensors: the caller holds x as [N, H, W, C] and wants the result
    in the same order, and says so with typed changes of layout around the block:
    y = to_last(relu(conv3x3(relu(conv3x3(to_first(x)) + b1)) + b2 + to_first(x)))."""
    rng = rng_for(config)
    g = GraphSpec("channel_last_block")
    data = {}
    xl = g.input("x", dtype, (batch, h, w, c))
    data["x"] = as_dtype(normal(rng, (batch, h, w, c)), dtype)
    ot = (dtype, (batch, c, h, w))
    o, (x,) = g.op("layout_transform", [xl], [ot], perm=(0, 3, 1, 2))
    g.group([o])

    def conv(name, xin, extra=None):
        wt = g.param(name + ".w", dtype, (c, c, 3, 3))
        data[name + ".w"] = as_dtype(kaiming_normal(rng, (c, c, 3, 3), c * 9), dtype)
        b = g.param(name + ".b", "f32", (c,))
        data[name + ".b"] = as_dtype(uniform(rng, (c,), -0.1, 0.1), "f32")
        ids = []
        o, (y,) = g.op("conv2d", [xin, wt], [ot], stride=(1, 1), pad=(1, 1)); ids.append(o)
        o, (y,) = g.op("bias_add", [y, b], [ot], axis=1); ids.append(o)
        if extra is not None:
            o, (y,) = g.op("add", [y, extra], [ot]); ids.append(o)
        o, (y,) = g.op("relu", [y], [ot]); ids.append(o)
        g.group(ids)
        return y

    c1 = conv("c1", x)
    c2 = conv("c2", c1, extra=x)
    o, (yl,) = g.op("layout_transform", [c2], [(dtype, (batch, h, w, c))], perm=(0, 2, 3, 1))
    g.group([o])
    g.output(yl)
    return g, data


# --------------------------------------------------------------------------
# configs 3 and 4: ResNet-18-shaped inference graph with folded batch-norm
# --------------------------------------------------------------------------
def resnet18(batch=1, dtype="f32", image=224, width=64, classes=1000, config=3,
             blocks=(2, 2, 2, 2), taps=False):
    """Returns (graph, data, bn) where `data` holds x, the *unfolded* conv
    weights, dense weight/bias, and `bn` maps each conv name to its batch-norm
    statistics (gamma, beta, mean, var).  The graph refers to folded parameters
    "<conv>.wf" / "<conv>.bf"; each consumer folds with its own code and casts
    to the graph dtype.  Random draws never depend on `batch` beyond x, nor on
    dtype, so the b64/bf16 graph has the b1/f32 graph's weights.
    taps=True makes the pooled stem tensor and every basic block's result graph outputs as well (behind the
    logits), each as its channel-last view (a layout_transform, which costs the plan no kernel and leaves every
    group's kernel what it is without the taps)."""
    rng = rng_for(3)          # configs 3 and 4 share weights by design
    tapped = []

    def tap(v, c, hw):
        if taps:
            o, (t,) = g.op("layout_transform", [v], [(dtype, (batch, hw, hw, c))], perm=(0, 2, 3, 1))
            g.group([o])
            tapped.append(t)

    xrng = rng_for(3, salt=1)
    g = GraphSpec(f"resnet18_b{batch}_{dtype}")
    raw: Dict[str, np.ndarray] = {}
    bn: Dict[str, Dict[str, np.ndarray]] = {}

    x = g.input("x", dtype, (batch, 3, image, image))
    raw["x"] = as_dtype(normal(xrng, (batch, 3, image, image)), dtype)

    def conv_bn(name, xin, cin, cout, k, s, p, hin, res=None, relu=True):
        ho = conv_out(hin, k, s, p)
        raw[name + ".w"] = as_dtype(kaiming_normal(rng, (cout, cin, k, k), cin * k * k), "f32")
        bn[name] = dict(
            gamma=as_dtype(uniform(rng, (cout,), 0.5, 1.5), "f32"),
            beta=as_dtype(uniform(rng, (cout,), -0.1, 0.1), "f32"),
            mean=as_dtype(normal(rng, (cout,), 0.1), "f32"),
            var=as_dtype(uniform(rng, (cout,), 0.5, 1.5), "f32"))
        wv = g.param(name + ".wf", dtype, (cout, cin, k, k))
        bv = g.param(name + ".bf", "f32", (cout,))
        ot = (dtype, (batch, cout, ho, ho))
        ids = []
        o, (y,) = g.op("conv2d", [xin, wv], [ot], name=name, stride=(s, s), pad=(p, p)); ids.append(o)
        o, (y,) = g.op("bias_add", [y, bv], [ot], axis=1); ids.append(o)
        if res is not None:
            o, (y,) = g.op("add", [y, res], [ot]); ids.append(o)
        if relu:
            o, (y,) = g.op("relu", [y], [ot]); ids.append(o)
        g.group(ids)
        return y, ho

    h = image
    y, h = conv_bn("conv1", x, 3, width, 7, 2, 3, h)
    ho = conv_out(h, 3, 2, 1)
    o, (y,) = g.op("maxpool2d", [y], [(dtype, (batch, width, ho, ho))], kernel=(3, 3), stride=(2, 2), pad=(1, 1))
    g.group([o])
    h = ho
    tap(y, width, h)
    cin = width
    for stage, nblk in enumerate(blocks):
        cout = width << stage
        for blk in range(nblk):
            s = 2 if (stage > 0 and blk == 0) else 1
            name = f"l{stage + 1}.b{blk}"
            skip = y
            y1, h1 = conv_bn(name + ".c1", y, cin, cout, 3, s, 1, h)
            if s != 1 or cin != cout:
                skip, _ = conv_bn(name + ".ds", y, cin, cout, 1, s, 0, h, relu=False)
            y, h = conv_bn(name + ".c2", y1, cout, cout, 3, 1, 1, h1, res=skip)
            cin = cout
            tap(y, cout, h)
    o, (y,) = g.op("global_avgpool", [y], [(dtype, (batch, cin, 1, 1))]); g.group([o])
    o, (y,) = g.op("flatten", [y], [(dtype, (batch, cin))]); g.group([o])
    raw["fc.w"] = as_dtype(kaiming_uniform(rng, (classes, cin), cin), dtype)
    raw["fc.b"] = as_dtype(uniform(rng, (classes,), -0.1, 0.1), "f32")
    wv = g.param("fc.w", dtype, (classes, cin))
    bv = g.param("fc.b", "f32", (classes,))
    o0, (y,) = g.op("dense", [y, wv], [(dtype, (batch, classes))])
    o1, (y,) = g.op("bias_add", [y, bv], [(dtype, (batch, classes))], axis=1)
    g.group([o0, o1])
    g.output(y)
    for t in tapped:
        g.output(t)
    return g, raw, bn


def conv_pool(batch=2, cin=3, cout=64, h=224, w=224, k=7, stride=2, pad=3, dtype="bf16", relu=True, tail=False, config=9):
    """conv2d + bias (+ ReLU) as one group, then max-pool 3x3 / 2 / pad 1 as the next: the ResNet stem's shape.
    tail=True appends neg as a third group, so the pooled tensor is an intermediate too."""
    rng = rng_for(config)
    g = GraphSpec("conv_pool")
    data = {}
    oh, ow = conv_out(h, k, stride, pad), conv_out(w, k, stride, pad)
    x = g.input("x", dtype, (batch, cin, h, w))
    data["x"] = as_dtype(normal(rng, (batch, cin, h, w)), dtype)
    wt = g.param("w", dtype, (cout, cin, k, k))
    data["w"] = as_dtype(kaiming_normal(rng, (cout, cin, k, k), cin * k * k), dtype)
    b = g.param("b", "f32", (cout,))
    data["b"] = as_dtype(uniform(rng, (cout,), -0.5, 0.5), "f32")
    ot = (dtype, (batch, cout, oh, ow))
    ids = []
    o, (y,) = g.op("conv2d", [x, wt], [ot], stride=(stride, stride), pad=(pad, pad)); ids.append(o)
    o, (y,) = g.op("bias_add", [y, b], [ot], axis=1); ids.append(o)
    if relu:
        o, (y,) = g.op("relu", [y], [ot]); ids.append(o)
    g.group(ids)
    ph, pw = conv_out(oh, 3, 2, 1), conv_out(ow, 3, 2, 1)
    pt = (dtype, (batch, cout, ph, pw))
    o, (y,) = g.op("maxpool2d", [y], [pt], kernel=(3, 3), stride=(2, 2), pad=(1, 1))
    g.group([o])
    if tail:
        o, (y,) = g.op("neg", [y], [pt])
        g.group([o])
    g.output(y)
    return g, data


# --------------------------------------------------------------------------
# the LeNet-shaped graph of the paper's decorator example (Fig. "dec_ex"): the
# only model the paper writes down.  Shapes only: inputs are synthetic.
# --------------------------------------------------------------------------
def lenet(batch=64, dtype="f32", config=8):
    """conv 5x5 (1->20) + bias + tanh | maxpool 2x2/2 | conv 5x5 (20->50) + bias + tanh | maxpool 2x2/2 | flatten |
    dense 800->500 + bias + tanh | dense 500->10 + bias; one fusion group per `|` part.  x is N(0,1) of shape
    (batch, 1, 28, 28) (MNIST-shaped, no dataset item), weights Kaiming-uniform, biases U(-0.1, 0.1)."""
    rng = rng_for(config)
    g = GraphSpec(f"lenet_b{batch}_{dtype}")
    data = {}
    x = g.input("x", dtype, (batch, 1, 28, 28))
    data["x"] = as_dtype(normal(rng, (batch, 1, 28, 28)), dtype)

    def conv_tanh(name, xin, cin, cout, k, hin):
        ho = conv_out(hin, k, 1, 0)
        data[name + ".w"] = as_dtype(kaiming_uniform(rng, (cout, cin, k, k), cin * k * k), dtype)
        data[name + ".b"] = as_dtype(uniform(rng, (cout,), -0.1, 0.1), "f32")
        wv = g.param(name + ".w", dtype, (cout, cin, k, k))
        bv = g.param(name + ".b", "f32", (cout,))
        ot = (dtype, (batch, cout, ho, ho))
        o0, (y,) = g.op("conv2d", [xin, wv], [ot], name=name, stride=(1, 1), pad=(0, 0))
        o1, (y,) = g.op("bias_add", [y, bv], [ot], axis=1)
        o2, (y,) = g.op("tanh", [y], [ot])
        g.group([o0, o1, o2])
        return y, ho

    def pool(xin, c, hin):
        ho = conv_out(hin, 2, 2, 0)
        o, (y,) = g.op("maxpool2d", [xin], [(dtype, (batch, c, ho, ho))], kernel=(2, 2), stride=(2, 2), pad=(0, 0))
        g.group([o])
        return y, ho

    def dense(name, xin, cin, cout, act):
        data[name + ".w"] = as_dtype(kaiming_uniform(rng, (cout, cin), cin), dtype)
        data[name + ".b"] = as_dtype(uniform(rng, (cout,), -0.1, 0.1), "f32")
        wv = g.param(name + ".w", dtype, (cout, cin))
        bv = g.param(name + ".b", "f32", (cout,))
        ot = (dtype, (batch, cout))
        ids = []
        o, (y,) = g.op("dense", [xin, wv], [ot], name=name); ids.append(o)
        o, (y,) = g.op("bias_add", [y, bv], [ot], axis=1); ids.append(o)
        if act:
            o, (y,) = g.op("tanh", [y], [ot]); ids.append(o)
        g.group(ids)
        return y

    y, h = conv_tanh("conv1", x, 1, 20, 5, 28)      # 24 x 24
    y, h = pool(y, 20, h)                            # 12 x 12
    y, h = conv_tanh("conv2", y, 20, 50, 5, h)       # 8 x 8
    y, h = pool(y, 50, h)                            # 4 x 4
    o, (y,) = g.op("flatten", [y], [(dtype, (batch, 50 * h * h))]); g.group([o])
    y = dense("fc1", y, 50 * h * h, 500, True)
    y = dense("fc2", y, 500, 10, False)
    g.output(y)
    return g, data


BN_EPS = 1e-5


# --------------------------------------------------------------------------
# config 5: LSTM
# --------------------------------------------------------------------------
def lstm_data(steps=128, batch=64, d_in=1024, hidden=1024, dtype="bf16", config=5):
    rng = rng_for(config)
    bound = 1.0 / 32.0
    return {
        "x": as_dtype(normal(rng, (steps, batch, d_in)), dtype),
        "w": as_dtype(uniform(rng, (4 * hidden, d_in + hidden), -bound, bound), dtype),
        "b": as_dtype(uniform(rng, (4 * hidden,), -bound, bound), "f32"),
    }


def lstm_cell_graph(batch=64, d_in=1024, hidden=1024, dtype="bf16", fused=True):
    """One time step.  z = [x, h] W^T + b in f32, then the gate op.  With
    fused=True the whole cell is one fusion group (GEMM anchor with the gate
    math as its epilogue); otherwise GEMM+bias is one group and the gate op a
    second, purely elementwise, group."""
    g = GraphSpec("lstm_cell")
    x = g.input("x", dtype, (batch, d_in))
    h = g.input("h", dtype, (batch, hidden))
    c = g.input("c", "f32", (batch, hidden))
    w = g.param("w", dtype, (4 * hidden, d_in + hidden))
    b = g.param("b", "f32", (4 * hidden,))
    o0, (xh,) = g.op("concat", [x, h], [(dtype, (batch, d_in + hidden))], axis=1)
    o1, (z,) = g.op("dense", [xh, w], [("f32", (batch, 4 * hidden))], out_dtype="f32")
    o2, (z,) = g.op("bias_add", [z, b], [("f32", (batch, 4 * hidden))], axis=1)
    o3, (c2, h2) = g.op("lstm_gates", [z, c], [("f32", (batch, hidden)), (dtype, (batch, hidden))])
    if fused:
        g.group([o0, o1, o2, o3])
    else:
        g.group([o0, o1, o2])
        g.group([o3])
    g.output(c2)
    g.output(h2)
    return g


def lstm_unrolled_graph(steps, batch, d_in, hidden, dtype="bf16", fused=True):
    """The same recurrence written out as `steps` chained cells with
    h_0 = c_0 = 0 supplied as inputs; outputs every h_t and the last c."""
    g = GraphSpec("lstm_unrolled")
    xs = [g.input(f"x{t}", dtype, (batch, d_in)) for t in range(steps)]
    h = g.input("h0", dtype, (batch, hidden))
    c = g.input("c0", "f32", (batch, hidden))
    w = g.param("w", dtype, (4 * hidden, d_in + hidden))
    b = g.param("b", "f32", (4 * hidden,))
    for t in range(steps):
        o0, (xh,) = g.op("concat", [xs[t], h], [(dtype, (batch, d_in + hidden))], axis=1)
        o1, (z,) = g.op("dense", [xh, w], [("f32", (batch, 4 * hidden))], out_dtype="f32")
        o2, (z,) = g.op("bias_add", [z, b], [("f32", (batch, 4 * hidden))], axis=1)
        o3, (c, h) = g.op("lstm_gates", [z, c], [("f32", (batch, hidden)), (dtype, (batch, hidden))])
        if fused:
            g.group([o0, o1, o2, o3])
        else:
            g.group([o0, o1, o2])
            g.group([o3])
        g.output(h)
    g.output(c)
    return g


# --------------------------------------------------------------------------
# supplementary set E: purely elementwise groups
# --------------------------------------------------------------------------
def eltwise_bias_res_relu(shape=(256, 64, 112, 112), dtype="bf16", config=6):
    """relu(bias_add(x, b) + r) over an NCHW tensor, one fusion group."""
    rng = rng_for(config)
    g = GraphSpec("eltwise_bias_res_relu")
    n, c = shape[0], shape[1]
    x = g.input("x", dtype, shape)
    r = g.input("r", dtype, shape)
    b = g.param("b", "f32", (c,))
    t = (dtype, shape)
    o0, (y,) = g.op("bias_add", [x, b], [t], axis=1)
    o1, (y,) = g.op("add", [y, r], [t])
    o2, (y,) = g.op("relu", [y], [t])
    g.group([o0, o1, o2])
    g.output(y)

    def make_data():
        return {"x": as_dtype(normal(rng, shape), dtype), "r": as_dtype(normal(rng, shape), dtype),
                "b": as_dtype(uniform(rng, (c,), -0.1, 0.1), "f32")}
    return g, make_data


def eltwise_chain(shape=(7, 5, 33), dtype="f32", config=7):
    """sq(neg(tanh(sigmoid(((a+b)*c - d)/e)))) -- every elementwise op kind in
    one anchor-less group; e is kept away from zero."""
    rng = rng_for(config)
    g = GraphSpec("eltwise_chain")
    t = (dtype, shape)
    ids = [g.input(nm, dtype, shape) for nm in "abcde"]
    data = {nm: as_dtype(normal(rng, shape), dtype) for nm in "abcd"}
    data["e"] = as_dtype(uniform(rng, shape, 1.0, 2.0), dtype)
    ops = []
    o, (y,) = g.op("add", [ids[0], ids[1]], [t]); ops.append(o)
    o, (y,) = g.op("mul", [y, ids[2]], [t]); ops.append(o)
    o, (y,) = g.op("sub", [y, ids[3]], [t]); ops.append(o)
    o, (y,) = g.op("div", [y, ids[4]], [t]); ops.append(o)
    o, (y,) = g.op("sigmoid", [y], [t]); ops.append(o)
    o, (y,) = g.op("tanh", [y], [t]); ops.append(o)
    o, (y,) = g.op("neg", [y], [t]); ops.append(o)
    o, (y,) = g.op("sq", [y], [t]); ops.append(o)
    g.group(ops)
    g.output(y)
    return g, data
