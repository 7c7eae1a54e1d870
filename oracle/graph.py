"""Oracle-side type checker and op-by-op graph runner -- TEST INFRASTRUCTURE ONLY.

Typing follows the paper's rules (figures "Rules for constructing types" and
"Rules for deriving types of expressions"):
  * Shape-T / Tensor-T: a tensor type is one base type and one shape of
    natural-number constants (here every dim >= 1, rank <= 6);
  * Type-UnaryOp: a unary operator keeps Tensor(b, s);
  * Type-Noncomp-BinaryOp: + - * / need both operands of the *same* b and s
    (so: no implicit broadcast, no implicit promotion) and return that type;
  * Type-Call: a call of a declared operator is well typed only when each
    argument has exactly the parameter type of the operator's arrow type; the
    result is the arrow's result type.  Here an operator's arrow type is
    instantiated from its argument types and attributes (the figure's caption
    notes quantified variables are already instantiated), and the caller's
    declared result type must equal it.

A change of layout is typed like any declared operator: its arrow type
permutes the Shape (the paper's types carry no layout; its section on
extensions proposes tracking it in types, and with row-major storage the
order of the Shape is the layout).

Execution evaluates one operator at a time in float64 and materialises every
intermediate.  A value leaving a fusion group is rounded once (nearest-even)
to its declared dtype; inside a group nothing is rounded.
"""
from __future__ import annotations

from typing import Dict, List, Tuple

import numpy as np

import oracle as O

DTYPES = ("f32", "bf16")
MAX_RANK = 6


class IllTyped(Exception):
    """category in {"kind", "shape", "type", "group", "unsupported"}"""

    def __init__(self, category: str, msg: str):
        super().__init__(f"[{category}] {msg}")
        self.category = category


def _check_tensor_type(t) -> None:
    if t.dtype not in DTYPES:
        raise IllTyped("kind", f"unknown base type {t.dtype!r}")
    if len(t.shape) > MAX_RANK:
        raise IllTyped("kind", f"rank {len(t.shape)} > {MAX_RANK}")
    for d in t.shape:
        if not isinstance(d, (int, np.integer)) or d < 1:
            raise IllTyped("shape", f"dimension {d!r} is not a positive constant")


def _pair(v, name):
    if not (isinstance(v, (tuple, list)) and len(v) == 2):
        raise IllTyped("kind", f"attribute {name} must be a pair")
    return int(v[0]), int(v[1])


def _out_dtype(attrs, in_dtype):
    od = attrs.get("out_dtype", in_dtype)
    if od not in (in_dtype, "f32"):
        raise IllTyped("type", f"out_dtype {od} not allowed for {in_dtype} operands")
    return od


def infer(kind: str, ins: List[Tuple[str, Tuple[int, ...]]], attrs: Dict) -> List[Tuple[str, Tuple[int, ...]]]:
    """Result type(s) of operator `kind` applied to argument types `ins`."""
    def need(n):
        if len(ins) != n:
            raise IllTyped("type", f"{kind} takes {n} arguments, got {len(ins)}")

    if kind in ("neg", "sq", "relu", "sigmoid", "tanh"):
        need(1)
        return [ins[0]]
    if kind in ("add", "sub", "mul", "div"):
        need(2)
        if ins[0] != ins[1]:
            raise IllTyped("type", f"{kind}: operands {ins[0]} and {ins[1]} differ")
        return [ins[0]]
    if kind == "bias_add":
        need(2)
        (dx, sx), (db, sb) = ins
        axis = int(attrs.get("axis", 1))
        if not 0 <= axis < len(sx):
            raise IllTyped("type", "bias_add axis out of range")
        if sb != (sx[axis],):
            raise IllTyped("type", f"bias shape {sb} != ({sx[axis]},)")
        if not (db == dx or (dx == "bf16" and db == "f32")):
            raise IllTyped("type", f"bias dtype {db} not allowed with {dx}")
        return [ins[0]]
    if kind == "dense":
        need(2)
        (dx, sx), (dw, sw) = ins
        if len(sx) != 2 or len(sw) != 2:
            raise IllTyped("type", "dense wants rank-2 operands")
        if dx != dw:
            raise IllTyped("type", "dense operands differ in base type")
        if sx[1] != sw[1]:
            raise IllTyped("type", f"dense inner dims {sx[1]} vs {sw[1]}")
        return [(_out_dtype(attrs, dx), (sx[0], sw[0]))]
    if kind == "conv2d":
        need(2)
        (dx, sx), (dw, sw) = ins
        if len(sx) != 4 or len(sw) != 4:
            raise IllTyped("type", "conv2d wants rank-4 operands")
        if dx != dw:
            raise IllTyped("type", "conv2d operands differ in base type")
        if sx[1] != sw[1]:
            raise IllTyped("type", f"conv2d channels {sx[1]} vs {sw[1]}")
        (s0, s1), (p0, p1) = _pair(attrs.get("stride", (1, 1)), "stride"), _pair(attrs.get("pad", (0, 0)), "pad")
        if s0 < 1 or s1 < 1 or p0 < 0 or p1 < 0:
            raise IllTyped("kind", "bad stride/pad")
        if _pair(attrs.get("dilation", (1, 1)), "dilation") != (1, 1) or int(attrs.get("groups", 1)) != 1:
            raise IllTyped("unsupported", "dilation/groups")
        oh = (sx[2] + 2 * p0 - sw[2]) // s0 + 1
        ow = (sx[3] + 2 * p1 - sw[3]) // s1 + 1
        if sx[2] + 2 * p0 < sw[2] or sx[3] + 2 * p1 < sw[3]:
            raise IllTyped("shape", "kernel larger than padded input")
        return [(_out_dtype(attrs, dx), (sx[0], sw[0], oh, ow))]
    # partial derivatives of the contractions: the arrow types of the operators a reverse-mode gradient calls
    if kind == "dense_grad_x":              # (dy[M,N], W[N,K]) -> [M,K]
        need(2)
        (dy, sy), (dw, sw) = ins
        if len(sy) != 2 or len(sw) != 2:
            raise IllTyped("type", "dense_grad_x wants rank-2 operands")
        if dy != dw:
            raise IllTyped("type", "dense_grad_x operands differ in base type")
        if sy[1] != sw[0]:
            raise IllTyped("type", f"dense_grad_x: dy has {sy[1]} columns, W {sw[0]} rows")
        return [(_out_dtype(attrs, dy), (sy[0], sw[1]))]
    if kind == "dense_grad_w":              # (dy[M,N], x[M,K]) -> [N,K]
        need(2)
        (dy, sy), (dx, sx) = ins
        if len(sy) != 2 or len(sx) != 2:
            raise IllTyped("type", "dense_grad_w wants rank-2 operands")
        if dy != dx:
            raise IllTyped("type", "dense_grad_w operands differ in base type")
        if sy[0] != sx[0]:
            raise IllTyped("type", f"dense_grad_w: batch {sy[0]} vs {sx[0]}")
        return [(_out_dtype(attrs, dy), (sy[1], sx[1]))]
    if kind in ("conv2d_grad_x", "conv2d_grad_w"):
        # (dy[N,O,OH,OW], w[O,C,KH,KW]) -> [N,C,H,W]   /   (dy[N,O,OH,OW], x[N,C,H,W]) -> [O,C,KH,KW]
        # The forward output size floor((H + 2p - KH)/s) + 1 does not determine H (or KH) from the operands: the
        # declaration states the result's Shape and the forward relation is checked against it.
        need(2)
        (dy, sy), (d2, s2) = ins
        if len(sy) != 4 or len(s2) != 4:
            raise IllTyped("type", f"{kind} wants rank-4 operands")
        if dy != d2:
            raise IllTyped("type", f"{kind} operands differ in base type")
        (s0, s1), (p0, p1) = _pair(attrs.get("stride", (1, 1)), "stride"), _pair(attrs.get("pad", (0, 0)), "pad")
        if s0 < 1 or s1 < 1 or p0 < 0 or p1 < 0:
            raise IllTyped("kind", "bad stride/pad")
        decl = attrs.get("declared_shape")
        if decl is None or len(decl) != 4:
            raise IllTyped("type", f"{kind}: the declared result must be rank 4")
        if kind == "conv2d_grad_x":
            n, c, h, w = decl
            o, c2, kh, kw = s2
            x_shape = (sy[0], s2[1], h, w)
            ok = (n, c) == (sy[0], s2[1]) and sy[1] == o
        else:
            o, c, kh, kw = decl
            n, c2, h, w = s2
            x_shape = s2
            ok = (o, c) == (sy[1], s2[1]) and sy[0] == n
        if not ok:
            raise IllTyped("type", f"{kind}: batch / channel counts of operands and declared result disagree")
        if h + 2 * p0 < kh or w + 2 * p1 < kw:
            raise IllTyped("shape", "kernel larger than padded input")
        if ((h + 2 * p0 - kh) // s0 + 1, (w + 2 * p1 - kw) // s1 + 1) != tuple(sy[2:]):
            raise IllTyped("type", f"{kind}: the forward convolution of {x_shape} with a {kh}x{kw} kernel does not give dy's {sy[2:]}")
        return [(_out_dtype(attrs, dy), tuple(decl))]
    if kind == "maxpool2d":
        need(1)
        (dx, sx), = ins
        if len(sx) != 4:
            raise IllTyped("type", "maxpool2d wants rank 4")
        k, s, p = _pair(attrs["kernel"], "kernel"), _pair(attrs.get("stride", (1, 1)), "stride"), _pair(attrs.get("pad", (0, 0)), "pad")
        if min(k) < 1 or min(s) < 1 or min(p) < 0 or p[0] >= k[0] or p[1] >= k[1]:
            raise IllTyped("kind", "bad pool attributes")
        if sx[2] + 2 * p[0] < k[0] or sx[3] + 2 * p[1] < k[1]:
            raise IllTyped("shape", "window larger than padded input")
        return [(dx, (sx[0], sx[1], (sx[2] + 2 * p[0] - k[0]) // s[0] + 1, (sx[3] + 2 * p[1] - k[1]) // s[1] + 1))]
    if kind == "global_avgpool":
        need(1)
        (dx, sx), = ins
        if len(sx) != 4:
            raise IllTyped("type", "global_avgpool wants rank 4")
        return [(dx, (sx[0], sx[1], 1, 1))]
    if kind == "flatten":
        need(1)
        (dx, sx), = ins
        if len(sx) < 2:
            raise IllTyped("type", "flatten wants rank >= 2")
        return [(dx, (sx[0], int(np.prod(sx[1:], dtype=np.int64))))]
    if kind == "concat":
        need(2)
        (da, sa), (db, sb) = ins
        if int(attrs.get("axis", 1)) != 1 or len(sa) != 2 or len(sb) != 2:
            raise IllTyped("unsupported", "concat: rank 2, axis 1 only")
        if da != db or sa[0] != sb[0]:
            raise IllTyped("type", "concat operands disagree")
        return [(da, (sa[0], sa[1] + sb[1]))]
    if kind == "cast":
        need(1)
        to = attrs.get("to")
        if to not in DTYPES:
            raise IllTyped("kind", f"cast to {to!r}")
        return [(to, ins[0][1])]
    if kind == "layout_transform":
        need(1)
        (dx, sx), = ins
        perm = tuple(int(v) for v in attrs.get("perm", ()))
        if sorted(perm) != list(range(len(sx))):
            raise IllTyped("kind", f"perm {perm} is not a permutation of the {len(sx)} axes")
        return [(dx, tuple(sx[p] for p in perm))]
    if kind == "lstm_gates":
        need(2)
        (dz, sz), (dc, sc) = ins
        if dz != "f32" or dc != "f32":
            raise IllTyped("type", "lstm_gates wants f32 pre-activations and cell state")
        if len(sz) != 2 or len(sc) != 2 or sz[0] != sc[0] or sz[1] != 4 * sc[1]:
            raise IllTyped("type", f"lstm_gates shapes {sz} / {sc}")
        hd = attrs.get("h_dtype", None)
        return [("f32", sc), (hd, sc)]   # h' dtype is taken from the declaration
    raise IllTyped("kind", f"unknown operator {kind!r}")


INJECTIVE = {"neg", "sq", "relu", "sigmoid", "tanh", "add", "sub", "mul", "div", "bias_add", "cast"}
ANCHORS = {"dense", "conv2d"}


def check(spec) -> None:
    """Type-check a workloads.GraphSpec and validate its fusion groups."""
    for v in spec.values:
        _check_tensor_type(v.type)
    defined = {i for i, v in enumerate(spec.values) if v.role in ("input", "param")}
    producer = {}
    for oi, op in enumerate(spec.ops):
        for vid in op.inputs:
            if vid not in defined:
                raise IllTyped("type", f"op {oi} uses value {vid} before its definition")
        ins = [(spec.values[v].type.dtype, spec.values[v].type.shape) for v in op.inputs]
        attrs = dict(op.attrs)
        declared = [(spec.values[v].type.dtype, spec.values[v].type.shape) for v in op.outputs]
        if op.kind == "lstm_gates" and len(declared) == 2:
            attrs["h_dtype"] = declared[1][0]
        if op.kind in ("conv2d_grad_x", "conv2d_grad_w") and len(declared) == 1:
            attrs["declared_shape"] = tuple(declared[0][1])
        got = infer(op.kind, ins, attrs)
        if got != declared:
            raise IllTyped("type", f"op {oi} ({op.kind}): declared {declared}, inferred {got}")
        for v in op.outputs:
            defined.add(v)
            producer[v] = oi
    for vid in spec.outputs:
        if vid not in defined:
            raise IllTyped("type", f"output {vid} undefined")

    # ---- fusion groups: connected, one anchor at most and first, the rest
    # injective on the group's output shape, no intermediate escapes
    seen = set()
    consumers: Dict[int, List[int]] = {}
    for oi, op in enumerate(spec.ops):
        for v in op.inputs:
            consumers.setdefault(v, []).append(oi)
    for grp in spec.groups:
        if not grp:
            raise IllTyped("group", "empty group")
        for oi in grp:
            if not 0 <= oi < len(spec.ops) or oi in seen:
                raise IllTyped("group", f"op {oi} missing or in two groups")
            seen.add(oi)
        gset = set(grp)
        ops = [spec.ops[i] for i in sorted(grp)]
        kinds = [o.kind for o in ops]
        lead = 0
        if kinds[0] == "concat" and len(kinds) > 1 and kinds[1] == "dense":
            lead = 1        # concatenation of the GEMM's operand rows is part of the anchor's load
        anchors = [k for k in kinds if k in ANCHORS]
        if len(anchors) > 1:
            raise IllTyped("group", "more than one anchor")
        if anchors and kinds[lead] not in ANCHORS:
            raise IllTyped("group", "anchor is not the group's first operator")
        tail = ops[lead + 1:] if anchors else ops
        if len(ops) > 1:
            for idx, o in enumerate(tail):
                # the gate operator closes a group only as the epilogue of a dense contraction: its pre-activations
                # are the value the rest of the group computes and its cell state comes from outside
                last_gate = o.kind == "lstm_gates" and o is ops[-1] and bool(anchors) and kinds[lead] == "dense"
                if o.kind not in INJECTIVE and not last_gate:
                    raise IllTyped("group", f"{o.kind} cannot be fused")
                if last_gate:
                    prev = ops[-2]
                    if o.inputs[0] not in prev.outputs:
                        raise IllTyped("group", "lstm_gates must take the group's last result as its first operand")
                    if producer.get(o.inputs[1]) in gset:
                        raise IllTyped("group", "lstm_gates' cell state must come from outside the group")
        # connectivity + single escape
        for idx, o in enumerate(ops):
            if idx > 0 and not any(producer.get(v) in gset for v in o.inputs):
                raise IllTyped("group", "group is not connected")
        escaping_ops = set()
        for o in ops:
            for v in o.outputs:
                if v in spec.outputs or any(c not in gset for c in consumers.get(v, [])):
                    escaping_ops.add(id(o))
        if len(escaping_ops) > 1 or (escaping_ops and id(ops[-1]) not in escaping_ops):
            raise IllTyped("group", "an intermediate of the group is used outside it")
        if len(ops) > 1:
            out_shape = spec.values[ops[lead if anchors else 0].outputs[0]].type.shape
            for o in tail:
                if o.kind == "lstm_gates":
                    continue
                if spec.values[o.outputs[0]].type.shape != out_shape:
                    raise IllTyped("group", "fused operators differ in output shape")


def run(spec, data: Dict[str, np.ndarray], keep_all: bool = False, keep=()) -> Dict[int, np.ndarray]:
    """Evaluate the graph.  `data` maps the names of input/param values to
    stored arrays (float32, or uint16 bf16 bits).  Returns float64 arrays for
    the graph outputs (every value when keep_all; the outputs and the value ids
    in `keep` otherwise), each holding numbers exactly representable in that
    value's declared dtype if it crossed a group boundary."""
    check(spec)
    keep = set(keep)
    group_of = {}
    for gi, grp in enumerate(spec.groups):
        for oi in grp:
            group_of[oi] = gi
    nxt = len(spec.groups)
    for oi in range(len(spec.ops)):
        if oi not in group_of:
            group_of[oi] = nxt
            nxt += 1
    consumers: Dict[int, List[int]] = {}
    for oi, op in enumerate(spec.ops):
        for v in op.inputs:
            consumers.setdefault(v, []).append(oi)

    val: Dict[int, np.ndarray] = {}
    for i, v in enumerate(spec.values):
        if v.role in ("input", "param"):
            a = O.widen(data[v.name], v.type.dtype)
            if a.shape != v.type.shape:
                raise ValueError(f"{v.name}: data shape {a.shape} != declared {v.type.shape}")
            val[i] = a
    for oi, op in enumerate(spec.ops):
        a = [val[v] for v in op.inputs]
        k = op.kind
        if k == "dense":
            out = [O.dense(a[0], a[1])]
        elif k == "conv2d":
            out = [O.conv2d(a[0], a[1], tuple(op.attrs.get("stride", (1, 1))), tuple(op.attrs.get("pad", (0, 0))))]
        elif k == "dense_grad_x":
            out = [O.dense_grad_x(a[0], a[1])]
        elif k == "dense_grad_w":
            out = [O.dense_grad_w(a[0], a[1])]
        elif k == "conv2d_grad_x":
            out = [O.conv2d_grad_x(a[0], a[1], spec.values[op.outputs[0]].type.shape, tuple(op.attrs.get("stride", (1, 1))),
                                   tuple(op.attrs.get("pad", (0, 0))))]
        elif k == "conv2d_grad_w":
            out = [O.conv2d_grad_w(a[0], a[1], spec.values[op.outputs[0]].type.shape[2:], tuple(op.attrs.get("stride", (1, 1))),
                                   tuple(op.attrs.get("pad", (0, 0))))]
        elif k == "bias_add":
            out = [O.bias_add(a[0], a[1], int(op.attrs.get("axis", 1)))]
        elif k in ("add", "sub", "mul", "div"):
            out = [O.binary(k, a[0], a[1])]
        elif k in ("neg", "sq", "relu", "sigmoid", "tanh"):
            out = [O.unary(k, a[0])]
        elif k == "maxpool2d":
            out = [O.maxpool2d(a[0], tuple(op.attrs["kernel"]), tuple(op.attrs.get("stride", (1, 1))),
                               tuple(op.attrs.get("pad", (0, 0))))]
        elif k == "global_avgpool":
            out = [O.global_avgpool(a[0])]
        elif k == "flatten":
            out = [a[0].reshape(a[0].shape[0], -1)]
        elif k == "concat":
            out = [np.concatenate([a[0], a[1]], axis=1)]
        elif k == "layout_transform":
            # result[i0, i1, ...] = operand[j] with j[perm[k]] = i[k]: the library routine for exactly that
            out = [np.ascontiguousarray(np.transpose(a[0], tuple(int(v) for v in op.attrs["perm"])))]
        elif k == "cast":
            out = [a[0]]
        elif k == "lstm_gates":
            out = list(O.lstm_gates(a[0], a[1]))
        else:
            raise IllTyped("kind", k)
        for vid, arr in zip(op.outputs, out):
            crosses = vid in spec.outputs or any(group_of[c] != group_of[oi] for c in consumers.get(vid, []))
            if crosses or k == "cast":
                arr = O.round_to(arr, spec.values[vid].type.dtype)
            val[vid] = arr
        if not keep_all:
            # free operands no later op needs
            for v in op.inputs:
                if v in val and all(c <= oi for c in consumers.get(v, [])) and v not in spec.outputs and v not in keep:
                    del val[v]
    if keep_all:
        return val
    return {v: val[v] for v in list(spec.outputs) + [k for k in keep if k not in spec.outputs]}
