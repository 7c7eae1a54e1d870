"""Shared helpers of the GPU parity tests: tolerances, running a graph
description through the HIP library, extracting one fusion group as a graph."""
import numpy as np

import oracle as O
from oracle import graph as OG
import workloads as W

# fp32 paths, the stated gate:  |g - o| <= 1e-5 + 1e-4 |o|  for every element.
#   An element outside it is accepted only with a reason computed from the oracle's own numbers:
#   (a) `budget`: a first-order worst-case bound on what fp32 arithmetic in *any* summation order can be off by at
#       that element (error_budget below: (K + 1) 2^-24 sum |x w| per contraction, pushed through the rest of the
#       graph with each operator's Lipschitz constant), or
#   (b) `rms_scaled=True`, for deep graphs where (a) is vacuous after twenty layers of worst-case amplification: the
#       absolute term grows to 1e-5 max(1, RMS(o)) -- the error of a sum scales with its terms, not with a result
#       that cancels.
#   Either way the count of such elements and the worst excess over the stated gate are reported (printed, and
#   appended to the file named by PARITY_REPORT if that is set).
# bf16-in / fp32-accumulate paths: |g - o| <= 2e-2 RMS(o) + 2e-2 |o|
#   (a purely relative bound is undefined where outputs change sign; elements outside the pure relative bound
#   are counted in the same report)
F32_RTOL, F32_ATOL = 1e-4, 1e-5
BF16_RTOL = 2e-2
U32 = 2.0 ** -24

REPORT = []


def _report(line):
    import os
    REPORT.append(line)
    print("PARITY " + line, flush=True)
    path = os.environ.get("PARITY_REPORT")
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def assert_close(got, ref, dtype, what="", budget=None, rms_scaled=False):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    err = np.abs(got - ref)
    rms = float(np.sqrt(np.mean(ref ** 2))) if ref.size else 0.0
    if dtype == "bf16":
        n_rel = int((err > BF16_RTOL * np.abs(ref)).sum())
        bound = BF16_RTOL * rms + BF16_RTOL * np.abs(ref)
        how = "rms"
        stated = BF16_RTOL * np.abs(ref)
    else:
        stated = F32_ATOL + F32_RTOL * np.abs(ref)
        n_rel = int((err > stated).sum())
        bound, how = stated, "stated"
        if n_rel and budget is not None:
            bound, how = stated + np.asarray(budget() if callable(budget) else budget, dtype=np.float64), "budget"
        if n_rel and rms_scaled and (err > bound).any():
            bound, how = np.maximum(bound, F32_ATOL * max(1.0, rms) + F32_RTOL * np.abs(ref)), "rms"
    bad = err > bound
    if n_rel or bad.any():
        _report(f"{what}: dtype {dtype} n {err.size} outside_stated_gate {n_rel} worst_excess_over_stated {float((err - stated).max()):.3e} "
                f"max_abs_err {float(err.max()) if err.size else 0.0:.3e} rms_ref {rms:.3e} accepted_by {how} rejected {int(bad.sum())}")
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())}/{bad.size} outside tolerance ({how}); worst at {i}: got {got[i]!r} ref {ref[i]!r} "
                             f"(max abs err {err.max():.3e}, rms {rms:.3e})")


def error_budget(spec, data):
    """For an fp32 graph: {value id: array e} with |fp32 result - oracle result| <= e to first order, whatever the order
    of the fp32 sums -- computed with the oracle's operators on the oracle's values: a contraction of K terms adds
    (K + 1) 2^-24 sum|x w| and passes its operand's error on through |w|; the injective operators pass errors on with
    their Lipschitz constants and add one rounding (a few for the transcendental ones); a value stored at a group
    boundary is rounded once on either side."""
    val = OG.run(spec, data, keep_all=True)
    e = {}
    for i, v in enumerate(spec.values):
        if v.role in ("input", "param"):
            e[i] = np.zeros(v.type.shape)
    for op in spec.ops:
        a = [np.abs(val[v]) for v in op.inputs]
        ea = [e[v] for v in op.inputs]
        y = np.abs(val[op.outputs[0]])
        k = op.kind
        if k == "dense":
            out = O.dense(ea[0], a[1]) + O.dense(a[0], ea[1]) + (a[0].shape[1] + 1) * U32 * O.dense(a[0], a[1])
        elif k == "conv2d":
            st, pd = tuple(op.attrs.get("stride", (1, 1))), tuple(op.attrs.get("pad", (0, 0)))
            K = a[1].shape[1] * a[1].shape[2] * a[1].shape[3]
            out = O.conv2d(ea[0], a[1], st, pd) + O.conv2d(a[0], ea[1], st, pd) + (K + 1) * U32 * O.conv2d(a[0], a[1], st, pd)
        elif k in ("dense_grad_x", "dense_grad_w", "conv2d_grad_x", "conv2d_grad_w"):
            st, pd = tuple(op.attrs.get("stride", (1, 1))), tuple(op.attrs.get("pad", (0, 0)))
            oshape = spec.values[op.outputs[0]].type.shape
            f = {"dense_grad_x": lambda p, q: O.dense_grad_x(p, q), "dense_grad_w": lambda p, q: O.dense_grad_w(p, q),
                 "conv2d_grad_x": lambda p, q: O.conv2d_grad_x(p, q, oshape, st, pd),
                 "conv2d_grad_w": lambda p, q: O.conv2d_grad_w(p, q, oshape[2:], st, pd)}[k]
            terms = {"dense_grad_x": a[0].shape[1], "dense_grad_w": a[0].shape[0],
                     "conv2d_grad_x": a[0].shape[1] * a[1].shape[2] * a[1].shape[3] if k == "conv2d_grad_x" else 0,
                     "conv2d_grad_w": a[0].shape[0] * a[0].shape[2] * a[0].shape[3] if k == "conv2d_grad_w" else 0}[k]
            out = f(ea[0], a[1]) + f(a[0], ea[1]) + (terms + 1) * U32 * f(a[0], a[1])
        elif k == "bias_add":
            out = O.bias_add(ea[0], ea[1], int(op.attrs.get("axis", 1))) + U32 * y
        elif k in ("add", "sub"):
            out = ea[0] + ea[1] + U32 * y
        elif k == "mul":
            out = a[0] * ea[1] + a[1] * ea[0] + U32 * y
        elif k == "div":
            out = ea[0] / a[1] + a[0] * ea[1] / (a[1] * a[1]) + 2 * U32 * y
        elif k == "neg" or k == "relu":
            out = ea[0]
        elif k == "sq":
            out = 2 * a[0] * ea[0] + U32 * y
        elif k == "sigmoid":
            out = 0.25 * ea[0] + 8 * U32
        elif k == "tanh":
            out = ea[0] + 8 * U32
        elif k == "maxpool2d":
            out = O.maxpool2d(ea[0], tuple(op.attrs["kernel"]), tuple(op.attrs.get("stride", (1, 1))), tuple(op.attrs.get("pad", (0, 0))))
        elif k == "global_avgpool":
            hw = a[0].shape[2] * a[0].shape[3]
            out = O.global_avgpool(ea[0]) + (hw + 1) * U32 * O.global_avgpool(a[0])
        elif k == "flatten":
            out = ea[0].reshape(ea[0].shape[0], -1)
        elif k == "concat":
            out = np.concatenate(ea, axis=1)
        elif k == "layout_transform":
            out = np.ascontiguousarray(np.transpose(ea[0], tuple(int(v) for v in op.attrs["perm"])))
        elif k == "cast":
            out = ea[0]
        else:
            raise NotImplementedError(k)
        e[op.outputs[0]] = out + 2 * U32 * y        # stored once by either side
    return e


def run_hip(spec, data, auto_groups=False, opts=None):
    """Run a graph description through the C ABI on cuda:0; returns {output value id: float64 array}.
    auto_groups: let the library form the fusion groups instead of declaring the description's.
    opts: plan-time switches ({field of rl_plan_opts: value})."""
    import torch
    from paper_1810_00952_amd import harness
    s = harness.Session(spec, auto_groups=auto_groups, opts=opts)
    s.load(data)
    s.alloc()
    s.run()
    torch.cuda.synchronize()
    out = {}
    for vid in spec.outputs:
        dt = spec.values[vid].type.dtype
        out[vid] = O.widen(harness.to_host(s.tensors[vid]), dt)
    return out, s


def store_as(arr64, dtype):
    """float64 values exactly representable in dtype -> stored array (float32 / bf16 bits)."""
    a = np.asarray(arr64, dtype=np.float64).astype(np.float32)
    return W.f32_to_bf16_bits(a) if dtype == "bf16" else a


def extract_group(spec, gi):
    """One fusion group as a graph of its own: everything it reads from outside
    becomes an input (weights stay params).  Returns (sub-spec, {old value id: new value id})."""
    ops = sorted(spec.groups[gi])
    gset = set(ops)
    sub = W.GraphSpec(f"{spec.name}.g{gi}")
    vmap = {}
    produced = {v for oi in ops for v in spec.ops[oi].outputs}
    for oi in ops:
        for v in spec.ops[oi].inputs:
            if v not in produced and v not in vmap:
                val = spec.values[v]
                role_param = val.role == "param"
                vmap[v] = (sub.param if role_param else sub.input)(val.name if val.role != "op" else f"v{v}", val.type.dtype, val.type.shape)
    new_ops = []
    for oi in ops:
        op = spec.ops[oi]
        no, outs = sub.op(op.kind, [vmap[v] for v in op.inputs],
                          [(spec.values[v].type.dtype, spec.values[v].type.shape) for v in op.outputs], **op.attrs)
        for a, b in zip(op.outputs, outs):
            vmap[a] = b
        new_ops.append(no)
    sub.group(new_ops)
    consumers = {}
    for oi, op in enumerate(spec.ops):
        for v in op.inputs:
            consumers.setdefault(v, []).append(oi)
    for v in spec.ops[ops[-1]].outputs:
        if v in spec.outputs or any(c not in gset for c in consumers.get(v, [])):
            sub.output(vmap[v])
    return sub, vmap


def extract_groups_channel_last(spec, gis, native_inputs=()):
    """Several fusion groups of `spec` as a graph of their own whose rank-4 activations arrive and leave channel-last:
    every rank-4 value the groups read from outside becomes a channel-last input behind a (0,3,1,2) view (ids in
    native_inputs keep their Shape order), every result used outside leaves through a (0,2,3,1) view.  The views cost a
    plan no kernel, so each group gets the kernel and launch shape it has inside the whole graph.
    Returns (sub-spec, {old input value id: (name, is_channel_last)}, {old result value id: new output value id})."""
    ops = sorted(o for gi in gis for o in spec.groups[gi])
    gset = set(ops)
    sub = W.GraphSpec(f"{spec.name}.g{'_'.join(map(str, gis))}")
    vmap, feeds = {}, {}
    produced = {v for oi in ops for v in spec.ops[oi].outputs}
    for oi in ops:
        for v in spec.ops[oi].inputs:
            if v in produced or v in vmap:
                continue
            val = spec.values[v]
            name = val.name if val.role != "op" else f"v{v}"
            if val.role == "param":
                vmap[v] = sub.param(name, val.type.dtype, val.type.shape)
            elif len(val.type.shape) == 4 and v not in native_inputs:
                n, c, h, w = val.type.shape
                xin = sub.input(name, val.type.dtype, (n, h, w, c))
                o, (xf,) = sub.op("layout_transform", [xin], [(val.type.dtype, val.type.shape)], perm=(0, 3, 1, 2))
                sub.group([o])
                vmap[v] = xf
                feeds[v] = (name, True)
            else:
                vmap[v] = sub.input(name, val.type.dtype, val.type.shape)
                feeds[v] = (name, False)
    for gi in gis:
        new_ops = []
        for oi in sorted(spec.groups[gi]):
            op = spec.ops[oi]
            no, outs = sub.op(op.kind, [vmap[v] for v in op.inputs],
                              [(spec.values[v].type.dtype, spec.values[v].type.shape) for v in op.outputs], **op.attrs)
            for a, b in zip(op.outputs, outs):
                vmap[a] = b
            new_ops.append(no)
        sub.group(new_ops)
    consumers = {}
    for oi, op in enumerate(spec.ops):
        for v in op.inputs:
            consumers.setdefault(v, []).append(oi)
    results = {}
    for gi in gis:
        for v in spec.ops[sorted(spec.groups[gi])[-1]].outputs:
            if v in spec.outputs or any(c not in gset for c in consumers.get(v, [])):
                t = spec.values[v].type
                if len(t.shape) == 4:
                    n, c, h, w = t.shape
                    o, (yl,) = sub.op("layout_transform", [vmap[v]], [(t.dtype, (n, h, w, c))], perm=(0, 2, 3, 1))
                    sub.group([o])
                    sub.output(yl)
                    results[v] = yl
                else:
                    sub.output(vmap[v])
                    results[v] = vmap[v]
    return sub, feeds, results


def fold_resnet_oracle(raw, bn, dtype):
    """Folded parameters computed by the oracle (float64 fold, rounded to f32, then to dtype)."""
    data = {"x": raw["x"], "fc.w": raw["fc.w"], "fc.b": raw["fc.b"]}
    for name, st in bn.items():
        wf, bf = O.fold_batchnorm(raw[name + ".w"], st["gamma"], st["beta"], st["mean"], st["var"], W.BN_EPS)
        data[name + ".wf"] = store_as(O.round_to(wf, "f32"), dtype)
        data[name + ".bf"] = bf.astype(np.float32)
    return data


def fold_resnet_hip(session, raw, bn, dtype):
    """Folded parameters computed on the device by the library's preparation call and bound to the session."""
    import torch
    from paper_1810_00952_amd import harness
    ctx = session.ctx
    dev = session.device
    tdt = torch.bfloat16 if dtype == "bf16" else torch.float32
    for name, st in bn.items():
        w = harness.to_device(raw[name + ".w"], "f32", dev)
        g, b, m, v = (harness.to_device(st[k], "f32", dev) for k in ("gamma", "beta", "mean", "var"))
        wf = torch.empty(w.shape, dtype=tdt, device=dev)
        bf = torch.empty(w.shape[0], dtype=torch.float32, device=dev)
        ctx.fold_batchnorm(w.data_ptr(), g.data_ptr(), b.data_ptr(), m.data_ptr(), v.data_ptr(), W.BN_EPS, wf.data_ptr(), dtype,
                           bf.data_ptr(), w.shape[0], w[0].numel(), harness.stream_handle())
        session.set_value(session.by_name[name + ".wf"], wf)
        session.set_value(session.by_name[name + ".bf"], bf)
    session.load({"x": raw["x"], "fc.w": raw["fc.w"], "fc.b": raw["fc.b"]})
