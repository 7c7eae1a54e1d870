"""Shared helpers of the GPU parity tests: tolerances, running a graph
description through the HIP library, extracting one fusion group as a graph."""
import numpy as np

import oracle as O
from oracle import graph as OG
import workloads as W

# fp32 paths: |g - o| <= 1e-5 max(1, RMS(o)) + 1e-4 |o|
#   The absolute term is 1e-5 for tensors of unit scale and grows with the
#   tensor's scale: the rounding error of an fp32 sum is proportional to the
#   size of its terms, not of a result that cancels to near zero.
# bf16-in / fp32-accumulate paths: |g - o| <= 2e-2 RMS(o) + 2e-2 |o|
#   (a purely relative bound is undefined where outputs change sign)
F32_RTOL, F32_ATOL = 1e-4, 1e-5
BF16_RTOL = 2e-2


def assert_close(got, ref, dtype, what="", atol_scale=1.0):
    got = np.asarray(got, dtype=np.float64)
    ref = np.asarray(ref, dtype=np.float64)
    assert got.shape == ref.shape, (what, got.shape, ref.shape)
    assert np.all(np.isfinite(got)), what
    if dtype == "bf16":
        atol = BF16_RTOL * float(np.sqrt(np.mean(ref ** 2)))
        rtol = BF16_RTOL
    else:
        atol, rtol = F32_ATOL * atol_scale * max(1.0, float(np.sqrt(np.mean(ref ** 2)))), F32_RTOL
    err = np.abs(got - ref)
    bound = atol + rtol * np.abs(ref)
    bad = err > bound
    if bad.any():
        i = np.unravel_index(np.argmax(err - bound), err.shape)
        raise AssertionError(f"{what}: {int(bad.sum())}/{bad.size} outside tolerance; worst at {i}: got {got[i]!r} ref {ref[i]!r} "
                             f"(max abs err {err.max():.3e}, atol {atol:.3e}, rtol {rtol})")


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
