"""The allocation-free entry point (rl_plan_run_static) against rl_plan_run: same plans, same bindings, the library's
built-in workspace instead of the caller's -- bit for bit, on calls in a row that share the built-in array, the later
ones with smaller inputs (so stale contents of the array from the earlier call lie behind what they use)."""
import numpy as np
import pytest

import workloads as W

pytestmark = pytest.mark.gpu


def _both_ways(spec, data, fold=None):
    import torch
    from paper_1810_00952_amd import binding, harness
    s = harness.Session(spec)
    if fold is not None:
        from helpers import fold_resnet_hip
        fold_resnet_hip(s, *fold)
    else:
        s.load(data)
    s.alloc()
    assert 0 < s.plan.workspace_bytes() <= binding.STATIC_WORKSPACE_BYTES
    s.workspace.fill_(0xA5)                      # the caller's workspace starts from junk as well
    s.run()
    torch.cuda.synchronize()
    want = [harness.to_host(s.tensors[v]).copy() for v in spec.outputs]
    for v in spec.outputs:
        s.tensors[v].zero_()
    torch.cuda.synchronize()
    s.plan.run_static({vid: t.data_ptr() for vid, t in s.tensors.items()}, harness.stream_handle())
    torch.cuda.synchronize()
    got = [harness.to_host(s.tensors[v]) for v in spec.outputs]
    for a, b in zip(got, want):
        assert np.any(b != 0)
        np.testing.assert_array_equal(a, b)
    return want


def test_static_workspace_matches_callers_workspace_on_calls_in_a_row():
    # K split over workgroups: partial sums [slices][M][N] and the hidden layer live in the workspace
    print("mlp batch 32", flush=True)
    big = _both_ways(*W.mlp(32, 784, 128, 10, "f32"))
    print("mlp batch 8 (smaller, right behind it)", flush=True)
    small = _both_ways(*W.mlp(8, 784, 128, 10, "f32"))
    assert big[0].shape == (32, 10) and small[0].shape == (8, 10)
    # a whole graph with liveness-packed intermediates, then a smaller one of the same kind
    for batch, image in ((4, 64), (2, 32)):
        print(f"resnet-shaped graph batch {batch} image {image}", flush=True)
        spec, raw, bn = W.resnet18(batch=batch, dtype="bf16", image=image, width=16, classes=24)
        _both_ways(spec, None, fold=(raw, bn, "bf16"))
    # and against the oracle once, through the static entry point only
    import torch
    from oracle import graph as OG
    from helpers import assert_close
    from paper_1810_00952_amd import harness
    import oracle as O
    spec, data = W.conv_group(2, 64, 64, 14, 14, 3, 1, 1, "f32", residual=True)
    s = harness.Session(spec); s.load(data); s.alloc()
    s.plan.run_static({vid: t.data_ptr() for vid, t in s.tensors.items()}, harness.stream_handle())
    torch.cuda.synchronize()
    assert_close(O.widen(harness.to_host(s.output()), "f32"), OG.run(spec, data)[spec.outputs[0]], "f32", "static entry point vs oracle")
