"""Graph-level pins for the oracle's runner (CPU only): fused == unfused
composition, folded batch-norm == explicit batch-norm inside a graph, the
unrolled LSTM graph == the plain recurrence, bf16 rounding points."""
import numpy as np

import oracle as O
from oracle import graph as OG
import workloads as W


def test_fused_equals_unfused_f32():
    g, data = W.conv_group(batch=2, cin=4, cout=6, h=7, w=6, residual=True)
    fused = OG.run(g, data)[g.outputs[0]]
    unf = OG.run(g.ungrouped(), data)[g.outputs[0]]
    # unfused rounds to f32 after every operator, fused once: a few f32 ulps apart
    np.testing.assert_allclose(fused, unf, rtol=1e-6, atol=1e-6)
    # and both equal the composition written out with the op functions
    x, w, b, r = (O.widen(data[k], "f32") for k in ("x", "w", "b", "r"))
    ref = O.unary("relu", O.binary("add", O.bias_add(O.conv2d(x, w, (1, 1), (1, 1)), b, 1), r))
    np.testing.assert_array_equal(fused, O.round_to(ref, "f32"))


def test_fused_equals_unfused_bf16_within_rounding():
    g, data = W.conv_group(batch=1, cin=8, cout=8, h=6, w=6, dtype="bf16", residual=True)
    fused = OG.run(g, data)[g.outputs[0]]
    unf = OG.run(g.ungrouped(), data)[g.outputs[0]]
    # each fused-away boundary costs at most one bf16 rounding (2^-8 relative) of a value of the output's scale
    scale = np.sqrt(np.mean(fused ** 2)) + np.abs(fused)
    assert np.all(np.abs(fused - unf) <= 4 * 2.0 ** -8 * scale)
    # group outputs are bf16-representable
    np.testing.assert_array_equal(O.round_to(fused, "bf16"), fused)


def test_mlp_graph_matches_numpy():
    g, data = W.mlp(batch=4, d_in=16, d_hidden=8, d_out=3)
    y = OG.run(g, data)[g.outputs[0]]
    x, w1, b1, w2, b2 = (data[k].astype(np.float64) for k in ("x", "w1", "b1", "w2", "b2"))
    h = np.maximum(x @ w1.T + b1, 0).astype(np.float32).astype(np.float64)
    ref = (h @ w2.T + b2).astype(np.float32).astype(np.float64)
    np.testing.assert_allclose(y, ref, rtol=1e-6, atol=1e-7)


def test_resnet_folded_equals_explicit_bn_small():
    g, raw, bn = W.resnet18(batch=1, dtype="f32", image=32, width=8, classes=10, blocks=(1, 1, 1, 1))
    data = {"x": raw["x"], "fc.w": raw["fc.w"], "fc.b": raw["fc.b"]}
    for name, st in bn.items():
        wf, bf = O.fold_batchnorm(raw[name + ".w"], st["gamma"], st["beta"], st["mean"], st["var"], W.BN_EPS)
        data[name + ".wf"] = wf.astype(np.float32)
        data[name + ".bf"] = bf.astype(np.float32)
    got = OG.run(g, data)[g.outputs[0]]
    assert got.shape == (1, 10)

    # the same network written with explicit conv -> batch-norm, float64 throughout
    def cbn(x, name, s, p):
        st = bn[name]
        return O.batchnorm(O.conv2d(x, raw[name + ".w"], (s, s), (p, p)), st["gamma"], st["beta"], st["mean"], st["var"], W.BN_EPS)
    relu = lambda v: O.unary("relu", v)
    y = relu(cbn(O.widen(raw["x"], "f32"), "conv1", 2, 3))
    y = O.maxpool2d(y, (3, 3), (2, 2), (1, 1))
    for stage in range(4):
        s = 2 if stage > 0 else 1
        name = f"l{stage + 1}.b0"
        skip = y if stage == 0 else cbn(y, name + ".ds", s, 0)
        y1 = relu(cbn(y, name + ".c1", s, 1))
        y = relu(cbn(y1, name + ".c2", 1, 1) + skip)
    y = O.global_avgpool(y).reshape(1, -1)
    ref = O.bias_add(O.dense(y, raw["fc.w"]), raw["fc.b"], 1)
    np.testing.assert_allclose(got, ref, rtol=2e-5, atol=2e-5)


def test_resnet18_shape_inventory():
    g, raw, bn = W.resnet18(batch=1, dtype="f32")
    OG.check(g)
    convs = [o for o in g.ops if o.kind == "conv2d"]
    assert len(convs) == 20 and len(g.groups) == 24      # 20 conv groups + maxpool + avgpool + flatten + dense
    macs = 0
    for o in convs:
        (n, co, oh, ow), (_, ci, kh, kw) = g.values[o.outputs[0]].type.shape, g.values[o.inputs[1]].type.shape
        macs += n * co * oh * ow * ci * kh * kw
    assert macs == 1813561344
    assert sum(raw[k].size for k in raw if k.endswith(".w")) == 11678912
    assert g.values[g.outputs[0]].type.shape == (1, 1000)


def test_unrolled_lstm_equals_recurrence():
    T, B, I, H = 3, 2, 8, 8
    d = W.lstm_data(T, B, I, H, "bf16")
    g = W.lstm_unrolled_graph(T, B, I, H, "bf16", fused=True)
    data = {f"x{t}": d["x"][t] for t in range(T)}
    data.update(h0=np.zeros((B, H), np.uint16), c0=np.zeros((B, H), np.float32), w=d["w"], b=d["b"])
    out = OG.run(g, data)
    hs, c = O.lstm_sequence(O.widen(d["x"], "bf16"), O.widen(d["w"], "bf16"), O.widen(d["b"], "f32"),
                            np.zeros((B, H)), np.zeros((B, H)))
    for t in range(T):
        np.testing.assert_array_equal(out[g.outputs[t]], hs[t])
    np.testing.assert_array_equal(out[g.outputs[T]], c)
    # unfused grouping differs only by the f32 rounding of z
    out2 = OG.run(W.lstm_unrolled_graph(T, B, I, H, "bf16", fused=False), data)
    np.testing.assert_allclose(out2[g.outputs[T]], c, rtol=1e-2, atol=1e-3)


def test_layout_transform_is_the_index_permutation():
    # pin: written out with loops over every index of small tensors of rank 2..5: y[i] = x[j], j[perm[k]] = i[k]
    import itertools
    for shape, perm in (((3, 4), (1, 0)), ((2, 3, 4), (2, 0, 1)), ((2, 3, 4, 5), (0, 2, 3, 1)), ((2, 3, 4, 5), (0, 3, 1, 2)),
                        ((2, 3, 2, 3, 2), (4, 0, 3, 1, 2))):
        g, data = W.layout_case(shape, perm, "f32")
        y = OG.run(g, data)[g.outputs[0]]
        x = data["x"].astype(np.float64)
        assert y.shape == tuple(shape[p] for p in perm)
        for i in itertools.product(*(range(d) for d in y.shape)):
            j = [0] * len(shape)
            for k, p in enumerate(perm):
                j[p] = i[k]
            assert y[i] == x[tuple(j)]
        # the inverse permutation brings the operand back
        inv = tuple(int(v) for v in np.argsort(perm))
        g2 = W.GraphSpec("back")
        a = g2.input("x", "f32", y.shape)
        o, (b,) = g2.op("layout_transform", [a], [("f32", shape)], perm=inv)
        g2.output(b)
        np.testing.assert_array_equal(OG.run(g2, {"x": y.astype(np.float32)})[b], x)


def test_channel_last_block_equals_the_channel_first_block():
    # the typed changes of layout around a block do not change its values: compare with the same block on the
    # transposed input, written with the op functions
    g, data = W.channel_last_block(batch=2, c=8, h=5, w=6, dtype="f32")
    y = OG.run(g, data)[g.outputs[0]]
    x = np.transpose(O.widen(data["x"], "f32"), (0, 3, 1, 2))
    w1, b1, w2, b2 = (O.widen(data[k], "f32") for k in ("c1.w", "c1.b", "c2.w", "c2.b"))
    c1 = O.round_to(O.unary("relu", O.bias_add(O.conv2d(x, w1, (1, 1), (1, 1)), b1, 1)), "f32")
    c2 = O.round_to(O.unary("relu", O.binary("add", O.bias_add(O.conv2d(c1, w2, (1, 1), (1, 1)), b2, 1), x)), "f32")
    np.testing.assert_array_equal(y, np.transpose(c2, (0, 2, 3, 1)))


def _bits32(a):
    return np.asarray(a, dtype=np.float64).astype(np.float32).view(np.uint32).ravel()


def test_cast_rounds_where_it_stands_and_nothing_else_does_inside_a_group():
    # The cast expression rounds at once, also in the middle of a fusion group; every other operator's result is
    # rounded only when it leaves its group.  Expected values are bit patterns worked out by hand:
    #   x0 = 1 + 2^-8            tie between 1 and 1 + 2^-7          -> bf16 0x3F80 (even)
    #   x1 = 1 + 3 * 2^-8        tie between 1 + 2^-7 and 1 + 2^-6   -> bf16 0x3F82 (even)
    #   x2 = 1 + 2^-8 + 2^-12    above the tie                       -> bf16 0x3F81
    x = np.array([[1 + 2.0 ** -8, 1 + 3 * 2.0 ** -8, 1 + 2.0 ** -8 + 2.0 ** -12]], dtype=np.float32)
    g = W.GraphSpec("cast_out")
    xv = g.input("x", "f32", (1, 3))
    o0, (y,) = g.op("cast", [xv], [("bf16", (1, 3))], to="bf16")
    g.group([o0]); g.output(y)
    out = OG.run(g, {"x": x})[y]
    np.testing.assert_array_equal(_bits32(out) >> 16, [0x3F80, 0x3F82, 0x3F81])
    np.testing.assert_array_equal(_bits32(out) & 0xFFFF, [0, 0, 0])

    # cast -> sq -> cast back, as one group: the first cast rounds (1 + 2^-7 for x2), the square (1 + 2^-6 + 2^-14) is
    # *not* rounded to bf16 although its declared type is bf16, the cast to f32 keeps it: 0x3F820200.
    # (cast as identity would give (1 + 2^-8 + 2^-12)^2; rounding the square to bf16 would give 0x3F820000.)
    def chain(grouped):
        g = W.GraphSpec("cast_chain")
        xv = g.input("x", "f32", (1, 3))
        o0, (a,) = g.op("cast", [xv], [("bf16", (1, 3))], to="bf16")
        o1, (b,) = g.op("sq", [a], [("bf16", (1, 3))])
        o2, (c,) = g.op("cast", [b], [("f32", (1, 3))], to="f32")
        if grouped:
            g.group([o0, o1, o2])
        g.output(c)
        return g, c
    g, c = chain(True)
    np.testing.assert_array_equal(_bits32(OG.run(g, {"x": x})[c]), [0x3F800000, 0x3F840800, 0x3F820200])
    # the same calls each in a group of its own: the square leaves its group as a bf16 value (1 + 2^-6 for x2;
    # (1 + 2^-6)^2 = 1 + 2^-5 + 2^-12 -> 1 + 2^-5 for x1)
    g, c = chain(False)
    np.testing.assert_array_equal(_bits32(OG.run(g, {"x": x})[c]), [0x3F800000, 0x3F840000, 0x3F820000])
    # a cast to the type the value already has changes nothing, grouped or not
    g = W.GraphSpec("cast_same")
    xv = g.input("x", "f32", (1, 3))
    o0, (a,) = g.op("cast", [xv], [("f32", (1, 3))], to="f32")
    g.output(a)
    np.testing.assert_array_equal(_bits32(OG.run(g, {"x": x})[a]), x.view(np.uint32).ravel())
