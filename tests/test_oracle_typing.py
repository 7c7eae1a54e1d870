"""The oracle's type checker against the paper's typing rules, one case per
rule (positive and negative) -- CPU only."""
import pytest

from oracle import graph as OG
from typing_corpus import CASES


@pytest.mark.parametrize("name,builder,expected", CASES, ids=[c[0] for c in CASES])
def test_oracle_checker(name, builder, expected):
    spec = builder()
    if expected is None:
        OG.check(spec)
    else:
        with pytest.raises(OG.IllTyped) as ei:
            OG.check(spec)
        assert ei.value.category == expected, str(ei.value)


def test_infer_examples():
    # Type-UnaryOp / Type-Noncomp-BinaryOp keep Tensor(b, s)
    assert OG.infer("sq", [("f32", (2, 3))], {}) == [("f32", (2, 3))]
    assert OG.infer("add", [("bf16", (2, 3)), ("bf16", (2, 3))], {}) == [("bf16", (2, 3))]
    # conv output size uses floor
    assert OG.infer("conv2d", [("f32", (1, 3, 224, 224)), ("f32", (64, 3, 7, 7))],
                    {"stride": (2, 2), "pad": (3, 3)}) == [("f32", (1, 64, 112, 112))]
    assert OG.infer("conv2d", [("f32", (1, 2, 8, 8)), ("f32", (4, 2, 3, 3))],
                    {"stride": (2, 2), "pad": (0, 0)}) == [("f32", (1, 4, 3, 3))]
    assert OG.infer("maxpool2d", [("f32", (1, 64, 112, 112))],
                    {"kernel": (3, 3), "stride": (2, 2), "pad": (1, 1)}) == [("f32", (1, 64, 56, 56))]
    assert OG.infer("dense", [("bf16", (64, 2048)), ("bf16", (4096, 2048))], {"out_dtype": "f32"}) == [("f32", (64, 4096))]


def test_types_along_the_papers_example():
    # tests/golden/lenet_example_types.txt: the types the example's calls must get, derived by hand
    import os
    import re
    import workloads as W
    path = os.path.join(os.path.dirname(os.path.abspath(__file__)), "golden", "lenet_example_types.txt")

    def ty(text):
        m = re.fullmatch(r"(f32|bf16)\[([0-9,]*)\]", text)
        return m.group(1), tuple(int(v) for v in m.group(2).split(",") if v)

    rows = [l for l in open(path) if l.strip() and not l.startswith("#")]
    assert len(rows) == 8
    for line in rows:
        kind, attrs, args, res = (f.strip() for f in line.split("|"))
        a = {}
        for item in attrs.split():
            k, v = item.split("=")
            a[k] = tuple(int(x) for x in v.split(","))
        assert OG.infer(kind, [ty(t) for t in args.split()], a) == [ty(res)], line
    # and the workload that stands for the example declares exactly these types, in this order
    g, _ = W.lenet(64, "f32")
    declared = [(op.kind, g.values[op.outputs[0]].type.shape) for op in g.ops if op.kind in ("conv2d", "maxpool2d", "flatten", "dense")]
    want = [(l.split("|")[0].strip(), ty(l.split("|")[3].strip())[1]) for l in rows if l.split("|")[0].strip() != "tanh"]
    assert declared == want
