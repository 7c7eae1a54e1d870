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
