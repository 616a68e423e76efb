"""Pins the oracle to the only numbers the paper prints for this path: the worked example of Appendix B."""
import os

import numpy as np
import pytest

from oracle import ref
from paper_2411_09909_amd import synth

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "appendix_b_example.txt")


def _golden():
    out = {}
    for line in open(GOLDEN):
        line = line.strip()
        if not line or line.startswith("#"):
            continue
        name, vals = line.split(":")
        out[name] = [float(v) for v in vals.split()]
    return out


def _example_row(as_bf16=True):
    x = np.linspace(-4.9, 31.0, 1024, dtype=np.float64).astype(np.float32)
    return synth.f32_to_bf16_bits(x).reshape(1, -1)


@pytest.mark.parametrize("name,scale,asym", [("mxfp4_pot_floor", ref.E8M0_FLOOR, 0),
                                             ("amxfp4_pot_floor", ref.E8M0_FLOOR, 1),
                                             ("amxfp4_fp8_e5m2", ref.FP8_E5M2, 1)])
def test_distinct_dequantized_values_match_paper(name, scale, asym):
    x = _example_row()
    codes, scales = ref.quantize(x, group_size=-1, scale=scale, asymmetric=asym)
    dq = ref.dequantize(codes, scales, group_size=-1, scale=scale, asymmetric=asym)
    assert sorted(np.unique(dq).tolist()) == _golden()[name]


def test_largest_value_31_becomes_24_pot_and_30_fp8():
    x = _example_row()
    for scale, want in [(ref.E8M0_FLOOR, 24.0), (ref.FP8_E5M2, 30.0)]:
        c, s = ref.quantize(x, -1, scale, 1)
        assert ref.dequantize(c, s, -1, scale, 1)[0, -1] == want


def test_scale_bytes_implied_by_the_example():
    # 15 distinct values on a 5x grid (positives) and a 0.875x grid (negatives) => S_p = 5 = 1.25 * 2^2,
    # S_n = 0.875 = 1.75 * 2^-1; E5M2 with bias 15: (17 << 2) | 1 = 0x45, (14 << 2) | 3 = 0x3B.
    x = _example_row()
    _, s = ref.quantize(x, -1, ref.FP8_E5M2, 1)
    assert s.ravel().tolist() == [0x45, 0x3B]
    # power-of-two: positives 2^2 (31 -> floor(log2) = 4, minus 2), negatives 2^0 (4.9 -> 2, minus 2)
    _, s = ref.quantize(x, -1, ref.E8M0_FLOOR, 1)
    assert s.ravel().tolist() == [127 + 2, 127 + 0]
    _, s = ref.quantize(x, -1, ref.E8M0_FLOOR, 0)
    assert s.ravel().tolist() == [127 + 2]
