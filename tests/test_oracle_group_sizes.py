"""Pins the oracle at the design-space points around the paper's choice (Sec. 5.3 and Table 5: group sizes 16 to 128;
Sec. 4.2: the FP8 scale with 4 exponent and 3 mantissa bits) against exact rational re-derivations written out here:
a wrong group index, a scale taken from a neighbouring group or a wrong E4M3 bias / subnormal rule fails them."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from paper_2411_09909_amd import synth
from tests import helpers as H

CASES = [(16, ref.FP8_E5M2, 1), (64, ref.FP8_E5M2, 1), (128, ref.FP8_E5M2, 0), (16, ref.FP8_E4M3, 1),
         (32, ref.FP8_E4M3, 0), (64, ref.FP8_E4M3, 1), (128, ref.E8M0_FLOOR, 1), (16, ref.E8M0_FLOOR, 0)]


def _x(rows, K, seed):
    return synth.activations(rows, K, seed=seed, n_outlier=4, outlier_gain=60.0, shift=0.5)


@pytest.mark.parametrize("gs,scale,asym", CASES)
def test_quantize_matches_rational_bruteforce(gs, scale, asym):
    rows, K = 2, 256
    x = _x(rows, K, seed=gs + scale)
    x[0, 40:60] = 0
    x[1, 128:] = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(x[1, 128:]) * np.float32(2.0 ** -9))  # tiny scales
    c, s = ref.quantize(x, gs, scale, asym)
    G = K // gs
    assert c.shape == (rows, K // 2) and s.shape == ((rows, G, 2) if asym else (rows, G))
    nib = H.unpack_codes(c)
    sc = s.reshape(rows, G, 2 if asym else 1)
    table = {ref.FP8_E5M2: H.E5M2_FINITE, ref.FP8_E4M3: H.E4M3_FINITE}.get(scale)
    for r in range(rows):
        for g in range(G):
            xs = [H.bf16_fraction(int(b)) for b in x[r, gs * g:gs * (g + 1)]]
            ap = max([v for v in xs if v > 0], default=Fraction(0))
            an = max([-v for v in xs if v < 0], default=Fraction(0))
            if not asym:
                ap = an = max(ap, an)
            for cls, amax in ((0, ap), (1, an)) if asym else ((0, ap),):
                if amax == 0:
                    want = 0
                elif table is not None:
                    want = H.nearest_scale_bruteforce(amax / 6, table)
                else:
                    e = -140
                    while Fraction(2) ** (e + 1) <= amax:
                        e += 1
                    want = e - 2 + 127
                assert sc[r, g, cls] == want
            for i, v in enumerate(xs):
                neg = int(x[r, gs * g + i]) >> 15
                S = H.scale_fraction(scale, int(sc[r, g, neg if asym else 0]))
                amax = an if neg else ap
                mag = 0 if (amax == 0 or S == 0) else H.nearest_e2m1_bruteforce(min(abs(v) / S, Fraction(6)))
                assert nib[r, gs * g + i] == (neg << 3 | mag)


@pytest.mark.parametrize("gs,scale,asym", CASES)
def test_dequantize_and_gemm_match_rational_arithmetic(gs, scale, asym):
    M, N, K = 3, 2, 256
    a = _x(M, K, seed=21)
    b = synth.weights(N, K, seed=22, std=0.02)
    ac, as_ = ref.quantize(a, gs, scale, asym)
    bc, bs = ref.quantize(b, gs, scale, asym)
    A = H.dequant_fraction(ac, as_, scale, asym, gs)
    B = H.dequant_fraction(bc, bs, scale, asym, gs)
    assert [[float(v) for v in row] for row in A] == ref.dequantize(ac, as_, gs, scale, asym).tolist()
    C = ref.gemm(ac, as_, bc, bs, gs, scale, asym)
    for i in range(M):
        for j in range(N):
            exact = sum((A[i][k] * B[j][k] for k in range(K)), Fraction(0))
            assert C[i, j] == np.float32(float(exact))


def test_e4m3_scale_saturates_and_keeps_subnormals():
    """amax / 6 above 448 stays at byte 0x7E (0x7F is not a number in the OCP format); below 2^-6 the grid is m * 2^-9;
    below 2^-10 the scale is 0 and the group is flushed."""
    assert ref.scale_encode(ref.FP8_E4M3, 6.0 * 448.0) == 0x7E
    assert ref.scale_encode(ref.FP8_E4M3, 1.0e30) == 0x7E
    assert ref.scale_encode(ref.FP8_E4M3, 6.0 * 5 * 2.0 ** -9) == 5
    assert ref.scale_encode(ref.FP8_E4M3, 6.0 * 2.0 ** -10) == 0      # tie between 0 and 2^-9: even byte
    assert ref.scale_encode(ref.FP8_E4M3, 6.0 * 1.5 * 2.0 ** -9) == 2  # tie between 1 and 2: even byte
    assert ref.scale_decode(ref.FP8_E4M3, 0x7E) == 448.0 and ref.scale_decode(ref.FP8_E4M3, 1) == 2.0 ** -9
    x = synth.f32_to_bf16_bits(np.full((1, 32), 1.0e-4, np.float32))
    c, s = ref.quantize(x, 32, ref.FP8_E4M3, 1)
    assert np.all(s == 0) and np.all(c == 0)


@pytest.mark.parametrize("gs", [16, 64, 128])
def test_groups_are_independent_rows(gs):
    """A [rows, K] operand with groups of gs quantizes like the [rows * K / gs, gs] operand with one group per row."""
    x = _x(4, 256, seed=30)
    c, s = ref.quantize(x, gs, ref.FP8_E5M2, 1)
    c1, s1 = ref.quantize(np.ascontiguousarray(x.reshape(-1, gs)), -1, ref.FP8_E5M2, 1)
    assert np.array_equal(c.reshape(-1, gs // 2), c1) and np.array_equal(s.reshape(-1, 1, 2), s1)
