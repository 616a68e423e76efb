"""Algebraic invariants and special cases that any correct implementation of the format must satisfy; each is chosen
so that a plausible slip (swapped scales, wrong sign class, off-by-one group index, wrong nibble) breaks it."""
import numpy as np
import pytest

from oracle import ref
from paper_2411_09909_amd import synth
from tests import helpers as H

FORMATS = [(ref.FP8_E5M2, 1), (ref.FP8_E5M2, 0), (ref.E8M0_FLOOR, 1), (ref.E8M0_FLOOR, 0)]


def _x(rows=16, K=256, seed=1):
    return synth.activations(rows, K, seed=seed, n_outlier=4, outlier_gain=60.0, shift=0.5)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_idempotent(scale, asym):
    """quantize(dequantize(q)) == q: amax / S lies in [5.4, 6.75] (E5M2) or [4, 8) (E8M0 floor), so the group maximum
    always maps to the code 6 and reproduces the same scale."""
    x = _x()
    c, s = ref.quantize(x, 32, scale, asym)
    dq = ref.dequantize(c, s, 32, scale, asym)
    xb = synth.f32_to_bf16_bits(dq.astype(np.float32))
    assert np.array_equal(synth.bf16_bits_to_f32(xb).astype(np.float64), dq)  # dequantized values are BF16-exact
    c2, s2 = ref.quantize(xb, 32, scale, asym)
    # -0 inputs that became +0 codes keep their sign bit in our convention, so compare through the magnitudes too
    assert np.array_equal(s2, s)
    assert np.array_equal(c2, c)


@pytest.mark.parametrize("scale", [ref.FP8_E5M2, ref.E8M0_FLOOR])
def test_negation_swaps_scales_and_flips_signs(scale):
    x = _x(seed=2)
    c, s = ref.quantize(x, 32, scale, 1)
    cn, sn = ref.quantize(x ^ np.uint16(0x8000), 32, scale, 1)
    assert np.array_equal(cn, c ^ np.uint8(0x88))
    assert np.array_equal(sn, s[..., ::-1])


@pytest.mark.parametrize("scale,asym", FORMATS)
@pytest.mark.parametrize("k", [-7, 3, 10])
def test_power_of_two_equivariance(scale, asym, k):
    x = _x(seed=3)
    xf = synth.bf16_bits_to_f32(x)
    x2 = synth.f32_to_bf16_bits(xf * np.float32(2.0 ** k))
    c, s = ref.quantize(x, 32, scale, asym)
    c2, s2 = ref.quantize(x2, 32, scale, asym)
    assert np.array_equal(c2, c)
    step = 4 if scale == ref.FP8_E5M2 else 1  # exponent field sits above 2 mantissa bits in E5M2
    nz = s != 0
    assert np.array_equal(s2[nz].astype(int), s[nz].astype(int) + k * step)
    assert np.all(s2[~nz] == 0)


@pytest.mark.parametrize("scale", [ref.FP8_E5M2, ref.E8M0_FLOOR])
def test_reduces_to_symmetric_format(scale):
    # all-positive rows: AMXFP4 == MXFP4 with the positive scale; the negative scale byte is 0
    xf = np.abs(synth.bf16_bits_to_f32(_x(seed=4)))
    x = synth.f32_to_bf16_bits(xf)
    ca, sa = ref.quantize(x, 32, scale, 1)
    cs, ss = ref.quantize(x, 32, scale, 0)
    assert np.array_equal(ca, cs) and np.array_equal(sa[..., 0], ss) and np.all(sa[..., 1] == 0)
    # all-negative: mirrored
    xn = x | np.uint16(0x8000)
    ca, sa = ref.quantize(xn, 32, scale, 1)
    assert np.array_equal(ca, cs | np.uint8(0x88)) and np.array_equal(sa[..., 1], ss) and np.all(sa[..., 0] == 0)
    # groups whose positive and negative maxima coincide: identical codes in both formats
    g = x[:, :32].copy()
    g[:, 1] = g[:, 0] | np.uint16(0x8000)
    big = synth.f32_to_bf16_bits(np.full((g.shape[0],), 1000.0, np.float32))
    g[:, 0] = big
    g[:, 1] = big | np.uint16(0x8000)
    g[:, 2::2] |= np.uint16(0x8000)
    ca, sa = ref.quantize(g, 32, scale, 1)
    cs, ss = ref.quantize(g, 32, scale, 0)
    assert np.array_equal(ca, cs) and np.array_equal(sa[..., 0], ss) and np.array_equal(sa[..., 1], ss)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_zero_group_and_signed_zero(scale, asym):
    x = np.zeros((2, 64), np.uint16)
    x[1, 5] = 0x8000  # -0.0
    c, s = ref.quantize(x, 32, scale, asym)
    assert np.all(s == 0)
    want = np.zeros((2, 32), np.uint8)
    want[1, 2] = 0x80  # element 5 = high nibble of byte 2: sign bit kept, magnitude 0
    assert np.array_equal(c, want)
    assert np.all(ref.dequantize(c, s, 32, scale, asym) == 0)


def test_outlier_group_hand_worked():
    """One hand-worked AMXFP4-E5M2 group: positives up to 96 (outlier), negatives down to -0.75.
    S_p = RNE_E5M2(16) = 16 (byte (19<<2)|0 = 0x4C); S_n = RNE_E5M2(0.125) = 0.125 (byte (12<<2) = 0x30).
    96 -> 6 (code 7); 20 -> 20/16 = 1.25 tie -> 1.0 (code 2); 7 -> 0.4375 -> 0.5 (code 1); 3 -> .1875 -> 0;
    -0.75 -> 6 (0xF); -0.5 -> 4 (0xE); -0.3125 -> 2.5 tie -> 2 (0xC); -0.0625 -> 0.5 (0x9)."""
    vals = [96.0, 20.0, 7.0, 3.0, -0.75, -0.5, -0.3125, -0.0625] + [0.0] * 24
    x = synth.f32_to_bf16_bits(np.array(vals, np.float32)).reshape(1, 32)
    c, s = ref.quantize(x, 32, ref.FP8_E5M2, 1)
    assert s.ravel().tolist() == [0x4C, 0x30]
    assert H.unpack_codes(c)[0, :8].tolist() == [7, 2, 1, 0, 0xF, 0xE, 0xC, 0x9]
    # the symmetric format shares S = 16 and wipes out every negative element
    c, s = ref.quantize(x, 32, ref.FP8_E5M2, 0)
    assert s.ravel().tolist() == [0x4C]
    assert H.unpack_codes(c)[0, :8].tolist() == [7, 2, 1, 0, 0x8, 0x8, 0x8, 0x8]


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_dequantize_matches_rational_decode(scale, asym):
    x = _x(rows=4, K=128, seed=5)
    c, s = ref.quantize(x, 32, scale, asym)
    dq = ref.dequantize(c, s, 32, scale, asym)
    want = H.dequant_fraction(c, s, scale, asym, 32)
    assert [[float(v) for v in row] for row in want] == dq.tolist()


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_quantize_matches_rational_bruteforce_on_small_input(scale, asym):
    """Whole quantizer against an independent exact re-derivation (group extrema, nearest scale, nearest element)."""
    from fractions import Fraction
    x = _x(rows=3, K=96, seed=6)
    x[0, 40:50] = 0
    c, s = ref.quantize(x, 32, scale, asym)
    nib = H.unpack_codes(c)
    sc = s.reshape(3, 3, 2 if asym else 1)
    for r in range(3):
        for g in range(3):
            xs = [H.bf16_fraction(int(b)) for b in x[r, 32 * g:32 * g + 32]]
            ap = max([v for v in xs if v > 0], default=Fraction(0))
            an = max([-v for v in xs if v < 0], default=Fraction(0))
            if not asym:
                ap = an = max(ap, an)
            for cls, amax in ((0, ap), (1, an)) if asym else ((0, ap),):
                if amax == 0:
                    want = 0
                elif scale == ref.FP8_E5M2:
                    want = H.nearest_scale_bruteforce(amax / 6, H.E5M2_FINITE)
                else:
                    e = -140
                    while Fraction(2) ** (e + 1) <= amax:
                        e += 1
                    want = e - 2 + 127
                assert sc[r, g, cls] == want
            for i, v in enumerate(xs):
                neg = int(x[r, 32 * g + i]) >> 15
                S = H.scale_fraction(scale, int(sc[r, g, neg if asym else 0]))
                amax = (an if neg else ap)
                mag = 0 if (amax == 0 or S == 0) else H.nearest_e2m1_bruteforce(min(abs(v) / S, Fraction(6)))
                assert nib[r, 32 * g + i] == (neg << 3 | mag)


def test_strided_axis_equals_transposed_input():
    x = _x(rows=64, K=48, seed=7)  # groups along axis 0 of a [64, 48] array == rows of its transpose
    c1, s1 = ref.quantize(x, 32, ref.FP8_E5M2, 1, k_axis=0)
    c2, s2 = ref.quantize(np.ascontiguousarray(x.T), 32, ref.FP8_E5M2, 1)
    assert np.array_equal(c1, c2) and np.array_equal(s1, s2)


def test_asymmetric_format_has_lower_error_on_shifted_data():
    """Non-binding sanity (Sec. 4.1, Sec. 4.2): on shifted, outlier-bearing activations the asymmetric format's MSE is
    below the symmetric one's, and the floored power-of-two scale is worse than the FP8 scale."""
    x, _ = synth.linear_operands("c1_linear_64x1024x1024")
    xf = synth.bf16_bits_to_f32(x).astype(np.float64)

    def mse(scale, asym):
        c, s = ref.quantize(x, 32, scale, asym)
        return float(np.mean((ref.dequantize(c, s, 32, scale, asym) - xf) ** 2))

    assert mse(ref.FP8_E5M2, 1) < mse(ref.FP8_E5M2, 0)
    assert mse(ref.FP8_E5M2, 0) < mse(ref.E8M0_FLOOR, 0)
    assert mse(ref.FP8_E5M2, 1) < mse(ref.E8M0_FLOOR, 1)
