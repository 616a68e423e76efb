"""Pins the oracle's double-scaling functions (Sec. 5.3: a tensor-wise FP32 scale under the group-wise FP8 scale, as
in NVFP4 and its asymmetric variant) against rational arithmetic written out here. The paper names the scheme without
giving its arithmetic, so the reading itself (S_t = amax / 2688, elements multiplied by 1 / S_t in single precision
before the group-wise cast) is this repository's; what is pinned is that the oracle computes that reading."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from paper_2411_09909_amd import synth
from tests import helpers as H

NVFP4 = (16, ref.FP8_E4M3, 0)
ANVFP4 = (16, ref.FP8_E4M3, 1)


def _x(rows, K, seed, gain=1.0):
    x = synth.activations(rows, K, seed=seed, n_outlier=2, outlier_gain=60.0, shift=0.5)
    return synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(x) * np.float32(gain))


def _frac_of_f32(v):
    return Fraction(float(np.float32(v)))


@pytest.mark.parametrize("gain", [1.0, 3.0e-7, 2.5e9])
def test_tensor_scale_is_amax_over_2688_in_single_precision(gain):
    x = _x(8, 64, seed=1, gain=gain)
    st, rt = ref.tensor_scale(x)
    amax = max(abs(H.bf16_fraction(int(b))) for b in x.ravel())
    want_st = H.f32_round_fraction(amax / 2688)
    assert _frac_of_f32(st) == want_st
    assert _frac_of_f32(rt) == H.f32_round_fraction(1 / want_st)
    # the largest element then lands within an ulp or two of 2688, the top of what scale * element can express
    assert abs(amax * _frac_of_f32(rt) - 2688) < Fraction(2688, 2 ** 21)


def test_tensor_scale_of_zero_and_tiny_tensors():
    z = np.zeros((2, 32), np.uint16)
    assert ref.tensor_scale(z) == (1.0, 1.0)
    z[1, 3] = 0x8001  # smallest negative subnormal: S_t clamps at 2^-96 and its reciprocal stays finite
    st, rt = ref.tensor_scale(z)
    assert st == np.float32(2.0 ** -96) and rt == np.float32(2.0 ** 96)


@pytest.mark.parametrize("gs,scale,asym", [NVFP4, ANVFP4, (32, ref.FP8_E5M2, 1), (32, ref.E8M0_ROUND, 1)])
@pytest.mark.parametrize("gain", [1.0, 7.0e-4, 900.0])
def test_scaled_quantize_matches_rational_bruteforce(gs, scale, asym, gain):
    rows, K = 2, 128
    x = _x(rows, K, seed=5, gain=gain)
    x[0, 16:32] = 0
    st, rt = ref.tensor_scale(x)
    c, s = ref.quantize(x, gs, scale, asym, tensor_rcp=rt)
    G = K // gs
    nib = H.unpack_codes(c)
    sc = s.reshape(rows, G, 2 if asym else 1)
    table = {ref.FP8_E5M2: H.E5M2_FINITE, ref.FP8_E4M3: H.E4M3_FINITE}.get(scale)
    R = _frac_of_f32(rt)
    for r in range(rows):
        for g in range(G):
            bits = [int(b) for b in x[r, gs * g:gs * (g + 1)]]
            ys = [H.f32_round_fraction(H.bf16_fraction(b) * R) for b in bits]   # one single-precision rounding
            ap = max([abs(v) for v, b in zip(ys, bits) if not b & 0x8000], default=Fraction(0))
            an = max([abs(v) for v, b in zip(ys, bits) if b & 0x8000], default=Fraction(0))
            if not asym:
                ap = an = max(ap, an)
            for cls, amax in ((0, ap), (1, an)) if asym else ((0, ap),):
                if amax == 0:
                    want = 0
                elif table is not None:
                    want = H.nearest_scale_bruteforce(amax / 6, table)
                else:
                    e = -160
                    while Fraction(2) ** (e + 1) <= amax:
                        e += 1
                    if amax * amax > 2 * Fraction(4) ** e:   # significand above sqrt(2): exponent rounds up
                        e += 1
                    want = e - 2 + 127
                assert sc[r, g, cls] == want
            for i, (v, b) in enumerate(zip(ys, bits)):
                neg = b >> 15
                S = H.scale_fraction(scale, int(sc[r, g, neg if asym else 0]))
                amax = an if neg else ap
                mag = 0 if (amax == 0 or S == 0) else H.nearest_e2m1_bruteforce(min(abs(v) / S, Fraction(6)))
                assert nib[r, gs * g + i] == (neg << 3 | mag)
    # with the tensor scale the group scales sit at the top of the E4M3 range: the largest is the maximum, 448
    if scale == ref.FP8_E4M3:
        assert s.max() >= 0x7D


@pytest.mark.parametrize("gs,scale,asym", [NVFP4, ANVFP4, (32, ref.FP8_E5M2, 1)])
@pytest.mark.parametrize("k", [-9, 4])
def test_power_of_two_tensor_factor_equals_casting_the_scaled_tensor(gs, scale, asym, k):
    """R_t = 2^k: x * R_t is exact, so the scaled cast must equal the plain cast of the tensor 2^k * x."""
    x = _x(4, 128, seed=6)
    x2 = synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(x) * np.float32(2.0 ** k))
    c, s = ref.quantize(x, gs, scale, asym, tensor_rcp=2.0 ** k)
    c2, s2 = ref.quantize(x2, gs, scale, asym)
    assert np.array_equal(c, c2) and np.array_equal(s, s2)


def test_without_the_tensor_scale_small_tensors_are_flushed_and_with_it_they_are_not():
    """Why the scheme exists: E4M3 group scales bottom out at 2^-9, so a tensor of magnitude 1e-4 casts to all zeros
    on its own and keeps its structure under the tensor scale."""
    x = _x(4, 64, seed=7, gain=1.0e-5)
    c0, s0 = ref.quantize(x, *NVFP4)
    assert not s0.any() and not (c0 & 0x77).any()
    st, rt = ref.tensor_scale(x)
    c, s = ref.quantize(x, *NVFP4, tensor_rcp=rt)
    dq = ref.dequantize(c, s, *NVFP4, tensor_scale=st)
    xf = synth.bf16_bits_to_f32(x).astype(np.float64)
    assert np.linalg.norm(dq - xf) / np.linalg.norm(xf) < 0.15


@pytest.mark.parametrize("gs,scale,asym", [NVFP4, ANVFP4])
def test_scaled_gemm_matches_rational_arithmetic(gs, scale, asym):
    M, N, K = 3, 2, 64
    a = _x(M, K, seed=8, gain=30.0)
    b = synth.weights(N, K, seed=9, std=0.02)
    sa, ra = ref.tensor_scale(a)
    sb, rb = ref.tensor_scale(b)
    ac, as_ = ref.quantize(a, gs, scale, asym, tensor_rcp=ra)
    bc, bs = ref.quantize(b, gs, scale, asym, tensor_rcp=rb)
    C = ref.gemm(ac, as_, bc, bs, gs, scale, asym, a_tensor_scale=sa, b_tensor_scale=sb)
    A = H.dequant_fraction(ac, as_, scale, asym, gs)
    B = H.dequant_fraction(bc, bs, scale, asym, gs)
    dq = ref.dequantize(ac, as_, gs, scale, asym, tensor_scale=sa)
    for i in range(M):
        assert [float(v * _frac_of_f32(sa)) for v in A[i]] == dq[i].tolist()
        for j in range(N):
            exact = sum((A[i][k] * B[j][k] for k in range(K)), Fraction(0)) * _frac_of_f32(sa) * _frac_of_f32(sb)
            # the oracle rounds the double product chain once more than the rational value: allow one float32 ulp
            assert abs(Fraction(float(C[i, j])) - exact) <= abs(exact) * Fraction(1, 2 ** 23)
    # and the product approximates the BF16 one
    ref_c = synth.bf16_bits_to_f32(a).astype(np.float64) @ synth.bf16_bits_to_f32(b).astype(np.float64).T
    assert np.linalg.norm(C - ref_c) / np.linalg.norm(ref_c) < 0.3
