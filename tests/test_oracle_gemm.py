"""Pins the oracle GEMM: brute force in rationals on tiny shapes, and cases whose result is an exact integer."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from paper_2411_09909_amd import synth
from tests import helpers as H


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.FP8_E5M2, 0), (ref.E8M0_FLOOR, 1), (ref.E8M0_FLOOR, 0)])
@pytest.mark.parametrize("M,N,K", [(3, 4, 32), (2, 3, 64), (4, 2, 96)])
def test_gemm_bruteforce_rational(scale, asym, M, N, K):
    a = synth.activations(M, K, seed=11, n_outlier=2, outlier_gain=60.0, shift=0.5)
    b = synth.weights(N, K, seed=12, std=0.02)
    ac, as_ = ref.quantize(a, 32, scale, asym)
    bc, bs = ref.quantize(b, 32, scale, asym)
    C = ref.gemm(ac, as_, bc, bs, 32, scale, asym)
    A = H.dequant_fraction(ac, as_, scale, asym, 32)
    B = H.dequant_fraction(bc, bs, scale, asym, 32)
    for i in range(M):
        for j in range(N):
            exact = sum((A[i][k] * B[j][k] for k in range(K)), Fraction(0))
            assert C[i, j] == np.float32(float(exact))  # float(Fraction) rounds correctly; then one rounding to f32
            # (double -> float double rounding cannot bite here: the exact sums have < 53 significant bits)


def test_sign_pair_selects_scale_pair():
    """Sec. 4.3: a product uses the scale of each factor's own sign. One group, hand-built codes and scales:
    A = [+6, -6, +1, -1, 0...], S_p = 2, S_n = 0.5; B = [+4, +4, -2, -2, 0...], S_p = 1, S_n = 8.
    dot = (6*2)(4*1) + (-6*.5)(4*1) + (1*2)(-2*8) + (-1*.5)(-2*8) = 48 - 12 - 32 + 8 = 12."""
    def pack(nibbles):
        n = np.array(nibbles + [0] * (32 - len(nibbles)), np.uint8)
        return (n[0::2] | (n[1::2] << 4)).reshape(1, 16)

    e5 = lambda v: ref.scale_encode(ref.FP8_E5M2, v * 6)
    ac, bc = pack([0x7, 0xF, 0x2, 0xA]), pack([0x6, 0x6, 0xC, 0xC])
    as_ = np.array([[[e5(2.0), e5(0.5)]]], np.uint8)
    bs = np.array([[[e5(1.0), e5(8.0)]]], np.uint8)
    assert ref.gemm(ac, as_, bc, bs, 32, ref.FP8_E5M2, 1)[0, 0] == 12.0
    # swapping the two scales of A changes the answer to (6*.5)(4) + (-6*2)(4) + (1*.5)(-16) + (-1*2)(-16) = -12
    assert ref.gemm(ac, as_[..., ::-1].copy(), bc, bs, 32, ref.FP8_E5M2, 1)[0, 0] == -12.0


def test_integer_exact_case_and_batch():
    """All scales 1 (E8M0 byte 127) and codes from {0, 1, 2, 3, 4, 6}: every product is an integer, the result is an
    exact small integer and equals an int64 matmul. Also checks batch indexing."""
    rng = np.random.default_rng(5)
    batch, M, N, K = 3, 5, 7, 128
    mags = np.array([0, 2, 4, 5, 6, 7])  # codes of 0, 1, 2, 3, 4, 6
    vals = np.array([0, 0, 1, 0, 2, 3, 4, 6])

    def operand(rows):
        mag = rng.choice(mags, size=(batch, rows, K))
        sgn = rng.integers(0, 2, size=(batch, rows, K))
        nib = (mag | (sgn << 3)).astype(np.uint8)
        codes = nib[..., 0::2] | (nib[..., 1::2] << 4)
        ints = np.where(sgn == 1, -vals[mag], vals[mag]).astype(np.int64)
        return codes, np.full((batch, rows, K // 32, 2), 127, np.uint8), ints

    ac, as_, ai = operand(M)
    bc, bs, bi = operand(N)
    C = ref.gemm(ac, as_, bc, bs, 32, ref.E8M0_FLOOR, 1)
    want = np.einsum("bik,bjk->bij", ai, bi)
    assert np.array_equal(C.astype(np.int64), want) and C.dtype == np.float32


def test_gemm_equals_numpy_matmul_of_dequantized_operands():
    a, w = synth.linear_operands("c1_linear_64x1024x1024", M=16, N=24)
    ac, as_ = ref.quantize(a)
    bc, bs = ref.quantize(w)
    C = ref.gemm(ac, as_, bc, bs)
    want = ref.dequantize(ac, as_) @ ref.dequantize(bc, bs).T
    assert np.allclose(C, want, rtol=1e-6, atol=0)
