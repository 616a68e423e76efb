"""The GEMM kernels feed the matrix cores dequantized operands elem * S (Eq. 1) in a 16-bit float type and rely on
that value being exact there. Checked on every element code and every scale byte, in exact rational arithmetic:
  BF16 (8 significant bits):  elem * S for FP8-E5M2 and FP8-E4M3 scales (gemm_bf16.hip, gemm_skinny.hip);
  FP16 biased by 2^-3:        (elem / 8) * S for FP8-E5M2 scales, subnormal results included, and formed by one FP16
                              multiplication of the two exact factors (gemm_e5m2.hip, gemm_skinny.hip).
"""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref

ELEMS = [Fraction(v).limit_denominator(2) for v in (0, 0.5, 1, 1.5, 2, 3, 4, 6)]


def significant_bits(q):
    """Bits between the highest and the lowest set bit of the positive rational q (a dyadic number)."""
    n, d = q.numerator, q.denominator
    assert d & (d - 1) == 0
    return n.bit_length() - ((n & -n).bit_length() - 1)


@pytest.mark.parametrize("kind,last", [(ref.FP8_E5M2, 0x7B), (ref.FP8_E4M3, 0x7E)])
def test_products_fit_bf16(kind, last):
    for byte in range(1, last + 1):
        S = Fraction(ref.scale_decode(kind, byte))
        for e in ELEMS[1:]:
            p = e * S
            assert significant_bits(p) <= 8
            assert Fraction(2) ** -126 <= p < Fraction(2) ** 128  # a normal BF16 number


def test_biased_products_are_exact_fp16_products():
    for byte in range(1, 0x7C):
        S = ref.scale_decode(ref.FP8_E5M2, byte)
        assert float(np.float16(S)) == S                         # the scale is an FP16 number (its upper byte)
        for e in ELEMS[1:]:
            exact = e / 8 * Fraction(S)
            assert exact >= Fraction(2) ** -24 and exact <= 65504
            got = np.float16(float(e / 8)) * np.float16(S)       # one FP16 multiplication, as v_pk_mul_f16 does
            assert Fraction(float(got)) == exact, (byte, e)
