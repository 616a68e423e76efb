"""Exhaustive brute-force pins of the oracle's two roundings (scale and element), in exact rational arithmetic."""
from fractions import Fraction

import numpy as np
import pytest

from oracle import ref
from tests import helpers as H


def test_algorithm1_hand_cases():
    # Appendix B, Algorithm 1 with emax_elem = 2: X = 2^(floor(log2 amax) - 2)
    for amax, X in [(1.0, 0.25), (5.96875, 1.0), (6.0, 1.0), (7.96875, 1.0), (8.0, 2.0), (0.75, 0.125), (31.0, 4.0)]:
        assert ref.scale_decode(ref.E8M0_FLOOR, ref.scale_encode(ref.E8M0_FLOOR, amax)) == X


def _all_nonneg_bf16():
    return [b for b in range(0, 0x7F80)]  # +0 .. largest finite


def test_e5m2_scale_every_bf16_amax_bruteforce():
    """RNE(amax / 6) onto the finite E5M2 values for EVERY finite non-negative BF16 amax, against a nearest-value
    search over the whole E5M2 table in rationals (includes the tie amax = 6.75, the subnormal range, saturation)."""
    table = H.E5M2_FINITE
    vals = [v for _, v in table]
    import bisect
    bad = []
    for b in _all_nonneg_bf16():
        q = H.bf16_fraction(b) / 6
        i = bisect.bisect_left(vals, q)
        cand = table[max(0, i - 2):i + 2]
        want = H.nearest_scale_bruteforce(q, cand)
        got = ref.scale_encode(ref.FP8_E5M2, float(H.bf16_fraction(b)))
        if got != want:
            bad.append((hex(b), got, want))
    assert not bad, bad[:10]


def test_e5m2_scale_full_table_search_on_a_sample():
    # same check, but searching the full table (no bisect shortcut), on every 37th pattern and the known hard ones
    hard = [0x40D8]  # 6.75 -> 1.125, a tie between 1.0 and 1.25 -> 1.0 (even mantissa)
    for b in list(range(0, 0x7F80, 37)) + hard:
        q = H.bf16_fraction(b) / 6
        assert ref.scale_encode(ref.FP8_E5M2, float(H.bf16_fraction(b))) == H.nearest_scale_bruteforce(q, H.E5M2_FINITE)
    assert ref.scale_encode(ref.FP8_E5M2, 6.75) == (15 << 2) | 0
    assert ref.scale_encode(ref.FP8_E5M2, 8.25) == (15 << 2) | 2  # 1.375: tie 1.25 / 1.5 -> 1.5 (even mantissa 2)
    assert ref.scale_encode(ref.FP8_E5M2, 3.0e38) == 0x7B            # saturates at 57344


def test_e4m3_scale_bruteforce_sample():
    for b in range(0, 0x7F80, 11):
        q = H.bf16_fraction(b) / 6
        assert ref.scale_encode(ref.FP8_E4M3, float(H.bf16_fraction(b))) == H.nearest_scale_bruteforce(q, H.E4M3_FINITE)


def test_e8m0_floor_every_bf16_amax():
    for b in range(1, 0x7F80):
        v = H.bf16_fraction(b)
        byte = ref.scale_encode(ref.E8M0_FLOOR, float(v))
        # largest power of two <= v, divided by 4, clamped to the E8M0 range
        e = -140
        while Fraction(2) ** (e + 1) <= v:
            e += 1
        assert byte == min(254, max(0, e - 2 + 127)), hex(b)
    assert ref.scale_encode(ref.E8M0_FLOOR, 0.0) == 0


@pytest.mark.parametrize("kind,scale_bytes", [
    (ref.FP8_E5M2, [0x01, 0x02, 0x03, 0x04, 0x3C, 0x3D, 0x3E, 0x3F, 0x45, 0x3B, 0x7B, 0x20, 0x21, 0x5A, 0x5B]),
    (ref.E8M0_FLOOR, [0, 1, 100, 127, 129, 200, 254]),
])
def test_element_code_every_bf16_bruteforce(kind, scale_bytes):
    """For a set of scales covering all four mantissas, subnormal scales and the range ends: EVERY finite non-negative
    BF16 magnitude -> code equals the nearest E2M1 value to min(|x|/S, 6) found by exhaustive search in rationals."""
    for sb in scale_bytes:
        S = H.scale_fraction(kind, sb)
        Sf = ref.scale_decode(kind, sb)
        assert Fraction(Sf) == S
        # restrict to magnitudes within 0 .. 8*S plus a sweep of everything else (all saturate or flush)
        bad = []
        for b in range(0, 0x7F80):
            x = H.bf16_fraction(b)
            if x > 8 * S and b % 64:
                continue
            if x < S / 8 and b % 64:
                continue
            want = H.nearest_e2m1_bruteforce(min(x / S, Fraction(6)))
            got = ref.elem_encode(float(x), Sf)
            if got != want:
                bad.append((hex(b), sb, got, want))
        assert not bad, bad[:10]


def test_all_seven_ties_for_each_scale_mantissa():
    # tie points t in {0.25, .75, 1.25, 1.75, 2.5, 3.5, 5}: t * S is exactly representable, must go to the even code
    want = {0.25: 0, 0.75: 2, 1.25: 2, 1.75: 4, 2.5: 4, 3.5: 6, 5.0: 6}
    for m in range(4):
        S = ref.scale_decode(ref.FP8_E5M2, (15 << 2) | m)
        for t, code in want.items():
            assert ref.elem_encode(t * S, S) == code
    # just above / just below each tie moves to the neighbouring codes
    S = 1.0
    for t, (lo, hi) in {0.25: (0, 1), 0.75: (1, 2), 1.25: (2, 3), 1.75: (3, 4), 2.5: (4, 5), 3.5: (5, 6),
                        5.0: (6, 7)}.items():
        assert ref.elem_encode(t * (1 - 2 ** -9), S) == lo
        assert ref.elem_encode(t * (1 + 2 ** -9), S) == hi


def test_zero_scale_gives_zero_code():
    assert ref.elem_encode(3.0, 0.0) == 0
