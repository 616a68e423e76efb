"""Independent exact-arithmetic helpers for pinning the oracle. Nothing here is imported from oracle/ or from the GPU
library: decoders and nearest-value searches are written out again from the format definitions (Sec. 2.1, Sec. 4.2),
in integer / rational arithmetic, so that a mistake in the oracle's floating-point formulas shows up as a mismatch."""
from fractions import Fraction

import numpy as np

E2M1_GRID = [Fraction(0), Fraction(1, 2), Fraction(1), Fraction(3, 2), Fraction(2), Fraction(3), Fraction(4),
             Fraction(6)]


def bf16_fraction(bits):
    """Exact value of a BF16 bit pattern (finite)."""
    s = -1 if bits & 0x8000 else 1
    e = (bits >> 7) & 0xFF
    m = bits & 0x7F
    if e == 0:
        return s * Fraction(m, 128) * Fraction(2) ** -126
    return s * (1 + Fraction(m, 128)) * Fraction(2) ** (e - 127)


def e5m2_fraction(byte):
    e, m = (byte >> 2) & 31, byte & 3
    if e == 0:
        return Fraction(m, 4) * Fraction(2) ** -14
    return (1 + Fraction(m, 4)) * Fraction(2) ** (e - 15)


def e4m3_fraction(byte):
    e, m = (byte >> 3) & 15, byte & 7
    if e == 0:
        return Fraction(m, 8) * Fraction(2) ** -6
    return (1 + Fraction(m, 8)) * Fraction(2) ** (e - 7)


def e8m0_fraction(byte):
    return Fraction(2) ** (byte - 127)


def scale_fraction(kind, byte):
    return {0: e8m0_fraction, 1: e8m0_fraction, 2: e5m2_fraction, 3: e4m3_fraction}[kind](byte)


# finite, non-negative E5M2 bytes: exponent field 0..30 (31 = inf/nan)
E5M2_FINITE = [(b, e5m2_fraction(b)) for b in range(0, 0x7C)]
# finite E4M3 (OCP): all bytes 0..0x7E (0x7F = NaN), max 448
E4M3_FINITE = [(b, e4m3_fraction(b)) for b in range(0, 0x7F)]


def nearest_scale_bruteforce(q, table):
    """Byte of the table value nearest to the rational q; ties to the even byte (= even mantissa); q above the
    largest value saturates."""
    best = None
    for b, v in table:
        d = abs(q - v)
        if best is None or d < best[0] or (d == best[0] and b % 2 == 0 and best[1] % 2 == 1):
            best = (d, b)
    return best[1]


def nearest_e2m1_bruteforce(q):
    """3-bit code of the E2M1 magnitude nearest to the non-negative rational q (values above 6 clamp to 6);
    ties to the even code."""
    best = None
    for c, v in enumerate(E2M1_GRID):
        d = abs(q - v)
        if best is None or d < best[0] or (d == best[0] and c % 2 == 0 and best[1] % 2 == 1):
            best = (d, c)
    return best[1]


def unpack_codes(codes):
    """[rows, K/2] bytes -> [rows, K] nibbles (element 2b in the low nibble of byte b)."""
    codes = np.asarray(codes, np.uint8)
    out = np.empty(codes.shape[:-1] + (codes.shape[-1] * 2,), np.uint8)
    out[..., 0::2] = codes & 15
    out[..., 1::2] = codes >> 4
    return out


def dequant_fraction(codes, scales, kind, asymmetric, group_size):
    """Exact dequantized values (list of lists of Fractions), Eq. 1."""
    nib = unpack_codes(codes)
    rows, K = nib.shape
    gs = K if group_size == -1 else group_size
    sc = np.asarray(scales, np.uint8).reshape(rows, K // gs, 2 if asymmetric else 1)
    out = []
    for r in range(rows):
        row = []
        for k in range(K):
            n = int(nib[r, k])
            neg = n >> 3
            S = scale_fraction(kind, int(sc[r, k // gs, neg if asymmetric else 0]))
            v = E2M1_GRID[n & 7] * S
            row.append(-v if neg else v)
        out.append(row)
    return out


def f32_round_fraction(q):
    """The IEEE single-precision number nearest to the rational q (ties to even), as a Fraction; subnormals kept,
    no overflow handling (callers stay in range)."""
    if q == 0:
        return Fraction(0)
    s, a = (-1 if q < 0 else 1), abs(q)
    e = 0
    while Fraction(2) ** (e + 1) <= a:
        e += 1
    while Fraction(2) ** e > a:
        e -= 1
    e = max(e, -126)
    quantum = Fraction(2) ** (e - 23)
    n = a / quantum
    lo = n.numerator // n.denominator
    rem = n - lo
    if rem > Fraction(1, 2) or (rem == Fraction(1, 2) and lo % 2 == 1):
        lo += 1
    return s * lo * quantum
