"""The cast kernel's arithmetic for BF16 inputs, modelled step by step in NumPy float32 and checked against the
oracle on every input: the GPU kernel does not divide exactly, it multiplies by reciprocals and snaps, and the claim
is that this decides every scale byte and every E2M1 code as exact arithmetic does (Appendix B Algorithm 1 with the
FP8 scale of Sec. 4.2). The model below follows csrc/cast_math.h (fp8_scale_bf16) and csrc/cast_core.h (encode8_bf16):

  scale:    q0 = fl32(amax * fl32(1/6)); snap q0 to 13 significant bits (integer add 0x400, mask); clamp to the
            largest finite scale; round to the FP8 grid (nearest, ties to even, subnormals kept);
  element:  z = fl32(x * R), R = fl32(1 / S) give or take one ulp (the hardware reciprocal is accurate to one ulp);
            round z to binary16, then to E2M1 (nearest, ties to even, saturating).

The two roundings to FP8 and to E2M1 are the hardware conversions; the GPU parity tests check those on the machine.
Here they are exact by construction, so what is tested is the part the kernel adds: that the approximate quotients
never land on the wrong side of a rounding boundary, nor off a boundary the exact quotient is on.
"""
import numpy as np
import pytest

from oracle import ref
from paper_2411_09909_amd import synth

FP8 = {ref.FP8_E5M2: dict(mbits=2, emin=-14, maxv=57344.0, bias=15),
       ref.FP8_E4M3: dict(mbits=3, emin=-6, maxv=448.0, bias=7)}


def fp8_round(q, mbits, emin, maxv, **_):
    """q (float64, >= 0, already <= maxv) to the nearest FP8 value, ties to even, subnormals kept."""
    e = np.floor(np.log2(np.where(q > 0, q, 1.0)))
    e = np.maximum(e, emin)
    ulp = np.exp2(e - mbits)
    return np.minimum(np.rint(q / ulp) * ulp, maxv)  # np.rint rounds halves to even; q / ulp is exact


def fp8_byte(r, mbits, emin, bias, **_):
    e = np.floor(np.log2(np.where(r > 0, r, 1.0)))
    normal = r >= 2.0 ** emin
    mant = np.where(normal, r / np.exp2(e) - 1.0, r / 2.0 ** emin) * (1 << mbits)
    return np.where(normal, ((e + bias).astype(np.int64) << mbits) | mant.astype(np.int64), mant.astype(np.int64))


def model_scale(amax_f32, kind):
    p = FP8[kind]
    q0 = (amax_f32.astype(np.float32) * np.float32(1.0 / 6.0)).astype(np.float32)
    qb = (q0.view(np.uint32) + np.uint32(0x400)) & np.uint32(0xFFFFF800)
    q = np.minimum(qb.view(np.float32).astype(np.float64), p["maxv"])
    return fp8_round(q, **p)


E2M1 = np.array([0, 0.5, 1, 1.5, 2, 3, 4, 6])


def e2m1_round(z):
    """|z| (float64) to the index of the nearest E2M1 magnitude, ties to the even mantissa, saturating."""
    bounds = np.array([0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0])
    up_on_tie = np.array([False, True, False, True, False, True, False])  # the even neighbour is the upper one
    idx = np.zeros(z.shape, np.int64)
    for b, up in zip(bounds, up_on_tie):
        idx += (z > b) | ((z == b) & up)
    return idx


def model_codes(x_f32, S):
    """Codes (sign << 3 | magnitude index) of the BF16 numbers x under the scale S, for R = 1/S and its two
    neighbours: all three must agree."""
    if S == 0:  # the kernel sets R = 0 for a zero scale: every quotient is a zero with the element's sign
        return np.signbit(x_f32).astype(np.int64) << 3
    out = []
    R0 = (np.float32(1.0) / np.float32(S)).astype(np.float32)
    for R in (np.nextafter(R0, np.float32(0)), R0, np.nextafter(R0, np.float32(np.inf))):
        with np.errstate(over="ignore"):
            z = (x_f32 * np.float32(R)).astype(np.float32).astype(np.float16)
        mag = e2m1_round(np.minimum(np.abs(z.astype(np.float64)), 1e30))
        out.append(mag | (np.signbit(x_f32).astype(np.int64) << 3))
    assert np.array_equal(out[0], out[1]) and np.array_equal(out[1], out[2]), "the decision depends on the last bit of 1/S"
    return out[1]


@pytest.mark.parametrize("kind", [ref.FP8_E5M2, ref.FP8_E4M3])
def test_scale_model_equals_the_oracle_for_every_bf16_maximum(kind):
    bits = np.arange(0, 0x7F80, dtype=np.uint16)              # every finite non-negative BF16 number
    amax = synth.bf16_bits_to_f32(bits)
    groups = np.zeros((bits.size, 32), np.uint16)
    groups[:, 0] = bits                                        # the group's only non-zero element
    _, scales = ref.quantize(groups, 32, kind, False)
    got = fp8_byte(model_scale(amax, kind), **FP8[kind])
    bad = np.flatnonzero(got != scales[:, 0])
    assert bad.size == 0, "amax %s: model %s oracle %s" % (amax[bad[:5]], got[bad[:5]], scales[bad[:5], 0])


@pytest.mark.parametrize("kind", [ref.FP8_E5M2, ref.FP8_E4M3])
def test_element_model_equals_exact_division_for_every_bf16_value_and_scale(kind):
    """Every finite BF16 x against every positive scale value of the format: the model's code equals the code of the
    exact quotient (float64 division decides exactly here: a quotient that is not on an E2M1 boundary is at least
    2^-9 of it away, and one that is, is computed exactly)."""
    bits = np.concatenate([np.arange(0, 0x7F80, dtype=np.uint16), np.arange(0x8000, 0xFF80, dtype=np.uint16)])
    x = synth.bf16_bits_to_f32(bits)
    for byte in range(1, 0x7C if kind == ref.FP8_E5M2 else 0x7F):
        S = ref.scale_decode(kind, byte)
        exact = e2m1_round(np.abs(x.astype(np.float64)) / S) | (np.signbit(x).astype(np.int64) << 3)
        got = model_codes(x, S)
        bad = np.flatnonzero(got != exact)
        assert bad.size == 0, "scale byte %d, x %s: model %s exact %s" % (byte, x[bad[:5]], got[bad[:5]], exact[bad[:5]])


@pytest.mark.parametrize("kind", [ref.FP8_E5M2, ref.FP8_E4M3])
def test_element_model_equals_the_oracle_on_whole_groups(kind):
    """The same through the oracle's own cast: groups whose first element fixes the scale (one per scale mantissa and
    a few exponents), the other 31 sweeping every BF16 value below it."""
    for top in (0x3F80, 0x3FA0, 0x3FC0, 0x3FE0, 0x3F90, 0x3FB0, 0x4420, 0x2B40):
        below = np.arange(0, top, dtype=np.uint16)
        below = np.concatenate([below, below | 0x8000])
        pad = (-below.size) % 31
        body = np.concatenate([below, np.zeros(pad, np.uint16)]).reshape(-1, 31)
        groups = np.concatenate([np.full((body.shape[0], 1), top, np.uint16), body], axis=1)
        codes, scales = ref.quantize(groups, 32, kind, False)
        nib = np.stack([codes & 15, codes >> 4], axis=-1).reshape(groups.shape[0], 32)
        S = ref.scale_decode(kind, int(scales[0, 0]))
        assert (scales[:, 0] == scales[0, 0]).all()
        got = model_codes(synth.bf16_bits_to_f32(groups.reshape(-1)), S).reshape(groups.shape)
        assert np.array_equal(got, nib), "group maximum 0x%04x" % top
