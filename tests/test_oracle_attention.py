"""Pins of the fused-attention oracle (oracle/attention_ref.py) against closed forms and invariants that do not use
its code: constant scores, one-hot rows, causality, independence of heads, agreement with exact attention within the
quantization error, and the single-precision group cast it relies on."""
import numpy as np
import pytest

from oracle import attention_ref, ref
from paper_2411_09909_amd import synth
from tests import helpers as H


def bits(a):
    return synth.f32_to_bf16_bits(np.asarray(a, np.float32))


def f64(b):
    return synth.bf16_bits_to_f32(b).astype(np.float64)


def test_f32_cast_reduces_to_the_bf16_cast_and_matches_brute_force():
    x = synth.activations(8, 128, seed=1, n_outlier=2, outlier_gain=30.0, shift=0.5)
    for scale, asym in [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0), (ref.FP8_E4M3, 1)]:
        c1, s1 = ref.quantize(x, 32, scale, asym)
        c2, s2 = ref.quantize_f32(synth.bf16_bits_to_f32(x), 32, scale, asym)
        assert np.array_equal(c1, c2) and np.array_equal(s1, s2)
    # values with 24 significant bits: one group against the rational definition
    from fractions import Fraction
    rng = np.random.default_rng(2)
    y = (rng.random((1, 32)).astype(np.float32) * np.float32(0.9) + np.float32(1e-3))
    y[0, 5] = 1.0
    c, s = ref.quantize_f32(y, 32, ref.FP8_E5M2, 1)
    amax = max(Fraction(float(v)) for v in y[0])
    assert s[0, 0, 0] == H.nearest_scale_bruteforce(amax / 6, H.E5M2_FINITE) and s[0, 0, 1] == 0
    S = H.scale_fraction(ref.FP8_E5M2, int(s[0, 0, 0]))
    want = [H.nearest_e2m1_bruteforce(min(Fraction(float(v)) / S, Fraction(6))) for v in y[0]]
    assert H.unpack_codes(c)[0].tolist() == want


@pytest.mark.parametrize("asym", [1, 0])
def test_zero_queries_give_the_quantized_mean_of_v(asym):
    """Q = 0: every score is 0, every probability exp(0) = 1. A group of ones has the E5M2 scale RNE(1/6) = 0.15625
    and 1 / 0.15625 = 6.4 saturates at the element 6, so p_hat = 0.9375 for every key, and
    out[i] = 0.9375 * sum_{j <= i} V_hat[j] / (i + 1). In the diagonal tile the masked keys are zeros of the same
    group and change nothing."""
    Sq = Sk = 96
    D = 32
    v = synth.activations(Sk, D, seed=3)[None]
    q = np.zeros((1, Sq, D), np.uint16)
    k = synth.activations(Sk, D, seed=4)[None]
    out = attention_ref.fused_attention(q, k, v, 0.125, True, ref.FP8_E5M2, asym)
    vc, vs = ref.quantize(np.ascontiguousarray(v[0]), 32, ref.FP8_E5M2, asym, k_axis=0)
    vh = ref.dequantize(vc, vs, 32, ref.FP8_E5M2, asym).T
    want = 0.9375 * np.cumsum(vh, axis=0) / np.arange(1, Sk + 1)[:, None]
    assert np.allclose(out[0], want.astype(np.float32), rtol=1e-6, atol=1e-30)


def test_one_dominant_key_selects_its_v_row():
    """Scores with one key far above the rest: p = 1 for it and exp(-huge) = 0 for the others. The running maximum
    changes when the dominant key arrives (tile 1), which wipes the earlier accumulation: out = 0.9375 * V_hat[j*]
    / (sum of p) with sum p = 1 up to e^-60 (so components where V_hat[j*] is 0 come out as ~1e-26, not 0)."""
    Sq, Sk, D = 32, 64, 32
    k = np.zeros((1, Sk, D), np.float32)
    k[0, :, 0] = 1.0
    k[0, 40, 0] = 64.0                      # E2M1 x E5M2 represent 1 and 64 exactly
    q = np.zeros((1, Sq, D), np.float32)
    q[0, :, 0] = 1.0
    v = synth.activations(Sk, D, seed=5)[None]
    out = attention_ref.fused_attention(bits(q), bits(k), v, 1.0, False)
    vc, vs = ref.quantize(np.ascontiguousarray(v[0]), 32, ref.FP8_E5M2, 1, k_axis=0)
    vh = ref.dequantize(vc, vs, 32, ref.FP8_E5M2, 1).T
    assert np.allclose(out[0], np.tile(0.9375 * vh[40], (Sq, 1)).astype(np.float32), rtol=1e-6, atol=1e-20)


def test_causality_heads_and_grouped_queries():
    Hq, Hkv, Sq, Sk, D = 4, 2, 64, 64, 32
    q = synth.activations(Hq * Sq, D, seed=6).reshape(Hq, Sq, D)
    k = synth.activations(Hkv * Sk, D, seed=7).reshape(Hkv, Sk, D)
    v = synth.activations(Hkv * Sk, D, seed=8).reshape(Hkv, Sk, D)
    base = attention_ref.fused_attention(q, k, v, D ** -0.5, True)
    # a query never sees later keys or values: change them, the earlier rows stay bit-identical
    k2, v2 = k.copy(), v.copy()
    k2[:, 40:] = synth.activations(Hkv * 24, D, seed=9).reshape(Hkv, 24, D)
    v2[:, 40:] ^= np.uint16(0x8000)
    out2 = attention_ref.fused_attention(q, k2, v2, D ** -0.5, True)
    # (V is quantized in groups of 32 keys: rows 32..39 share their V group with the changed rows, rows < 32 do not)
    assert np.array_equal(out2[:, :32], base[:, :32]) and not np.array_equal(out2[:, 40:], base[:, 40:])
    # heads are independent, and query heads 0, 1 read key/value head 0, heads 2, 3 read head 1
    k3 = k.copy()
    k3[1] = k[0]
    out3 = attention_ref.fused_attention(q, k3, v, D ** -0.5, True)
    assert np.array_equal(out3[:2], base[:2]) and not np.array_equal(out3[2:], base[2:])
    single = attention_ref.fused_attention(q[2:3], k[1:2], v[1:2], D ** -0.5, True)
    assert np.array_equal(single[0], base[2])


def test_longer_key_sequence_aligns_queries_to_its_end():
    """Sq < Sk (a chunk of new queries against a cache): query i may attend to keys <= i + Sk - Sq, so its row equals
    the row Sk - Sq + i of the square problem."""
    Sk, Sq, D = 96, 32, 32
    qa = synth.activations(Sk, D, seed=10)[None]
    k = synth.activations(Sk, D, seed=11)[None]
    v = synth.activations(Sk, D, seed=12)[None]
    full = attention_ref.fused_attention(qa, k, v, D ** -0.5, True)
    tail = attention_ref.fused_attention(qa[:, Sk - Sq:], k, v, D ** -0.5, True)
    assert np.array_equal(tail[0], full[0, Sk - Sq:])


@pytest.mark.parametrize("causal", [True, False])
def test_close_to_exact_attention_of_the_quantized_operands(causal):
    """The only difference to exact softmax attention over (Q_hat, K_hat, V_hat) is the 4-bit cast of the probability
    tiles: relative error of a few per cent, far from what a wrong recurrence (missing rescale, wrong normaliser)
    would give."""
    S, D = 128, 64
    q = synth.activations(S, D, seed=13)[None]
    k = synth.activations(S, D, seed=14)[None]
    v = synth.activations(S, D, seed=15)[None]
    out = attention_ref.fused_attention(q, k, v, D ** -0.5, causal)[0].astype(np.float64)
    dq = lambda b, ax: (ref.dequantize(*ref.quantize(np.ascontiguousarray(b), 32, ref.FP8_E5M2, 1, k_axis=ax), 32,
                                       ref.FP8_E5M2, 1))
    qh, kh, vh = dq(q[0], -1), dq(k[0], -1), dq(v[0], 0).T
    s = (qh @ kh.T) * np.float64(np.float32(D ** -0.5))
    if causal:
        s = np.where(np.arange(S)[None, :] <= np.arange(S)[:, None], s, -np.inf)
    p = np.exp(s - s.max(axis=1, keepdims=True))
    exact = (p / p.sum(axis=1, keepdims=True)) @ vh
    rel = np.linalg.norm(out - exact) / np.linalg.norm(exact)
    assert 1e-4 < rel < 0.12


# ---- split keys (the decoding shape) -----------------------------------------------------------------------------------

def _dequantized(b, ax):
    return ref.dequantize(*ref.quantize(np.ascontiguousarray(b), 32, ref.FP8_E5M2, 1, k_axis=ax), 32, ref.FP8_E5M2, 1)


@pytest.mark.parametrize("n", [2, 3, 5, 8, 64])
def test_split_keys_closed_forms(n):
    """Q = 0 makes every range's maximum 0 and every probability 1 (cast to 0.9375), so whatever the number of ranges
    the combination must give 0.9375 * mean of V_hat over the visible keys: checks the ranges' weights l_c and that
    ranges past the causal limit (and, for n = 64 > 8 tiles, empty ones) contribute nothing. And one dominant key:
    only the range that holds it survives the combination."""
    Sk, Sq, D = 256, 5, 32
    v = synth.activations(Sk, D, seed=3)[None]
    k = synth.activations(Sk, D, seed=4)[None]
    q = np.zeros((1, Sq, D), np.uint16)
    out = attention_ref.fused_attention(q, k, v, 0.125, True, key_splits=n)
    vh = _dequantized(v[0], 0).T
    want = 0.9375 * np.stack([vh[:Sk - Sq + i + 1].mean(axis=0) for i in range(Sq)])
    assert np.allclose(out[0], want.astype(np.float32), rtol=1e-6, atol=1e-30)
    # dominant key 77 (range depends on n): q = k[77] direction, scaled up
    kk = np.zeros((Sk, D), np.float32)
    kk[:, 0] = 1.0
    kk[77, 0] = 6.0
    qq = np.zeros((1, D), np.float32)
    qq[0, 0] = 4.0
    out = attention_ref.fused_attention(bits(qq)[None], bits(kk)[None], v, 4.0, False, key_splits=n)
    assert np.allclose(out[0, 0], 0.9375 * vh[77], rtol=1e-6, atol=1e-20)


@pytest.mark.parametrize("n,causal", [(2, False), (4, False), (3, True), (4, True)])
def test_split_keys_are_a_weighted_mean_of_the_ranges_own_attention(n, causal):
    """Each range's (l_c, m_c) is the exact softmax denominator of its keys, sum_j exp(s_j) = l_c exp(m_c), because l
    sums the un-quantized probabilities. So the split result must equal the single-range oracle (key_splits = 1) run on
    each key range alone, combined with weights W_c = sum over the range's visible keys of exp(s_j) computed here in
    float64 from the dequantized operands: pins the combination rule without using its code."""
    Sk, Sq, D = 256, 6, 64
    tiles_per_range = -(-(Sk // 32) // n)
    q = synth.activations(Sq, D, seed=21)[None]
    k = synth.activations(Sk, D, seed=22)[None]
    v = synth.activations(Sk, D, seed=23)[None]
    sc = D ** -0.5
    out = attention_ref.fused_attention(q, k, v, sc, causal, key_splits=n)[0].astype(np.float64)
    s = (_dequantized(q[0], -1) @ _dequantized(k[0], -1).T) * np.float64(np.float32(sc))
    num, den = np.zeros((Sq, D)), np.zeros(Sq)
    shift = s.max(axis=1)
    for r0 in range(0, Sk, tiles_per_range * 32):
        r1 = min(r0 + tiles_per_range * 32, Sk)
        for i in range(Sq):
            last = i + Sk - Sq if causal else Sk - 1
            hi = min(r1, last + 1)
            if hi <= r0:
                continue
            # this query against this range alone: non-causal call on the visible keys, padded to a whole tile with
            # keys the query cannot see in the causal call (the V group of the last tile must be the same group)
            if hi % 32 == 0 or not causal:
                part = attention_ref.fused_attention(q[:, i:i + 1], k[:, r0:hi], v[:, r0:hi], sc, False)[0, 0]
            else:
                top = -(-hi // 32) * 32
                # causal call whose single query sits at position hi - 1 of the range: Sq' = 1 aligned to the end of
                # top - r0 keys would see all of them, so align by passing top - hi extra queries in front
                qq = np.concatenate([q[:, i:i + 1]] + [q[:, i:i + 1]] * (top - hi), axis=1)
                part = attention_ref.fused_attention(qq, k[:, r0:top], v[:, r0:top], sc, True)[0, 0]
            w = np.exp(s[i, r0:hi] - shift[i]).sum()
            num[i] += w * part.astype(np.float64)
            den[i] += w
    assert np.allclose(out, num / den[:, None], rtol=2e-6, atol=1e-12)


def test_split_keys_stay_close_to_exact_attention_and_differ_from_one_range():
    S, Sq, D = 512, 4, 64
    q = synth.activations(Sq, D, seed=31)[None]
    k = synth.activations(S, D, seed=32)[None]
    v = synth.activations(S, D, seed=33)[None]
    one = attention_ref.fused_attention(q, k, v, D ** -0.5, True, key_splits=1)[0].astype(np.float64)
    four = attention_ref.fused_attention(q, k, v, D ** -0.5, True, key_splits=4)[0].astype(np.float64)
    s = (_dequantized(q[0], -1) @ _dequantized(k[0], -1).T) * np.float64(np.float32(D ** -0.5))
    s = np.where(np.arange(S)[None, :] <= np.arange(Sq)[:, None] + S - Sq, s, -np.inf)
    p = np.exp(s - s.max(axis=1, keepdims=True))
    exact = (p / p.sum(axis=1, keepdims=True)) @ _dequantized(v[0], 0).T
    for got in (one, four):
        assert 1e-4 < np.linalg.norm(got - exact) / np.linalg.norm(exact) < 0.12
    assert not np.array_equal(one, four)   # the ranges' probabilities are cast against their own maxima
