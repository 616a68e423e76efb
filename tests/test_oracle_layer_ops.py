"""Pins for the decoder-layer glue operators of the oracle (oracle/layer_ref.py): each is checked against something
other than itself — a library routine evaluated in float64 (torch's rms_norm, softmax, silu), a different closed form
(complex multiplication for the rotary embedding), exact special cases and invariants."""
from fractions import Fraction

import numpy as np
import torch

from oracle import layer_ref as L


def bits_of(f32):
    return (np.asarray(f32, np.float32).view(np.uint32) >> 16).astype(np.uint16)


def test_bf16_rounding_is_nearest_even_in_one_step():
    # exact ties between two BF16 neighbours go to the even one; just off a tie goes to the nearer one
    one, ulp = 1.0, 2.0 ** -7
    cases = {one + ulp / 2: one, one + 3 * ulp / 2: one + 2 * ulp, one + ulp / 2 + 2.0 ** -40: one + ulp,
             one + 3 * ulp / 2 - 2.0 ** -40: one + ulp, -(one + ulp / 2): -one, 0.0: 0.0,
             2.0 ** -133: 2.0 ** -133, 2.0 ** -134: 0.0, 3 * 2.0 ** -134: 2.0 ** -132,  # subnormal quantum 2^-133
             255.5: 256.0, 254.5: 254.0, 1.99999999: 2.0}
    for x, want in cases.items():
        got = L.f64_from_bf16(L.bf16_from_f64(np.array([x])))[0]
        assert got == want, (x, got, want)
    # brute force on random doubles: the result is the BF16 value nearest to x (rational arithmetic)
    rng = np.random.default_rng(0)
    xs = rng.standard_normal(300) * np.exp(rng.uniform(-30, 30, 300))
    for x in xs:
        got = Fraction(float(L.f64_from_bf16(L.bf16_from_f64(np.array([x])))[0]))
        b = int(bits_of(np.array([x], np.float32))[0])  # truncation of the float32 neighbour: a BF16 value close to x
        near = [Fraction(float(L.f64_from_bf16(np.array([c], np.uint16))[0])) for c in range(b - 2, b + 3)
                if (c & 0x7F80) != 0x7F80]
        best = min(abs(Fraction(float(x)) - c) for c in near)
        assert abs(Fraction(float(x)) - got) == best


def test_rmsnorm_against_torch_float64():
    rng = np.random.default_rng(1)
    x = bits_of(rng.standard_normal((37, 512)) * 3)
    w = (1 + 0.1 * rng.standard_normal(512)).astype(np.float32)
    eps = 1e-5
    mine = L.rmsnorm(x, w, eps, exact=True)
    xt = torch.from_numpy(L.f64_from_bf16(x))
    want = torch.nn.functional.rms_norm(xt, (512,), torch.from_numpy(w.astype(np.float64)),
                                        eps=float(np.float32(eps))).numpy()
    assert np.allclose(mine, want, rtol=1e-13, atol=0)
    # unit gain: every output row has mean square 1 / (1 + eps / ms)
    y = L.rmsnorm(x, np.ones(512, np.float32), eps, exact=True)
    ms = np.mean(L.f64_from_bf16(x) ** 2, axis=1)
    assert np.allclose(np.mean(y * y, axis=1), ms / (ms + float(np.float32(eps))), rtol=1e-12)


def test_rotary_against_complex_multiplication_and_invariants():
    rng = np.random.default_rng(2)
    seq, heads, d, theta = 50, 3, 128, 500000.0
    proj = rng.standard_normal((seq, 7 + heads * d)).astype(np.float32)
    out = L.split_heads_rope(proj, 7, heads, d, True, pos0=11, theta=theta, exact=True)  # [h, s, d]
    x = proj[:, 7:].astype(np.float64).reshape(seq, heads, d)
    for h in range(heads):
        for s in (0, 1, 17, 49):
            z = x[s, h, :64] + 1j * x[s, h, 64:]
            rot = z * np.exp(1j * (11 + s) * theta ** (-np.arange(64) / 64.0))
            assert np.allclose(out[h, s, :64], rot.real, rtol=1e-12, atol=1e-12)
            assert np.allclose(out[h, s, 64:], rot.imag, rtol=1e-12, atol=1e-12)
    # position 0 is the identity; without rotation it is a pure re-layout
    ident = L.split_heads_rope(proj[:1], 7, heads, d, True, pos0=0, theta=theta, exact=True)
    assert np.array_equal(ident[:, 0, :], x[0])
    plain = L.split_heads_rope(proj, 7, heads, d, False, exact=True)
    assert np.array_equal(plain, x.transpose(1, 0, 2))
    # the inner product of a rotated query and key depends only on the distance of their positions
    q = rng.standard_normal((1, d)).astype(np.float32)
    k = rng.standard_normal((1, d)).astype(np.float32)
    dots = []
    for p in (0, 5, 1000):
        rq = L.split_heads_rope(q, 0, 1, d, True, pos0=p + 3, theta=theta, exact=True)[0, 0]
        rk = L.split_heads_rope(k, 0, 1, d, True, pos0=p, theta=theta, exact=True)[0, 0]
        dots.append(rq @ rk)
    assert np.allclose(dots, dots[0], rtol=1e-9)


def test_causal_softmax_against_torch_and_invariants():
    rng = np.random.default_rng(3)
    batch, per, seq = 2, 3, 40
    s = (rng.standard_normal((batch, per * seq, seq)) * 4).astype(np.float32)
    scale = 0.125
    p = L.softmax_causal(s, scale, exact=True)
    st = torch.from_numpy(s.astype(np.float64)) * scale
    pos = torch.arange(per * seq) % seq
    mask = torch.arange(seq)[None, :] <= pos[:, None]
    want = torch.softmax(st.masked_fill(~mask, float("-inf")), dim=-1).numpy()
    assert np.allclose(p, want, rtol=1e-13, atol=0)
    assert np.allclose(p.sum(-1), 1.0, rtol=1e-13)
    assert np.all(p[:, :, :][~np.broadcast_to(mask.numpy(), p.shape)] == 0.0)
    assert np.all(p[:, 0, 0] == 1.0) and np.all(p[:, seq, 0] == 1.0)  # position 0 of each stacked head sees one key
    bits = L.softmax_causal(s, scale)
    assert np.all(bits[~np.broadcast_to(mask.numpy(), p.shape)] == 0)


def test_silu_mul_residual_and_merge():
    rng = np.random.default_rng(4)
    gu = (rng.standard_normal((9, 64)) * 3).astype(np.float32)
    mine = L.silu_mul(gu, exact=True)
    g, u = torch.from_numpy(gu[:, :32].astype(np.float64)), torch.from_numpy(gu[:, 32:].astype(np.float64))
    assert np.allclose(mine, (torch.nn.functional.silu(g) * u).numpy(), rtol=1e-13, atol=1e-300)
    # residual: BF16 + float32 rounded once
    x = bits_of(np.array([1.0, 1.0, -2.0, 100.0], np.float32))
    y = np.array([2.0 ** -8, 3 * 2.0 ** -8, 0.5, 0.25], np.float32)
    assert np.array_equal(L.f64_from_bf16(L.residual_add(x, y)), [1.0, 1.0 + 2.0 ** -6, -1.5, 100.0])
    # merge_heads undoes the head split (values that BF16 holds exactly)
    seq, groups, per, d = 6, 2, 3, 8
    tok = rng.integers(-100, 100, (seq, groups * per * d)).astype(np.float32)
    heads = L.split_heads_rope(tok, 0, groups * per, d, False, exact=True)          # [h, s, d]
    stacked = heads.reshape(groups, per * seq, d).astype(np.float32)                # per heads of a group along rows
    assert np.array_equal(L.f64_from_bf16(L.merge_heads(stacked, groups, per, seq, d)), tok)
