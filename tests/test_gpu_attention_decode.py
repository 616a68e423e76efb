"""GPU parity of the fused attention for few queries against many keys (amxfp4_attention_decode: K and V read as packed
codes, the keys cut into ranges that are combined exactly) against the oracle's split-key definition
(oracle/attention_ref.py, key_splits). Compared as the other attention kernel is (tests/test_gpu_attention_fused.py):
the GPU evaluates exp in FP32, the oracle in float64."""
import numpy as np
import pytest
import torch

from oracle import attention_ref, ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G
from tests.test_gpu_attention_fused import compare, heads

pytestmark = pytest.mark.gpu


def gpu_decode(q, k, v, scale, causal, scale_format, asym, key_splits):
    fmt = binding.make_format(scale_format, asym, 32)
    Hq, Sq, D = q.shape
    Hkv, Sk, _ = k.shape
    qc, qs = binding.quantize(fmt, G.to_dev_bf16(q.reshape(Hq * Sq, D)))
    kc, ks = binding.quantize(fmt, G.to_dev_bf16(k.reshape(Hkv * Sk, D)))
    vc, vs = binding.quantize_batched(fmt, G.to_dev_bf16(v.reshape(Hkv * Sk, D)).view(Hkv, Sk, D), k_axis=1)
    ns = qs.shape[1:]
    out = binding.attention_decode(fmt, qc.view(Hq, Sq, -1), qs.view(Hq, Sq, *ns), kc.view(Hkv, Sk, -1),
                                   ks.view(Hkv, Sk, *ns), vc, vs, scale, causal, key_splits)
    torch.cuda.synchronize()
    return out.cpu().numpy()


FORMATS = [(ref.FP8_E5M2, 1), (ref.FP8_E5M2, 0), (ref.E8M0_FLOOR, 1), (ref.FP8_E4M3, 1), (ref.E8M0_ROUND, 0)]

# Hq, Hkv, Sq, Sk, causal, key_splits, D
SHAPES = [
    (4, 1, 1, 256, True, 4, 128),      # one new token, four query heads on one key/value head
    (8, 2, 4, 512, True, 8, 128),      # a chunk of four tokens: the causal limit differs between the columns
    (2, 2, 16, 128, False, 3, 128),    # 4 tiles in 3 ranges (2, 2, 0 tiles: the last range is empty)
    (3, 3, 32, 96, True, 1, 128),      # all 32 columns one head's queries, one range: the other kernel's definition
    (1, 1, 5, 64, True, 2, 128),       # a range no query but the last sees in full
    (6, 2, 2, 320, True, 10, 128),     # one tile per range
    (4, 2, 3, 256, True, 5, 64),       # heads of 64
    (8, 8, 1, 512, False, 4, 64),
    # V goes through LDS in chunks of 8 tiles when Sk is a multiple of 256: ranges that start inside a chunk and run
    # across chunk boundaries (32 tiles in 3 ranges of 11, 11, 10; 24 tiles in 2 ranges of 12)
    (4, 1, 2, 1024, True, 3, 128),
    (4, 2, 1, 768, False, 2, 64),
]


@pytest.mark.parametrize("scale_format,asym", FORMATS)
@pytest.mark.parametrize("Hq,Hkv,Sq,Sk,causal,splits,D", SHAPES)
def test_decode_matches_the_split_key_oracle(Hq, Hkv, Sq, Sk, causal, splits, D, scale_format, asym):
    q, k, v = heads(Hq, Sq, 41, d=D), heads(Hkv, Sk, 42, d=D), heads(Hkv, Sk, 43, d=D)
    want = attention_ref.fused_attention(q, k, v, D ** -0.5, causal, scale_format, asym, key_splits=splits)
    compare(gpu_decode(q, k, v, D ** -0.5, causal, scale_format, asym, splits), want)


def test_one_range_agrees_with_the_many_queries_kernel():
    """key_splits = 1 is the definition amxfp4_attention implements; the two kernels differ in summation order only."""
    Hq, Hkv, Sq, Sk, D = 8, 2, 8, 384, 128
    q, k, v = heads(Hq, Sq, 51), heads(Hkv, Sk, 52), heads(Hkv, Sk, 53)
    fmt = binding.make_format(ref.FP8_E5M2, 1, 32)
    qc, qs = binding.quantize(fmt, G.to_dev_bf16(q.reshape(Hq * Sq, D)))
    kc, ks = binding.quantize(fmt, G.to_dev_bf16(k.reshape(Hkv * Sk, D)))
    vc, vs = binding.quantize_batched(fmt, G.to_dev_bf16(v.reshape(Hkv * Sk, D)).view(Hkv, Sk, D), k_axis=1)
    args = (fmt, qc.view(Hq, Sq, -1), qs.view(Hq, Sq, 4, 2), kc.view(Hkv, Sk, -1), ks.view(Hkv, Sk, 4, 2), vc, vs,
            D ** -0.5, True)
    a = binding.attention(*args)
    b = binding.attention_decode(*args, key_splits=1)
    torch.cuda.synchronize()
    compare(b.cpu().numpy(), a.cpu().numpy())


def test_closed_form_and_large_scores():
    """Q = 0: every probability is 1 in every range, cast to 0.9375; out = 0.9375 * mean of V_hat over the visible keys
    whatever the number of ranges. And scores large enough that all but one key vanish."""
    Sk, D = 256, 128
    q = np.zeros((2, 1, D), np.uint16)
    k, v = heads(1, Sk, 61), heads(1, Sk, 62)
    out = gpu_decode(q, k, v, 0.1, True, ref.FP8_E5M2, 1, 8)
    vc, vs = ref.quantize(np.ascontiguousarray(v[0]), 32, ref.FP8_E5M2, 1, k_axis=0)
    want = 0.9375 * ref.dequantize(vc, vs, 32, ref.FP8_E5M2, 1).T.mean(axis=0)
    assert np.allclose(out[0, 0], want, rtol=2e-6, atol=1e-6) and np.array_equal(out[0], out[1])
    q, k = heads(2, 1, 63, gain=30.0), heads(1, Sk, 64, gain=30.0)
    want = attention_ref.fused_attention(q, k, v, D ** -0.5, True, key_splits=8)
    compare(gpu_decode(q, k, v, D ** -0.5, True, ref.FP8_E5M2, 1, 8), want)


@pytest.mark.parametrize("scale_format,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0)])
def test_decoding_shape_at_full_size(scale_format, asym):
    """One new token of the decoder layer's attention (32 query / 8 key-value heads of 128) against 8192 cached keys,
    32 ranges of 8 tiles: every output row against the oracle."""
    Hq, Hkv, Sk, D = 32, 8, 8192, 128
    q, _, _ = synth.attention_qkv(Hq, 1, D, seed=5)
    _, k, v = synth.attention_qkv(Hkv, Sk, D, seed=6)
    out = gpu_decode(q, k, v, D ** -0.5, True, scale_format, asym, 32)
    want = attention_ref.fused_attention(q, k, v, D ** -0.5, True, scale_format, asym, key_splits=32)
    compare(out, want)


def test_invalid_arguments():
    fmt = binding.make_format(ref.FP8_E5M2, 1, 32)
    z = lambda *s: torch.zeros(s, dtype=torch.uint8, device="cuda")  # noqa: E731
    ok = (z(4, 2, 64), z(4, 2, 4, 2), z(1, 64, 64), z(1, 64, 4, 2), z(1, 128, 32), z(1, 128, 2, 2), 0.1, True)
    binding.attention_decode(fmt, *ok, key_splits=2)
    with pytest.raises(binding.AmxError):   # more ranges than key tiles
        binding.attention_decode(fmt, *ok, key_splits=3)
    with pytest.raises(binding.AmxError):   # 4 query heads x 9 queries on one key/value head: more than 32 columns
        binding.attention_decode(fmt, z(4, 9, 64), z(4, 9, 4, 2), *ok[2:], key_splits=1)
    with pytest.raises(binding.AmxError):   # head dimension 32
        binding.attention_decode(fmt, z(1, 1, 16), z(1, 1, 1, 2), z(1, 32, 16), z(1, 32, 1, 2), z(1, 32, 16), z(1, 32, 1, 2),
                                 0.1, True, key_splits=1)
    torch.cuda.synchronize()
