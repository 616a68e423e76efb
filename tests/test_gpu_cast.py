"""GPU cast / dequantize parity: codes and scales bit-exact against the CPU oracle on the same seeded inputs."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

FORMATS = [(ref.FP8_E5M2, 1), (ref.FP8_E5M2, 0), (ref.E8M0_FLOOR, 1), (ref.E8M0_FLOOR, 0), (ref.E8M0_ROUND, 1),
           (ref.E8M0_ROUND, 0)]


def check(bits, scale, asym):
    gc, gs = G.gpu_quantize(bits, scale, asym)
    rc, rs = ref.quantize(bits, 32, scale, asym)
    bad_s = np.argwhere(gs != rs)
    assert bad_s.size == 0, "scale mismatch at %s: gpu %s oracle %s" % (bad_s[:5].tolist(), gs[gs != rs][:5], rs[gs != rs][:5])
    bad_c = np.argwhere(gc != rc)
    assert bad_c.size == 0, "code mismatch at %s: gpu %s oracle %s" % (bad_c[:5].tolist(), gc[gc != rc][:5], rc[gc != rc][:5])


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_config1_operands(scale, asym):
    x, w = synth.linear_operands("c1_linear_64x1024x1024")
    check(x, scale, asym)
    check(w, scale, asym)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0)])
def test_llm_shaped_operands(scale, asym):
    x, w = synth.linear_operands("c2_llama7b_qkvo_2048x4096x4096", M=512, N=256)
    check(x, scale, asym)
    check(w, scale, asym)
    g = synth.glu_activations(256, 2048 + 32, seed=3)  # ragged: K not a multiple of the 128-bit-load quad pattern size
    check(g, scale, asym)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_every_bf16_value_as_group_maximum(scale, asym):
    """Every finite BF16 magnitude as the largest element of a group, once per sign: exercises the scale rounding
    (ties, subnormal scales, saturation) and the element rounding relative to each of those scales."""
    rng = np.random.default_rng(1)
    mags = np.arange(0, 0x7F80, dtype=np.uint16)
    for sign in (0, 0x8000):
        x = np.zeros((mags.size, 32), np.uint16)
        xf = synth.bf16_bits_to_f32(mags)
        frac = rng.random((mags.size, 31), dtype=np.float32)
        body = synth.f32_to_bf16_bits(frac * xf[:, None])
        body = np.minimum(body, mags[:, None])  # rounding must not exceed the intended maximum
        sgn = (rng.integers(0, 2, size=body.shape) * 0x8000).astype(np.uint16)
        x[:, 1:] = body | sgn
        x[:, 0] = mags | np.uint16(sign)
        check(x, scale, asym)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_every_bf16_value_under_fixed_scales(scale, asym):
    """For group maxima that produce each scale mantissa (and power-of-two scales), sweep ALL BF16 patterns through the
    other 31 slots: every rounding boundary, both signs, subnormal inputs."""
    allbits = np.arange(0, 0x10000, dtype=np.uint32)
    finite = allbits[(allbits & 0x7F80) != 0x7F80].astype(np.uint16)
    for amax in (6.0, 7.5, 9.0, 10.5, 0.046875, 3.0e-5, 1.0e-6, 1536.0):  # scales 1, 1.25, 1.5, 1.75, tiny, subnormal
        ab = synth.f32_to_bf16_bits(np.array([amax], np.float32))[0]
        cand = finite[(finite & 0x7FFF) <= ab]
        n = (cand.size + 29) // 30
        pad = np.zeros(n * 30 - cand.size, np.uint16)
        x = np.zeros((n, 32), np.uint16)
        x[:, 2:] = np.concatenate([cand, pad]).reshape(n, 30)
        x[:, 0] = ab
        x[:, 1] = ab | 0x8000
        check(x, scale, asym)
        # one-sided variants: the other class's scale comes from the swept values themselves
        x[:, 1] = 0
        check(x, scale, asym)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_degenerate_groups(scale, asym):
    x = np.zeros((8, 64), np.uint16)
    x[1, :] = 0x8000                       # all -0
    x[2, :] = 0x3F80                       # all +1
    x[3, :] = 0xBF80                       # all -1
    x[4, :32] = 0x0001                     # smallest subnormal
    x[4, 32:] = 0x7F7F                     # largest finite
    x[5, ::2] = 0x7F7F
    x[5, 1::2] = 0xFF7F
    x[6, 0] = 0x4300                       # one outlier 128, rest tiny
    x[6, 1:] = 0x3000
    x[7, :] = synth.f32_to_bf16_bits(np.linspace(-4.9, 31, 64).astype(np.float32))
    check(x, scale, asym)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.FP8_E5M2, 0), (ref.E8M0_FLOOR, 1)])
def test_row_stride_and_strided_axis(scale, asym):
    rng = np.random.default_rng(7)
    base = synth.activations(96, 512, seed=9)
    # contiguous cast of a column slice (row_stride > K)
    fmt = binding.make_format(scale, asym)
    xd = G.to_dev_bf16(base)
    view = xd[:, 128:128 + 256]
    c, s = binding.quantize(fmt, view)
    rc, rs = ref.quantize(np.ascontiguousarray(base[:, 128:384]), 32, scale, asym)
    assert np.array_equal(c.cpu().numpy(), rc) and np.array_equal(s.cpu().numpy(), rs)
    # groups down the columns (V in softmax(P).V): operand = x.T
    v = synth.activations(256, 80, seed=10)  # [seq 256, d 80] -> operand [80, 256]
    gc, gs = G.gpu_quantize(v, scale, asym, k_axis=0)
    rc, rs = ref.quantize(v, 32, scale, asym, k_axis=0)
    assert np.array_equal(gc, rc) and np.array_equal(gs, rs)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0)])
def test_batched_cast_equals_the_oracle_per_operand(scale, asym):
    """Several operands in one launch (the heads of an attention layer): along the rows (Q, K), down the columns (V),
    and with a batch stride larger than an operand; every operand's codes and scales against the oracle."""
    fmt = binding.make_format(scale, asym)
    heads, seq, d = 5, 96, 128
    x = np.stack([synth.activations(seq, d, seed=20 + h) for h in range(heads)])      # [heads, seq, d]
    xd = torch.from_numpy(x.view(np.int16)).cuda().view(torch.bfloat16)
    c, s = binding.quantize_batched(fmt, xd)                                           # groups along d
    for h in range(heads):
        rc, rs = ref.quantize(x[h], 32, scale, asym)
        assert np.array_equal(c[h].cpu().numpy(), rc) and np.array_equal(s[h].cpu().numpy(), rs)
    c, s = binding.quantize_batched(fmt, xd, k_axis=1)                                 # groups down the 96 keys
    assert tuple(c.shape) == (heads, d, seq // 2)
    for h in range(heads):
        rc, rs = ref.quantize(x[h], 32, scale, asym, k_axis=0)
        assert np.array_equal(c[h].cpu().numpy(), rc) and np.array_equal(s[h].cpu().numpy(), rs)
    c, s = binding.quantize_batched(fmt, xd[::2])                                      # batch stride = two operands
    for i, h in enumerate(range(0, heads, 2)):
        rc, rs = ref.quantize(x[h], 32, scale, asym)
        assert np.array_equal(c[i].cpu().numpy(), rc) and np.array_equal(s[i].cpu().numpy(), rs)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_dequantize_exact(scale, asym):
    x = synth.activations(40, 288, seed=11)
    rc, rs = ref.quantize(x, 32, scale, asym)
    want = ref.dequantize(rc, rs, 32, scale, asym)
    fmt = binding.make_format(scale, asym)
    for dt in (torch.float32, torch.bfloat16):
        out = binding.dequantize(fmt, G.to_dev_u8(rc), G.to_dev_u8(rs), dt)
        torch.cuda.synchronize()
        assert np.array_equal(out.float().cpu().numpy().astype(np.float64), want)


def test_mxfp4_baseline_entry_points_force_symmetric():
    x = synth.activations(32, 256, seed=12)
    fmt = binding.make_format(ref.FP8_E5M2, True)  # asymmetric flag set, but the mxfp4_* calls ignore it
    c, s = binding.quantize(fmt, G.to_dev_bf16(x), baseline=True)
    rc, rs = ref.quantize(x, 32, ref.FP8_E5M2, 0)
    assert np.array_equal(c.cpu().numpy(), rc) and np.array_equal(s.cpu().numpy(), rs)
    out = binding.dequantize(fmt, c, s, baseline=True)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), ref.dequantize(rc, rs, 32, ref.FP8_E5M2, 0))
