"""GPU parity for the design-space points around the paper's choice (Sec. 5.3 and Table 5: group sizes 16 .. 128;
Sec. 4.2: an FP8 scale with 4 exponent and 3 mantissa bits): cast and dequantize bit-exact against the CPU oracle,
GEMM within 1e-3 relative Frobenius error."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3
# (group size, scale format, asymmetric): every group size with the paper's format, E4M3 at every group size, and
# the power-of-two scales at the sizes that leave the block-scaled matrix instructions
CASES = ([(gs, ref.FP8_E5M2, a) for gs in (16, 64, 128) for a in (1, 0)] +
         [(gs, ref.FP8_E4M3, a) for gs in (16, 32, 64, 128) for a in (1, 0)] +
         [(gs, ref.E8M0_FLOOR, 1) for gs in (16, 64, 128)] + [(64, ref.E8M0_ROUND, 0), (16, ref.E8M0_FLOOR, 0)])


def check(bits, gs, scale, asym, k_axis=-1):
    gc, gsc = G.gpu_quantize(bits, scale, asym, k_axis=k_axis, group_size=gs)
    rc, rs = ref.quantize(bits, gs, scale, asym, k_axis=k_axis)
    assert gsc.shape == rs.shape and gc.shape == rc.shape
    bad_s = np.argwhere(gsc != rs)
    assert bad_s.size == 0, "scale mismatch at %s: gpu %s oracle %s" % (
        bad_s[:5].tolist(), gsc[gsc != rs][:5], rs[gsc != rs][:5])
    bad_c = np.argwhere(gc != rc)
    assert bad_c.size == 0, "code mismatch at %s: gpu %s oracle %s" % (
        bad_c[:5].tolist(), gc[gc != rc][:5], rc[gc != rc][:5])


@pytest.mark.parametrize("gs,scale,asym", CASES)
def test_cast_linear_operands_and_ragged_rows(gs, scale, asym):
    x, w = synth.linear_operands("c1_linear_64x1024x1024")
    check(x, gs, scale, asym)
    check(w, gs, scale, asym)
    # K = 128 * 17 + 128: chunk count not a power of two, a single row, and a one-group row
    check(synth.glu_activations(37, 2304, seed=3), gs, scale, asym)
    check(synth.activations(1, 128, seed=4, n_outlier=1, outlier_gain=80.0), gs, scale, asym)


@pytest.mark.parametrize("gs,scale,asym", [c for c in CASES if c[1] in (ref.FP8_E4M3, ref.FP8_E5M2)])
def test_every_bf16_value_as_group_maximum(gs, scale, asym):
    """Every finite BF16 magnitude as the largest element of a group, once per sign: scale rounding (ties, subnormal
    scales, saturation at 448 for E4M3) and the element rounding relative to each of those scales."""
    rng = np.random.default_rng(gs)
    mags = np.arange(0, 0x7F80, dtype=np.uint16)
    xf = synth.bf16_bits_to_f32(mags)
    for sign in (0, 0x8000):
        x = np.zeros((mags.size, gs), np.uint16)
        frac = rng.random((mags.size, gs - 1), dtype=np.float32)
        body = np.minimum(synth.f32_to_bf16_bits(frac * xf[:, None]), mags[:, None])
        sgn = (rng.integers(0, 2, size=body.shape) * 0x8000).astype(np.uint16)
        pos = int(rng.integers(0, gs))  # the maximum sits in a different lane of the group each time
        x[:, :pos] = (body | sgn)[:, :pos]
        x[:, pos + 1:] = (body | sgn)[:, pos:]
        x[:, pos] = mags | np.uint16(sign)
        if gs == 16:
            x = x.reshape(-1, 32)  # K must be a multiple of 32: two groups of 16 per row
        check(x, gs, scale, asym)


@pytest.mark.parametrize("asym", [1, 0])
def test_every_bf16_value_under_each_e4m3_scale_mantissa(asym):
    """Group maxima that give each of the eight E4M3 scale mantissas (6 * (1 + m/8)), a subnormal scale and the
    saturated one; ALL finite BF16 patterns not above the maximum go through the other slots."""
    allbits = np.arange(0, 0x10000, dtype=np.uint32)
    finite = allbits[(allbits & 0x7F80) != 0x7F80].astype(np.uint16)
    amaxes = [6.0 * (1 + m / 8.0) for m in range(8)] + [6.0 * 5 * 2.0 ** -9, 6.0 * 2.0 ** -7, 3000.0, 1.0e6]
    for amax in amaxes:
        ab = synth.f32_to_bf16_bits(np.array([amax], np.float32))[0]
        cand = finite[(finite & 0x7FFF) <= ab]
        n = (cand.size + 29) // 30
        x = np.zeros((n, 32), np.uint16)
        x[:, 2:] = np.concatenate([cand, np.zeros(n * 30 - cand.size, np.uint16)]).reshape(n, 30)
        x[:, 0] = ab
        x[:, 1] = ab | 0x8000
        check(x, 32, ref.FP8_E4M3, asym)
        x[:, 1] = 0
        check(x, 32, ref.FP8_E4M3, asym)


@pytest.mark.parametrize("gs,scale,asym", CASES)
def test_degenerate_groups(gs, scale, asym):
    x = np.zeros((8, 256), np.uint16)
    x[1, :] = 0x8000                       # all -0
    x[2, :] = 0x3F80                       # all +1
    x[3, :] = 0xBF80                       # all -1
    x[4, :128] = 0x0001                    # smallest subnormal
    x[4, 128:] = 0x7F7F                    # largest finite
    x[5, ::2] = 0x7F7F
    x[5, 1::2] = 0xFF7F
    x[6, 0] = 0x4300                       # one outlier 128, rest tiny
    x[6, 1:] = 0x3000
    x[7, :] = synth.f32_to_bf16_bits(np.linspace(-4.9, 31, 256).astype(np.float32))
    check(x, gs, scale, asym)


@pytest.mark.parametrize("gs,scale,asym", CASES)
def test_groups_down_the_columns_and_row_stride(gs, scale, asym):
    v = synth.activations(256, 80, seed=10)  # [seq 256, d 80] -> operand [80, 256], groups along seq
    check(v, gs, scale, asym, k_axis=0)
    v = synth.activations(384, 300, seed=11, n_outlier=2, outlier_gain=40.0)  # more than one block of rows
    check(v, gs, scale, asym, k_axis=0)
    base = synth.activations(96, 640, seed=9)
    fmt = binding.make_format(scale, asym, gs)
    c, s = binding.quantize(fmt, G.to_dev_bf16(base)[:, 128:128 + 384])
    rc, rs = ref.quantize(np.ascontiguousarray(base[:, 128:512]), gs, scale, asym)
    assert np.array_equal(c.cpu().numpy(), rc) and np.array_equal(s.cpu().numpy(), rs)


@pytest.mark.parametrize("gs,scale,asym", CASES)
def test_dequantize_exact(gs, scale, asym):
    x = synth.activations(40, 384, seed=11)
    rc, rs = ref.quantize(x, gs, scale, asym)
    want = ref.dequantize(rc, rs, gs, scale, asym)
    fmt = binding.make_format(scale, asym, gs)
    for dt in (torch.float32, torch.bfloat16):
        out = binding.dequantize(fmt, G.to_dev_u8(rc), G.to_dev_u8(rs), dt)
        torch.cuda.synchronize()
        assert np.array_equal(out.float().cpu().numpy().astype(np.float64), want)


def test_every_e4m3_scale_byte_dequantizes_exactly():
    """All 127 finite E4M3 scale bytes (the cast never produces most of them for BF16 data of ordinary range) times
    all 16 element codes, both classes."""
    codes = np.tile(np.array([0x10, 0x32, 0x54, 0x76, 0x98, 0xBA, 0xDC, 0xFE] * 2, np.uint8), (127, 1))  # K = 32
    scales = np.zeros((127, 1, 2), np.uint8)
    scales[:, 0, 0] = np.arange(127)
    scales[:, 0, 1] = np.arange(127)[::-1]
    want = ref.dequantize(codes, scales, 32, ref.FP8_E4M3, 1)
    fmt = binding.make_format(ref.FP8_E4M3, True, 32)
    out = binding.dequantize(fmt, G.to_dev_u8(codes), G.to_dev_u8(scales), torch.float32)
    assert np.array_equal(out.cpu().numpy().astype(np.float64), want)
    out = binding.dequantize(fmt, G.to_dev_u8(codes), G.to_dev_u8(scales), torch.bfloat16)
    assert np.array_equal(out.float().cpu().numpy().astype(np.float64), want)  # <= 6 significant bits: exact in BF16


@pytest.mark.parametrize("gs,scale,asym", CASES)
@pytest.mark.parametrize("M,N,K", [(64, 1024, 1024), (33, 65, 128), (257, 255, 640), (300, 520, 1152)])
def test_gemm(gs, scale, asym, M, N, K):
    a = synth.activations(M, K, seed=M + K, n_outlier=1, outlier_gain=60.0)
    b = synth.weights(N, K, seed=N)
    ac, as_ = ref.quantize(a, gs, scale, asym)
    bc, bs = ref.quantize(b, gs, scale, asym)
    C = G.gpu_gemm(ac, as_, bc, bs, scale, asym, group_size=gs)
    Cr = ref.gemm(ac, as_, bc, bs, gs, scale, asym)
    assert C.shape == (M, N)
    assert G.rel_fro(C, Cr) <= TOL
    assert np.allclose(C, Cr, rtol=1e-4, atol=1e-4 * np.abs(Cr).max())


@pytest.mark.parametrize("gs", [16, 64, 128])
def test_gemm_batched_with_scales_on_every_group(gs):
    """Batched operands whose scale bytes all differ, so a group index taken from the wrong row, batch entry or half
    of a 32-block shows up."""
    rng = np.random.default_rng(gs)
    batch, M, N, K = 3, 70, 90, 256
    G_ = K // gs

    def operand(rows):
        codes = rng.integers(0, 256, size=(batch, rows, K // 2), dtype=np.uint8)
        scales = rng.integers(40, 90, size=(batch, rows, G_, 2), dtype=np.uint8)  # E5M2 bytes 2^-5 .. 2^7
        return codes, scales

    ac, as_ = operand(M)
    bc, bs = operand(N)
    C = G.gpu_gemm(ac, as_, bc, bs, ref.FP8_E5M2, 1, group_size=gs)
    Cr = ref.gemm(ac, as_, bc, bs, gs, ref.FP8_E5M2, 1)
    assert G.rel_fro(C, Cr) <= TOL
