"""GPU parity for one group per row (group size -1, the granularity of the code example in Appendix B): cast and
dequantize bit-exact against the CPU oracle, the GEMM within 1e-3 relative Frobenius error, and the calls that do not
take such a format rejected on the host."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3
FORMATS = [(s, a) for s in (ref.FP8_E5M2, ref.FP8_E4M3, ref.E8M0_FLOOR, ref.E8M0_ROUND) for a in (1, 0)]


def check(bits, scale, asym, dev=None):
    fmt = binding.make_format(scale, asym, -1)
    gc, gs = binding.quantize(fmt, G.to_dev_bf16(bits) if dev is None else dev)
    torch.cuda.synchronize()
    gc, gs = gc.cpu().numpy(), gs.cpu().numpy()
    rc, rs = ref.quantize(bits, -1, scale, asym)
    assert gs.shape == rs.shape and gc.shape == rc.shape
    bad_s = np.argwhere(gs != rs)
    assert bad_s.size == 0, "scale mismatch at %s: gpu %s oracle %s" % (
        bad_s[:5].tolist(), gs[gs != rs][:5], rs[gs != rs][:5])
    bad_c = np.argwhere(gc != rc)
    assert bad_c.size == 0, "code mismatch at %s: gpu %s oracle %s" % (
        bad_c[:5].tolist(), gc[gc != rc][:5], rc[gc != rc][:5])


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_cast_matches_oracle(scale, asym):
    # the tensor of the Appendix B example: one row of 1024 values from -4.9 to 31
    check(synth.f32_to_bf16_bits(np.linspace(-4.9, 31, 1024).astype(np.float32)).reshape(1, -1), scale, asym)
    x, w = synth.linear_operands("c1_linear_64x1024x1024")
    check(x, scale, asym)
    check(w, scale, asym)
    check(synth.glu_activations(37, 2304, seed=3), scale, asym)                           # chunks not a power of two
    check(synth.activations(5, 32, seed=4, n_outlier=1, outlier_gain=80.0), scale, asym)    # four chunks, one wave
    check(synth.activations(3, 4096 + 32, seed=5, n_outlier=2, outlier_gain=50.0), scale, asym)  # first four-wave size
    check(synth.activations(2, 28672, seed=6, n_outlier=4, outlier_gain=60.0), scale, asym)  # 14 chunks a lane
    # the extreme of a class sits in the last chunk, which a lane of the last wave owns
    x = synth.activations(4, 8192, seed=7)
    x[:, -1] = 0x4700   # +32768
    x[:, -2] = 0xC680   # -16384
    check(x, scale, asym)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_degenerate_rows(scale, asym):
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
    x[7, 17] = 0x8001                      # one negative subnormal in a row of zeros
    check(x, scale, asym)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.FP8_E4M3, 0)])
def test_every_bf16_value_as_row_maximum(scale, asym):
    """Every finite BF16 magnitude as the largest element of a row, once per sign, in a different chunk each time."""
    rng = np.random.default_rng(5)
    mags = np.arange(0, 0x7F80, dtype=np.uint16)
    xf = synth.bf16_bits_to_f32(mags)
    for sign in (0, 0x8000):
        frac = rng.random((mags.size, 96), dtype=np.float32)
        body = np.minimum(synth.f32_to_bf16_bits(frac * xf[:, None]), mags[:, None])
        x = body | (rng.integers(0, 2, size=body.shape) * 0x8000).astype(np.uint16)
        x[np.arange(mags.size), rng.integers(0, 96, size=mags.size)] = mags | np.uint16(sign)
        check(x, scale, asym)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0)])
def test_row_stride_and_batch(scale, asym):
    base = synth.activations(96, 640, seed=9, n_outlier=2, outlier_gain=40.0)
    check(np.ascontiguousarray(base[:, 128:512]), scale, asym, dev=G.to_dev_bf16(base)[:, 128:512])
    fmt = binding.make_format(scale, asym, -1)
    xb = synth.activations(3 * 40, 8192, seed=10, n_outlier=1, outlier_gain=30.0).reshape(3, 40, 8192)
    c, s = binding.quantize_batched(fmt, G.to_dev_bf16(xb))
    for b in range(3):
        rc, rs = ref.quantize(xb[b], -1, scale, asym)
        assert np.array_equal(c[b].cpu().numpy(), rc) and np.array_equal(s[b].cpu().numpy(), rs)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E4M3, 1), (ref.FP8_E5M2, 0), (ref.E8M0_ROUND, 1)])
@pytest.mark.parametrize("rt", [1.0, 1234.567, 3.21e-6])
def test_cast_over_a_tensor_wise_scale(scale, asym, rt):
    """Sec. 5.3's double scaling with a row as the group: the elements are multiplied by the factor in FP32 first."""
    fmt = binding.make_format(scale, asym, -1)
    pair = torch.tensor([1.0, rt], dtype=torch.float32, device="cuda")
    for bits in (synth.activations(33, 2304, seed=2, n_outlier=2, outlier_gain=60.0),
                 synth.activations(2, 16384, seed=3)):
        gc, gs = binding.quantize(fmt, G.to_dev_bf16(bits), tensor_pair=pair)
        rc, rs = ref.quantize(bits, -1, scale, asym, tensor_rcp=np.float32(rt))
        assert np.array_equal(gs.cpu().numpy(), rs) and np.array_equal(gc.cpu().numpy(), rc)


@pytest.mark.parametrize("scale,asym", FORMATS)
def test_dequantize_exact(scale, asym):
    x = synth.activations(40, 384, seed=11, n_outlier=1, outlier_gain=20.0)
    rc, rs = ref.quantize(x, -1, scale, asym)
    want = ref.dequantize(rc, rs, -1, scale, asym)
    fmt = binding.make_format(scale, asym, -1)
    for dt in (torch.float32, torch.bfloat16):
        out = binding.dequantize(fmt, G.to_dev_u8(rc), G.to_dev_u8(rs), dt)
        torch.cuda.synchronize()
        assert np.array_equal(out.float().cpu().numpy().astype(np.float64), want)


@pytest.mark.parametrize("scale,asym", FORMATS)
@pytest.mark.parametrize("M,N,K", [(64, 1024, 1024), (33, 65, 128), (257, 255, 640), (1, 300, 2048)])
def test_gemm(scale, asym, M, N, K):
    a = synth.activations(M, K, seed=M + K, n_outlier=1, outlier_gain=60.0)
    b = synth.weights(N, K, seed=N)
    ac, as_ = ref.quantize(a, -1, scale, asym)
    bc, bs = ref.quantize(b, -1, scale, asym)
    C = G.gpu_gemm(ac, as_, bc, bs, scale, asym, group_size=-1)
    Cr = ref.gemm(ac, as_, bc, bs, -1, scale, asym)
    assert C.shape == (M, N)
    assert G.rel_fro(C, Cr) <= TOL
    assert np.allclose(C, Cr, rtol=1e-4, atol=1e-4 * np.abs(Cr).max())


def test_gemm_batched_with_a_scale_pair_of_its_own_on_every_row():
    """Random codes and scale bytes that all differ, so a scale taken from the wrong row or batch entry shows up; the
    same product from weights prepared beforehand."""
    rng = np.random.default_rng(1)
    batch, M, N, K = 3, 70, 90, 256

    def operand(rows):
        codes = rng.integers(0, 256, size=(batch, rows, K // 2), dtype=np.uint8)
        scales = rng.integers(40, 90, size=(batch, rows, 1, 2), dtype=np.uint8)  # E5M2 bytes 2^-5 .. 2^7
        return codes, scales

    ac, as_ = operand(M)
    bc, bs = operand(N)
    C = G.gpu_gemm(ac, as_, bc, bs, ref.FP8_E5M2, 1, group_size=-1)
    Cr = ref.gemm(ac, as_, bc, bs, -1, ref.FP8_E5M2, 1)
    assert G.rel_fro(C, Cr) <= TOL
    fmt = binding.make_format(ref.FP8_E5M2, 1, -1)
    dev = [G.to_dev_u8(t[1]) for t in (ac, as_, bc, bs)]
    prepared = binding.prepare_weights(fmt, dev[2], dev[3])
    Cp = binding.gemm_prepared(fmt, *dev, prepared)
    torch.cuda.synchronize()
    assert G.rel_fro(Cp.cpu().numpy(), Cr[1]) <= TOL


@pytest.mark.parametrize("K", [96, 4128, 28672])
def test_cast_writes_only_its_outputs(K):
    """Codes and scale bytes land in windows of pattern-filled buffers; the guard bytes around them stay untouched."""
    rows, guard = 7, 4096
    x = synth.activations(rows, K, seed=K, n_outlier=1, outlier_gain=30.0)
    fmt = binding.make_format(ref.FP8_E5M2, 1, -1)
    cbuf = torch.full((guard + rows * K // 2 + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    sbuf = torch.full((guard + rows * 2 + guard,), 0xA5, dtype=torch.uint8, device="cuda")
    codes = cbuf[guard:guard + rows * K // 2].view(rows, K // 2)
    scales = sbuf[guard:guard + rows * 2].view(rows, 1, 2)
    binding.quantize(fmt, G.to_dev_bf16(x), codes=codes, scales=scales)
    torch.cuda.synchronize()
    rc, rs = ref.quantize(x, -1, ref.FP8_E5M2, 1)
    assert np.array_equal(codes.cpu().numpy(), rc) and np.array_equal(scales.cpu().numpy(), rs)
    for buf, n in ((cbuf, rows * K // 2), (sbuf, rows * 2)):
        assert bool((buf[:guard] == 0xA5).all()) and bool((buf[guard + n:] == 0xA5).all())


def test_calls_without_a_whole_row_form_say_so():
    fmt = binding.make_format(ref.FP8_E5M2, 1, -1)
    x = G.to_dev_bf16(synth.activations(64, 128, seed=1))
    with pytest.raises(binding.AmxError, match="whole-row"):
        binding.quantize(fmt, x, k_axis=0)                      # groups down a column
    with pytest.raises(binding.AmxError, match="whole-row"):
        binding.rmsnorm_quantize(fmt, x, torch.ones(128, dtype=torch.float32, device="cuda"), 1e-5)
