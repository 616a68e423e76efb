"""GPU parity of the double-scaling calls (Sec. 5.3: tensor-wise FP32 scale under the group-wise scale, NVFP4 and its
asymmetric variant ANVFP4) against the CPU oracle: tensor scale pair, codes and scales bit-exact; dequantize equal
after the one FP32 rounding; GEMM within 1e-3 relative Frobenius error."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3
NVFP4 = (16, ref.FP8_E4M3, 0)
ANVFP4 = (16, ref.FP8_E4M3, 1)
CASES = [NVFP4, ANVFP4, (32, ref.FP8_E5M2, 1), (64, ref.E8M0_ROUND, 1), (32, ref.E8M0_FLOOR, 0), (128, ref.FP8_E4M3, 1)]


def pair_dev(st, rt):
    return torch.tensor([float(st), float(rt)], dtype=torch.float32, device="cuda")


def check_cast(bits, gs, scale, asym, rt, k_axis=-1):
    fmt = binding.make_format(scale, asym, gs)
    gc, gsc = binding.quantize(fmt, G.to_dev_bf16(bits), k_axis=k_axis, tensor_pair=pair_dev(1.0, rt))
    gc, gsc = gc.cpu().numpy(), gsc.cpu().numpy()
    rc, rs = ref.quantize(bits, gs, scale, asym, k_axis=k_axis, tensor_rcp=rt)
    bad_s = np.argwhere(gsc != rs)
    assert bad_s.size == 0, "R_t %r: scale mismatch at %s: gpu %s oracle %s" % (
        rt, bad_s[:5].tolist(), gsc[gsc != rs][:5], rs[gsc != rs][:5])
    bad_c = np.argwhere(gc != rc)
    assert bad_c.size == 0, "R_t %r: code mismatch at %s: gpu %s oracle %s" % (
        rt, bad_c[:5].tolist(), gc[gc != rc][:5], rc[gc != rc][:5])


def scaled_bits(bits, gain):
    return synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(bits) * np.float32(gain))


@pytest.mark.parametrize("gain", [1.0, 3.0e-7, 2.5e9, 0.0])
def test_tensor_scale_pair(gain):
    x = scaled_bits(synth.activations(300, 1032, seed=1, n_outlier=3, outlier_gain=60.0), gain)
    x[7, 5] |= 0x8000
    want = ref.tensor_scale(x)
    got = binding.tensor_scale(G.to_dev_bf16(x)).cpu().numpy()
    assert got[0] == want[0] and got[1] == want[1]
    # a column slice (row stride larger than the row), maximum outside the slice
    xs = np.ascontiguousarray(x[:, 64:64 + 512])
    got = binding.tensor_scale(G.to_dev_bf16(x)[:, 64:64 + 512]).cpu().numpy()
    want = ref.tensor_scale(xs)
    assert got[0] == want[0] and got[1] == want[1]


def test_tensor_scale_of_extreme_tensors():
    z = np.zeros((4, 64), np.uint16)
    z[2, 9] = 0x8001   # one negative subnormal: the scale clamps at 2^-96
    got = binding.tensor_scale(G.to_dev_bf16(z)).cpu().numpy()
    assert got[0] == np.float32(2.0 ** -96) and got[1] == np.float32(2.0 ** 96)
    z[0, 0] = 0x7F7F   # largest finite BF16
    got, want = binding.tensor_scale(G.to_dev_bf16(z)).cpu().numpy(), ref.tensor_scale(z)
    assert got[0] == want[0] and got[1] == want[1]


@pytest.mark.parametrize("gs,scale,asym", CASES)
@pytest.mark.parametrize("gain", [1.0, 7.0e-4, 900.0])
def test_scaled_cast_of_linear_operands(gs, scale, asym, gain):
    x, w = synth.linear_operands("c1_linear_64x1024x1024")
    for t in (scaled_bits(x, gain), scaled_bits(w, gain), scaled_bits(synth.glu_activations(37, 2304, seed=3), gain)):
        _, rt = ref.tensor_scale(t)
        check_cast(t, gs, scale, asym, rt)
    # an arbitrary factor that has nothing to do with the data: saturation and flushing of whole groups
    check_cast(x, gs, scale, asym, np.float32(1234.567))
    check_cast(x, gs, scale, asym, np.float32(3.21e-6))


@pytest.mark.parametrize("gs,scale,asym", [NVFP4, ANVFP4, (32, ref.FP8_E5M2, 1)])
def test_scaled_cast_all_bf16_values(gs, scale, asym):
    """Every finite BF16 pattern through the multiply and the cast, under two non-trivial factors."""
    allbits = np.arange(0, 0x10000, dtype=np.uint32)
    finite = allbits[(allbits & 0x7F80) != 0x7F80].astype(np.uint16)
    x = np.sort(finite.view(np.int16)).view(np.uint16)          # neighbours in value share a group
    x = x[:x.size // 128 * 128].reshape(-1, 128)
    for rt in (np.float32(1.0 / 3.0), np.float32(2688.0 / 37.25)):
        check_cast(x, gs, scale, asym, rt)
    rng = np.random.default_rng(5)
    check_cast(rng.permutation(finite)[:65024].reshape(-1, 128), gs, scale, asym, np.float32(0.7071))


def _nudge(v, k):
    """The float32 k steps above (k > 0) or below v."""
    v = np.float32(v)
    for _ in range(abs(k)):
        v = np.nextafter(v, np.float32(np.inf if k > 0 else -np.inf), dtype=np.float32)
    return v


@pytest.mark.parametrize("scale,mbits,exps", [(ref.FP8_E4M3, 3, (-8, -3, 0, 5)), (ref.FP8_E5M2, 2, (-16, -3, 0, 9))])
@pytest.mark.parametrize("asym", [1, 0])
def test_group_maximum_next_to_a_scale_tie(scale, mbits, exps, asym):
    """The scaled values are arbitrary FP32 numbers, so max / 6 can sit one ulp beside a midpoint of the scale grid
    (where rounding the quotient to FP32 first and to FP8 second would go wrong). An element 1.0 carries the factor
    itself into the group: y = R_t."""
    x = np.zeros((2, 32), np.uint16)
    x[0, 3] = 0x3F80                    # +1.0 is the positive maximum of row 0
    x[0, 4:12] = synth.f32_to_bf16_bits(np.linspace(0.1, 0.95, 8).astype(np.float32))
    x[0, 12:20] = synth.f32_to_bf16_bits(-np.linspace(0.1, 0.9, 8).astype(np.float32))
    x[1] = x[0] ^ np.uint16(0x8000)     # mirrored: the maximum is in the negative class
    for e in exps:
        for m in range(1 << mbits):
            mid = (1.0 + (2 * m + 1) / float(2 << mbits)) * 2.0 ** e     # halfway between two scale values
            for k in (-2, -1, 0, 1, 2):
                check_cast(x, 32, scale, asym, _nudge(6.0 * mid, k))
    emin = -6 if scale == ref.FP8_E4M3 else -14
    for n in range(1 << mbits):          # midpoints of the subnormal part of the grid, n + 1/2 quanta
        for k in (-1, 0, 1):
            check_cast(x, 32, scale, asym, _nudge(6.0 * (n + 0.5) * 2.0 ** (emin - mbits), k))


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E4M3, 1), (ref.FP8_E4M3, 0), (ref.FP8_E5M2, 1)])
def test_element_next_to_a_rounding_boundary(scale, asym):
    """y / S one ulp beside each E2M1 rounding boundary, for every scale mantissa: the element 1.0 becomes
    y = R_t = boundary * S (nudged), and a larger element fixes the group scale at S."""
    nm = 8 if scale == ref.FP8_E4M3 else 4
    for m in range(nm):
        S = (1.0 + m / float(nm)) * 0.25
        for bnd in (0.25, 0.75, 1.25, 1.75, 2.5, 3.5, 5.0):
            for k in (-2, -1, 0, 1, 2):
                rt = _nudge(bnd * S, k)
                xmax = synth.f32_to_bf16_bits(np.array([6.0 * S / float(rt)], np.float32))[0]
                x = np.zeros((2, 32), np.uint16)
                x[0, 0] = xmax
                x[0, 1] = xmax | 0x8000
                x[0, 2] = 0x3F80          # +1.0 -> y = R_t
                x[0, 3] = 0xBF80          # -1.0 -> y = -R_t
                x[1] = x[0]
                x[1, 1] = 0               # negative class led by the -1.0 element itself
                check_cast(x, 32, scale, asym, rt)


@pytest.mark.parametrize("gs,scale,asym", CASES)
def test_scaled_cast_down_the_columns(gs, scale, asym):
    v = scaled_bits(synth.activations(384, 300, seed=11, n_outlier=2, outlier_gain=40.0), 0.013)
    _, rt = ref.tensor_scale(v)
    check_cast(v, gs, scale, asym, rt, k_axis=0)


@pytest.mark.parametrize("gs,scale,asym", [NVFP4, ANVFP4, (32, ref.E8M0_FLOOR, 1)])
def test_scaled_dequantize(gs, scale, asym):
    x = scaled_bits(synth.activations(40, 384, seed=11), 5.0e-3)
    st, rt = ref.tensor_scale(x)
    rc, rs = ref.quantize(x, gs, scale, asym, tensor_rcp=rt)
    want = ref.dequantize(rc, rs, gs, scale, asym, tensor_scale=st).astype(np.float32)  # one rounding of exact values
    fmt = binding.make_format(scale, asym, gs)
    out = binding.dequantize(fmt, G.to_dev_u8(rc), G.to_dev_u8(rs), tensor_pair=pair_dev(st, rt))
    assert np.array_equal(out.cpu().numpy(), want)
    with pytest.raises(binding.AmxError):
        binding.dequantize(fmt, G.to_dev_u8(rc), G.to_dev_u8(rs), torch.bfloat16, tensor_pair=pair_dev(st, rt))


@pytest.mark.parametrize("gs,scale,asym", [NVFP4, ANVFP4, (32, ref.FP8_E5M2, 1), (32, ref.E8M0_FLOOR, 1)])
@pytest.mark.parametrize("M,N,K", [(64, 1024, 1024), (33, 65, 128), (300, 520, 1152)])
def test_scaled_gemm(gs, scale, asym, M, N, K):
    a = scaled_bits(synth.activations(M, K, seed=M + K, n_outlier=1, outlier_gain=60.0), 2.0e-5)
    b = synth.weights(N, K, seed=N)
    (sa, ra), (sb, rb) = ref.tensor_scale(a), ref.tensor_scale(b)
    ac, as_ = ref.quantize(a, gs, scale, asym, tensor_rcp=ra)
    bc, bs = ref.quantize(b, gs, scale, asym, tensor_rcp=rb)
    Cr = ref.gemm(ac, as_, bc, bs, gs, scale, asym, a_tensor_scale=sa, b_tensor_scale=sb)
    fmt = binding.make_format(scale, asym, gs)
    C = binding.gemm(fmt, G.to_dev_u8(ac), G.to_dev_u8(as_), G.to_dev_u8(bc), G.to_dev_u8(bs),
                     a_pair=pair_dev(sa, ra), b_pair=pair_dev(sb, rb)).cpu().numpy()
    assert C.shape == (M, N)
    assert G.rel_fro(C, Cr) <= TOL
    assert np.allclose(C, Cr, rtol=1e-4, atol=1e-4 * np.abs(Cr).max())


@pytest.mark.parametrize("gs,scale,asym", [NVFP4, ANVFP4])
def test_whole_chain_on_the_device(gs, scale, asym):
    """tensor_scale -> quantize -> gemm with the pairs never leaving the device, batched, against the oracle chain;
    and the product approximates the BF16 one although the activations alone would flush to zero in E4M3 groups."""
    batch, M, N, K = 2, 96, 80, 256
    fmt = binding.make_format(scale, asym, gs)
    a = scaled_bits(synth.activations(batch * M, K, seed=3, n_outlier=1, outlier_gain=30.0), 1.0e-5)
    b = synth.weights(batch * N, K, seed=4)
    ad, bd = G.to_dev_bf16(a), G.to_dev_bf16(b)
    pa, pb = binding.tensor_scale(ad), binding.tensor_scale(bd)
    ac, as_ = binding.quantize(fmt, ad, tensor_pair=pa)
    bc, bs = binding.quantize(fmt, bd, tensor_pair=pb)
    ns = as_.shape[1:]
    C = binding.gemm(fmt, ac.view(batch, M, -1), as_.view(batch, M, *ns), bc.view(batch, N, -1),
                     bs.view(batch, N, *ns), a_pair=pa, b_pair=pb).cpu().numpy()
    (sa, ra), (sb, rb) = ref.tensor_scale(a), ref.tensor_scale(b)
    rac, ras = ref.quantize(a, gs, scale, asym, tensor_rcp=ra)
    rbc, rbs = ref.quantize(b, gs, scale, asym, tensor_rcp=rb)
    assert np.array_equal(ac.cpu().numpy(), rac) and np.array_equal(as_.cpu().numpy(), ras)
    Cr = ref.gemm(rac.reshape(batch, M, -1), ras.reshape(batch, M, *ns), rbc.reshape(batch, N, -1),
                  rbs.reshape(batch, N, *ns), gs, scale, asym, a_tensor_scale=sa, b_tensor_scale=sb)
    assert G.rel_fro(C, Cr) <= TOL
    af = synth.bf16_bits_to_f32(a).astype(np.float64).reshape(batch, M, K)
    bf = synth.bf16_bits_to_f32(b).astype(np.float64).reshape(batch, N, K)
    exact = np.einsum("bmk,bnk->bmn", af, bf)
    assert G.rel_fro(C, exact) < 0.25
    unscaled = binding.quantize(fmt, ad)[1]
    assert not unscaled.any()
