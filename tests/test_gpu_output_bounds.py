"""Output bounds: every GEMM kernel of the library, on shapes with partial tiles, writes C[b][i][j] for i < M, j < N and
nothing else. C is a window of a larger buffer filled with a bit pattern (a NaN payload no kernel produces): leading
dimension ldc > N, guard words in front of the first row and behind the last one. After the call the window must match
the oracle and every other word must still hold the pattern, bit for bit."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3
CANARY = 0x7FC0DEAD  # a quiet NaN with a payload, as int32
GUARD = 4096  # words in front of and behind the matrix


def canary_window(batch, M, N, pad, dtype=torch.float32):
    """A [batch, M, N] window with leading dimension N + pad inside a pattern-filled buffer. Returns (buffer as
    integers, window, mask of the words the call may write)."""
    ld = N + pad
    words = torch.int32 if dtype == torch.float32 else torch.int16
    pattern = CANARY if dtype == torch.float32 else 0x7FC5
    buf = torch.full((GUARD + batch * M * ld + GUARD,), pattern, dtype=words, device="cuda")
    body = buf[GUARD:GUARD + batch * M * ld].view(batch, M, ld)
    window = body.view(dtype)[:, :, :N]
    allowed = torch.zeros_like(buf, dtype=torch.bool)
    allowed[GUARD:GUARD + batch * M * ld].view(batch, M, ld)[:, :, :N] = True
    return buf, window, allowed, pattern


def assert_padding_untouched(buf, allowed, pattern, what):
    touched = (buf != pattern) & ~allowed
    n = int(touched.sum())
    assert n == 0, "%s: %d words outside C were written (first at flat index %d)" % (
        what, n, int(torch.nonzero(touched)[0]))


def operands(batch, M, N, K, scale, asym, gs=32):
    a = synth.activations(batch * M, K, seed=M + K, n_outlier=2, outlier_gain=60.0)
    b = synth.weights(batch * N, K, seed=N)
    ac, as_ = ref.quantize(a, gs, scale, asym)
    bc, bs = ref.quantize(b, gs, scale, asym)
    shp = lambda t, r: t.reshape((batch, r) + t.shape[1:])  # noqa: E731
    return shp(ac, M), shp(as_, M), shp(bc, N), shp(bs, N)


# (label, scale, asymmetric, group size, per-call options, shapes) — one entry per kernel and store path
KERNELS = [
    ("panel 256x256", ref.FP8_E5M2, 1, 32, dict(tile="256x256", few_rows=-1), [(1, 300, 270, 160), (2, 257, 31, 96)]),
    ("panel 256x128", ref.FP8_E5M2, 1, 32, dict(tile="256x128", few_rows=-1), [(1, 300, 270, 160), (2, 257, 31, 96)]),
    ("panel 64x256", ref.FP8_E5M2, 0, 32, dict(tile="64x256", few_rows=-1), [(1, 300, 270, 160), (2, 65, 257, 96)]),
    ("panel, groups of 16, E4M3", ref.FP8_E4M3, 1, 16, dict(few_rows=-1), [(1, 130, 100, 64)]),
    ("hybrid", ref.FP8_E5M2, 1, 32, dict(e5m2_kernel="hybrid", few_rows=-1), [(1, 300, 270, 384), (2, 257, 31, 128)]),
    ("fused", ref.FP8_E5M2, 1, 32, dict(e5m2_kernel="fused", few_rows=-1), [(1, 300, 270, 384), (2, 257, 31, 128)]),
    ("block-scaled FP4", ref.E8M0_FLOOR, 0, 32, dict(few_rows=-1), [(1, 300, 270, 384), (2, 257, 31, 128)]),
    ("sign-split FP4", ref.E8M0_FLOOR, 1, 32, dict(pot_kernel="split", few_rows=-1), [(1, 300, 270, 384), (2, 257, 31, 128)]),
    ("merged FP8", ref.E8M0_FLOOR, 1, 32, dict(pot_kernel="merged_fp8", few_rows=-1), [(1, 300, 270, 160), (2, 257, 31, 96)]),
    ("merged FP6", ref.E8M0_FLOOR, 1, 32, dict(pot_kernel="merged_fp6", few_rows=-1), [(1, 300, 270, 160), (2, 257, 31, 96)]),
    ("few rows, one K slice", ref.FP8_E5M2, 1, 32, dict(few_rows=1), [(1, 5, 70, 512), (2, 33, 100, 256), (1, 200, 45, 512)]),
    ("few rows, K slices", ref.FP8_E5M2, 1, 32, dict(few_rows=2), [(1, 5, 70, 512), (2, 100, 100, 1024), (1, 250, 33, 512)]),
    ("few rows, power-of-two scales", ref.E8M0_FLOOR, 1, 32, dict(few_rows=3), [(1, 31, 65, 768)]),
]


@pytest.mark.parametrize("label,scale,asym,gs,opts,shapes", KERNELS, ids=[k[0] for k in KERNELS])
def test_gemm_writes_only_its_window(label, scale, asym, gs, opts, shapes):
    for batch, M, N, K in shapes:
        ac, as_, bc, bs = operands(batch, M, N, K, scale, asym, gs)
        buf, window, allowed, pattern = canary_window(batch, M, N, pad=37)
        fmt = binding.make_format(scale, asym, gs)
        out = window if batch > 1 else window[0]
        binding.gemm(fmt, *(G.to_dev_u8(t if batch > 1 else t[0]) for t in (ac, as_, bc, bs)), out=out,
                     options=binding.gemm_options(**opts))
        torch.cuda.synchronize()
        what = "%s %dx%dx%dx%d" % (label, batch, M, N, K)
        assert_padding_untouched(buf, allowed, pattern, what)
        Cr = ref.gemm(ac, as_, bc, bs, gs, scale, asym)
        assert G.rel_fro(window.cpu().numpy(), Cr) <= TOL, what


def test_scaled_gemm_writes_only_its_window():
    """The double-scaling product (tensor-wise scales in the epilogue of the panel kernel)."""
    M, N, K = 130, 100, 64
    a = synth.activations(M, K, seed=1, n_outlier=1, outlier_gain=30.0)
    b = synth.weights(N, K, seed=2)
    fmt = binding.make_format(binding.FP8_E4M3, True, 16)
    ad, bd = G.to_dev_bf16(a), G.to_dev_bf16(b)
    pa, pb = binding.tensor_scale(ad), binding.tensor_scale(bd)
    ac, as_ = binding.quantize(fmt, ad, tensor_pair=pa)
    bc, bs = binding.quantize(fmt, bd, tensor_pair=pb)
    buf, window, allowed, pattern = canary_window(1, M, N, pad=5)
    binding.gemm(fmt, ac, as_, bc, bs, out=window[0], a_pair=pa, b_pair=pb)
    torch.cuda.synchronize()
    assert_padding_untouched(buf, allowed, pattern, "scaled GEMM")
    sa, sb = float(pa[0]), float(pb[0])
    Cr = ref.gemm(ac.cpu().numpy(), as_.cpu().numpy(), bc.cpu().numpy(), bs.cpu().numpy(), 16, ref.FP8_E4M3, 1, sa, sb)
    assert G.rel_fro(window[0].cpu().numpy(), Cr) <= TOL


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0), (ref.E8M0_FLOOR, 1)])
@pytest.mark.parametrize("M,width,K,pad", [(300, 96, 160, 8), (257, 160, 128, 3), (70, 32, 256, 0)])
def test_gated_gemm_writes_only_its_window(M, width, K, pad, scale, asym):
    """The GEMM with the gated activation as its epilogue writes BF16: through LDS with 16-byte stores when the output
    allows it (pad 8: leading dimension a multiple of 8), element by element otherwise (pad 3), on all three tiled
    kernels (BF16 panels, block-scaled FP4, merged FP6)."""
    import ctypes
    a = synth.activations(M, K, seed=M, n_outlier=1, outlier_gain=30.0)
    wg, wu = synth.weights(width, K, seed=3), synth.weights(width, K, seed=4)
    fmt = binding.make_format(scale, asym)
    ac, as_ = binding.quantize(fmt, G.to_dev_bf16(a))
    inter = binding.interleave_gate_up(G.to_dev_bf16(wg), G.to_dev_bf16(wu)).contiguous()
    ic, is_ = binding.quantize(fmt, inter)
    buf, window, allowed, pattern = canary_window(1, M, width, pad, dtype=torch.bfloat16)
    need = binding.gemm_silu_mul_workspace_bytes(fmt, M, width, K)
    ws = torch.empty(max(need, 1), dtype=torch.uint8, device="cuda")
    binding._check(binding.load().amxfp4_gemm_silu_mul(
        ctypes.byref(fmt), M, width, K, ac.data_ptr(), as_.data_ptr(), ic.data_ptr(), is_.data_ptr(),
        window.data_ptr(), width + pad, ws.data_ptr() if need else None, need, binding._stream()))
    torch.cuda.synchronize()
    assert_padding_untouched(buf, allowed, pattern, "gated GEMM %dx%dx%d" % (M, width, K))
    plain = binding.gemm_silu_mul(fmt, ac, as_, ic, is_)   # contiguous output of its own
    torch.cuda.synchronize()
    assert torch.equal(window[0].contiguous().view(torch.int16), plain.view(torch.int16))
