"""The library at the size limits its header states (K = 2^20, the largest GEMM row count, the largest batch) and
just inside them: launch grids and 32-bit offsets in the kernels are laid out for these bounds. Casts are compared
bit for bit, GEMMs on all or on sampled rows against the oracle."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

K_MAX = 1 << 20
ROWS_MAX = (1 << 21) - 256


@pytest.mark.parametrize("gs,scale,asym", [(32, ref.FP8_E5M2, 1), (16, ref.FP8_E4M3, 1), (128, ref.E8M0_FLOOR, 0)])
def test_cast_longest_rows(gs, scale, asym):
    x = synth.activations(3, K_MAX, seed=1, n_outlier=8, outlier_gain=60.0)
    gc, gsc = G.gpu_quantize(x, scale, asym, group_size=gs)
    rc, rs = ref.quantize(x, gs, scale, asym)
    assert np.array_equal(gc, rc) and np.array_equal(gsc, rs)
    # the same length down a strided axis: [K_MAX, 8] tensor, groups along axis 0
    v = np.ascontiguousarray(synth.activations(8, K_MAX, seed=2).T)
    gc, gsc = G.gpu_quantize(v, scale, asym, k_axis=0, group_size=gs)
    rc, rs = ref.quantize(v, gs, scale, asym, k_axis=0)
    assert np.array_equal(gc, rc) and np.array_equal(gsc, rs)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0), (ref.E8M0_FLOOR, 1)])
def test_gemm_longest_contraction(scale, asym):
    """K = 2^20 on each GEMM path (BF16 panels, block-scaled FP4, merged FP8): 32768 groups per row."""
    M, N = 33, 40
    a = synth.activations(M, K_MAX, seed=3, n_outlier=4, outlier_gain=30.0)
    b = synth.weights(N, K_MAX, seed=4)
    ac, as_ = ref.quantize(a, 32, scale, asym)
    bc, bs = ref.quantize(b, 32, scale, asym)
    C = G.gpu_gemm(ac, as_, bc, bs, scale, asym)
    assert G.rel_fro(C, ref.gemm(ac, as_, bc, bs, 32, scale, asym)) <= 1e-3


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0)])
def test_gemm_most_rows(scale, asym):
    """M = 2^21 - 256 rows (the largest the header allows) against a 33-row operand; sampled rows from the oracle."""
    M, N, K = ROWS_MAX, 33, 32
    rng = np.random.default_rng(5)
    ac = rng.integers(0, 256, size=(M, K // 2), dtype=np.uint8)
    as_ = rng.integers(44, 76, size=(M, 1, 2) if asym else (M, 1), dtype=np.uint8) + (0 if scale == ref.FP8_E5M2 else 60)
    b = synth.weights(N, K, seed=6)
    bc, bs = ref.quantize(b, 32, scale, asym)
    C = G.gpu_gemm(ac, as_.astype(np.uint8), bc, bs, scale, asym)
    assert C.shape == (M, N)
    rows = np.unique(np.concatenate([[0, 1, 255, 256, M - 257, M - 256, M - 1], rng.choice(M, 500, replace=False)]))
    want = ref.gemm(ac[rows], as_[rows].astype(np.uint8), bc, bs, 32, scale, asym)
    assert G.rel_fro(C[rows], want) <= 1e-3
    # and as the second operand (N large)
    Ct = G.gpu_gemm(bc, bs, ac, as_.astype(np.uint8), scale, asym)
    assert G.rel_fro(Ct[:, rows], want.T) <= 1e-3


def test_gemm_largest_batch():
    batch, M, N, K = 65535, 2, 3, 32
    rng = np.random.default_rng(7)
    ac = rng.integers(0, 256, size=(batch, M, K // 2), dtype=np.uint8)
    bc = rng.integers(0, 256, size=(batch, N, K // 2), dtype=np.uint8)
    as_ = rng.integers(44, 76, size=(batch, M, 1, 2), dtype=np.uint8)
    bs = rng.integers(44, 76, size=(batch, N, 1, 2), dtype=np.uint8)
    C = G.gpu_gemm(ac, as_, bc, bs, ref.FP8_E5M2, 1)
    pick = np.unique(np.concatenate([[0, 1, 65534], rng.choice(batch, 300, replace=False)]))
    want = ref.gemm(ac[pick], as_[pick], bc[pick], bs[pick], 32, ref.FP8_E5M2, 1)
    assert G.rel_fro(C[pick], want) <= 1e-3


def test_just_beyond_the_limits_is_rejected():
    fmt = binding.make_format(ref.FP8_E5M2, 1, 32)
    x = torch.zeros((1, K_MAX + 32), dtype=torch.bfloat16, device="cuda")
    with pytest.raises(binding.AmxError, match="maximum"):
        binding.quantize(fmt, x)
