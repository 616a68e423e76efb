"""amxfp4_gemm_static, the GEMM entry point that allocates nothing (its scratch is a static device array inside the
library): through the C ABI, against amxfp4_gemm on the same operands. The two run the same kernels in the same
order, so the results must be identical bit for bit, and both must match the oracle. Two calls in a row, the second
on a smaller problem (the array keeps the first call's contents: nothing stale may leak into the second result)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3


def both_ways(scale, asym, batch, M, N, K, seed):
    a = synth.activations(batch * M, K, seed=seed, n_outlier=2, outlier_gain=60.0)
    b = synth.weights(batch * N, K, seed=seed + 1)
    ac, as_ = ref.quantize(a, 32, scale, asym)
    bc, bs = ref.quantize(b, 32, scale, asym)
    shp = lambda t, r: t.reshape((batch, r) + t.shape[1:]) if batch > 1 else t  # noqa: E731
    ac, as_, bc, bs = shp(ac, M), shp(as_, M), shp(bc, N), shp(bs, N)
    fmt = binding.make_format(scale, asym)
    dev = [G.to_dev_u8(t) for t in (ac, as_, bc, bs)]
    shape = (batch, M, N) if batch > 1 else (M, N)
    # the outputs are the caller's; the static call gets a poisoned one so that an unwritten element shows
    C_static = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda")
    lib = binding.load()
    rc = lib.amxfp4_gemm_static(ctypes.byref(fmt), M, N, K, *(t.data_ptr() for t in dev), C_static.data_ptr(), N,
                                batch, binding._stream())
    assert rc == 0, lib.amxfp4_last_error()
    C_plain = binding.gemm(fmt, *dev)
    torch.cuda.synchronize()
    assert torch.equal(C_static.view(torch.int32), C_plain.view(torch.int32)), "static and workspace calls differ"
    Cr = ref.gemm(ac, as_, bc, bs, 32, scale, asym)
    assert G.rel_fro(C_static.cpu().numpy(), Cr) <= TOL


# (scale, asymmetric, first problem, second, smaller problem): one pair per kernel family that uses scratch
PAIRS = [
    # few-rows kernel: A panel + partial tiles of 4 outer K slices, then one slice
    (ref.FP8_E5M2, 1, (1, 64, 1024, 1024), (1, 5, 70, 512)),
    # BF16-panel kernel: both operands' panels (padded rows and K are rewritten as zeros by every call)
    (ref.FP8_E5M2, 1, (1, 600, 700, 1056), (2, 257, 130, 160)),
    # merged FP6 kernel: merged panels, anchor words, split flags and plan
    (ref.E8M0_FLOOR, 1, (1, 600, 700, 1056), (1, 300, 31, 96)),
    # few rows against a weight-matrix-sized B (32 tokens, 8 MB of weights): the decoding shape this call is for
    (ref.FP8_E5M2, 1, (1, 32, 4096, 4096), (1, 1, 4096, 4096)),
]


@pytest.mark.parametrize("scale,asym,first,second", PAIRS)
def test_static_scratch_gemm_matches_the_workspace_gemm(scale, asym, first, second):
    both_ways(scale, asym, *first, seed=11)
    both_ways(scale, asym, *second, seed=12)


def test_static_scratch_gemm_rejects_what_does_not_fit():
    """The headline product needs 537 MB of panels: refused on the host, nothing launched, the output untouched. The
    same K in the power-of-two symmetric format needs only its re-laid scale bytes and is accepted."""
    lib = binding.load()
    fmt = binding.make_format(binding.FP8_E5M2, True)
    assert binding.gemm_workspace_bytes(fmt, 4096, 28672, 8192) > binding.GEMM_STATIC_BYTES
    out = torch.full((8,), 7.0, device="cuda")
    p = ctypes.c_void_p(out.data_ptr())   # never dereferenced
    rc = lib.amxfp4_gemm_static(ctypes.byref(fmt), 4096, 28672, 8192, p, p, p, p, p, 28672, 1, binding._stream())
    assert rc == -3 and b"static array" in lib.amxfp4_last_error()
    torch.cuda.synchronize()
    assert bool((out == 7.0).all())
    both_ways(ref.E8M0_FLOOR, 0, 1, 4096, 512, 8192, seed=13)
