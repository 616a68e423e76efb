"""amxfp4_gemm_prepared: the product against weights whose kernel-private form was written once. Same kernels as
amxfp4_gemm, so the results must be bit-identical to it (and within the GEMM tolerance of the oracle)."""
import ctypes

import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3

FORMATS = [(ref.FP8_E5M2, 1, 32), (ref.FP8_E5M2, 0, 32), (ref.FP8_E4M3, 1, 16), (ref.E8M0_FLOOR, 0, 64),
           (ref.E8M0_FLOOR, 0, 32), (ref.E8M0_FLOOR, 1, 32)]


@pytest.mark.parametrize("scale,asym,gs", FORMATS)
@pytest.mark.parametrize("M,N,K", [(600, 700, 1088), (300, 130, 192), (2048, 512, 4096), (32, 512, 512), (257, 64, 256)])
def test_prepared_product_is_the_plain_product(M, N, K, scale, asym, gs):
    """Shapes with partial tiles and K tails, a long K, few rows (the kernel that reads B as packed codes ignores the
    prepared form) and formats with nothing to prepare (power-of-two scales of 32-groups: zero bytes)."""
    if K % gs:
        pytest.skip("K not a multiple of the group size")
    a = synth.activations(M, K, seed=M + K, n_outlier=2, outlier_gain=60.0)
    b = synth.weights(N, K, seed=N)
    ac, as_ = ref.quantize(a, gs, scale, asym)
    bc, bs = ref.quantize(b, gs, scale, asym)
    fmt = binding.make_format(scale, asym, gs)
    dac, das, dbc, dbs = (G.to_dev_u8(t) for t in (ac, as_, bc, bs))
    prepared = binding.prepare_weights(fmt, dbc, dbs)
    pot32 = gs == 32 and scale in (ref.E8M0_FLOOR, ref.E8M0_ROUND)
    assert (prepared.numel() == 0) == pot32
    plain = binding.gemm(fmt, dac, das, dbc, dbs)
    torch.cuda.synchronize()
    dbc_in = dbc
    if prepared.numel() and M > 768:
        # a large product must not read the canonical codes of B at all: hand it garbage in their place
        dbc_in = torch.randint(0, 256, dbc.shape, dtype=torch.uint8, device="cuda")
    got = binding.gemm_prepared(fmt, dac, das, dbc_in, dbs, prepared)
    again = binding.gemm_prepared(fmt, dac, das, dbc_in, dbs, prepared)   # the prepared form is not consumed
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int32), plain.view(torch.int32))
    assert torch.equal(again.view(torch.int32), plain.view(torch.int32))
    assert G.rel_fro(got.cpu().numpy(), ref.gemm(ac, as_, bc, bs, gs, scale, asym)) <= TOL


def test_prepared_workspace_is_the_activations_panel_only():
    fmt = binding.make_format(ref.FP8_E5M2, 1, 32)
    L = binding.load()
    M, N, K = 4096, 28672, 8192
    full = binding.gemm_workspace_bytes(fmt, M, N, K)
    prep = int(L.amxfp4_weights_prepared_bytes(ctypes.byref(fmt), N, K))
    ws = int(L.amxfp4_gemm_prepared_workspace_bytes(ctypes.byref(fmt), M, N, K))
    assert prep == N * K * 2 and ws == M * K * 2 and ws + prep == full
    pot = binding.make_format(ref.E8M0_FLOOR, 0, 32)
    assert int(L.amxfp4_weights_prepared_bytes(ctypes.byref(pot), N, K)) == 0
    assert int(L.amxfp4_gemm_prepared_workspace_bytes(ctypes.byref(pot), M, N, K)) == binding.gemm_workspace_bytes(pot, M, N, K)


def test_prepared_argument_errors():
    fmt = binding.make_format(ref.FP8_E5M2, 1, 32)
    L = binding.load()
    M, N, K = 300, 512, 256
    z = lambda *s: torch.zeros(s, dtype=torch.uint8, device="cuda")  # noqa: E731
    ac, as_, bc, bs = z(M, K // 2), z(M, K // 32, 2), z(N, K // 2), z(N, K // 32, 2)
    need = int(L.amxfp4_weights_prepared_bytes(ctypes.byref(fmt), N, K))
    small = z(need - 256)
    assert L.amxfp4_prepare_weights(ctypes.byref(fmt), N, K, bc.data_ptr(), bs.data_ptr(), small.data_ptr(),
                                    small.numel(), None) == -3
    assert L.amxfp4_prepare_weights(ctypes.byref(fmt), N, K, None, bs.data_ptr(), small.data_ptr(), need,
                                    None) == -1
    out = torch.empty((M, N), dtype=torch.float32, device="cuda")
    ws = z(int(L.amxfp4_gemm_prepared_workspace_bytes(ctypes.byref(fmt), M, N, K)))
    rc = L.amxfp4_gemm_prepared(ctypes.byref(fmt), M, N, K, ac.data_ptr(), as_.data_ptr(), bc.data_ptr(), bs.data_ptr(),
                                small.data_ptr(), small.numel(), out.data_ptr(), N, ws.data_ptr(), ws.numel(), None)
    assert rc == -3
    rc = L.amxfp4_gemm_prepared(ctypes.byref(fmt), M, N, K, ac.data_ptr(), as_.data_ptr(), bc.data_ptr(), bs.data_ptr(),
                                None, 0, out.data_ptr(), N, ws.data_ptr(), ws.numel(), None)
    assert rc == -3
    torch.cuda.synchronize()
