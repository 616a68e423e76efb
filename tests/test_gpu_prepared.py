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
@pytest.mark.parametrize("M,N,K", [(600, 700, 1088), (300, 130, 192), (2048, 512, 4096), (32, 512, 512), (257, 64, 256),
                                   (300, 290, 32), (1100, 260, 448)])
def test_prepared_product_is_the_plain_product(M, N, K, scale, asym, gs):
    """Shapes with partial tiles and K tails, a long K, few rows (the kernel that reads B as packed codes ignores the
    prepared form) and a format with nothing to prepare (symmetric power-of-two scales of 32-groups: zero bytes). The
    asymmetric power-of-two format prepares B's merged FP6 panel; its activations carry outlier channels, so some
    positions of A are split and B's blocks are repeated through the table."""
    if K % gs:
        pytest.skip("K not a multiple of the group size")
    a = synth.activations(M, K, seed=M + K, n_outlier=2, outlier_gain=60.0)
    b = synth.weights(N, K, seed=N)
    ac, as_ = ref.quantize(a, gs, scale, asym)
    bc, bs = ref.quantize(b, gs, scale, asym)
    fmt = binding.make_format(scale, asym, gs)
    dac, das, dbc, dbs = (G.to_dev_u8(t) for t in (ac, as_, bc, bs))
    prepared = binding.prepare_weights(fmt, dbc, dbs)
    nothing = gs == 32 and scale in (ref.E8M0_FLOOR, ref.E8M0_ROUND) and not asym
    assert (prepared.numel() == 0) == nothing
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
    apot = binding.make_format(ref.E8M0_FLOOR, 1, 32)
    # B alone: at most two 6-bit blocks per position (1.5 bytes per element) plus anchors and plan; the call's
    # workspace then holds A's worst case only
    prep = int(L.amxfp4_weights_prepared_bytes(ctypes.byref(apot), N, K))
    assert 1.5 * N * K < prep < 1.65 * N * K
    assert int(L.amxfp4_gemm_prepared_workspace_bytes(ctypes.byref(apot), M, N, K)) < 0.25 * binding.gemm_workspace_bytes(apot, M, N, K)


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


@pytest.mark.parametrize("gaps_a,gaps_b", [((0, 1, 2, 3, 4, 5), (5, 4, 3, 2, 1, 0)),      # nothing split
                                           ((0, 6, 3, 9, 5, 20), (0, 0, 1, 2, 3, 4)),      # A split at some positions
                                           ((1, 2, 3), (0, 7, 5, 30, 2)),                  # B split
                                           ((6, 0, 7, 2, 40, 5), (8, 0, 1, 6, 9, 5))])     # both, together and apart
def test_prepared_fp6_weights_with_split_positions(gaps_a, gaps_b):
    """The merged FP6 kernel on a prepared B: B's panel holds B's own blocks (one per position, two where a row of B
    leaves the window) and the call's table says which of them stands at each block of the lengthened K: repeated where
    only A is split, alternating (b+, b-, b+, b-) where both are. Same blocks in the same order as the unprepared
    kernel builds: bit-identical, and within FP32 accumulation accuracy of the oracle."""
    from tests.test_gpu_fp6_merged import hand_made
    rng = np.random.default_rng(11)
    M, N, K = 300, 290, 32 * 25
    ac, as_ = hand_made(M, K, rng, gaps_a)
    bc, bs = hand_made(N, K, rng, gaps_b)
    fmt = binding.make_format(ref.E8M0_FLOOR, 1, 32)
    dac, das, dbc, dbs = (G.to_dev_u8(t) for t in (ac, as_, bc, bs))
    prepared = binding.prepare_weights(fmt, dbc, dbs)
    plain = binding.gemm(fmt, dac, das, dbc, dbs, options=binding.gemm_options(few_rows=-1))
    garbage = torch.randint(0, 256, dbc.shape, dtype=torch.uint8, device="cuda")   # B's codes must not be read
    got = binding.gemm_prepared(fmt, dac, das, garbage, dbs, prepared)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int32), plain.view(torch.int32))
    assert G.rel_fro(got.cpu().numpy(), ref.gemm(ac, as_, bc, bs, 32, ref.E8M0_FLOOR, 1)) <= 2e-6


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 1), (ref.E8M0_FLOOR, 0)])
def test_prepared_gated_gemm(scale, asym):
    """amxfp4_gemm_silu_mul_prepared against the plain gated GEMM: the same bits."""
    M, width, K = 300, 160, 1088 if scale == ref.FP8_E5M2 else 1024
    a = synth.activations(M, K, seed=M, n_outlier=2, outlier_gain=60.0)
    wg, wu = synth.weights(width, K, seed=3), synth.weights(width, K, seed=4)
    fmt = binding.make_format(scale, asym)
    ac, as_ = binding.quantize(fmt, G.to_dev_bf16(a))
    inter = binding.interleave_gate_up(G.to_dev_bf16(wg), G.to_dev_bf16(wu)).contiguous()
    ic, is_ = binding.quantize(fmt, inter)
    prepared = binding.prepare_weights(fmt, ic, is_)
    plain = binding.gemm_silu_mul(fmt, ac, as_, ic, is_)
    got = binding.gemm_silu_mul(fmt, ac, as_, ic, is_, prepared=prepared)
    torch.cuda.synchronize()
    assert torch.equal(got.view(torch.int16), plain.view(torch.int16))
