"""Parity at the full benchmark sizes, through the same calls and launch configuration bench.py times (cast of X into
preallocated buffers + GEMM with a caller workspace): the casts are compared bit for bit over the whole tensors, the
GEMM on sampled rows (all N columns) and sampled columns (all M rows) that the oracle computes from operands it
quantized itself."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3
N_SAMPLE = 48


def run_full(name, scale, asym, seed=0):
    cfg = synth.CONFIGS[name]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    x, w = synth.linear_operands(name, seed=seed)
    fmt = binding.make_format(scale, asym)
    xd, wd = G.to_dev_bf16(x), G.to_dev_bf16(w)
    nsc = (2,) if asym else ()
    xc = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    xs = torch.empty((M, K // 32) + nsc, dtype=torch.uint8, device="cuda")
    binding.quantize(fmt, xd, codes=xc, scales=xs)
    wc, ws = binding.quantize(fmt, wd)
    need = binding.gemm_workspace_bytes(fmt, M, N, K)
    work = torch.empty(need, dtype=torch.uint8, device="cuda") if need else None
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    binding.gemm(fmt, xc, xs, wc, ws, out=C, workspace=work)
    torch.cuda.synchronize()

    rxc, rxs = ref.quantize(x, 32, scale, asym)
    rwc, rws = ref.quantize(w, 32, scale, asym)
    assert np.array_equal(xc.cpu().numpy(), rxc) and np.array_equal(xs.cpu().numpy(), rxs)
    assert np.array_equal(wc.cpu().numpy(), rwc) and np.array_equal(ws.cpu().numpy(), rws)

    rng = np.random.default_rng(seed + 1)
    rows = np.sort(rng.choice(M, min(N_SAMPLE, M), replace=False))
    cols = np.sort(rng.choice(N, N_SAMPLE, replace=False))
    # include the corners of the tile grid: first / last row and column
    rows[0], rows[-1], cols[0], cols[-1] = 0, M - 1, 0, N - 1
    Ch = C.cpu().numpy()
    Cr_rows = ref.gemm(rxc[rows], rxs[rows], rwc, rws, 32, scale, asym)
    Cr_cols = ref.gemm(rxc, rxs, rwc[cols], rws[cols], 32, scale, asym)
    assert G.rel_fro(Ch[rows], Cr_rows) <= TOL
    assert G.rel_fro(Ch[:, cols], Cr_cols) <= TOL
    # no row or column of the sample may be off as a whole (a misplaced tile would hide in a global norm)
    for i in range(len(rows)):
        assert G.rel_fro(Ch[rows[i]], Cr_rows[i]) <= 10 * TOL
    for i in range(N_SAMPLE):
        assert G.rel_fro(Ch[:, cols[i]], Cr_cols[:, i]) <= 10 * TOL


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0)])
def test_c3_up_projection_full_size(scale, asym):
    """The headline workload X[4096 x 8192] . W[28672 x 8192]^T: the paper's AMXFP4 (BF16 MFMA path) and OCP MXFP4
    (block-scaled FP4 MFMA path)."""
    run_full("c3_70b_up_4096x8192x28672", scale, asym)


def test_c3_down_projection_full_size():
    """X[4096 x 28672] (GLU-shaped, one-sided) . W[8192 x 28672]^T, K = 28672 = 224 stages of 128."""
    run_full("c3_70b_down_4096x28672x8192", ref.FP8_E5M2, 1)


@pytest.mark.parametrize("name,scale,asym", [("c3_70b_up_32tokens_32x8192x28672", ref.FP8_E5M2, 1),
                                             ("c3_70b_up_32tokens_32x8192x28672", ref.E8M0_FLOOR, 0),
                                             ("c3_70b_down_32tokens_32x28672x8192", ref.FP8_E5M2, 1)])
def test_c3_projections_with_32_tokens_full_size(name, scale, asym):
    """32 tokens against the 70B projections (the few-rows kernel, weights read as packed codes; two waves per column
    tile, one and several K slices): every row, sampled columns."""
    run_full(name, scale, asym)
