"""Parity at the shapes the benchmark configurations name, not cut-downs of them: the LLaMA-7B-shaped prefill linears
in full (every element of C against the oracle), the attention products with all 32 heads in one batched launch
(sampled heads against the oracle), and every workgroup tile shape of the BF16-panel kernel forced per call. The
launch configuration is the library's own choice for these shapes (what a benchmark run times) unless a test says
otherwise."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu

TOL = 1e-3


def check_rows_and_columns(C, Cr, what):
    """Whole-matrix norm, and no single row or column off as a whole (a misplaced tile would hide in a global norm)."""
    err = G.rel_fro(C, Cr)
    assert err <= TOL, "%s: relative Frobenius error %.3g" % (what, err)
    d = (np.asarray(C, np.float64) - Cr) ** 2
    r2 = np.asarray(Cr, np.float64) ** 2
    row = np.sqrt(d.sum(-1) / np.maximum(r2.sum(-1), 1e-300)).max()
    col = np.sqrt(d.sum(-2) / np.maximum(r2.sum(-2), 1e-300)).max()
    assert row <= 10 * TOL and col <= 10 * TOL, "%s: worst row %.3g, worst column %.3g" % (what, row, col)
    return err


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0), (ref.E8M0_FLOOR, 1)])
@pytest.mark.parametrize("name", ["c2_llama7b_qkvo_2048x4096x4096", "c2_llama7b_mlp_up_2048x4096x11008"])
def test_config2_linears_full_matrix(name, scale, asym):
    """X[2048 x 4096] against W[4096 x 4096] (128 tiles of 256 x 256: the panel kernel switches to its 256 x 128 tile)
    and against W[11008 x 4096] (344 tiles, ragged in N: 11008 = 43 * 256). The paper's AMXFP4, OCP MXFP4 and the
    asymmetric power-of-two format: casts bit for bit, the product in full."""
    cfg = synth.CONFIGS[name]
    M, N, K = cfg["M"], cfg["N"], cfg["K"]
    x, w = synth.linear_operands(name, seed=0)
    fmt = binding.make_format(scale, asym)
    xc, xs = binding.quantize(fmt, G.to_dev_bf16(x))
    wc, ws = binding.quantize(fmt, G.to_dev_bf16(w))
    C = binding.gemm(fmt, xc, xs, wc, ws)
    torch.cuda.synchronize()
    rxc, rxs = ref.quantize(x, 32, scale, asym)
    rwc, rws = ref.quantize(w, 32, scale, asym)
    assert np.array_equal(xc.cpu().numpy(), rxc) and np.array_equal(xs.cpu().numpy(), rxs)
    assert np.array_equal(wc.cpu().numpy(), rwc) and np.array_equal(ws.cpu().numpy(), rws)
    Cr = ref.gemm(rxc, rxs, rwc, rws, 32, scale, asym)
    assert C.shape == (M, N)
    err = check_rows_and_columns(C.cpu().numpy(), Cr, name)
    print("%s scale %d asym %d: rel. Frobenius error %.3g" % (name, scale, asym, err))


HEADS, SEQ, D = 32, 4096, 128
SAMPLED_HEADS = (0, 13, 31)


@pytest.fixture(scope="module")
def attention_inputs():
    """Q, K, V of the attention configuration (32 heads, 4096 tokens, head size 128) and the BF16 causal softmax map of
    every head (1 GiB on the host), drawn once for all formats."""
    q, k, v = synth.attention_qkv(HEADS, SEQ, D, seed=0)
    p = np.empty((HEADS, SEQ, SEQ), np.uint16)
    for h in range(HEADS):
        p[h] = synth.causal_softmax_probs(q[h], k[h])
    return q, k, v, p


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0), (ref.E8M0_FLOOR, 1)])
def test_config4_attention_products_all_heads(attention_inputs, scale, asym):
    """Both attention products with the 32 heads as the batch of ONE launch each, as a benchmark run issues them:
    Q.K^T (8192 tiles of 256 x 256, K = 128) and P.V (M = 4096, N = 128, K = 4096 per head: the panel kernel's
    256 x 128 tile). The casts of the sampled heads are compared bit for bit, their products in full."""
    q, k, v, p = attention_inputs
    fmt = binding.make_format(scale, asym)
    ns = (2,) if asym else ()
    qc, qs = binding.quantize(fmt, G.to_dev_bf16(q.reshape(HEADS * SEQ, D)))
    kc, ks = binding.quantize(fmt, G.to_dev_bf16(k.reshape(HEADS * SEQ, D)))
    S = binding.gemm(fmt, qc.view(HEADS, SEQ, D // 2), qs.view(HEADS, SEQ, D // 32, *ns),
                     kc.view(HEADS, SEQ, D // 2), ks.view(HEADS, SEQ, D // 32, *ns))
    torch.cuda.synchronize()
    for h in SAMPLED_HEADS:
        rq = ref.quantize(q[h], 32, scale, asym)
        rk = ref.quantize(k[h], 32, scale, asym)
        assert np.array_equal(qc.view(HEADS, SEQ, -1)[h].cpu().numpy(), rq[0])
        assert np.array_equal(ks.view(HEADS, SEQ, D // 32, *ns)[h].cpu().numpy(), rk[1])
        check_rows_and_columns(S[h].cpu().numpy(), ref.gemm(*rq, *rk, 32, scale, asym), "scores of head %d" % h)
    del S

    pd = G.to_dev_bf16(p.reshape(HEADS * SEQ, SEQ))
    pc, ps = binding.quantize(fmt, pd)
    del pd
    vd = G.to_dev_bf16(v.reshape(HEADS * SEQ, D)).view(HEADS, SEQ, D)
    vc, vs = binding.quantize_batched(fmt, vd, k_axis=1)   # every head's V down its keys, one launch
    O = binding.gemm(fmt, pc.view(HEADS, SEQ, SEQ // 2), ps.view(HEADS, SEQ, SEQ // 32, *ns), vc, vs)
    torch.cuda.synchronize()
    assert O.shape == (HEADS, SEQ, D)
    for h in SAMPLED_HEADS:
        rp = ref.quantize(p[h], 32, scale, asym)
        rv = ref.quantize(v[h], 32, scale, asym, k_axis=0)
        assert np.array_equal(pc.view(HEADS, SEQ, -1)[h].cpu().numpy(), rp[0])
        assert np.array_equal(ps.view(HEADS, SEQ, SEQ // 32, *ns)[h].cpu().numpy(), rp[1])
        assert np.array_equal(vc[h].cpu().numpy(), rv[0]) and np.array_equal(vs[h].cpu().numpy(), rv[1])
        err = check_rows_and_columns(O[h].cpu().numpy(), ref.gemm(*rp, *rv, 32, scale, asym), "P.V of head %d" % h)
        print("head %d scale %d asym %d: P.V rel. Frobenius error %.3g" % (h, scale, asym, err))


@pytest.mark.parametrize("tile", ["256x256", "256x128", "64x256"])
@pytest.mark.parametrize("scale,asym,gs", [(ref.FP8_E5M2, 1, 32), (ref.FP8_E4M3, 1, 16), (ref.E8M0_FLOOR, 0, 64)])
@pytest.mark.parametrize("batch,M,N,K", [(1, 600, 700, 1088), (3, 257, 130, 192), (1, 64, 1024, 1024),
                                         (2, 513, 129, 4096)])
def test_every_tile_shape_of_the_panel_kernel(batch, M, N, K, scale, asym, gs, tile):
    """The three workgroup tiles of the BF16-panel kernel, each forced on shapes with partial tiles in M and N, K tails
    (K = 1088, 192: not a multiple of the 128 the panels are padded to), a batch, a K long enough for the ring to wrap
    many times, and group sizes whose scales the expansion indexes differently."""
    a = synth.activations(batch * M, K, seed=M + K, n_outlier=2, outlier_gain=60.0)
    b = synth.weights(batch * N, K, seed=N)
    ac, as_ = ref.quantize(a, gs, scale, asym)
    bc, bs = ref.quantize(b, gs, scale, asym)
    shp = lambda t, r: t.reshape((batch, r) + t.shape[1:]) if batch > 1 else t  # noqa: E731
    ac, as_, bc, bs = shp(ac, M), shp(as_, M), shp(bc, N), shp(bs, N)
    opts = binding.gemm_options(tile=tile, few_rows=-1)
    C = G.gpu_gemm(ac, as_, bc, bs, scale, asym, group_size=gs, options=opts)
    Cr = ref.gemm(ac, as_, bc, bs, gs, scale, asym)
    assert C.shape == Cr.shape
    check_rows_and_columns(C, Cr, "tile %s" % tile)
