"""Fully quantized attention matmuls (the attention workload, 32 heads of 128, cut down): Q.K^T grouped along
head_dim, softmax(P).V grouped along the key sequence (P strongly one-sided; V cast along a strided axis), heads as
the GEMM batch."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.FP8_E5M2, 0), (ref.E8M0_FLOOR, 1), (ref.E8M0_FLOOR, 0)])
def test_attention_matmuls(scale, asym):
    run_attention(3, 256, 128, scale, asym)


@pytest.mark.parametrize("scale,asym", [(ref.FP8_E5M2, 1), (ref.E8M0_FLOOR, 0)])
def test_attention_matmuls_full_sequence(scale, asym):
    """Sequence length and head size of the benchmark configuration (4096, 128), two heads instead of 32 so that the
    host-side softmax and the oracle finish in seconds; per-head shapes and the batched launch are the real ones."""
    run_attention(2, 4096, 128, scale, asym)


def run_attention(heads, seq, d, scale, asym):
    q, k, v = synth.attention_qkv(heads, seq, d, seed=0)
    fmt = binding.make_format(scale, asym)
    ns = (2,) if asym else ()

    # scores: cast Q, K along head_dim (all heads in one call: rows = heads * seq), batched GEMM
    qd, kd = G.to_dev_bf16(q.reshape(heads * seq, d)), G.to_dev_bf16(k.reshape(heads * seq, d))
    qc, qs = binding.quantize(fmt, qd)
    kc, ks = binding.quantize(fmt, kd)
    rqc, rqs = ref.quantize(q.reshape(heads * seq, d), 32, scale, asym)
    rkc, rks = ref.quantize(k.reshape(heads * seq, d), 32, scale, asym)
    assert np.array_equal(qc.cpu().numpy(), rqc) and np.array_equal(qs.cpu().numpy(), rqs)
    assert np.array_equal(kc.cpu().numpy(), rkc) and np.array_equal(ks.cpu().numpy(), rks)
    S = binding.gemm(fmt, qc.view(heads, seq, d // 2), qs.view(heads, seq, d // 32, *ns),
                     kc.view(heads, seq, d // 2), ks.view(heads, seq, d // 32, *ns))
    torch.cuda.synchronize()
    Sr = ref.gemm(rqc.reshape(heads, seq, -1), rqs.reshape(heads, seq, d // 32, *ns),
                  rkc.reshape(heads, seq, -1), rks.reshape(heads, seq, d // 32, *ns), 32, scale, asym)
    assert G.rel_fro(S.cpu().numpy(), Sr) <= 1e-3

    # P.V: P = causal softmax (host, from the BF16 Q and K), cast along the key axis; V cast down its columns per head
    p = np.stack([synth.causal_softmax_probs(q[h], k[h]) for h in range(heads)])
    pd = G.to_dev_bf16(p.reshape(heads * seq, seq))
    pc, ps = binding.quantize(fmt, pd)
    rpc, rps = ref.quantize(p.reshape(heads * seq, seq), 32, scale, asym)
    assert np.array_equal(pc.cpu().numpy(), rpc) and np.array_equal(ps.cpu().numpy(), rps)
    if asym:
        assert np.all(rps[..., 1] == 0)  # P >= 0: the negative scale is never used

    vd = G.to_dev_bf16(v.reshape(heads * seq, d)).view(heads, seq, d)
    vc = torch.empty((heads, d, seq // 2), dtype=torch.uint8, device="cuda")
    vs = torch.empty((heads, d, seq // 32) + ns, dtype=torch.uint8, device="cuda")
    rvc, rvs = [], []
    for h in range(heads):
        binding.quantize(fmt, vd[h], k_axis=0, codes=vc[h], scales=vs[h])
        c, s = ref.quantize(v[h], 32, scale, asym, k_axis=0)
        rvc.append(c)
        rvs.append(s)
    rvc, rvs = np.stack(rvc), np.stack(rvs)
    assert np.array_equal(vc.cpu().numpy(), rvc) and np.array_equal(vs.cpu().numpy(), rvs)

    O = binding.gemm(fmt, pc.view(heads, seq, seq // 2), ps.view(heads, seq, seq // 32, *ns), vc, vs)
    torch.cuda.synchronize()
    Or = ref.gemm(rpc.reshape(heads, seq, -1), rps.reshape(heads, seq, seq // 32, *ns), rvc, rvs, 32, scale, asym)
    assert O.shape == (heads, seq, d)
    assert G.rel_fro(O.cpu().numpy(), Or) <= 1e-3
