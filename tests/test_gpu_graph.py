"""The library allocates nothing, clears nothing with memset and keeps no state between calls, so a sequence of its
calls can be captured into a HIP graph and replayed: cast + GEMM of a launch-bound shape, the tensor-scaled chain (whose
scale pair is produced and consumed on the device) and the fused attention. Every replay runs on new input data, with
eager work and synchronisations between the replays, and is compared with the eager result of the same calls."""
import numpy as np
import pytest
import torch

from oracle import ref
from paper_2411_09909_amd import binding, synth
from tests import gpu_util as G

pytestmark = pytest.mark.gpu


def replay_and_compare(build_inputs, run, outputs, n_replays=3):
    """build_inputs(i) refreshes the static input tensors for trial i; run() issues the library calls; outputs() lists
    the tensors to compare."""
    build_inputs(0)
    side = torch.cuda.Stream()
    side.wait_stream(torch.cuda.current_stream())
    with torch.cuda.stream(side):
        run()  # warm-up outside the capture (module loads)
    torch.cuda.current_stream().wait_stream(side)
    torch.cuda.synchronize()
    graph = torch.cuda.CUDAGraph()
    with torch.cuda.graph(graph):
        run()
    for i in range(1, n_replays + 1):
        build_inputs(i)
        graph.replay()
        torch.cuda.synchronize()
        got = [t.clone() for t in outputs()]
        for t in outputs():
            t.zero_()
        run()  # eager, same inputs
        torch.cuda.synchronize()
        for a, b in zip(got, outputs()):
            assert torch.equal(a, b), "replay %d differs from the eager run" % i


def test_cast_and_gemm_in_a_graph():
    M, N, K = 64, 1024, 1024
    fmt = binding.make_format(ref.FP8_E5M2, 1)
    _, w = synth.linear_operands("c1_linear_64x1024x1024")
    wc, ws = binding.quantize(fmt, G.to_dev_bf16(w))
    x = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    xc = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    xs = torch.empty((M, K // 32, 2), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    work = torch.empty(binding.gemm_workspace_bytes(fmt, M, N, K), dtype=torch.uint8, device="cuda")

    def build(i):
        x.copy_(G.to_dev_bf16(synth.activations(M, K, seed=100 + i, n_outlier=4, outlier_gain=30.0)))

    def run():
        binding.quantize(fmt, x, codes=xc, scales=xs)
        binding.gemm(fmt, xc, xs, wc, ws, out=C, workspace=work)

    replay_and_compare(build, run, lambda: [xc, xs, C])
    # and the last replayed result against the oracle
    xb = x.view(torch.int16).cpu().numpy().view(np.uint16)
    rc, rs = ref.quantize(xb, 32, ref.FP8_E5M2, 1)
    want = ref.gemm(rc, rs, wc.cpu().numpy(), ws.cpu().numpy(), 32, ref.FP8_E5M2, 1)
    assert G.rel_fro(C.cpu().numpy(), want) <= 1e-3


def test_tensor_scaled_chain_in_a_graph():
    M, N, K = 96, 160, 256
    fmt = binding.make_format(ref.FP8_E4M3, 1, 16)
    a = torch.empty((M, K), dtype=torch.bfloat16, device="cuda")
    b = G.to_dev_bf16(synth.weights(N, K, seed=3))
    pb = binding.tensor_scale(b)
    bc, bs = binding.quantize(fmt, b, tensor_pair=pb)
    pa = torch.empty(2, dtype=torch.float32, device="cuda")
    ac = torch.empty((M, K // 2), dtype=torch.uint8, device="cuda")
    as_ = torch.empty((M, K // 16, 2), dtype=torch.uint8, device="cuda")
    C = torch.empty((M, N), dtype=torch.float32, device="cuda")
    work = torch.empty(binding.load().amxfp4_gemm_scaled_workspace_bytes(__import__("ctypes").byref(fmt), M, N, K, 1), dtype=torch.uint8, device="cuda")

    def build(i):
        bits = synth.activations(M, K, seed=200 + i, n_outlier=2, outlier_gain=20.0)
        a.copy_(G.to_dev_bf16(synth.f32_to_bf16_bits(synth.bf16_bits_to_f32(bits) * np.float32(10.0 ** (-2 * i)))))

    def run():
        binding.tensor_scale(a, out=pa)
        binding.quantize(fmt, a, codes=ac, scales=as_, tensor_pair=pa)
        binding.gemm(fmt, ac, as_, bc, bs, out=C, workspace=work, a_pair=pa, b_pair=pb)

    replay_and_compare(build, run, lambda: [pa, ac, as_, C])


def test_fused_attention_in_a_graph():
    H, S, D = 2, 160, 128
    fmt = binding.make_format(ref.FP8_E5M2, 1)
    q = torch.empty((H * S, D), dtype=torch.bfloat16, device="cuda")
    _, kb, vb = synth.attention_qkv(H, S, D, seed=5)
    kc, ks = binding.quantize(fmt, G.to_dev_bf16(kb.reshape(H * S, D)))
    vd = G.to_dev_bf16(vb.reshape(H * S, D)).view(H, S, D)
    vcs = [binding.quantize(fmt, vd[h], k_axis=0) for h in range(H)]
    vc, vs = torch.stack([t[0] for t in vcs]), torch.stack([t[1] for t in vcs])
    qc = torch.empty((H * S, D // 2), dtype=torch.uint8, device="cuda")
    qs = torch.empty((H * S, D // 32, 2), dtype=torch.uint8, device="cuda")
    out = torch.empty((H, S, D), dtype=torch.float32, device="cuda")
    work = torch.empty(binding.attention_workspace_bytes(fmt, H, H, S, S, D), dtype=torch.uint8, device="cuda")

    def build(i):
        qb, _, _ = synth.attention_qkv(H, S, D, seed=300 + i)
        q.copy_(G.to_dev_bf16(qb.reshape(H * S, D)))

    def run():
        binding.quantize(fmt, q, codes=qc, scales=qs)
        binding.attention(fmt, qc.view(H, S, -1), qs.view(H, S, D // 32, 2), kc.view(H, S, -1), ks.view(H, S, D // 32, 2),
                          vc, vs, D ** -0.5, True, out=out, workspace=work)

    replay_and_compare(build, run, lambda: [qc, out])
