"""Attention workload (32 heads, sequence 4096, head size 128 by default; synthetic Q, K, V with outlier head
dimensions): the two quantized products of Sec. 5.1 timed two ways on one GPU,
  materialised: cast Q, K -> Q.K^T (FP32 scores) -> causal softmax (BF16 map) -> cast map and V -> map . V
  fused:        cast Q, K, V -> amxfp4_attention (online softmax, probability tiles cast in registers)
and the two outputs compared with the exact softmax attention of the BF16 inputs. Prints one JSON line.

    python -m paper_2411_09909_amd.attention_bench [--heads 32 --kv-heads 32 --seq 4096 --steps 10 --format amxfp4_e5m2]
"""
import argparse
import json
import math
import time

import numpy as np
import torch

from . import binding, synth

FORMATS = {"amxfp4_e5m2": (2, True), "mxfp4_e5m2": (2, False), "amxfp4_e8m0": (0, True), "mxfp4_e8m0": (0, False)}


def timed(fn, steps):
    fn()
    torch.cuda.synchronize()
    t0 = time.perf_counter()
    for _ in range(steps):
        fn()
    torch.cuda.synchronize()
    return (time.perf_counter() - t0) / steps * 1e3


def run(heads=32, kv_heads=32, seq=4096, steps=10, fmt_name="amxfp4_e5m2", no_materialised=False):
    """Returns the dictionary main() prints."""
    import types
    return _run(types.SimpleNamespace(heads=heads, kv_heads=kv_heads, seq=seq, steps=steps, format=fmt_name,
                                      no_materialised=no_materialised))


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--heads", type=int, default=32)
    ap.add_argument("--kv-heads", type=int, default=32)
    ap.add_argument("--seq", type=int, default=4096)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--format", default="amxfp4_e5m2", choices=sorted(FORMATS))
    ap.add_argument("--no-materialised", action="store_true", help="time the fused call only")
    print(json.dumps(_run(ap.parse_args())))


def _run(args):
    H, G, S, D = args.heads, args.kv_heads, args.seq, 128
    per = H // G
    dev = torch.device("cuda:0")
    binding.load()
    kind, asym = FORMATS[args.format]
    fmt = binding.make_format(kind, asym)
    ns = (2,) if asym else ()
    qb, _, _ = synth.attention_qkv(H, S, D, seed=0)
    _, kb, vb = synth.attention_qkv(G, S, D, seed=1)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)  # noqa: E731
    q, k, v = to_dev(qb), to_dev(kb), to_dev(vb)
    scale = 1.0 / math.sqrt(D)

    qc = torch.empty((H * S, D // 2), dtype=torch.uint8, device=dev)
    qs = torch.empty((H * S, D // 32) + ns, dtype=torch.uint8, device=dev)
    kc = torch.empty((G * S, D // 2), dtype=torch.uint8, device=dev)
    ks = torch.empty((G * S, D // 32) + ns, dtype=torch.uint8, device=dev)
    vc = torch.empty((G, D, S // 2), dtype=torch.uint8, device=dev)
    vs = torch.empty((G, D, S // 32) + ns, dtype=torch.uint8, device=dev)

    def cast_qkv():
        binding.quantize(fmt, q.view(H * S, D), codes=qc, scales=qs)
        binding.quantize(fmt, k.view(G * S, D), codes=kc, scales=ks)
        binding.quantize_batched(fmt, v, k_axis=1, codes=vc, scales=vs)  # every head's V down its keys, one launch

    out_f = torch.empty((H, S, D), dtype=torch.float32, device=dev)
    ws_f = torch.empty(binding.attention_workspace_bytes(fmt, H, G, S, S, D), dtype=torch.uint8, device=dev)
    qa = (qc.view(H, S, D // 2), qs.view(H, S, D // 32, *ns), kc.view(G, S, D // 2), ks.view(G, S, D // 32, *ns))

    def fused():
        binding.attention(fmt, *qa, vc, vs, scale, True, out=out_f, workspace=ws_f)

    cast_qkv()
    res = {"workload": "c4_attention", "heads": H, "kv_heads": G, "seq": S, "head_dim": D, "format": args.format,
           "causal": True, "data": "synthetic", "flops_full": 4.0 * H * S * S * D}
    res["cast_qkv_ms"] = round(timed(cast_qkv, args.steps), 4)
    res["fused_ms"] = round(timed(fused, args.steps), 4)
    res["fused_TFLOPs_causal"] = round(2.0 * H * S * S * D / (res["fused_ms"] * 1e-3) / 1e12, 1)

    # exact attention of the BF16 inputs, one query head at a time
    def exact(h):
        s = (q[h].float() @ k[h // per].float().T) * scale
        s = s.masked_fill(torch.ones(S, S, dtype=torch.bool, device=dev).triu(1), float("-inf"))
        return torch.softmax(s, dim=-1) @ v[h // per].float()

    def rel_err(o):
        num = den = 0.0
        for h in range(0, H, max(1, H // 4)):
            e = exact(h)
            num += (o[h] - e).pow(2).sum().item()
            den += e.pow(2).sum().item()
        return math.sqrt(num / den)

    fused()
    res["fused_rel_err_vs_exact"] = round(rel_err(out_f), 5)

    if not args.no_materialised:
        scores = torch.empty((G, per * S, S), dtype=torch.float32, device=dev)
        o = torch.empty((G, per * S, D), dtype=torch.float32, device=dev)
        pc = torch.empty((G * per * S, S // 2), dtype=torch.uint8, device=dev)
        ps = torch.empty((G * per * S, S // 32) + ns, dtype=torch.uint8, device=dev)
        need = max(binding.gemm_workspace_bytes(fmt, per * S, S, D, G), binding.gemm_workspace_bytes(fmt, per * S, D, S, G), 1)
        ws = torch.empty(need, dtype=torch.uint8, device=dev)
        ga = (qc.view(G, per * S, D // 2), qs.view(G, per * S, D // 32, *ns), kc.view(G, S, D // 2),
              ks.view(G, S, D // 32, *ns))
        state = {}

        def qk():
            binding.gemm(fmt, *ga, out=scores, workspace=ws)

        def softmax():
            state["p"] = binding.softmax_causal(scores, scale)

        def cast_p():
            binding.quantize(fmt, state["p"].view(G * per * S, S), codes=pc, scales=ps)

        def pv():
            binding.gemm(fmt, pc.view(G, per * S, S // 2), ps.view(G, per * S, S // 32, *ns), vc, vs, out=o, workspace=ws)

        parts = {}
        for name, fn in (("qk_gemm", qk), ("softmax", softmax), ("cast_map", cast_p), ("pv_gemm", pv)):
            parts[name] = round(timed(fn, args.steps), 4)
        res["materialised_ms"] = parts
        res["materialised_total_ms"] = round(sum(parts.values()), 4)
        res["materialised_rel_err_vs_exact"] = round(rel_err(o.view(H, S, D)), 5)
        res["speedup_fused"] = round(res["materialised_total_ms"] / res["fused_ms"], 2)
    return res


if __name__ == "__main__":
    main()
