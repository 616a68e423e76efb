"""Decoding-shaped attention: a few new queries per sequence against a long key / value cache (synthetic Q, K, V with
outlier head dimensions, already cast: a cache holds codes and scales). Times amxfp4_attention_decode (K and V read as
packed codes, keys cut into ranges) for several numbers of ranges, beside amxfp4_attention on the same operands (which
expands K and V to BF16 panels on every call). A batch of sequences is a larger number of heads. Prints one JSON line.

    python -m paper_2411_09909_amd.decode_bench [--batch 1 --heads 32 --kv-heads 8 --keys 8192 --queries 1]
"""
import argparse
import json
import math

import numpy as np
import torch

from . import binding, synth
from .attention_bench import FORMATS, timed


def run(batch=1, heads=32, kv_heads=8, keys=8192, queries=1, steps=50, fmt_name="amxfp4_e5m2", splits=None):
    """Times the decode call for each number of key ranges in `splits` (default: a sweep) and the many-queries kernel
    on the same operands; returns the dictionary main() prints."""
    import types
    args = types.SimpleNamespace(batch=batch, heads=heads, kv_heads=kv_heads, keys=keys, queries=queries, steps=steps,
                                 format=fmt_name)
    return _run(args, splits)


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--batch", type=int, default=1, help="sequences (each with its own heads and cache)")
    ap.add_argument("--heads", type=int, default=32)
    ap.add_argument("--kv-heads", type=int, default=8)
    ap.add_argument("--keys", type=int, default=8192)
    ap.add_argument("--queries", type=int, default=1)
    ap.add_argument("--steps", type=int, default=50)
    ap.add_argument("--format", default="amxfp4_e5m2", choices=sorted(FORMATS))
    print(json.dumps(_run(ap.parse_args(), None)))


def _run(args, splits_wanted):
    H, G, Sk, Sq, D = args.batch * args.heads, args.batch * args.kv_heads, args.keys, args.queries, 128
    dev = torch.device("cuda:0")
    binding.load()
    kind, asym = FORMATS[args.format]
    fmt = binding.make_format(kind, asym)
    ns = (2,) if asym else ()
    qb, _, _ = synth.attention_qkv(H, Sq, D, seed=0)
    _, kb, vb = synth.attention_qkv(G, Sk, D, seed=1)
    to_dev = lambda a: torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16)  # noqa: E731
    qc, qs = binding.quantize(fmt, to_dev(qb).view(H * Sq, D))
    kc, ks = binding.quantize(fmt, to_dev(kb).view(G * Sk, D))
    vc, vs = binding.quantize_batched(fmt, to_dev(vb), k_axis=1)
    ops = (qc.view(H, Sq, D // 2), qs.view(H, Sq, D // 32, *ns), kc.view(G, Sk, D // 2), ks.view(G, Sk, D // 32, *ns),
           vc, vs)
    scale = 1.0 / math.sqrt(D)
    cache_bytes = sum(t.numel() for t in (kc, ks, vc, vs))
    res = {"workload": "decode_attention", "batch": args.batch, "heads": args.heads, "kv_heads": args.kv_heads,
           "keys": Sk, "queries": Sq, "head_dim": D, "format": args.format, "data": "synthetic",
           "cache_MB": round(cache_bytes / 1e6, 2), "decode": {}}
    out = torch.empty((H, Sq, D), dtype=torch.float32, device=dev)
    tiles = Sk // 32
    for splits in sorted(set(splits_wanted or (1, 4, 16, 32, 64, 128, 256)) & set(range(1, tiles + 1))):
        ws = torch.empty(max(256, G * splits * 32 * (D + 2) * 4), dtype=torch.uint8, device=dev)
        ms = timed(lambda: binding.attention_decode(fmt, *ops, scale, True, key_splits=splits, out=out, workspace=ws),
                   args.steps)
        res["decode"][str(splits)] = {"us": round(ms * 1e3, 1), "cache_GB_per_s": round(cache_bytes / (ms * 1e-3) / 1e9, 1),
                                      "waves": G * splits}
    ws = torch.empty(binding.attention_workspace_bytes(fmt, H, G, Sq, Sk, D), dtype=torch.uint8, device=dev)
    ms = timed(lambda: binding.attention(fmt, *ops, scale, True, out=out, workspace=ws), args.steps)
    res["many_queries_kernel_us"] = round(ms * 1e3, 1)
    return res


if __name__ == "__main__":
    main()
