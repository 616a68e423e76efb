"""Times one LLaMA-3-8B-shaped decoder layer (d 4096, 32 query / 8 key-value heads of 128, MLP 14336, RMSNorm, rotary
embedding) with every matrix multiplication quantized, and compares its output with a BF16 reference of the same
layer (torch matmuls in BF16, FP32 softmax) on the same random-init weights and synthetic hidden states.

    python -m paper_2411_09909_amd.layer_bench [--seq 8192] [--steps 5]

Prints one JSON object: per format the time of a forward pass, TFLOP/s over the flops the seven quantized matmuls
execute (the fused attention skips key tiles behind the causal mask; the dense-attention credit is listed beside it), and
the mean squared error of the layer output against the BF16 reference (lower is better; the paper's argument is that
the asymmetric scales lower it at equal bit width, Sec. 4.2 / Table 2 for model-level perplexity).
"""
import argparse
import json
import math
import time

import numpy as np
import torch

from . import binding, layer, synth

FORMATS = {"amxfp4_e5m2": (binding.FP8_E5M2, True), "mxfp4_e5m2": (binding.FP8_E5M2, False),
           "amxfp4_e8m0": (binding.E8M0_FLOOR, True), "mxfp4_e8m0": (binding.E8M0_FLOOR, False)}


def bf16_reference(x, w, cfg, chunk_heads=4):
    """The same layer without quantization: BF16 tensors, torch matmuls (FP32 accumulate), FP32 softmax."""
    S, H, G, D = x.shape[0], cfg.n_heads, cfg.n_kv_heads, cfg.head_dim
    f32 = torch.float32

    def norm(t, g):
        tf = t.to(f32)
        return (tf * torch.rsqrt((tf * tf).mean(-1, keepdim=True) + cfg.eps) * g).to(torch.bfloat16)

    def rope(t):  # [S, heads, D] float32
        half = D // 2
        ang = torch.arange(S, device=t.device, dtype=torch.float64)[:, None] * torch.exp(
            -math.log(cfg.rope_theta) * torch.arange(half, device=t.device, dtype=torch.float64) / half)
        cs, sn = ang.cos().to(f32)[:, None, :], ang.sin().to(f32)[:, None, :]
        t1, t2 = t[..., :half], t[..., half:]
        return torch.cat([t1 * cs - t2 * sn, t2 * cs + t1 * sn], -1)

    h = norm(x, w["norm1"])
    q = rope((h @ w["wq"].T).to(f32).view(S, H, D)).to(torch.bfloat16)
    k = rope((h @ w["wk"].T).to(f32).view(S, G, D)).to(torch.bfloat16)
    v = (h @ w["wv"].T).view(S, G, D)
    attn = torch.empty((S, H * D), dtype=torch.bfloat16, device=x.device)
    mask = torch.ones((S, S), dtype=torch.bool, device=x.device).tril()
    for h0 in range(0, H, chunk_heads):
        for hh in range(h0, min(H, h0 + chunk_heads)):
            g = hh // (H // G)
            s = (q[:, hh] @ k[:, g].T).to(f32) / math.sqrt(D)
            p = torch.softmax(s.masked_fill(~mask, float("-inf")), -1).to(torch.bfloat16)
            attn[:, hh * D:(hh + 1) * D] = p @ v[:, g]
    x2 = (x.to(f32) + (attn @ w["wo"].T).to(f32)).to(torch.bfloat16)
    h2 = norm(x2, w["norm2"])
    act = (torch.nn.functional.silu((h2 @ w["wg"].T).to(f32)) * (h2 @ w["wu"].T).to(f32)).to(torch.bfloat16)
    return (x2.to(f32) + (act @ w["wd"].T).to(f32)).to(torch.bfloat16)


def run(seq=8192, steps=5, formats=tuple(FORMATS), fused_attention=True, separate_norm=False, prepared_weights=False):
    """Times the layer in each format; returns the dictionary main() prints."""
    cfg = layer.LayerConfig()
    dev = torch.device("cuda:0")
    binding.load()
    w_host = synth.layer_weights(cfg, seed=0)
    to_dev = lambda a: (torch.from_numpy(a).to(dev) if a.dtype == np.float32  # noqa: E731
                        else torch.from_numpy(a.view(np.int16)).to(dev).view(torch.bfloat16))
    w = {k: to_dev(v) for k, v in w_host.items()}
    x = to_dev(synth.layer_input(seq, cfg.d_model, seed=0))
    ref_out = bf16_reference(x, w, cfg).to(torch.float32)
    upd = (ref_out - x.to(torch.float32)).pow(2).mean().item()
    out = {"workload": "c5_llama3_8b_decoder_layer", "seq": seq, "d_model": cfg.d_model, "heads": cfg.n_heads,
           "kv_heads": cfg.n_kv_heads, "d_ff": cfg.d_ff, "data": "synthetic, random-init weights", "fused_attention": fused_attention,
           "prepared_weights": prepared_weights,
           "reference_update_mean_square": upd, "formats": {}}
    for name in formats:
        # "<format>[prepared_w]": this entry on prepared weights whatever the argument says
        kind, asym = FORMATS[name.replace("[prepared_w]", "")]
        lay = layer.DecoderLayer(cfg, w, binding.make_format(kind, asym), fused_attention=fused_attention,
                                 fused_norm=False if separate_norm else None,
                                 prepared_weights=prepared_weights or name.endswith("[prepared_w]"))
        y = lay.forward(x)  # warm-up, also the output that is compared
        torch.cuda.synchronize()
        t0 = time.perf_counter()
        for _ in range(steps):
            lay.forward(x)
        torch.cuda.synchronize()
        dt = (time.perf_counter() - t0) / steps
        mse = (y.to(torch.float32) - ref_out).pow(2).mean().item()
        out["formats"][name] = {"ms_per_layer": round(dt * 1e3, 3),
                                # flops the layer executes (the fused attention skips the masked key tiles) ...
                                "matmul_TFLOPs": round(lay.matmul_flops(seq) / dt / 1e12, 1),
                                # ... and with the attention products counted in full whatever runs
                                "matmul_TFLOPs_dense_attention_credit": round(
                                    lay.matmul_flops(seq, nominal=True) / dt / 1e12, 1),
                                "mse_vs_bf16": mse, "mse_over_update": mse / upd}
        del lay, y
        torch.cuda.empty_cache()
    return out


def main():
    ap = argparse.ArgumentParser()
    ap.add_argument("--seq", type=int, default=8192)
    ap.add_argument("--steps", type=int, default=5)
    ap.add_argument("--formats", default=",".join(FORMATS))
    ap.add_argument("--fused-attention", action="store_true",
                    help="one fused attention call instead of Q.K^T, softmax, cast and P.V with a materialised map")
    ap.add_argument("--separate-norm", action="store_true",
                    help="residual addition, RMS normalisation and cast as three calls instead of one")
    ap.add_argument("--prepared-weights", action="store_true",
                    help="the weights' kernel-private form (BF16 panels for FP8 scales) written once, not per call")
    args = ap.parse_args()
    print(json.dumps(run(args.seq, args.steps, args.formats.split(","), args.fused_attention, args.separate_norm,
                         args.prepared_weights)))


if __name__ == "__main__":
    main()
