"""One LLaMA-style decoder layer (grouped-query attention, rotary embedding, gated MLP) whose seven matrix
multiplications all go through the quantized path: every operand is cast with amxfp4_quantize and multiplied with
amxfp4_gemm (Sec. 5.1: the linear projections and both attention products are quantized, the rest stays BF16).

This module only sequences library calls; the arithmetic is in libamxfp4 (binding.py marshals the arguments).
Shapes for a sequence of S tokens, H query heads, G key/value heads (H = G * per), head size D, model width W = H * D,
MLP width F:
  qkv    = cast(rmsnorm(x)) . Wqkv^T                  [S, W + 2 G D]
  scores = cast(rope(q)) . cast(rope(k))^T            batch G, [per * S, S]   (the `per` query heads that share a key
                                                                                head are stacked along the rows)
  o      = cast(softmax(scores)) . cast(v)^T          batch G, [per * S, D]   (P grouped along the keys, V cast down
                                                                                its columns)
  x2     = x + cast(merge(o)) . Wo^T
  out    = x2 + cast(silu(g) * u) . Wd^T,  (g | u) = cast(rmsnorm(x2)) . Wgu^T
With fused_attention=True the two attention products and the softmax between them are one call (binding.attention):
the attention map is not materialised and its tiles are cast relative to the running row maximum, which gives
slightly different numbers than casting the normalised map.
"""
import math
from dataclasses import dataclass

import torch

from . import binding


@dataclass
class LayerConfig:
    d_model: int = 4096
    n_heads: int = 32
    n_kv_heads: int = 8
    head_dim: int = 128
    d_ff: int = 14336
    eps: float = 1e-5
    rope_theta: float = 500000.0


WEIGHT_SHAPES = lambda c: {  # noqa: E731  (name -> [out features, in features])
    "wq": (c.n_heads * c.head_dim, c.d_model), "wk": (c.n_kv_heads * c.head_dim, c.d_model),
    "wv": (c.n_kv_heads * c.head_dim, c.d_model), "wo": (c.d_model, c.n_heads * c.head_dim),
    "wg": (c.d_ff, c.d_model), "wu": (c.d_ff, c.d_model), "wd": (c.d_model, c.d_ff)}


class DecoderLayer:
    """weights: dict name -> BF16 CUDA tensor (WEIGHT_SHAPES) plus "norm1" / "norm2" FP32 [d_model]. The weights are
    cast once here (they are static in inference); forward() casts the activations."""

    def __init__(self, cfg, weights, fmt, baseline=False, fused_attention=False, fused_glu=None, fused_norm=None,
                 fused_rope=None, prepared_weights=False):
        self.cfg, self.fmt, self.baseline, self.fused_attention = cfg, fmt, baseline, fused_attention
        # the rotary embedding casts its result (Q and K never exist as BF16 tensors): same bits
        if fused_rope is None:
            fused_rope = fmt.group_size == 32 and cfg.head_dim % 64 == 0 and cfg.head_dim <= 256
        self.fused_rope = fused_rope
        # the two normalisations cast their result in registers (and the second adds the residual first): same bits
        if fused_norm is None:
            fused_norm = fmt.group_size in (16, 32, 64) and cfg.d_model <= 16384
        self.fused_norm = fused_norm
        # the gate / up projection with the gated activation in its epilogue (the FP32 product is never written)
        if fused_glu is None:
            fused_glu = cfg.d_ff % 32 == 0
        self.fused_glu = fused_glu
        q = lambda w: binding.quantize(fmt, w.contiguous(), baseline=baseline)  # noqa: E731
        self.wqkv = q(torch.cat([weights["wq"], weights["wk"], weights["wv"]], 0))
        self.wo = q(weights["wo"])
        self.wgu = q(binding.interleave_gate_up(weights["wg"], weights["wu"]) if fused_glu
                     else torch.cat([weights["wg"], weights["wu"]], 0))
        self.wd = q(weights["wd"])
        self.norm1, self.norm2 = weights["norm1"].contiguous(), weights["norm2"].contiguous()
        self._ws = None
        # static weights: their kernel-private form written once (2 bytes per element of extra memory for the formats
        # that multiply on BF16 panels, nothing for the power-of-two formats); same bits
        self.prepared = None
        if prepared_weights and not baseline:
            self.prepared = {id(w): binding.prepare_weights(fmt, w[0], w[1])
                             for w in (self.wqkv, self.wo, self.wgu, self.wd)}

    def _gemm(self, a, b):
        fmt = self.fmt
        batch = a[0].shape[0] if a[0].dim() == 3 else 1
        need = binding.gemm_workspace_bytes(fmt, a[0].shape[-2], b[0].shape[-2], a[0].shape[-1] * 2, batch)
        if need and (self._ws is None or self._ws.numel() < need):
            self._ws = torch.empty(need, dtype=torch.uint8, device=a[0].device)
        if self.prepared is not None and id(b) in self.prepared and batch == 1:
            return binding.gemm_prepared(fmt, a[0], a[1], b[0], b[1], self.prepared[id(b)], workspace=self._ws)
        return binding.gemm(fmt, a[0], a[1], b[0], b[1], workspace=self._ws if need else None, baseline=self.baseline)

    def _plain_fmt(self):
        """the format for the entry points that have no mxfp4_* twin: symmetric when this layer is the baseline"""
        return binding.make_format(self.fmt.scale, False, self.fmt.group_size) if self.baseline else self.fmt

    def _cast(self, x, k_axis=-1):
        return binding.quantize(self.fmt, x, k_axis=k_axis, baseline=self.baseline)

    def forward(self, x, pos0=0):
        c = self.cfg
        S, G, D = x.shape[0], c.n_kv_heads, c.head_dim
        per = c.n_heads // G
        nsc = self.wqkv[1].shape[2:]  # () or (2,): scale entries per group

        if self.fused_norm:
            qkv = self._gemm(binding.rmsnorm_quantize(self._plain_fmt(), x, self.norm1, c.eps), self.wqkv)
        else:
            qkv = self._gemm(self._cast(binding.rmsnorm(x, self.norm1, c.eps)), self.wqkv)
        v = binding.split_heads_rope(qkv, (c.n_heads + G) * D, G, D, False)
        if self.fused_rope:
            # rotary embedding and the cast of Q and K along the head dimension in one launch each (same bits)
            qc, qs = binding.split_heads_rope_quantize(self._plain_fmt(), qkv, 0, c.n_heads, D, pos0, c.rope_theta)
            kc, ks = binding.split_heads_rope_quantize(self._plain_fmt(), qkv, c.n_heads * D, G, D, pos0, c.rope_theta)
        else:
            q = binding.split_heads_rope(qkv, 0, c.n_heads, D, True, pos0, c.rope_theta)
            k = binding.split_heads_rope(qkv, c.n_heads * D, G, D, True, pos0, c.rope_theta)
            qc, qs = self._cast(q.view(c.n_heads * S, D))
            kc, ks = self._cast(k.view(G * S, D))
        if self.fused_attention:
            vc, vs = self._cast_v(v, nsc)
            fmt = binding.make_format(self.fmt.scale, False, 32) if self.baseline else self.fmt
            need = binding.attention_workspace_bytes(fmt, c.n_heads, G, S, S, D)
            if self._ws is None or self._ws.numel() < need:
                self._ws = torch.empty(need, dtype=torch.uint8, device=x.device)
            # (the kernel writes its output merged and in BF16: what merge_heads would make of the FP32 result)
            o = binding.attention(fmt, qc.view(c.n_heads, S, D // 2), qs.view(c.n_heads, S, D // 32, *nsc),
                                  kc.view(G, S, D // 2), ks.view(G, S, D // 32, *nsc), vc, vs, 1.0 / math.sqrt(D),
                                  True, workspace=self._ws, merged=True)
            return self._after_attention(x, o)
        scores = self._gemm((qc.view(G, per * S, D // 2), qs.view(G, per * S, D // 32, *nsc)),
                            (kc.view(G, S, D // 2), ks.view(G, S, D // 32, *nsc)))
        p = binding.softmax_causal(scores, 1.0 / math.sqrt(D))
        del scores
        pc, ps = self._cast(p.view(G * per * S, S))
        del p
        vc, vs = self._cast_v(v, nsc)
        o = self._gemm((pc.view(G, per * S, S // 2), ps.view(G, per * S, S // 32, *nsc)), (vc, vs))
        return self._after_attention(x, binding.merge_heads(o, G, per, S, D))

    def _cast_v(self, v, nsc):
        G, S, D = v.shape
        vc = torch.empty((G, D, S // 2), dtype=torch.uint8, device=v.device)
        vs = torch.empty((G, D, S // 32) + tuple(nsc), dtype=torch.uint8, device=v.device)
        # V of one head is [S, D]; its groups run down the columns (along the keys); all heads in one launch
        fmt = binding.make_format(self.fmt.scale, False, self.fmt.group_size) if self.baseline else self.fmt
        binding.quantize_batched(fmt, v, k_axis=1, codes=vc, scales=vs)
        return vc, vs

    def _after_attention(self, x, attn):
        c = self.cfg
        if self.fused_norm:
            x2, *hc = binding.rmsnorm_quantize(self._plain_fmt(), x, self.norm2, c.eps,
                                               y=self._gemm(self._cast(attn), self.wo))
        else:
            x2 = binding.residual_add(x, self._gemm(self._cast(attn), self.wo))
            hc = self._cast(binding.rmsnorm(x2, self.norm2, c.eps))
        if self.fused_glu:
            fmt = self._plain_fmt()
            need = binding.gemm_silu_mul_workspace_bytes(fmt, hc[0].shape[0], c.d_ff, c.d_model)
            if need and (self._ws is None or self._ws.numel() < need):
                self._ws = torch.empty(need, dtype=torch.uint8, device=x.device)
            act = binding.gemm_silu_mul(fmt, hc[0], hc[1], self.wgu[0], self.wgu[1], workspace=self._ws,
                                        prepared=self.prepared[id(self.wgu)] if self.prepared is not None else None)
        else:
            act = binding.silu_mul(self._gemm(hc, self.wgu))
        return binding.residual_add(x2, self._gemm(self._cast(act), self.wd))

    def matmul_flops(self, S, nominal=False):
        """2 * M * N * K summed over the seven quantized matmuls, counting what this layer EXECUTES: with the
        materialised map both attention products run in full (no causal skipping); the fused attention skips the key
        tiles of 32 that lie wholly behind the causal mask of a block of 32 queries, so a head multiplies
        S * (S + 32) / 2 query-key pairs instead of S * S. nominal=True counts the attention products in full
        whatever runs (the figure a dense-attention layer would be credited with)."""
        c = self.cfg
        W, F, kv = c.n_heads * c.head_dim, c.d_ff, c.n_kv_heads * c.head_dim
        lin = S * c.d_model * (W + 2 * kv) + S * W * c.d_model + S * c.d_model * 2 * F + S * F * c.d_model
        pairs = S * (S + 32) // 2 if (self.fused_attention and not nominal) else S * S
        att = 2 * c.n_heads * pairs * c.head_dim
        return 2.0 * (lin + att)
