"""Oracle of the decoder-layer workload (TEST INFRASTRUCTURE: only tests/, the smoke check and a benchmark's CPU
baseline may import this; it shares no code with the HIP path).

Plain NumPy in float64, one function per operator between the quantized matrix multiplications of a LLaMA-style
decoder layer, and the layer itself with every matmul going through the quantization oracle (ref.quantize /
ref.gemm). The paper (Sec. 5.1) quantizes all matmuls of the decoder layers and leaves the other operators in BF16;
it does not define those operators, so they are the textbook ones:
  RMSNorm        y = x / sqrt(mean(x^2) + eps) * w
  rotary         pairs (i, i + d/2) of a head rotated by pos * theta^(-2i/d)   ("rotate-half" convention)
  causal softmax over keys c <= query position, scores scaled by 1/sqrt(d)
  gated MLP      silu(g) * u with silu(g) = g / (1 + exp(-g))
Every operator output is rounded ONCE from the float64 result to BF16 (nearest even), which is where the BF16
tensors of such a layer live; matmul outputs are FP32 as the library's GEMM returns them.
"""
import numpy as np

from . import attention_ref, ref


def bf16_from_f64(x):
    """float64 array -> BF16 bit patterns (uint16), round to nearest even in ONE step from the double value
    (finite inputs; BF16 has 8 significant bits, exponent range of float32, subnormal quantum 2^-133)."""
    x = np.asarray(x, np.float64)
    m, e = np.frexp(x)                       # x = m * 2^e, 0.5 <= |m| < 1
    e = np.maximum(e, -125)                  # below 2^-126 the quantum stays 2^-133 (subnormals)
    q = np.rint(np.ldexp(x, 8 - e))          # integer multiple of the quantum 2^(e-8); rint rounds ties to even
    y = np.ldexp(q, e - 8)                   # exactly representable in BF16 (or rounds up into the next binade)
    y32 = y.astype(np.float32)               # exact: at most 8 significant bits
    return (y32.view(np.uint32) >> 16).astype(np.uint16)


def f64_from_bf16(bits):
    return (np.asarray(bits, np.uint16).astype(np.uint32) << 16).view(np.float32).astype(np.float64)


def _out(y, exact):
    """Operator results are BF16 bits; exact=True hands back the float64 values before that one rounding (tests)."""
    return y if exact else bf16_from_f64(y)


def rmsnorm(x_bits, weight, eps, exact=False):
    x = f64_from_bf16(x_bits)
    inv = 1.0 / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + np.float64(np.float32(eps)))
    return _out(x * inv * np.asarray(weight, np.float64), exact)


def split_heads_rope(proj, col0, heads, head_dim, rotate, pos0=0, theta=10000.0, exact=False):
    """proj [seq, ld] float32 -> BF16 bits [heads, seq, head_dim]."""
    proj = np.asarray(proj, np.float64)
    seq = proj.shape[0]
    x = proj[:, col0:col0 + heads * head_dim].reshape(seq, heads, head_dim).transpose(1, 0, 2)  # [h, s, d]
    if rotate:
        half = head_dim // 2
        i = np.arange(half, dtype=np.float64)
        ang = (pos0 + np.arange(seq, dtype=np.float64))[:, None] * np.exp(-np.log(np.float64(theta)) * i / half)
        cs, sn = np.cos(ang), np.sin(ang)                    # [s, half]
        x1, x2 = x[..., :half], x[..., half:]
        x = np.concatenate([x1 * cs - x2 * sn, x2 * cs + x1 * sn], axis=-1)
    return _out(x, exact)


def softmax_causal(scores, scale, exact=False):
    """scores [batch, rows, cols] float32; row r is the query at position r % cols -> BF16 bits, masked entries 0."""
    s = np.asarray(scores, np.float64) * np.float64(np.float32(scale))
    rows, cols = s.shape[-2], s.shape[-1]
    allowed = np.arange(cols)[None, :] <= (np.arange(rows) % cols)[:, None]
    s = np.where(allowed, s, -np.inf)
    s = s - s.max(axis=-1, keepdims=True)
    e = np.exp(s)
    return _out(e / e.sum(axis=-1, keepdims=True), exact)


def silu_mul(gate_up, exact=False):
    gu = np.asarray(gate_up, np.float64)
    w = gu.shape[-1] // 2
    g, u = gu[..., :w], gu[..., w:]
    return _out(g / (1.0 + np.exp(-g)) * u, exact)


def residual_add(x_bits, y):
    return bf16_from_f64(f64_from_bf16(x_bits) + np.asarray(y, np.float64))


def merge_heads(o, groups, per_group, seq, head_dim):
    """o [groups, per_group * seq, head_dim] float32 -> BF16 bits [seq, groups * per_group * head_dim]."""
    o = np.asarray(o, np.float64).reshape(groups, per_group, seq, head_dim)
    return bf16_from_f64(o.transpose(2, 0, 1, 3).reshape(seq, groups * per_group * head_dim))


def _matmul(a_bits, b_codes_scales, scale, asym):
    ac, as_ = ref.quantize(np.ascontiguousarray(a_bits), 32, scale, asym)
    return ref.gemm(ac, as_, b_codes_scales[0], b_codes_scales[1], 32, scale, asym)


def decoder_layer(x_bits, w, cfg, scale=ref.FP8_E5M2, asym=1, pos0=0, fused_attention=False):
    """x_bits [S, d_model] BF16 bits; w: dict of BF16-bit weight matrices wq wk wv wo wg wu wd ([out, in]) and float32
    norm1 / norm2; cfg: object with d_model, n_heads, n_kv_heads, head_dim, d_ff, eps, rope_theta.
    fused_attention: the tile-wise attention of attention_ref instead of the materialised, normalised map.
    Returns the layer output as BF16 bits [S, d_model]."""
    S, G, D, H = x_bits.shape[0], cfg.n_kv_heads, cfg.head_dim, cfg.n_heads
    per = H // G
    q_ = lambda bits: ref.quantize(np.ascontiguousarray(bits), 32, scale, asym)  # noqa: E731
    wqkv = q_(np.concatenate([w["wq"], w["wk"], w["wv"]], 0))
    wo, wgu, wd = q_(w["wo"]), q_(np.concatenate([w["wg"], w["wu"]], 0)), q_(w["wd"])

    h = rmsnorm(x_bits, w["norm1"], cfg.eps)
    qkv = _matmul(h, wqkv, scale, asym)
    q = split_heads_rope(qkv, 0, H, D, True, pos0, cfg.rope_theta)
    k = split_heads_rope(qkv, H * D, G, D, True, pos0, cfg.rope_theta)
    v = split_heads_rope(qkv, (H + G) * D, G, D, False)

    if fused_attention:
        o = attention_ref.fused_attention(q, k, v, 1.0 / np.sqrt(np.float64(D)), True, scale, asym)   # [H, S, D]
        attn = merge_heads(o.reshape(G, per * S, D), G, per, S, D)
        return _after_attention(x_bits, attn, w, cfg, wo, wgu, wd, scale, asym)
    qc, qs = ref.quantize(q.reshape(H * S, D), 32, scale, asym)
    kc, ks = ref.quantize(k.reshape(G * S, D), 32, scale, asym)
    nsc = qs.shape[2:]
    scores = ref.gemm(qc.reshape(G, per * S, -1), qs.reshape(G, per * S, D // 32, *nsc),
                      kc.reshape(G, S, -1), ks.reshape(G, S, D // 32, *nsc), 32, scale, asym)
    p = softmax_causal(scores, 1.0 / np.sqrt(np.float64(D)))
    pc, ps = ref.quantize(p.reshape(G * per * S, S), 32, scale, asym)
    vcs = [ref.quantize(v[g], 32, scale, asym, k_axis=0) for g in range(G)]
    vc, vs = np.stack([t[0] for t in vcs]), np.stack([t[1] for t in vcs])
    o = ref.gemm(pc.reshape(G, per * S, -1), ps.reshape(G, per * S, S // 32, *nsc), vc, vs, 32, scale, asym)
    attn = merge_heads(o, G, per, S, D)
    return _after_attention(x_bits, attn, w, cfg, wo, wgu, wd, scale, asym)


def _after_attention(x_bits, attn, w, cfg, wo, wgu, wd, scale, asym):
    x2 = residual_add(x_bits, _matmul(attn, wo, scale, asym))
    h2 = rmsnorm(x2, w["norm2"], cfg.eps)
    act = silu_mul(_matmul(h2, wgu, scale, asym))
    return residual_add(x2, _matmul(act, wd, scale, asym))
