"""Seeded synthetic operands shaped like the paper's LLM workloads.

This module holds no arithmetic of the quantization method: it only draws random tensors and rounds them to BF16.
It serves the GPU tests, the benchmark and the CPU oracle's tests alike.

Structure follows what the paper reports about activations (Sec. 3.1-3.3): outliers concentrated in a few hidden
channels, group means scattered away from zero at group size 32 (asymmetry), and GLU-amplified, skewed inputs to the
second FFN matmul. Weights are plain small-variance Gaussians.

All generators return BF16 bit patterns as numpy uint16 arrays (host memory).
"""
import numpy as np


def f32_to_bf16_bits(x):
    """Round float32 to BF16 (nearest, ties to even) and return the 16-bit patterns."""
    u = np.ascontiguousarray(x, np.float32).view(np.uint32)
    r = (u + np.uint32(0x7FFF) + ((u >> np.uint32(16)) & np.uint32(1))) >> np.uint32(16)
    return r.astype(np.uint16)


def bf16_bits_to_f32(b):
    return (np.ascontiguousarray(b, np.uint16).astype(np.uint32) << np.uint32(16)).view(np.float32)


def _rng(seed, stream):
    return np.random.Generator(np.random.PCG64(np.random.SeedSequence(seed).spawn(stream + 1)[stream]))


def _normal(rng, shape, std=1.0, chunk_rows=4096):
    """float32 N(0, std) drawn in row chunks (keeps peak host memory low for the 70B-shaped weights)."""
    out = np.empty(shape, np.float32)
    for r0 in range(0, shape[0], chunk_rows):
        blk = out[r0:r0 + chunk_rows]
        rng.standard_normal(blk.shape, dtype=np.float32, out=blk)
    if std != 1.0:
        out *= np.float32(std)
    return out


def activations(rows, K, seed=0, n_outlier=8, outlier_gain=60.0, shift=0.5, stream=0):
    """X ~ N(0,1); `n_outlier` random channels multiplied by `outlier_gain`; `shift` added to a random half of the
    channels (group means move away from zero)."""
    rng = _rng(seed, stream)
    x = _normal(rng, (rows, K))
    ch = rng.choice(K, n_outlier, replace=False)
    x[:, ch] *= np.float32(outlier_gain)
    if shift:
        half = rng.choice(K, K // 2, replace=False)
        x[:, half] += np.float32(shift)
    return f32_to_bf16_bits(x)


def glu_activations(rows, K, seed=0, n_outlier=29, outlier_gain=100.0, stream=2):
    """silu(g), g ~ N(0,1): skewed, bounded below by -0.278, with outlier channels (input of a down projection)."""
    rng = _rng(seed, stream)
    g = _normal(rng, (rows, K))
    x = g / (1.0 + np.exp(-g))
    ch = rng.choice(K, n_outlier, replace=False)
    x[:, ch] *= np.float32(outlier_gain)
    return f32_to_bf16_bits(x.astype(np.float32))


def weights(N, K, seed=0, std=0.02, stream=1):
    """W ~ N(0, std), stored [N, K] (output features x input features, K contiguous)."""
    return f32_to_bf16_bits(_normal(_rng(seed, stream), (N, K), std))


def attention_qkv(heads, seq, head_dim, seed=0, n_outlier=2, outlier_gain=20.0, stream=3):
    """Q, K, V ~ N(0,1) [heads, seq, head_dim]; per head `n_outlier` head dims multiplied by `outlier_gain`
    (the same dims for Q and K of a head, independent ones for V)."""
    rng = _rng(seed, stream)
    q = _normal(rng, (heads * seq, head_dim)).reshape(heads, seq, head_dim)
    k = _normal(rng, (heads * seq, head_dim)).reshape(heads, seq, head_dim)
    v = _normal(rng, (heads * seq, head_dim)).reshape(heads, seq, head_dim)
    for h in range(heads):
        d_qk = rng.choice(head_dim, n_outlier, replace=False)
        d_v = rng.choice(head_dim, n_outlier, replace=False)
        q[h][:, d_qk] *= np.float32(outlier_gain)
        k[h][:, d_qk] *= np.float32(outlier_gain)
        v[h][:, d_v] *= np.float32(outlier_gain)
    return f32_to_bf16_bits(q), f32_to_bf16_bits(k), f32_to_bf16_bits(v)


def causal_softmax_probs(q_bits, k_bits):
    """P = softmax(causal(Q.K^T / sqrt(d))) in float32 from BF16 Q, K of ONE head ([seq, d] each), rounded to BF16.
    Masked entries are exactly 0 and all entries are >= 0 (a strongly one-sided operand)."""
    q = bf16_bits_to_f32(q_bits)
    k = bf16_bits_to_f32(k_bits)
    s = (q @ k.T) / np.float32(np.sqrt(q.shape[1]))
    seq = s.shape[0]
    mask = np.tril(np.ones((seq, seq), bool))
    s = np.where(mask, s, -np.inf)
    s -= s.max(axis=1, keepdims=True)
    p = np.exp(s)
    p /= p.sum(axis=1, keepdims=True)
    return f32_to_bf16_bits(p.astype(np.float32))


# The benchmark configurations (shapes only; distributions as above).
CONFIGS = {
    "c1_linear_64x1024x1024": dict(M=64, K=1024, N=1024, n_outlier=8, outlier_gain=60.0, shift=0.5),
    "c2_llama7b_qkvo_2048x4096x4096": dict(M=2048, K=4096, N=4096, n_outlier=8, outlier_gain=60.0, shift=0.5),
    "c2_llama7b_mlp_up_2048x4096x11008": dict(M=2048, K=4096, N=11008, n_outlier=8, outlier_gain=60.0, shift=0.5),
    "c3_70b_up_4096x8192x28672": dict(M=4096, K=8192, N=28672, n_outlier=8, outlier_gain=100.0, shift=0.0),
    "c3_70b_down_4096x28672x8192": dict(M=4096, K=28672, N=8192, n_outlier=29, outlier_gain=100.0, glu=True),
    # the same projections with a few tokens (decoding a batch of 32 sequences): weights-bound
    "c3_70b_up_32tokens_32x8192x28672": dict(M=32, K=8192, N=28672, n_outlier=8, outlier_gain=100.0, shift=0.0),
    "c3_70b_down_32tokens_32x28672x8192": dict(M=32, K=28672, N=8192, n_outlier=29, outlier_gain=100.0, glu=True),
}


def linear_operands(name, seed=0, M=None, N=None):
    """(X bits [M,K], W bits [N,K]) for a named linear configuration; M / N can be cut down for sampled checks."""
    c = CONFIGS[name]
    m = c["M"] if M is None else M
    n = c["N"] if N is None else N
    if c.get("glu"):
        x = glu_activations(m, c["K"], seed, c["n_outlier"], c["outlier_gain"])
    else:
        x = activations(m, c["K"], seed, c["n_outlier"], c["outlier_gain"], c["shift"])
    return x, weights(n, c["K"], seed)


def layer_weights(cfg, seed=0, stream=20):
    """Random-init weights of one decoder layer: projection matrices ~ N(0, 0.02) as BF16 bits ([out, in]), RMSNorm
    gains 1 + 0.1 N(0,1) as float32. cfg: d_model, n_heads, n_kv_heads, head_dim, d_ff."""
    shapes = {"wq": (cfg.n_heads * cfg.head_dim, cfg.d_model), "wk": (cfg.n_kv_heads * cfg.head_dim, cfg.d_model),
              "wv": (cfg.n_kv_heads * cfg.head_dim, cfg.d_model), "wo": (cfg.d_model, cfg.n_heads * cfg.head_dim),
              "wg": (cfg.d_ff, cfg.d_model), "wu": (cfg.d_ff, cfg.d_model), "wd": (cfg.d_model, cfg.d_ff)}
    w = {}
    for i, (name, shape) in enumerate(shapes.items()):
        w[name] = weights(shape[0], shape[1], seed, stream=stream + i)
    rng = _rng(seed, stream + 10)
    w["norm1"] = (1.0 + 0.1 * rng.standard_normal(cfg.d_model)).astype(np.float32)
    w["norm2"] = (1.0 + 0.1 * rng.standard_normal(cfg.d_model)).astype(np.float32)
    return w


def layer_input(seq, d_model, seed=0, n_outlier=4, outlier_gain=20.0):
    """Hidden states entering a decoder layer: N(0,1) with a few outlier channels, BF16 bits [seq, d_model]."""
    return activations(seq, d_model, seed, n_outlier, outlier_gain, shift=0.0, stream=31)
