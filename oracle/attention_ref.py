"""Oracle of the fused quantized attention (TEST INFRASTRUCTURE: only tests/, the smoke check and a benchmark's CPU
baseline may import this; it shares no code with the HIP path).

The paper quantizes both attention products, Q.K^T and the attention map times V (Sec. 5.1), and discusses attention
at long context as the case where they dominate (Sec. 5.2, long-context evaluation). It defines no fused kernel. This
file states, in plain NumPy float64 loops, the tile-wise variant in which the attention map is never materialised:
the scores of one tile of keys are turned into un-normalised probabilities against the running row maximum (the
online-softmax recurrence), that tile of probabilities is quantized as one group per query along the keys, and
multiplied with the quantized V tile; the normalisation by the row sum happens at the end.

Definition (per head, per query i; T = 32 keys per tile = the group size along the keys; key tiles in ascending order):
  Q_hat, K_hat   = dequantized casts of Q and K, groups along the head dimension
  V_hat          = dequantized cast of V, groups along the keys (so one V group = one key tile)
  s_j            = scale * sum_d Q_hat[i, d] * K_hat[j, d];  causal: keys j > i + (Sk - Sq) are masked
  a tile with no unmasked key is skipped; otherwise
  m'             = max(m, max over unmasked j of s_j)                      (m starts at -inf)
  p_j            = float32(exp(s_j - m'))  for unmasked j, 0 for masked j
  l              = l * exp(m - m') + sum_j p_j                             (l starts at 0)
  p_hat          = dequantize(quantize(the 32 values p_j as ONE group))    (same element / scale format as the operands)
  O              = O * exp(m - m') + sum_j p_hat_j * V_hat[j, :]           (O starts at 0);  m = m'
  out[i, :]      = float32(O / l)
This differs numerically from quantizing the normalised map (the probabilities are quantized relative to the running
maximum, tile by tile), which is why it has its own definition here.                         -- parity unpinned
(against the paper: it prints no attention output; pinned against closed forms and invariants in the tests)

Split keys (key_splits = n > 1; the decoding shape, a few queries against many keys, where the keys are the only
parallelism): the Sk / 32 key tiles are cut into n contiguous ranges of ceil((Sk / 32) / n) tiles (the last ones may be
shorter or empty); the recurrence above runs over each range on its own, from m = -inf, l = 0, O = 0, giving
(m_c, l_c, O_c); a range in which the query sees no key contributes nothing. Then, exactly,
  m*  = max_c m_c;   out[i, :] = float32( sum_c O_c exp(m_c - m*)  /  sum_c l_c exp(m_c - m*) )
The probabilities of a range are quantized relative to that range's running maximum, so the result depends on n
(n = 1 is the definition above); without quantization every n would give the same softmax.
"""
import numpy as np

from . import ref

TILE = 32


def fused_attention(q_bits, k_bits, v_bits, scale, causal=True, scale_format=ref.FP8_E5M2, asymmetric=True,
                    heads=None, rows=None, key_splits=1):
    """q_bits [Hq, Sq, D], k_bits / v_bits [Hkv, Sk, D]: BF16 bit patterns (uint16); Hq a multiple of Hkv (query
    head h reads key/value head h // (Hq // Hkv)). Returns float32 [Hq, Sq, D]. heads / rows: compute only these
    query heads / query positions (the other entries of the result stay 0): every output row depends on its own
    query and on the keys and values only, so a sample of rows is computed exactly as in the full problem."""
    Hq, Sq, D = q_bits.shape
    Hkv, Sk, _ = k_bits.shape
    assert Hq % Hkv == 0 and Sk % TILE == 0 and D % 32 == 0
    per = Hq // Hkv
    assert key_splits >= 1
    tiles_per_range = -(-(Sk // TILE) // key_splits)
    out = np.zeros((Hq, Sq, D), np.float32)
    heads = range(Hq) if heads is None else list(heads)
    rows = range(Sq) if rows is None else list(rows)
    kv = {}
    for g in sorted({h // per for h in heads}):
        kc, ks = ref.quantize(np.ascontiguousarray(k_bits[g]), 32, scale_format, asymmetric)
        vc, vs = ref.quantize(np.ascontiguousarray(v_bits[g]), 32, scale_format, asymmetric, k_axis=0)  # [D, Sk]
        kv[g] = (ref.dequantize(kc, ks, 32, scale_format, asymmetric),
                 ref.dequantize(vc, vs, 32, scale_format, asymmetric).T)                       # [Sk, D] each
    sc = np.float64(np.float32(scale))
    for h in heads:
        qc, qs = ref.quantize(np.ascontiguousarray(q_bits[h]), 32, scale_format, asymmetric)
        qh = ref.dequantize(qc, qs, 32, scale_format, asymmetric)
        kh, vh = kv[h // per]
        for i in rows:
            s_row = (kh @ qh[i]) * sc                                                          # [Sk] float64
            last = i + (Sk - Sq) if causal else Sk - 1          # last key this query may attend to
            parts = []                                          # (m_c, l_c, O_c) of every range with a visible key
            for r0 in range(0, Sk, tiles_per_range * TILE):
                m, l, o = -np.inf, 0.0, np.zeros(D, np.float64)
                for t0 in range(r0, min(r0 + tiles_per_range * TILE, Sk), TILE):
                    n_ok = min(TILE, last - t0 + 1)
                    if n_ok <= 0:
                        break
                    s = s_row[t0:t0 + TILE]
                    m_new = max(m, float(np.max(s[:n_ok])))
                    alpha = np.exp(m - m_new)                   # exp(-inf) = 0 on the first tile
                    p = np.zeros(TILE, np.float32)
                    p[:n_ok] = np.exp(s[:n_ok] - m_new).astype(np.float32)
                    l = l * alpha + float(np.sum(p.astype(np.float64)))
                    pc, ps = ref.quantize_f32(p.reshape(1, TILE), 32, scale_format, asymmetric)
                    p_hat = ref.dequantize(pc, ps, 32, scale_format, asymmetric)[0]
                    o = o * alpha + p_hat @ vh[t0:t0 + TILE]
                    m = m_new
                if l > 0.0:
                    parts.append((m, l, o))
            m_all = max(pm for pm, _, _ in parts)
            num = sum(po * np.exp(pm - m_all) for pm, _, po in parts)
            den = sum(pl * np.exp(pm - m_all) for pm, pl, _ in parts)
            out[h, i] = (num / den).astype(np.float32)
    return out
