"""A second, independent statement of the decoder in NumPy float64 (test-only).

Written in matrix form (whole sequences at once, explicit causal mask matrix, library matmul), i.e.
structured differently from the oracle's per-token loops, so that agreement between the two is evidence
for both.  Shares nothing with the oracle or the GPU path.
"""
import numpy as np


def _norm(x, g, eps):
    return g * x / np.sqrt((x * x).mean(-1, keepdims=True) + eps)


def _rope(t, base, style):
    # t: [T, H, hd]; position = row index
    T, H, hd = t.shape
    half = hd // 2
    ang = np.arange(T)[:, None] * base ** (-2.0 * np.arange(half) / hd)[None, :]   # [T, half]
    c, s = np.cos(ang)[:, None, :], np.sin(ang)[:, None, :]
    out = np.empty_like(t)
    if style == 0:
        a, b = t[..., 0::2], t[..., 1::2]
        out[..., 0::2], out[..., 1::2] = a * c - b * s, a * s + b * c
    else:
        a, b = t[..., :half], t[..., half:]
        out[..., :half], out[..., half:] = a * c - b * s, a * s + b * c
    return out


def forward_all(shape, W, tokens):
    """W: dict of float64 arrays (lists for layer tensors); tokens [B, T] -> logits [B, T, V]"""
    B, T = tokens.shape
    Hq, Hkv, hd = shape.n_heads, shape.n_kv_heads, shape.head_dim
    mask = np.tril(np.ones((T, T), dtype=bool))
    # the shape record carries eps and the rotary base as single-precision numbers
    shape = type("S", (), dict(vars(shape), rms_eps=float(np.float32(shape.rms_eps)),
                               rope_base=float(np.float32(shape.rope_base))))
    out = np.empty((B, T, shape.vocab))
    for b in range(B):
        x = W["tok_emb"][tokens[b]]
        for l in range(shape.n_layers):
            h = _norm(x, W["attn_norm"][l], shape.rms_eps)
            q = _rope((h @ W["wq"][l].T).reshape(T, Hq, hd), shape.rope_base, shape.rope_style)
            k = _rope((h @ W["wk"][l].T).reshape(T, Hkv, hd), shape.rope_base, shape.rope_style)
            v = (h @ W["wv"][l].T).reshape(T, Hkv, hd)
            k = np.repeat(k, Hq // Hkv, axis=1)
            v = np.repeat(v, Hq // Hkv, axis=1)
            s = np.einsum("ihe,jhe->hij", q, k) / np.sqrt(hd)
            s = np.where(mask[None], s, -np.inf)
            p = np.exp(s - s.max(-1, keepdims=True))
            p /= p.sum(-1, keepdims=True)
            o = np.einsum("hij,jhe->ihe", p, v).reshape(T, Hq * hd)
            x = x + o @ W["wo"][l].T
            h = _norm(x, W["ffn_norm"][l], shape.rms_eps)
            g = h @ W["w_gate"][l].T
            x = x + ((g / (1.0 + np.exp(-g))) * (h @ W["w_up"][l].T)) @ W["w_down"][l].T
        out[b] = _norm(x, W["final_norm"], shape.rms_eps) @ W["lm_head"].T
    return out
