"""Independent float64 NumPy derivation of the decoder forward pass (test helper).

Written separately from the C oracle and vectorised over positions: rotary
embedding by complex multiplication, attention by batched matrix products with
an explicit lower-triangular mask, grouped-query attention by repeating KV heads.
"""
import numpy as np


def forward(shape, W, tokens):
    f8 = lambda a: np.asarray(a, dtype=np.float64)
    T = len(tokens)
    H, KV, hd, d = shape.n_heads, shape.n_kv_heads, shape.head_dim, shape.d_model
    x = f8(W["embed"])[np.asarray(tokens)]                              # [T, d]

    def norm(v, g):
        return v / np.sqrt((v * v).mean(-1, keepdims=True) + shape.rms_eps) * f8(g)

    def rot(v):                                                         # v: [T, heads, hd]
        half = hd // 2
        freq = shape.rope_theta ** (-np.arange(half) * 2.0 / hd)
        ph = np.exp(1j * np.arange(T)[:, None] * freq[None, :])         # [T, half]
        z = (v[..., :half] + 1j * v[..., half:]) * ph[:, None, :]
        return np.concatenate([z.real, z.imag], -1)

    mask = np.tril(np.ones((T, T), bool))
    for l in range(shape.n_layers):
        p = f"layers.{l}."
        a = norm(x, W[p + "norm_attn"])
        q = rot((a @ f8(W[p + "wq"]).T).reshape(T, H, hd))
        k = rot((a @ f8(W[p + "wk"]).T).reshape(T, KV, hd))
        v = (a @ f8(W[p + "wv"]).T).reshape(T, KV, hd)
        k = np.repeat(k, H // KV, axis=1)
        v = np.repeat(v, H // KV, axis=1)
        s = np.einsum("thd,shd->hts", q, k) / np.sqrt(hd)
        s = np.where(mask[None], s, -np.inf)
        s = np.exp(s - s.max(-1, keepdims=True))
        s /= s.sum(-1, keepdims=True)
        o = np.einsum("hts,shd->thd", s, v).reshape(T, H * hd)
        x = x + o @ f8(W[p + "wo"]).T
        b = norm(x, W[p + "norm_ffn"])
        g = b @ f8(W[p + "w_gate"]).T
        u = b @ f8(W[p + "w_up"]).T
        x = x + (g / (1 + np.exp(-g)) * u) @ f8(W[p + "w_down"]).T
    return norm(x, W["norm_final"]) @ f8(W["lm_head"]).T
