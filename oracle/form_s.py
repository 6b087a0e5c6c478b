"""Brute-force definition ("form S") -- TEST INFRASTRUCTURE, not the product.

Speculative decoding is lossless (paper Sec. II-B): whatever the target model
returns for a tree node must be what it would return when it simply decodes,
causally and with no cache, the committed prefix followed by the tokens on the
root-to-node path.  This module is that plain decoder, in numpy float64, written
independently of the C oracle: whole-matrix products, a lower-triangular mask,
rotary embedding as a complex multiplication.  It knows nothing about trees
except how to read a root-to-node path from a parent array.
"""
import numpy as np


def widen(a):
    """Storage array (float32 / float64 / uint16 bf16 bits) -> float64, exactly."""
    a = np.asarray(a)
    if a.dtype == np.uint16:
        return (a.astype(np.uint32) << 16).view(np.float32).astype(np.float64)
    return a.astype(np.float64)


def _rms(x, g, eps):
    return x / np.sqrt(np.mean(x * x, axis=-1, keepdims=True) + eps) * g


def _rotary(x, theta):
    """x: [T, heads, hd]; row t is at position t.  The pair (j, j+hd/2) is one
    complex number, multiplied by exp(i * t * theta^(-2j/hd))."""
    T, _, hd = x.shape
    half = hd // 2
    freq = theta ** (-np.arange(half, dtype=np.float64) * 2.0 / hd)
    phase = np.exp(1j * np.arange(T, dtype=np.float64)[:, None] * freq[None, :])
    z = (x[..., :half] + 1j * x[..., half:]) * phase[:, None, :]
    return np.concatenate([z.real, z.imag], axis=-1)


def causal_decoder(cfg, w, inputs):
    """Logits [T, vocab] of a causal decoder over input rows ``inputs`` [T, d_model]
    at positions 0..T-1."""
    H, Hkv, hd = cfg["n_heads"], cfg["n_kv_heads"], cfg["head_dim"]
    eps, theta = cfg.get("rms_eps", 1e-5), cfg.get("rope_theta", 10000.0)
    x = np.array(inputs, np.float64)
    T = x.shape[0]
    causal = np.tril(np.ones((T, T), bool))
    for lw in w["layers"]:
        h = _rms(x, widen(lw["attn_norm"]), eps)
        q = (h @ widen(lw["wq"]).T).reshape(T, H, hd)
        k = (h @ widen(lw["wk"]).T).reshape(T, Hkv, hd)
        v = (h @ widen(lw["wv"]).T).reshape(T, Hkv, hd)
        q, k = _rotary(q, theta), _rotary(k, theta)
        k = np.repeat(k, H // Hkv, axis=1)   # query head a uses KV head a // (H/Hkv)
        v = np.repeat(v, H // Hkv, axis=1)
        s = np.einsum("thc,shc->hts", q, k) / np.sqrt(hd)
        s = np.where(causal[None], s, -np.inf)
        s = s - s.max(axis=-1, keepdims=True)
        p = np.exp(s)
        p /= p.sum(axis=-1, keepdims=True)
        o = np.einsum("hts,shc->thc", p, v).reshape(T, H * hd)
        x = x + o @ widen(lw["wo"]).T
        h = _rms(x, widen(lw["ffn_norm"]), eps)
        g = h @ widen(lw["w_gate"]).T
        u = h @ widen(lw["w_up"]).T
        x = x + ((g / (1.0 + np.exp(-g))) * u) @ widen(lw["w_down"]).T
    return _rms(x, widen(w["final_norm"]), eps) @ widen(w["lm_head"]).T


def root_path(parents, i):
    path = []
    while i >= 0:
        path.append(i)
        i = int(parents[i])
    return path[::-1]


def node_logits(cfg, w, prefix_inputs, tokens, parents, i):
    """Logits the target returns at tree node i = last row of a causal decode of
    [prefix ; tokens on the root-to-i path]."""
    E = widen(w["tok_embed"])
    rows = [np.asarray(prefix_inputs, np.float64).reshape(-1, cfg["d_model"])]
    rows.append(E[[int(tokens[j]) for j in root_path(parents, i)]])
    return causal_decoder(cfg, w, np.concatenate(rows, axis=0))[-1]


def greedy_decode(cfg, w, prefix_inputs, first_token, n_new):
    """Autoregressive greedy decoding, one full causal pass per token: returns the
    n_new tokens emitted after ``first_token`` (the last committed token)."""
    E = widen(w["tok_embed"])
    seq = np.concatenate([np.asarray(prefix_inputs, np.float64).reshape(-1, cfg["d_model"]),
                          E[[int(first_token)]]], axis=0)
    out = []
    for _ in range(n_new):
        t = int(np.argmax(causal_decoder(cfg, w, seq)[-1]))
        out.append(t)
        seq = np.concatenate([seq, E[[t]]], axis=0)
    return out
