"""LLaMA-style target forward and EAGLE-style draft forward (test infrastructure).

Target model: the paper's targets are LLaMA2-Chat / LLaMA3-Instruct (Sec. 4.1,
Target LLMs): pre-norm decoder, RMSNorm, rotary positions, grouped-query
attention, SwiGLU feed-forward, no biases.  The "feature" handed to the draft
model is the LM head's input (appendix A.1 applies the head directly to the
target hidden state), i.e. the final-RMSNorm output.

Draft model (Sec. 2, EAGLE): one decoder layer whose input is the target
feature of the previous position concatenated with the embedding of the current
token, mapped 2d -> d by a bias-free linear layer; the target's LM head is
applied to its output with no extra norm (Sec. 3.2, Head(f)).

Every row of a forward names explicitly which cache slots it may attend to, so
the same routine serves plain causal decoding, tree verification and the
brute-force path-by-path check.
"""
from __future__ import annotations

from typing import Dict, List, Sequence

import numpy as np

Weights = Dict[str, np.ndarray]


class KVCache:
    """Per-layer key/value rows, keys stored AFTER rotary embedding."""

    def __init__(self, n_layers: int, max_seq: int, n_kv_heads: int, head_dim: int, dtype=np.float64):
        self.k = np.zeros((n_layers, max_seq, n_kv_heads, head_dim), dtype=dtype)
        self.v = np.zeros((n_layers, max_seq, n_kv_heads, head_dim), dtype=dtype)

    def copy(self) -> "KVCache":
        c = KVCache.__new__(KVCache)
        c.k = self.k.copy()
        c.v = self.v.copy()
        return c


def rmsnorm(x: np.ndarray, w: np.ndarray, eps: float) -> np.ndarray:
    ms = np.mean(x * x, axis=-1, keepdims=True)
    return x / np.sqrt(ms + eps) * w


def rope(x: np.ndarray, pos: np.ndarray, theta: float) -> np.ndarray:
    """Rotary embedding, rotate-half pairing: dims (j, j + hd/2) form one 2-D
    plane rotated by angle pos * theta**(-2j/hd).  x: [rows, heads, hd]."""
    hd = x.shape[-1]
    half = hd // 2
    j = np.arange(half, dtype=np.float64)
    inv = theta ** (-2.0 * j / hd)
    ang = pos.astype(np.float64)[:, None] * inv[None, :]          # [rows, half]
    c = np.cos(ang)[:, None, :].astype(x.dtype)
    s = np.sin(ang)[:, None, :].astype(x.dtype)
    x1, x2 = x[..., :half], x[..., half:]
    return np.concatenate([x1 * c - x2 * s, x2 * c + x1 * s], axis=-1)


def attention_row(q: np.ndarray, keys: np.ndarray, vals: np.ndarray) -> np.ndarray:
    """Softmax attention of one query head over the given keys.  q:[hd] keys,vals:[n,hd]."""
    s = keys @ q / np.sqrt(np.asarray(q.shape[0], dtype=q.dtype))
    s = s - s.max()
    p = np.exp(s)
    p = p / p.sum()
    return p @ vals


def _identity(x: np.ndarray) -> np.ndarray:
    return x


def decoder_layer(h: np.ndarray, w: Weights, prefix: str, shape, layer_idx: int, cache: KVCache,
                  pos: np.ndarray, slots: Sequence[int], visible: Sequence[Sequence[int]], store=_identity) -> np.ndarray:
    """One pre-norm decoder layer over `rows` inputs.

    Row i is at position pos[i]; its key/value are written to cache slot slots[i];
    it attends to the cache slots visible[i] (which must include slots[i]).

    `store` models the configuration's storage type: it is applied to every
    tensor that is held in memory between two operations (norm outputs, cached
    keys and values, the attention output, the SwiGLU output).  The residual
    stream, the queries and all accumulations stay in the compute dtype.  The
    default is the identity (the plain definition); a bf16 configuration may
    pass a round-to-bf16 function to ask what a bf16-storage pipeline computes.
    """
    rows = h.shape[0]
    hq, hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    a = store(rmsnorm(h, w[prefix + "attn_norm"], shape.rms_eps))
    q = (a @ w[prefix + "wq"].T).reshape(rows, hq, hd)
    k = (a @ w[prefix + "wk"].T).reshape(rows, hkv, hd)
    v = store((a @ w[prefix + "wv"].T).reshape(rows, hkv, hd))
    q = rope(q, pos, shape.rope_theta)
    k = store(rope(k, pos, shape.rope_theta))
    for i in range(rows):
        cache.k[layer_idx, slots[i]] = k[i]
        cache.v[layer_idx, slots[i]] = v[i]
    group = hq // hkv
    att = np.zeros((rows, hq, hd), dtype=h.dtype)
    for i in range(rows):
        vis = np.asarray(visible[i], dtype=np.int64)
        for hh in range(hq):
            kvh = hh // group
            att[i, hh] = attention_row(q[i, hh], cache.k[layer_idx, vis, kvh], cache.v[layer_idx, vis, kvh])
    h = h + store(att.reshape(rows, hq * hd)) @ w[prefix + "wo"].T
    b = store(rmsnorm(h, w[prefix + "ffn_norm"], shape.rms_eps))
    g = b @ w[prefix + "w_gate"].T
    u = b @ w[prefix + "w_up"].T
    act = store(g / (1.0 + np.exp(-g)) * u)
    return h + act @ w[prefix + "w_down"].T


def target_forward(w: Weights, shape, cache: KVCache, tokens: np.ndarray, pos: np.ndarray,
                   slots: Sequence[int], visible: Sequence[Sequence[int]], store=_identity):
    """Target LLM over rows -> (logits [rows, V], features [rows, d])."""
    h = w["embed"][np.asarray(tokens, dtype=np.int64)].astype(cache.k.dtype)
    for l in range(shape.n_layers):
        h = decoder_layer(h, w, f"layers.{l}.", shape, l, cache, pos, slots, visible, store)
    f = store(rmsnorm(h, w["final_norm"], shape.rms_eps))
    return f @ w["lm_head"].T, f


def draft_forward(w: Weights, shape, dcache: KVCache, feats: np.ndarray, tokens: np.ndarray, pos: np.ndarray,
                  slots: Sequence[int], visible: Sequence[Sequence[int]], store=_identity):
    """Draft model over rows of (previous-position feature, current token).

    -> (draft logits [rows, V], predicted features g [rows, d])."""
    e = w["embed"][np.asarray(tokens, dtype=np.int64)].astype(dcache.k.dtype)
    z = np.concatenate([feats.astype(dcache.k.dtype), e], axis=-1) @ w["draft.fc"].T
    g = store(decoder_layer(z, w, "draft.", shape, 0, dcache, pos, slots, visible, store))
    return g @ w["lm_head"].T, g


def as_dtype(w: Weights, dtype) -> Weights:
    return {k: v.astype(dtype) for k, v in w.items()}
