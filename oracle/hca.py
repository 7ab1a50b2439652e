"""Harmonized context alignment: the draft model's batched training forward
(test infrastructure; nothing on the product path imports this).

Sec. 3.2: training step j (j = 1 .. n, n = 3 by default) runs the draft model
over the whole sequence at once, but every position must see the context it
will see at decoding time after j autoregressive draft calls: its query comes
from the draft feature of step j-1, the key/value of the position itself comes
from step j-1 too, the one before it from step j-2, ..., the one j-2 positions
back from step 1, and everything older from the target LLM's features.

Notation.  "Stream" m (0 <= m < J, J = j) is one [T, ...] sequence of per-position
tensors: stream 0 derives from the target's features, stream m from the draft
features of training step m.  For query position t and key position s <= t with
offset o = t - s, the key/value used is the one of stream J-1-o if o <= J-2 and
of stream 0 otherwise.  With J = 1 this is plain causal attention (Sec. 3.2,
first step).

The function below is that definition written out: for every query it gathers,
position by position, the key and the value of the stream the rule names, and
runs plain softmax attention over them.

reading: the appendix reaches the same thing in a batched way (target-stream
scores with some diagonals replaced, then a correction of the output along those
diagonals), but its correction is weighted by the scores taken BEFORE the
softmax.  That cannot be meant (it would not be an attention over the mixed
key/value set of the Sec. 3.2 formula, and step j would not equal j
autoregressive draft calls); the softmax probabilities weight every value.
"""
from __future__ import annotations

from typing import List, Optional, Sequence

import numpy as np

from .llama import Weights, attention_row, rmsnorm, rope, _identity


def hca_attention(q: np.ndarray, ks: Sequence[np.ndarray], vs: Sequence[np.ndarray],
                  heads: Optional[Sequence[int]] = None) -> np.ndarray:
    """q: [T, hq, hd] (queries of stream J-1, rotary already applied);
    ks[m], vs[m]: [T, hkv, hd] for streams m = 0 .. J-1.  -> [T, hq, hd].
    `heads`: compute only these query heads (the others stay zero)."""
    n_streams = len(ks)
    t_len, hq, hd = q.shape
    group = hq // ks[0].shape[1]
    k_all, v_all = np.stack(ks), np.stack(vs)                   # [stream, position, kv head, hd]
    out = np.zeros_like(q)
    for h in (range(hq) if heads is None else heads):
        kv = h // group
        for t in range(t_len):
            s = np.arange(t + 1)                                # key positions of query t
            o = t - s                                           # how far back each one lies
            stream = np.where(o <= n_streams - 2, n_streams - 1 - o, 0)
            out[t, h] = attention_row(q[t, h], k_all[stream, s, kv], v_all[stream, s, kv])
    return out


def draft_train_pass(w: Weights, shape, inputs: Sequence[np.ndarray], tokens: np.ndarray, pos: np.ndarray,
                     store=_identity) -> np.ndarray:
    """Training step J = len(inputs) of the draft layer over T positions at once.

    inputs[m][t]: the feature handed to position t in stream m (inputs[0] from the
    target LLM, inputs[m] from training step m); tokens[t], pos[t]: the token paired
    with it and its rotary position.  Every stream goes through the draft model's
    input layer and attention norm; the query and the residual stream are those of
    the newest stream (at decoding time a draft call continues from its own previous
    output).  -> predicted features [T, d].

    `store` has the meaning it has in llama.decoder_layer.
    """
    hq, hkv, hd = shape.n_q_heads, shape.n_kv_heads, shape.head_dim
    t_len = tokens.shape[0]
    dt = inputs[0].dtype
    e = w["embed"][np.asarray(tokens, dtype=np.int64)].astype(dt)
    zs = [np.concatenate([u.astype(dt), e], axis=-1) @ w["draft.fc"].T for u in inputs]
    ks: List[np.ndarray] = []
    vs: List[np.ndarray] = []
    a_new = None
    for z in zs:
        a = store(rmsnorm(z, w["draft.attn_norm"], shape.rms_eps))
        k = (a @ w["draft.wk"].T).reshape(t_len, hkv, hd)
        ks.append(store(rope(k, pos, shape.rope_theta)))
        vs.append(store((a @ w["draft.wv"].T).reshape(t_len, hkv, hd)))
        a_new = a
    q = rope((a_new @ w["draft.wq"].T).reshape(t_len, hq, hd), pos, shape.rope_theta)
    att = hca_attention(q, ks, vs)
    h = zs[-1] + store(att.reshape(t_len, hq * hd)) @ w["draft.wo"].T
    b = store(rmsnorm(h, w["draft.ffn_norm"], shape.rms_eps))
    g = b @ w["draft.w_gate"].T
    u = b @ w["draft.w_up"].T
    act = store(g / (1.0 + np.exp(-g)) * u)
    return store(h + act @ w["draft.w_down"].T)


def next_stream(target_inputs: np.ndarray, predicted: np.ndarray) -> np.ndarray:
    """Input features of the next training step's new stream (appendix A.1, training loop):
    position t receives the feature just predicted for position t-1; position 0, which
    has no predecessor, keeps the target's."""
    return np.concatenate([target_inputs[:1], predicted[:-1]], axis=0)
