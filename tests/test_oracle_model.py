"""Pins for the oracle's target forward: library building blocks, closed forms, invariants."""
import numpy as np
import pytest
import torch
import torch.nn.functional as F

import workload as wl
from oracle import KVCache, attention_row, rmsnorm, rope, target_forward
from oracle.llama import as_dtype

GQA = wl.Shape("gqa-micro", 2, 64, 4, 2, 16, 96, 50, 1e4, "fp32", 9, 2, 2, 4, 0.0, 4, seed=7)


def causal(n):
    return [list(range(i + 1)) for i in range(n)]


def torch_llama(w, sh, tokens):
    """LLaMA forward assembled from torch library routines; rotary as a complex product."""
    tw = {k: torch.from_numpy(v).double() for k, v in w.items()}
    n = len(tokens)
    h = F.embedding(torch.as_tensor(tokens, dtype=torch.long), tw["embed"])
    half = sh.head_dim // 2
    ang = torch.arange(n).double()[:, None] * sh.rope_theta ** (-torch.arange(half).double() * 2 / sh.head_dim)[None]
    rot = torch.polar(torch.ones_like(ang), ang)[:, None, :]          # e^{i pos theta_j}

    def rotary(x):                                                    # [n, heads, hd]
        z = torch.complex(x[..., :half], x[..., half:]) * rot
        return torch.cat([z.real, z.imag], dim=-1)

    for l in range(sh.n_layers):
        p = f"layers.{l}."
        a = F.rms_norm(h, (sh.d_model,), tw[p + "attn_norm"], sh.rms_eps)
        q = rotary(F.linear(a, tw[p + "wq"]).view(n, sh.n_q_heads, sh.head_dim)).transpose(0, 1)
        k = rotary(F.linear(a, tw[p + "wk"]).view(n, sh.n_kv_heads, sh.head_dim)).transpose(0, 1)
        v = F.linear(a, tw[p + "wv"]).view(n, sh.n_kv_heads, sh.head_dim).transpose(0, 1)
        rep = sh.n_q_heads // sh.n_kv_heads
        k, v = k.repeat_interleave(rep, dim=0), v.repeat_interleave(rep, dim=0)
        o = F.scaled_dot_product_attention(q[None], k[None], v[None], is_causal=True)[0]
        h = h + F.linear(o.transpose(0, 1).reshape(n, -1), tw[p + "wo"])
        b = F.rms_norm(h, (sh.d_model,), tw[p + "ffn_norm"], sh.rms_eps)
        h = h + F.linear(F.silu(F.linear(b, tw[p + "w_gate"])) * F.linear(b, tw[p + "w_up"]), tw[p + "w_down"])
    f = F.rms_norm(h, (sh.d_model,), tw["final_norm"], sh.rms_eps)
    return F.linear(f, tw["lm_head"]).numpy(), f.numpy()


@pytest.mark.parametrize("sh", [GQA, wl.TINY], ids=["gqa", "tiny"])
def test_forward_matches_torch_library_blocks(sh):
    w = wl.make_weights(sh, std=0.2 if sh is GQA else 0.02)
    # non-trivial norm weights so that a dropped norm weight shows
    rng = np.random.default_rng(1)
    for k in w:
        if k.endswith("norm"):
            w[k] = (1 + 0.3 * rng.standard_normal(w[k].shape)).astype(np.float32)
    w = as_dtype(w, np.float64)
    tokens = wl.make_prompt(sh)
    n = len(tokens)
    cache = KVCache(sh.n_layers, n, sh.n_kv_heads, sh.head_dim)
    logits, feats = target_forward(w, sh, cache, tokens, np.arange(n), list(range(n)), causal(n))
    ref_logits, ref_feats = torch_llama(w, sh, tokens)
    assert np.abs(logits - ref_logits).max() < 1e-10
    assert np.abs(feats - ref_feats).max() < 1e-10


def test_incremental_equals_full_recompute(tiny):
    sh, w, prompt = tiny
    n = len(prompt)
    full_cache = KVCache(sh.n_layers, n, sh.n_kv_heads, sh.head_dim)
    full, _ = target_forward(w, sh, full_cache, prompt, np.arange(n), list(range(n)), causal(n))
    inc_cache = KVCache(sh.n_layers, n, sh.n_kv_heads, sh.head_dim)
    for i in range(n):
        row, _ = target_forward(w, sh, inc_cache, prompt[i:i + 1], np.array([i]), [i], [list(range(i + 1))])
        assert np.abs(row[0] - full[i]).max() < 1e-10
    assert np.abs(inc_cache.k - full_cache.k).max() < 1e-12


def test_rope_is_rotation_with_right_sign():
    rng = np.random.default_rng(0)
    x = rng.standard_normal((5, 3, 16))
    pos = np.array([0, 1, 2, 7, 100])
    y = rope(x, pos, 1e4)
    assert np.allclose(y[0], x[0])                                       # position 0 is the identity
    assert np.allclose(np.linalg.norm(y, axis=-1), np.linalg.norm(x, axis=-1))
    # plane j rotates counter-clockwise by pos * theta^(-2j/hd): complex form
    half = 8
    z = (x[..., :half] + 1j * x[..., half:]) * np.exp(1j * pos[:, None, None] * 1e4 ** (-np.arange(half) * 2 / 16))
    assert np.allclose(y[..., :half], z.real) and np.allclose(y[..., half:], z.imag)
    # first plane has frequency 1: a quarter turn at pos = pi/2 (checked through linearity in pos)
    e = np.zeros((1, 1, 16)); e[0, 0, 0] = 1.0
    r = rope(e, np.array([1]), 1e4)[0, 0]
    assert np.isclose(r[0], np.cos(1.0)) and np.isclose(r[half], np.sin(1.0))


def test_rope_scores_depend_on_relative_position_only():
    rng = np.random.default_rng(1)
    q, k = rng.standard_normal((1, 1, 32)), rng.standard_normal((1, 1, 32))
    s0 = (rope(q, np.array([9]), 5e5) * rope(k, np.array([4]), 5e5)).sum()
    s1 = (rope(q, np.array([1009]), 5e5) * rope(k, np.array([1004]), 5e5)).sum()
    s2 = (rope(q, np.array([9]), 5e5) * rope(k, np.array([5]), 5e5)).sum()
    assert np.isclose(s0, s1) and not np.isclose(s0, s2)


def test_rmsnorm_closed_form():
    x = np.full((1, 8), 3.0)
    w = np.arange(1, 9, dtype=np.float64)
    assert np.allclose(rmsnorm(x, w, 1e-5), 3.0 / np.sqrt(9.0 + 1e-5) * w)
    y = rmsnorm(np.array([[3.0, -4.0]]), np.ones(2), 0.0)              # rms = sqrt(12.5)
    assert np.allclose(y, np.array([[3.0, -4.0]]) / np.sqrt(12.5))


def test_attention_closed_forms():
    rng = np.random.default_rng(2)
    q = rng.standard_normal(8)
    v = rng.standard_normal((5, 8))
    same = np.tile(rng.standard_normal(8), (5, 1))
    assert np.allclose(attention_row(q, same, v), v.mean(axis=0))       # equal keys -> mean of values
    assert np.allclose(attention_row(q, same[:1], v[:1]), v[0])         # one key -> its value
    # two keys, scores s and 0: weights are sigmoid(s / sqrt(hd))
    keys = np.stack([q, np.zeros(8)])
    s = q @ q / np.sqrt(8)
    pw = 1 / (1 + np.exp(-s))
    assert np.allclose(attention_row(q, keys, v[:2]), pw * v[0] + (1 - pw) * v[1])


def test_gqa_heads_share_kv(tiny):
    """With the q heads of one group fed identical queries, their outputs coincide."""
    sh = GQA
    w = as_dtype(wl.make_weights(sh, std=0.2), np.float64)
    p = "layers.0."
    w[p + "wq"][sh.head_dim:2 * sh.head_dim] = w[p + "wq"][:sh.head_dim]   # head 1 := head 0 (same kv group)
    from oracle import decoder_layer
    h = np.random.default_rng(3).standard_normal((4, sh.d_model))
    cache = KVCache(sh.n_layers, 4, sh.n_kv_heads, sh.head_dim)
    # recover the attention output through wo = identity on the first two heads
    w[p + "wo"] = np.eye(sh.d_model, sh.d_q)
    w[p + "w_down"] = np.zeros_like(w[p + "w_down"])
    out = decoder_layer(h, w, p, sh, 0, cache, np.arange(4), list(range(4)), causal(4)) - h
    assert np.allclose(out[:, :sh.head_dim], out[:, sh.head_dim:2 * sh.head_dim])
    assert not np.allclose(out[:, :sh.head_dim], out[:, 2 * sh.head_dim:3 * sh.head_dim])
