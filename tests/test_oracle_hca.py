"""Pins of the training-attention oracle (oracle/hca.py) against things other than itself:
a library attention routine, the per-query definition of Sec. 3.2 built by explicit concatenation,
and the statement that training step j equals j autoregressive draft calls (Sec. 3.2, Figure 2 caption),
checked against the decode-side draft model with its KV cache."""
import numpy as np
import pytest
import torch

import workload as wl
from oracle import hca
from oracle.llama import KVCache, as_dtype, draft_forward


def _streams(seed, n_streams, t_len, hq, hkv, hd):
    g = np.random.default_rng(seed)
    q = g.standard_normal((t_len, hq, hd))
    ks = [g.standard_normal((t_len, hkv, hd)) for _ in range(n_streams)]
    vs = [g.standard_normal((t_len, hkv, hd)) for _ in range(n_streams)]
    return q, ks, vs


def _sdpa(q, k, v, causal):
    """torch's attention; q [Tq, hd], k, v [Tk, hd], float64."""
    o = torch.nn.functional.scaled_dot_product_attention(torch.from_numpy(q)[None], torch.from_numpy(k)[None],
                                                         torch.from_numpy(v)[None], is_causal=causal)
    return o[0].numpy()


def test_single_stream_is_causal_attention():
    # Sec. 3.2, first step: the mask is the plain causal one.
    q, ks, vs = _streams(1, 1, 37, 4, 2, 16)
    out = hca.hca_attention(q, ks, vs)
    for h in range(4):
        np.testing.assert_allclose(out[:, h], _sdpa(q[:, h], ks[0][:, h // 2], vs[0][:, h // 2], True), rtol=1e-12, atol=1e-13)


@pytest.mark.parametrize("n_streams", [2, 3, 4, 5])
def test_equals_attention_over_the_concatenated_context(n_streams):
    # Sec. 3.2 formula: at position t the context is target entries 1..t-j+1 followed by one entry of each
    # earlier draft step, oldest step first, the newest step's entry at position t itself.
    t_len, hq, hkv, hd = 23, 4, 2, 8
    q, ks, vs = _streams(10 + n_streams, n_streams, t_len, hq, hkv, hd)
    out = hca.hca_attention(q, ks, vs)
    for t in range(t_len):
        n_target = max(t - n_streams + 2, 0)                  # entries 0 .. t-J+1
        for h in range(hq):
            kv = h // (hq // hkv)
            keys = [ks[0][s, kv] for s in range(n_target)]
            vals = [vs[0][s, kv] for s in range(n_target)]
            for m in range(1, n_streams):                     # stream m sits at position t - (J-1-m)
                s = t - (n_streams - 1 - m)
                if s >= 0:
                    keys.append(ks[m][s, kv])
                    vals.append(vs[m][s, kv])
            assert len(keys) == t + 1
            ref = _sdpa(q[t:t + 1, h], np.stack(keys), np.stack(vals), False)[0]
            np.testing.assert_allclose(out[t, h], ref, rtol=1e-11, atol=1e-12)


def test_identical_streams_reduce_to_causal_attention():
    q, ks, vs = _streams(3, 1, 29, 2, 2, 8)
    out1 = hca.hca_attention(q, ks, vs)
    out3 = hca.hca_attention(q, ks * 3, vs * 3)
    np.testing.assert_allclose(out3, out1, rtol=1e-12, atol=1e-13)


def test_which_entries_of_a_stream_matter():
    # Entry s of stream m (m >= 1) is seen by query s + (J-1-m) only; entry s of stream 0 by queries >= s + J-1.
    n_streams, t_len = 3, 19
    q, ks, vs = _streams(4, n_streams, t_len, 2, 1, 8)
    base = hca.hca_attention(q, ks, vs)
    for m in range(n_streams):
        for s in (0, 7, t_len - 2, t_len - 1):
            ks2 = [k.copy() for k in ks]
            vs2 = [v.copy() for v in vs]
            ks2[m][s] += 1.0
            vs2[m][s] -= 2.0
            changed = np.abs(hca.hca_attention(q, ks2, vs2) - base).max(axis=(1, 2)) > 1e-9
            if m == 0:
                expect = np.arange(t_len) >= s + n_streams - 1
            else:
                expect = np.arange(t_len) == s + (n_streams - 1 - m)
            assert (changed == expect).all(), (m, s)


def test_heads_argument_selects_heads():
    q, ks, vs = _streams(5, 2, 11, 4, 2, 8)
    full = hca.hca_attention(q, ks, vs)
    some = hca.hca_attention(q, ks, vs, heads=[1, 3])
    np.testing.assert_array_equal(some[:, [1, 3]], full[:, [1, 3]])
    assert not some[:, [0, 2]].any()


def _passes(sh, w, target_in, tokens, pos, n_steps):
    """Training steps 1..n_steps -> list of predicted features, each [T, d]."""
    inputs = [target_in]
    preds = []
    for _ in range(n_steps):
        g = hca.draft_train_pass(w, sh, inputs, tokens, pos)
        preds.append(g)
        inputs.append(hca.next_stream(target_in, g))
    return preds


@pytest.fixture(scope="module")
def tiny_train():
    sh = wl.TINY
    w = as_dtype(wl.make_weights(sh), np.float64)
    g = np.random.default_rng(7)
    t_len = 12
    target_in = g.standard_normal((t_len, sh.d_model))
    tokens = g.integers(0, sh.vocab, t_len)
    pos = np.arange(t_len)
    return sh, w, target_in, tokens, pos, _passes(sh, w, target_in, tokens, pos, 4)


@pytest.mark.parametrize("step", [1, 2, 3, 4])
def test_training_step_equals_autoregressive_draft_calls(tiny_train, step):
    # Figure 2 caption / Sec. 3.2: step j in a batch = the j-th autoregressive draft call at decoding time.
    # The decode-side draft model (its own KV cache, one row at a time) is run that way for every position.
    sh, w, target_in, tokens, pos, preds = tiny_train
    t_len = len(tokens)
    for t in range(step - 1, t_len):
        p0 = t - (step - 1)
        cache = KVCache(1, t_len, sh.n_kv_heads, sh.head_dim)
        rows = list(range(p0 + 1))
        _, g = draft_forward(w, sh, cache, target_in[:p0 + 1], tokens[:p0 + 1], pos[:p0 + 1], rows,
                             [list(range(i + 1)) for i in rows])
        feat = g[-1]
        for p in range(p0 + 1, t + 1):                        # the draft continues from its own output
            _, g = draft_forward(w, sh, cache, feat[None], tokens[p:p + 1], pos[p:p + 1], [p], [list(range(p + 1))])
            feat = g[0]
        np.testing.assert_allclose(preds[step - 1][t], feat, rtol=1e-9, atol=1e-10)


def test_first_positions_repeat_the_earlier_step(tiny_train):
    # Positions with fewer than j-1 predecessors have no older draft entries to see: step j there equals step t+1.
    *_, preds = tiny_train
    for step in range(2, 5):
        for t in range(step - 1):
            np.testing.assert_allclose(preds[step - 1][t], preds[t][t], rtol=1e-10, atol=1e-11)


def test_later_steps_differ_from_the_first(tiny_train):
    # guards the pins above against a vacuous pass (streams ignored)
    *_, preds = tiny_train
    assert np.abs(preds[2][5:] - preds[0][5:]).max() > 1e-3
