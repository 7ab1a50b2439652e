"""Pins for the T > 0 acceptance rule and the counter-based RNG."""
import os

import numpy as np
import pytest
from scipy import stats

import workload as wl
from oracle import Tree, accept_sample, draft_tree, prefill, verify_tree, sample_decode, spec_decode
from oracle.rng import GOLDEN, gumbel, mix64, uniform01

HERE = os.path.dirname(os.path.abspath(__file__))


def test_mix64_is_splitmix64_finaliser():
    want = [int(l, 16) for l in open(os.path.join(HERE, "golden", "splitmix64_seed0.txt")) if not l.startswith("#")]
    s, got = 0, []
    for _ in range(3):
        s = (s + GOLDEN) & ((1 << 64) - 1)
        got.append(mix64(s))
    assert got == want
    assert list(mix64(np.array([GOLDEN], dtype=np.uint64))) == want[:1]          # array form agrees


def test_uniform_and_gumbel_statistics():
    u = uniform01(3, 1, 2, np.arange(200000))
    assert u.min() > 0 and u.max() < 1 and u.dtype == np.float32
    assert stats.kstest(u, "uniform").pvalue > 0.01
    assert uniform01(3, 1, 2, 5) == u[5]
    assert uniform01(4, 1, 2, 5) != u[5] and uniform01(3, 2, 2, 5) != u[5] and uniform01(3, 1, 3, 5) != u[5]
    g = gumbel(9, 1, 0, 200000)
    assert stats.kstest(g, "gumbel_r").pvalue > 0.01


def chi2_p(counts, probs):
    exp = probs * counts.sum()
    keep = exp >= 5
    obs = np.append(counts[keep], counts[~keep].sum())
    ex = np.append(exp[keep], exp[~keep].sum())
    if ex[-1] == 0:
        obs, ex = obs[:-1], ex[:-1]
    return stats.chisquare(obs, ex).pvalue


def test_first_token_distribution_tiny_1e5_seeds(tiny):
    """Check (b): over 1e5 seeds the token a cycle emits first follows softmax(logits[root]) (T = 1)."""
    sh, w, prompt = tiny
    st, _ = prefill(w, sh, prompt, 128, temperature=1.0, seed=0)
    st.cycle = 1
    tree = draft_tree(st, sh.tree_depth, sh.tree_topk, sh.tree_total)
    logits, _ = verify_tree(st, tree)
    x = logits[0].astype(np.float64)
    p = np.exp(x - x.max()); p /= p.sum()
    counts = np.zeros(sh.vocab)
    for seed in range(100000):
        acc, bonus = accept_sample(tree, logits, 1.0, seed, 1)
        counts[int(tree.token[acc[0]]) if acc else bonus] += 1
    assert (p * 1e5).min() >= 5                      # every bin is populated enough for the test
    assert chi2_p(counts, p) > 0.01


def test_joint_distribution_micro_vocab():
    """Peaky synthetic logits over 12 tokens, a two-level tree with duplicate and low-probability
    children: the first two emitted tokens follow p(x1) p(x2 | x1) of the target."""
    V = 12
    rng = np.random.default_rng(0)
    #          0  1  2  3  4  5  6
    tok = [0, 3, 5, 3, 7, 1, 2]          # node 3 duplicates node 1's token under the same parent
    par = [-1, 0, 0, 0, 1, 1, 2]
    dep = [0, 1, 1, 1, 2, 2, 2]
    tree = Tree(np.array(tok, np.int32), np.array(par, np.int32), np.array(dep, np.int32), np.zeros(7, np.float32))
    logits = rng.standard_normal((7, V)) * 2.0
    P = np.exp(logits - logits.max(1, keepdims=True)); P /= P.sum(1, keepdims=True)
    child_by_tok = {0: {3: 1, 5: 2}, 1: {7: 4, 1: 5}, 2: {2: 6}}
    n_seeds = 60000
    c1 = np.zeros(V)
    c2 = {1: np.zeros(V), 2: np.zeros(V)}
    for seed in range(n_seeds):
        acc, bonus = accept_sample(tree, logits, 1.0, seed, 3)
        seq = [tok[j] for j in acc] + [bonus]
        c1[seq[0]] += 1
        if acc and len(seq) >= 2:
            c2[acc[0]][seq[1]] += 1
        # an accepted node is always the first child carrying that token
        if acc:
            assert acc[0] == child_by_tok[0][seq[0]]
    assert chi2_p(c1, P[0]) > 0.01
    for node in (1, 2):
        assert c2[node].sum() > 2000
        assert chi2_p(c2[node], P[node]) > 0.01


def test_chain_accept_probability_is_min_1_p_over_q():
    """K = 1 chain with a point-mass proposal q: the textbook accept probability min(1, p/q) = p."""
    V = 6
    tree = Tree(np.array([0, 4], np.int32), np.array([-1, 0], np.int32), np.array([0, 1], np.int32), np.zeros(2, np.float32))
    logits = np.log(np.array([[0.05, 0.1, 0.15, 0.2, 0.37, 0.13], [1 / 6] * 6]))
    n = 40000
    hits = sum(1 for s in range(n) if accept_sample(tree, logits, 1.0, s, 0)[0])
    assert abs(hits / n - 0.37) < 4 * np.sqrt(0.37 * 0.63 / n)
    # temperature: T = 0.5 squares the probabilities
    p2 = np.array([0.05, 0.1, 0.15, 0.2, 0.37, 0.13]) ** 2
    p2 /= p2.sum()
    hits = sum(1 for s in range(n) if accept_sample(tree, logits, 0.5, s, 0)[0])
    assert abs(hits / n - p2[4]) < 4 * np.sqrt(p2[4] * (1 - p2[4]) / n)


def test_certain_child_is_accepted_and_residual_excludes_rejected():
    V = 5
    tree = Tree(np.array([0, 2], np.int32), np.array([-1, 0], np.int32), np.array([0, 1], np.int32), np.zeros(2, np.float32))
    logits = np.full((2, V), -1e4); logits[0, 2] = 0.0; logits[1, 1] = 0.0      # p(2) == 1 exactly
    for s in range(50):
        acc, bonus = accept_sample(tree, logits, 1.0, s, 0)
        assert acc == [1] and bonus == 1
    logits = np.zeros((2, V))                                                       # uniform: child 2 w.p. 1/5
    for s in range(300):
        acc, bonus = accept_sample(tree, logits, 1.0, s, 0)
        assert acc or bonus != 2                                                    # a rejected token is never the bonus


def test_plain_sampling_definition_matches_softmax(tiny):
    """The T > 0 definition layer itself: the first sampled token follows softmax(last prompt logits)."""
    sh, w, prompt = tiny
    from oracle import KVCache, target_forward
    n = 8
    cache = KVCache(sh.n_layers, n + 2, sh.n_kv_heads, sh.head_dim)
    logits, _ = target_forward(w, sh, cache, prompt[:n], np.arange(n), list(range(n)), [list(range(i + 1)) for i in range(n)])
    x = logits[-1] * 8.0                                     # sharpen so that 2e4 draws populate the bins
    p = np.exp(x - x.max()); p /= p.sum()
    counts = np.zeros(sh.vocab)
    for seed in range(20000):
        counts[int(np.argmax(x.astype(np.float32) + gumbel(seed, 0, 0, sh.vocab)))] += 1
    assert chi2_p(counts, p) > 0.01
    a = sample_decode(w, sh, prompt[:n], 3, 1.0, seed=5)
    b = sample_decode(w, sh, prompt[:n], 3, 1.0, seed=5)
    assert a == b and len(a) == 3


def test_spec_sampling_run_is_reproducible_and_counts_tokens(tiny):
    sh, w, prompt = tiny
    a, ta = spec_decode(w, sh, prompt, 10, temperature=1.0, seed=3)
    b, tb = spec_decode(w, sh, prompt, 10, temperature=1.0, seed=3)
    c, _ = spec_decode(w, sh, prompt, 10, temperature=1.0, seed=4)
    assert a == b and ta == tb and a != c and len(a) == 10
