"""Pins of the ratio acceptance rule for sampled draft tokens (oracle/qratio.py): losslessness by chi-square
(the emitted token follows the target distribution whatever the draft distribution is: Sec. 2, third step),
the closed-form acceptance rate 1 - TV(p, q), and the reduction to the already pinned point-mass rule."""
import numpy as np
import pytest
import scipy.stats

from oracle import qratio
from oracle.spec import Tree, accept_sample


def _softmax(x):
    e = np.exp(x - x.max())
    return e / e.sum()


def _first_token_counts(p_logits, q_logits, m, temperature, n_draws, seed):
    v = p_logits.shape[1]
    counts = np.zeros(v)
    accepted = 0
    for cycle in range(n_draws):
        kids = qratio.sample_children(q_logits[0], temperature, m, seed, cycle, 0)
        token = [0] + kids
        parent = [-1] + [0] * m
        acc, nxt, _ = qratio.accept_qratio(token, parent, p_logits, q_logits, temperature, seed, cycle)
        first = token[acc[0]] if acc else nxt
        counts[first] += 1
        accepted += bool(acc)
    return counts, accepted


@pytest.mark.parametrize("m,temperature", [(1, 1.0), (3, 1.0), (2, 0.7)])
def test_emitted_token_follows_the_target_distribution(m, temperature):
    g = np.random.default_rng(100 + m)
    v = 7
    p_logits = g.standard_normal((1 + m, v)) * 1.5
    q_logits = g.standard_normal((1 + m, v)) * 1.5            # a draft that disagrees with the target
    n = 30000
    counts, _ = _first_token_counts(p_logits, q_logits, m, temperature, n, seed=5)
    expect = _softmax(p_logits[0] / temperature) * n
    chi2, pval = scipy.stats.chisquare(counts, expect)
    assert pval > 0.01, (chi2, pval, counts, expect)


def test_a_biased_rule_would_fail_the_chi_square():
    # the same test detects the draft distribution leaking through: always accepting the first child emits q, not p
    g = np.random.default_rng(7)
    v, n = 7, 30000
    p_logits, q_logits = g.standard_normal((2, v)) * 1.5, g.standard_normal((2, v)) * 1.5
    counts = np.zeros(v)
    for cycle in range(n):
        counts[qratio.sample_children(q_logits[0], 1.0, 1, 5, cycle, 0)[0]] += 1
    assert scipy.stats.chisquare(counts, _softmax(p_logits[0]) * n)[1] < 1e-6
    assert scipy.stats.chisquare(counts, _softmax(q_logits[0]) * n)[1] > 0.01   # and the sampler itself follows q


def test_acceptance_rate_of_one_child_is_one_minus_total_variation():
    g = np.random.default_rng(8)
    v, n = 5, 30000
    p_logits, q_logits = g.standard_normal((2, v)), g.standard_normal((2, v)) * 2
    _, accepted = _first_token_counts(p_logits, q_logits, 1, 1.0, n, seed=9)
    p, q = _softmax(p_logits[0]), _softmax(q_logits[0])
    rate = np.minimum(p, q).sum()                              # sum_x q(x) min(1, p(x)/q(x))
    assert abs(accepted / n - rate) < 4 * np.sqrt(rate * (1 - rate) / n)


def test_second_token_follows_the_accepted_nodes_target_distribution():
    # two levels: given that child c was accepted, the next emitted token follows p at node c
    g = np.random.default_rng(9)
    v, n, temperature = 5, 40000, 1.0
    counts = {}
    for cycle in range(n):
        p_logits = np.zeros((4, v)); q_logits = np.zeros((4, v))
        gg = np.random.default_rng(1234)                       # the same rows every cycle
        p_logits[:] = gg.standard_normal((4, v)); q_logits[:] = gg.standard_normal((4, v))
        kids = qratio.sample_children(q_logits[0], temperature, 2, 3, cycle, 0)
        token = [0] + kids
        parent = [-1, 0, 0]
        # each child gets one sampled child of its own
        for c in (1, 2):
            token.append(qratio.sample_children(q_logits[c], temperature, 1, 3, cycle, c)[0])
            parent.append(c)
        acc, nxt, _ = qratio.accept_qratio(token, parent, np.vstack([p_logits, p_logits[:1]]), np.vstack([q_logits, q_logits[:1]]),
                                           temperature, 3, cycle)
        if acc:
            c = acc[0]
            second = token[acc[1]] if len(acc) > 1 else nxt
            counts.setdefault(c, np.zeros(v))[second] += 1
    gg = np.random.default_rng(1234)
    p_rows = gg.standard_normal((4, v))
    for c, cnt in counts.items():
        assert cnt.sum() > 2000
        pval = scipy.stats.chisquare(cnt, _softmax(p_rows[c]) * cnt.sum())[1]
        assert pval > 0.01, (c, cnt)


def test_identical_distributions_always_accept():
    g = np.random.default_rng(10)
    z = g.standard_normal((2, 9))
    for cycle in range(200):
        kid = qratio.sample_children(z[0], 1.0, 1, 1, cycle, 0)
        acc, _, _ = qratio.accept_qratio([0] + kid, [-1, 0], z, z, 1.0, 1, cycle)
        assert acc == [1]


def test_point_mass_draft_reduces_to_the_deterministic_children_rule():
    # a chain whose draft distribution is (numerically) a point mass on the drafted token: the ratio rule makes the
    # decisions of the rule for deterministic children (oracle/spec.py: accept_sample), draw for draw
    g = np.random.default_rng(11)
    v, depth = 12, 4
    p_logits = g.standard_normal((depth + 1, v)).astype(np.float32)
    token = np.array([0] + [int(t) for t in g.integers(0, v, depth)], dtype=np.int32)
    parent = np.arange(-1, depth, dtype=np.int32)
    q_logits = np.full((depth + 1, v), -1e4)
    for i in range(depth):
        q_logits[i, token[i + 1]] = 0.0
    tree = Tree(token, parent, np.arange(depth + 1, dtype=np.int32), np.zeros(depth + 1, dtype=np.float32))
    same = 0
    for cycle in range(300):
        a1, b1, margin = qratio.accept_qratio(token, parent, p_logits, q_logits, 1.0, 2, cycle)
        a2, b2 = accept_sample(tree, p_logits, 1.0, 2, cycle)
        if margin > 1e-5:                                     # fp32 (accept_sample) and fp64 agree away from the boundary
            assert a1 == a2
            assert b1 == b2                                   # the bonus: the same residual, the same Gumbel noise
            same += 1
    assert same > 250
