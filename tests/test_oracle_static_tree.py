"""Pins of the static-tree drafting oracle (oracle/static_tree.py): at T = 0 any tree shape leaves the output equal
to plain greedy decoding (the lossless-acceptance statement of Sec. 4.1, Metrics); a static shape with the dynamic
tree's own nodes drafts the same tokens as the dynamic tree; sampled children make honest draws (chi-square on the
first emitted token with the model's own rows)."""
import numpy as np
import pytest
from scipy import stats

import workload as wl
from oracle import draft_tree, greedy_decode, prefill, verify_tree
from oracle import qratio
from oracle.static_tree import StaticShape, draft_static, spec_decode_static

# a small tree in the style of the static-tree comparison system: 4 / 3+2+1 / 2+1 / 1 nodes per depth
EAGLE_LIKE = StaticShape(parent=[-1, 0, 0, 0, 0, 1, 1, 1, 2, 2, 3, 5, 5, 6, 11],
                         rank=[0, 0, 1, 2, 3, 0, 1, 2, 0, 1, 0, 0, 1, 0, 0])


@pytest.mark.parametrize("shape_", [StaticShape.chain(1), StaticShape.chain(5), EAGLE_LIKE], ids=["chain1", "chain5", "tree15"])
def test_greedy_output_is_unchanged_by_any_static_shape(tiny, shape_):
    sh, w, prompt = tiny
    want = greedy_decode(w, sh, prompt, 24)
    got, taus = spec_decode_static(w, sh, prompt, 24, shape_)
    assert got == want and sum(taus) >= 23 and min(taus) >= 1


def test_static_shape_of_the_dynamic_trees_first_levels_drafts_the_same_tokens(tiny):
    # depth-1 and depth-2 nodes of a top-k tree: children of the root are its top-3, children of the best are its top-2
    sh, w, prompt = tiny
    st, _ = prefill(w, sh, prompt, 128)
    st.cycle = 1
    dyn = draft_tree(st.__class__(**{**st.__dict__, "tcache": st.tcache.copy(), "dcache": st.dcache.copy()}), 2, 3, 1 + 3 + 9)
    ss = StaticShape(parent=[-1, 0, 0, 0, 1, 1, 1], rank=[0, 0, 1, 2, 0, 1, 2])
    tree, _ = draft_static(st, ss)
    # the dynamic tree's depth-1 nodes are the root's top-3 in order; its node 1 is the best of them
    d1 = [j for j in range(dyn.n_nodes) if dyn.depth[j] == 1]
    assert [int(dyn.token[j]) for j in d1] == [int(t) for t in tree.token[1:4]]
    kids_dyn = [int(dyn.token[j]) for j in range(dyn.n_nodes) if dyn.parent[j] == d1[0]]
    assert kids_dyn == [int(t) for t in tree.token[4:7]]
    np.testing.assert_allclose(tree.score[1:4], [dyn.score[j] for j in d1], rtol=1e-6)


def test_sampled_children_first_token_chi_square_with_model_rows(tiny):
    # T = 1, three sampled children of the root: over many seeds the first emitted token follows the target's softmax
    sh, w, prompt = tiny
    st, _ = prefill(w, sh, prompt, 128, temperature=1.0, seed=0)
    st.cycle = 1
    ss = StaticShape(parent=[-1, 0, 0, 0], rank=[0, 0, 1, 2])
    tree0, q_logits = draft_static(st, ss, 1.0, True, 0)       # the draft's root row does not depend on the seed
    logits, _ = verify_tree(st, tree0)
    p_rows = np.repeat(logits[:1], 4, axis=0)                  # only node 0's row matters for the first token
    x = logits[0].astype(np.float64)
    p = np.exp(x - x.max()); p /= p.sum()
    counts = np.zeros(sh.vocab)
    n = 40000
    for seed in range(n):
        kids = qratio.sample_children(q_logits[0], 1.0, 3, seed, 1, 0)
        acc, nxt, _ = qratio.accept_qratio([int(tree0.token[0])] + kids, [-1, 0, 0, 0], p_rows, q_logits, 1.0, seed, 1)
        counts[kids[acc[0] - 1] if acc else nxt] += 1
    exp = p * n
    keep = exp >= 5
    obs = np.append(counts[keep], counts[~keep].sum()); ex = np.append(exp[keep], exp[~keep].sum())
    if ex[-1] == 0:
        obs, ex = obs[:-1], ex[:-1]
    assert stats.chisquare(obs, ex).pvalue > 0.01


def test_sampled_run_is_reproducible_and_differs_across_seeds(tiny):
    sh, w, prompt = tiny
    a, ta = spec_decode_static(w, sh, prompt, 20, EAGLE_LIKE, temperature=1.0, seed=3, sampled=True)
    b, tb = spec_decode_static(w, sh, prompt, 20, EAGLE_LIKE, temperature=1.0, seed=3, sampled=True)
    c, _ = spec_decode_static(w, sh, prompt, 20, EAGLE_LIKE, temperature=1.0, seed=4, sampled=True)
    assert a == b and ta == tb and a != c and len(a) == 20


def test_shape_validation():
    with pytest.raises(AssertionError):
        StaticShape([-1, 0, 0], [0, 1, 1])                    # two children with the same rank
    with pytest.raises(AssertionError):
        StaticShape([-1, 2, 0], [0, 0, 0])                    # a child before its parent
    with pytest.raises(AssertionError):
        StaticShape([0, 0], [0, 0])                           # node 0 is not a root
    # what the paper leaves open is accepted: any order of the nodes that keeps parents first, any rank, any size
    ss = StaticShape([-1, 0, 1, 0], [0, 0, 0, 1])             # not in order of depth
    assert ss.depth == [0, 1, 2, 1]
    big = StaticShape([-1] + list(range(40)) + [0] * 200, [0] * 41 + list(range(2, 202)))   # depth 40, 241 nodes, rank 201
    assert big.n_nodes == 241 and max(big.depth) == 40 and big.width[0] == 202
    assert not big.children_are_successive_draws() and StaticShape.chain(3).children_are_successive_draws()


def test_unordered_and_deep_shapes_leave_greedy_output_unchanged(tiny):
    sh, w, prompt = tiny
    want = greedy_decode(w, sh, prompt, 16)
    for ss in (StaticShape([-1, 0, 1, 0, 3, 2], [0, 0, 0, 1, 0, 1]),        # depths 0 1 2 1 2 3: not depth-major
               StaticShape.chain(18),                                       # deeper than any product limit
               StaticShape([-1] + [0] * 20, [0] + list(range(20)))):        # 20 proposals at the root
        got, _ = spec_decode_static(w, sh, prompt, 16, ss)
        assert got == want


def test_sampled_children_must_be_the_first_draws(tiny):
    """Why sampled shapes may not skip a rank: the ratio rule divides by the draft distribution renormalised over
    the tokens not yet listed, which is the law of a child only if every earlier draw is listed before it.  With a
    12-token vocabulary and a draft that disagrees with the target, listing draws (0, 1) keeps the emitted token
    target-distributed; listing only draw 1 does not."""
    rng = np.random.default_rng(5)
    V, n = 12, 30000
    p_log, q_log = rng.standard_normal(V) * 1.5, rng.standard_normal(V) * 1.5
    p = np.exp(p_log - p_log.max()); p /= p.sum()

    def pvalue(listed):
        counts = np.zeros(V)
        rows_p, rows_q = np.tile(p_log, (1 + len(listed), 1)), np.tile(q_log, (1 + len(listed), 1))
        for seed in range(n):
            draws = qratio.sample_children(q_log, 1.0, 2, seed, 1, 0)
            kids = [draws[i] for i in listed]
            acc, nxt, _ = qratio.accept_qratio([0] + kids, [-1] + [0] * len(kids), rows_p, rows_q, 1.0, seed, 1)
            counts[kids[acc[0] - 1] if acc else nxt] += 1
        return stats.chisquare(counts, p * n).pvalue

    assert pvalue([0, 1]) > 0.01
    assert pvalue([1]) < 1e-6
    sh, w, prompt = tiny
    st, _ = prefill(w, sh, prompt, 64, temperature=1.0, seed=0)
    st.cycle = 1
    for parent, rank in (([-1, 0], [0, 1]), ([-1, 0, 0], [0, 0, 2]), ([-1, 0, 0], [0, 1, 0])):
        with pytest.raises(AssertionError):
            draft_static(st, StaticShape(parent, rank), 1.0, True, 0)
        draft_static(st.__class__(**{**st.__dict__, "tcache": st.tcache.copy(), "dcache": st.dcache.copy()}),
                     StaticShape(parent, rank))                # the same shapes are fine with deterministic children
