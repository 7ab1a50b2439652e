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
        StaticShape([-1, 0, 1, 0], [0, 0, 0, 1])              # not in order of depth
    with pytest.raises(AssertionError):
        StaticShape([-1, 0], [0, 16])                         # rank beyond the proposal limit
