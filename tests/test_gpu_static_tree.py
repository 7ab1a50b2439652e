"""GPU parity of static-tree drafting (spec_set_static_tree + the usual draft / verify / accept calls) against
oracle/static_tree.py: deterministic children at T = 0 (tokens, trees, logits per cycle; output equal to plain
greedy decoding), deterministic children at T = 1 (the point-mass rule), and SAMPLED children at T = 1 (Gumbel-top-m
drafting + the ratio rule; the oracle reports each cycle's smallest decision margin, and the comparison stops at
the first cycle whose fp64 decision sits within 1e-4 of the boundary, since the kernel decides in fp32)."""
import numpy as np
import pytest

import workload as wl
import oracle
from oracle.llama import as_dtype
from oracle.static_tree import StaticShape, spec_decode_static

pytestmark = pytest.mark.gpu

EAGLE_LIKE = StaticShape(parent=[-1, 0, 0, 0, 0, 1, 1, 1, 2, 2, 3, 5, 5, 6, 11],
                         rank=[0, 0, 1, 2, 3, 0, 1, 2, 0, 1, 0, 0, 1, 0, 0])
SHAPES = {"chain1": StaticShape.chain(1), "chain5": StaticShape.chain(5), "tree15": EAGLE_LIKE,
          "wide": StaticShape(parent=[-1] + [0] * 16 + [1, 1, 16], rank=[0] + list(range(16)) + [0, 3, 2]),
          # the same width with gap-free ranks: what sampled children need (each child is the next draw)
          "wide_draws": StaticShape(parent=[-1] + [0] * 16 + [1, 1, 16], rank=[0] + list(range(16)) + [0, 1, 0])}
CAP = (6, 8, 40)            # configured capacity: depth * top-k bounds the expanded nodes, total bounds the nodes


@pytest.fixture(scope="module")
def env():
    import torch
    import paper_2408_15766_amd as P
    assert torch.cuda.is_available()
    return torch, P


@pytest.fixture(scope="module")
def tiny_gpu(env):
    torch, P = env
    sh = wl.TINY
    hw = wl.make_weights(sh)
    return sh, hw, as_dtype(hw, np.float64), wl.make_prompt(sh), P.upload_weights(hw, sh.dtype)


def run_gpu(P, sh, dw, prompt, gen, ss, temperature=0.0, seed=0, sampled=False):
    eng = P.Engine(sh, dw, tree=CAP, temperature=temperature, seed=seed)
    eng.set_static_tree(ss.parent, ss.rank, sampled)
    rec = []
    got, taus = eng.generate(prompt, gen, record=rec)
    return got, taus, rec


@pytest.mark.parametrize("name", list(SHAPES))
def test_static_shapes_greedy_match_oracle(env, tiny_gpu, name):
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    ss = SHAPES[name]
    gen = 24
    got, taus, grec = run_gpu(P, sh, dw, prompt, gen, ss)
    orec = []
    want, wt = spec_decode_static(w64, sh, prompt, gen, ss, record=orec)
    assert want == oracle.greedy_decode(w64, sh, prompt, gen)
    assert got == want and taus == wt and len(grec) == len(orec)
    for a, b in zip(grec, orec):
        ta, tb = a["tree"], b["tree"]
        assert ta.n_nodes == tb.n_nodes == ss.n_nodes
        assert list(ta.token) == list(tb.token) and list(ta.parent) == list(tb.parent) and list(ta.depth) == list(tb.depth)
        assert np.abs(ta.score - tb.score).max() < 5e-5
        assert np.abs(a["logits"] - b["logits"]).max() < 1e-4


def test_static_tree_filling_the_configured_total_uses_the_replayed_verify(env, tiny_gpu):
    # with n_nodes == tree_total the verify forward is the captured graph (as for the dynamic tree); same results
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    eng = P.Engine(sh, dw, tree=(6, 8, EAGLE_LIKE.n_nodes))
    eng.set_static_tree(EAGLE_LIKE.parent, EAGLE_LIKE.rank)
    rec = []
    got, taus = eng.generate(prompt, 24, record=rec)
    orec = []
    want, wt = spec_decode_static(w64, sh, prompt, 24, EAGLE_LIKE, record=orec)
    assert got == want and taus == wt
    for a, b in zip(rec, orec):
        assert list(a["tree"].token) == list(b["tree"].token)
        assert np.abs(a["logits"] - b["logits"]).max() < 1e-4


def test_static_tree_point_mass_rule_matches_oracle(env, tiny_gpu):
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    got, taus, _ = run_gpu(P, sh, dw, prompt, 30, EAGLE_LIKE, temperature=1.0, seed=5)
    want, wt = spec_decode_static(w64, sh, prompt, 30, EAGLE_LIKE, temperature=1.0, seed=5)
    assert got == want and taus == wt


@pytest.mark.parametrize("name,seed", [("tree15", 1), ("tree15", 2), ("chain5", 3), ("wide_draws", 4)])
def test_static_tree_sampled_children_match_oracle(env, tiny_gpu, name, seed):
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    ss = SHAPES[name]
    gen = 30
    got, taus, grec = run_gpu(P, sh, dw, prompt, gen, ss, temperature=1.0, seed=seed, sampled=True)
    orec = []
    want, wt = spec_decode_static(w64, sh, prompt, gen, ss, temperature=1.0, seed=seed, sampled=True, record=orec)
    compared = 0
    for a, b in zip(grec, orec):
        assert list(a["tree"].token) == list(b["tree"].token), "sampled children differ"
        if b["margin"] < 1e-4:
            break
        assert a["emitted"] == [int(b["tree"].token[j]) for j in b["accepted"]] + [b["bonus"]]
        compared += 1
    assert compared >= min(len(orec), 5)
    if compared == len(orec):
        assert got == want and taus == wt


def test_static_tree_errors_and_return_to_dynamic(env, tiny_gpu):
    torch, P = env
    sh, hw, w64, prompt, dw = tiny_gpu
    eng = P.Engine(sh, dw, tree=CAP)
    for parent, rank in [([-1, 0, 0], [0, 1, 1]),            # equal ranks
                         ([-1, 0, 0], [0, 1, 0]),            # ranks not increasing
                         ([-1, 0, 1, 0], [0, 0, 0, 1]),      # not in order of depth
                         ([0, 0], [0, 0]),                   # node 0 is not a root
                         ([-1, 0], [0, 16])]:                # rank beyond the proposal limit
        with pytest.raises(P.SpecError):
            eng.set_static_tree(parent, rank)
    with pytest.raises(P.SpecError):
        eng.set_static_tree([-1] + list(range(45)), [0] * 46)            # more nodes than tree_total = 40
    with pytest.raises(P.SpecError):
        eng.set_static_tree([-1, 0], [0, 0], sampled=True)               # sampled children need T > 0
    hot = P.Engine(sh, dw, tree=CAP, temperature=1.0, seed=1)
    for parent, rank in [([-1, 0], [0, 1]), ([-1, 0, 0], [0, 0, 2]), (SHAPES["wide"].parent, SHAPES["wide"].rank)]:
        with pytest.raises(P.SpecError) as e:                             # sampled children with a rank skipped
            hot.set_static_tree(parent, rank, sampled=True)
        assert e.value.code == P.binding.SPEC_EINVAL
        hot.set_static_tree(parent, rank)                                 # fine with deterministic children
    hot.close()
    # a shape, then back to the dynamic tree: the dynamic result is the one of a fresh context
    eng.set_static_tree(EAGLE_LIKE.parent, EAGLE_LIKE.rank)
    first = eng.prefill(prompt)
    t = eng.draft_tree()
    assert t.n_nodes == 15 and list(t.parent[:15]) == EAGLE_LIKE.parent
    eng.verify(t)
    out = eng.accept(t)
    eng.set_static_tree([], [])
    rest, _ = [], None
    toks = [first] + out
    while len(toks) < 20:
        t = eng.draft_tree()
        assert t.n_nodes == CAP[2]
        eng.verify(t)
        toks += eng.accept(t)
    assert toks[:20] == oracle.greedy_decode(w64, sh, prompt, 20)
    with pytest.raises(P.SpecError):                                      # not between cycles
        t = eng.draft_tree()
        eng.set_static_tree(EAGLE_LIKE.parent, EAGLE_LIKE.rank)


def test_bf16_static_chain_equals_greedy_bit_exact(env):
    torch, P = env
    sh = wl.LLAMA2_7B.with_(name="llama2-7b-2layer", n_layers=2, prompt_len=96, gen_tokens=24)
    hw = wl.make_weights(sh)
    dw = P.upload_weights(hw, sh.dtype)
    prompt = wl.make_prompt(sh)
    plain = P.Engine(sh, dw, tree=(1, 1, 1))
    greedy, _ = plain.generate(prompt, 24)
    for ss in (StaticShape.chain(4), EAGLE_LIKE):
        eng = P.Engine(sh, dw)
        eng.set_static_tree(ss.parent, ss.rank)
        got, _ = eng.generate(prompt, 24)
        assert got == greedy
