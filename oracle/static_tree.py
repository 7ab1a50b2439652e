"""Static draft trees with deterministic or SAMPLED children (test infrastructure; nothing on the product path
imports this).

Sec. 4.1, Comparisons and Sec. 2: EAGLE drafts a tree whose SHAPE is fixed in advance (EAGLE-2 / HASS replace
it by the dynamic tree of oracle/spec.py), and chain speculative sampling is the shape with one child per
node.  A shape is given per node (node 0 = root, nodes in order of depth, parents before children) by its
parent and by its RANK among the parent's proposals: rank r is the r-th best token of the draft distribution
at the parent (deterministic children) or the r-th token drawn from it without replacement (sampled children,
oracle/qratio.py).  Every node that has children is run through the draft model once, all nodes of a depth
in one forward, exactly as the dynamic tree's expansion steps are.  With sampled children the acceptance is
the ratio rule of oracle/qratio.py; with deterministic children it is the point-mass rule of oracle/spec.py.

reading: the paper fixes no particular shape, so any tree is accepted: parents before children, and the
children of a node carrying distinct ranks.  Sampled children have one more condition, which the acceptance rule
itself imposes: the ratio rule tries the children of a node as successive draws without replacement from the
draft distribution, so they must BE the first c draws, in draw order (ranks 0, 1, ..., c-1 in node order).  A
child of rank r whose earlier draws are missing from the tree follows the marginal of the (r+1)-th draw, not
the renormalised draft distribution the rule divides by, and the output would no longer be target-distributed
(tests/test_oracle_static_tree.py shows the chi-square test failing for such a shape).
"""
from __future__ import annotations

import dataclasses
from typing import Dict, List, Optional, Sequence, Tuple

import numpy as np

from . import qratio
from .llama import draft_forward
from .spec import SpecState, Tree, _kw, accept_greedy, accept_sample, commit, log_softmax, prefill, top_k, verify_tree


@dataclasses.dataclass
class StaticShape:
    parent: List[int]        # parent[0] = -1
    rank: List[int]          # rank[0] = 0

    def __post_init__(self):
        n = len(self.parent)
        assert n == len(self.rank) and n >= 1 and self.parent[0] == -1
        self.depth = [0] * n
        for i in range(1, n):
            assert 0 <= self.parent[i] < i, "a parent precedes its children"
            assert self.rank[i] >= 0
            self.depth[i] = self.depth[self.parent[i]] + 1
        self.n_nodes = n
        self.children = [[i for i in range(1, n) if self.parent[i] == u] for u in range(n)]
        for u in range(n):
            ranks = [self.rank[c] for c in self.children[u]]
            assert len(set(ranks)) == len(ranks), "the children of a node carry distinct ranks"
        self.expanded = [u for u in range(n) if self.children[u]]           # nodes run through the draft model
        self.width = [1 + max((self.rank[c] for c in self.children[u]), default=-1) for u in range(n)]

    def children_are_successive_draws(self) -> bool:
        """True when every node's children have ranks 0, 1, ..., c-1 in node order (what sampled children need)."""
        return all([self.rank[c] for c in self.children[u]] == list(range(len(self.children[u]))) for u in range(self.n_nodes))

    @staticmethod
    def chain(length: int) -> "StaticShape":
        return StaticShape([-1] + list(range(length)), [0] * (length + 1))


def draft_static(st: SpecState, shape_: StaticShape, temperature: float = 0.0, sampled: bool = False,
                 seed: int = 0) -> Tuple[Tree, np.ndarray]:
    """-> (tree, q_logits [n_nodes, V]: the draft's logit row at every expanded node, zeros elsewhere)."""
    w, shape, n = st.w, st.shape, st.n
    ss = shape_
    assert not sampled or ss.children_are_successive_draws(), "sampled children must be the first draws, in draw order"
    m1 = len(st.pend_tokens)
    pos = np.arange(n - m1 + 1, n + 1)
    logits, g = draft_forward(w, shape, st.dcache, st.pend_feats, st.pend_tokens, pos, list(pos),
                              [list(range(1, p + 1)) for p in pos], **_kw(st))
    q_logits = np.zeros((ss.n_nodes, shape.vocab), dtype=np.float32)
    g_of: Dict[int, np.ndarray] = {0: g[-1]}
    token = np.zeros(ss.n_nodes, dtype=np.int32)
    score = np.zeros(ss.n_nodes, dtype=np.float32)
    token[0] = st.root
    slot_of: Dict[int, int] = {}
    next_slot = n + 1

    def propose(u: int, row: np.ndarray):
        """Fill tokens and scores of u's children from the draft's logit row at u."""
        q_logits[u] = row.astype(np.float32)
        lp = log_softmax(row).astype(np.float32)
        if sampled:
            picks = qratio.sample_children(row, temperature, ss.width[u], seed, st.cycle, u)
        else:
            picks = [int(v) for v in top_k(lp, ss.width[u])]
        for c in ss.children[u]:
            token[c] = picks[ss.rank[c]]
            score[c] = np.float32(score[u] + lp[token[c]])

    if ss.children[0]:
        propose(0, logits[-1])
    max_depth = max(ss.depth)
    for t in range(1, max_depth):
        rows = [u for u in ss.expanded if ss.depth[u] == t]
        if not rows:
            continue
        feats = np.stack([g_of[ss.parent[u]] for u in rows])
        toks = np.array([token[u] for u in rows])
        slots, vis = [], []
        for u in rows:
            slot_of[u] = next_slot; next_slot += 1
            anc, a = [], u
            while a > 0:
                anc.append(slot_of[a]); a = ss.parent[a]
            slots.append(slot_of[u]); vis.append(list(range(1, n + 1)) + anc[::-1])
        lg, gg = draft_forward(w, shape, st.dcache, feats, toks, np.full(len(rows), n + t), slots, vis, **_kw(st))
        for r, u in enumerate(rows):
            g_of[u] = gg[r]
            propose(u, lg[r])
    tree = Tree(token, np.array(ss.parent, dtype=np.int32), np.array(ss.depth, dtype=np.int32), score)
    return tree, q_logits


def spec_decode_static(w, shape, prompt: np.ndarray, gen: int, shape_: StaticShape, *, temperature: float = 0.0, seed: int = 0,
                       sampled: bool = False, dtype=np.float64, record: Optional[list] = None):
    """Whole run with a static tree.  Returns (tokens[:gen], emitted-per-cycle list)."""
    assert not sampled or temperature > 0
    max_seq = len(prompt) + gen + 2 * shape_.n_nodes + 20
    st, first = prefill(w, shape, prompt, max_seq, temperature, seed, dtype)
    out, taus = [first], []
    while len(out) < gen:
        st.cycle += 1
        tree, q_logits = draft_static(st, shape_, temperature, sampled, seed)
        logits, feats = verify_tree(st, tree)
        margin = np.inf
        if temperature > 0 and sampled:
            acc, bonus, margin = qratio.accept_qratio(tree.token, tree.parent, logits, q_logits, temperature, seed, st.cycle)
        elif temperature > 0:
            acc, bonus = accept_sample(tree, logits, temperature, seed, st.cycle)
        else:
            acc, bonus = accept_greedy(tree, logits)
        if record is not None:
            record.append(dict(n=st.n, tree=tree, logits=logits, feats=feats, q_logits=q_logits, accepted=list(acc), bonus=bonus,
                               margin=margin))
        emitted = commit(st, tree, feats, acc, bonus)
        out += emitted
        taus.append(len(emitted))
    return out[:gen], taus
