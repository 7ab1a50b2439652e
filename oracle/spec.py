"""Speculative decoding with a dynamic draft tree (test infrastructure).

Follows the three-step statement of speculative sampling (Sec. 2, Preliminary):
the draft model proposes, the target scores all proposals in one parallel
forward, and a lossless acceptance rule keeps a prefix.  The proposal is a
tree: an expansion phase governed by `depth` and a reranking phase that keeps
`number of tokens` (appendix Drafting Hyper-Parameters; 60 tokens / depth 6 in
Sec. 4.1, Implementation), scored by the draft's cumulative log-probability
(its confidence score).  Acceptance is greedy matching at T=0 and multi-round
rejection sampling at T>0, neither of which relaxes the target distribution
(Sec. 4.1, Metrics).  The acceptance length of a cycle is the number of tokens
it emits (Sec. 4.1, Metrics).

Readings taken where the paper is silent are listed in the repository's design
notes; each is marked "reading:" below.

Notation: n = tokens already in the target cache, r = pending root token
(chosen from the target distribution, not yet run through the target),
D = depth, K = top-k, N = rows verified including the root.
"""
from __future__ import annotations

import dataclasses
from typing import Callable, List, Optional, Sequence, Tuple

import numpy as np

from . import rng as _rng
from .llama import KVCache, Weights, draft_forward, target_forward


# --------------------------------------------------------------------------- helpers

def log_softmax(x: np.ndarray) -> np.ndarray:
    m = x.max(axis=-1, keepdims=True)
    return x - m - np.log(np.exp(x - m).sum(axis=-1, keepdims=True))


def top_k(x: np.ndarray, k: int) -> np.ndarray:
    """Indices of the k largest entries, larger first, equal values by lower index."""
    return np.argsort(-x, kind="stable")[:k]


def argmax_low(x: np.ndarray) -> int:
    return int(np.argmax(x))          # numpy returns the first maximal index


@dataclasses.dataclass
class Tree:
    """Flattened draft tree; node 0 is the root, parents precede children."""
    token: np.ndarray    # int32 [n_nodes]
    parent: np.ndarray   # int32 [n_nodes], parent[0] = -1
    depth: np.ndarray    # int32 [n_nodes], depth[0] = 0
    score: np.ndarray    # float32 [n_nodes], cumulative draft log-prob, score[0] = 0

    @property
    def n_nodes(self) -> int:
        return int(self.token.shape[0])

    def path(self, j: int) -> List[int]:
        """Nodes from the root to j, inclusive."""
        p = []
        while j >= 0:
            p.append(j)
            j = int(self.parent[j])
        return p[::-1]

    def children(self, j: int) -> List[int]:
        return [c for c in range(self.n_nodes) if int(self.parent[c]) == j]


@dataclasses.dataclass
class SpecState:
    w: Weights
    shape: object
    tcache: KVCache
    dcache: KVCache
    n: int = 0                      # committed tokens in the target cache
    root: int = -1                  # pending root token
    pend_feats: Optional[np.ndarray] = None   # [m+1, d] true target features of positions n-m-1 .. n-1
    pend_tokens: Optional[np.ndarray] = None  # [m+1] tokens at positions n-m .. n (last one is the root)
    cycle: int = 0
    g_root: Optional[np.ndarray] = None
    store: Callable = None            # storage-type model handed to the forwards (None = identity)


# --------------------------------------------------------------------------- definition layer

def greedy_decode(w: Weights, shape, prompt: np.ndarray, gen: int, dtype=np.float64) -> List[int]:
    """Plain autoregressive greedy decoding of the target: the 1.00x baseline
    and the definition that speculative decoding at T=0 must reproduce."""
    n = len(prompt)
    cache = KVCache(shape.n_layers, n + gen + 1, shape.n_kv_heads, shape.head_dim, dtype)
    logits, _ = target_forward(w, shape, cache, prompt, np.arange(n), list(range(n)),
                               [list(range(i + 1)) for i in range(n)])
    out = [argmax_low(logits[-1].astype(np.float32))]
    while len(out) < gen:
        p = n + len(out) - 1
        logits, _ = target_forward(w, shape, cache, np.array([out[-1]]), np.array([p]), [p], [list(range(p + 1))])
        out.append(argmax_low(logits[0].astype(np.float32)))
    return out


def sample_decode(w: Weights, shape, prompt: np.ndarray, gen: int, temperature: float, seed: int,
                  dtype=np.float64) -> List[int]:
    """Plain ancestral sampling from softmax(logits / T): the definition for T > 0."""
    n = len(prompt)
    cache = KVCache(shape.n_layers, n + gen + 1, shape.n_kv_heads, shape.head_dim, dtype)
    logits, _ = target_forward(w, shape, cache, prompt, np.arange(n), list(range(n)),
                               [list(range(i + 1)) for i in range(n)])
    out: List[int] = []
    row = logits[-1]
    while True:
        g = _rng.gumbel(seed, len(out), 0, shape.vocab)
        out.append(argmax_low(row.astype(np.float32) / np.float32(temperature) + g))
        if len(out) >= gen:
            return out
        p = n + len(out) - 1
        logits, _ = target_forward(w, shape, cache, np.array([out[-1]]), np.array([p]), [p], [list(range(p + 1))])
        row = logits[0]


# --------------------------------------------------------------------------- algorithm layer

def _kw(st_or_store):
    store = st_or_store.store if isinstance(st_or_store, SpecState) else st_or_store
    return {} if store is None else {"store": store}


def prefill(w: Weights, shape, prompt: np.ndarray, max_seq: int, temperature: float = 0.0, seed: int = 0,
            dtype=np.float64, store=None) -> Tuple[SpecState, int]:
    """Target forward over the prompt, first token, and the draft over the prompt pairs.

    reading: pair i = (target feature of position i-1, token at position i) sits
    at rotary position i and predicts the feature of position i."""
    n = len(prompt)
    st = SpecState(w, shape, KVCache(shape.n_layers, max_seq, shape.n_kv_heads, shape.head_dim, dtype),
                   KVCache(1, max_seq, shape.n_kv_heads, shape.head_dim, dtype), store=store)
    logits, feats = target_forward(w, shape, st.tcache, prompt, np.arange(n), list(range(n)),
                                   [list(range(i + 1)) for i in range(n)], **_kw(st))
    last = logits[-1].astype(np.float32)
    if temperature > 0:
        first = argmax_low(last / np.float32(temperature) + _rng.gumbel(seed, 0, 0, shape.vocab))
    else:
        first = argmax_low(last)
    if n > 1:
        pos = np.arange(1, n)
        draft_forward(w, shape, st.dcache, feats[:-1], prompt[1:], pos, list(pos), [list(range(1, p + 1)) for p in pos],
                      **_kw(st))
    st.n, st.root = n, first
    st.pend_feats = feats[-1:].copy()
    st.pend_tokens = np.array([first], dtype=np.int32)
    return st, first


def draft_tree(st: SpecState, depth: int, topk: int, total: int) -> Tree:
    """Expansion (depth) then rerank (number of tokens) -> flattened tree of <= total nodes."""
    w, shape, n = st.w, st.shape, st.n
    # -- root step: draft over the pending pairs, all of which carry true target features
    m1 = len(st.pend_tokens)
    pos = np.arange(n - m1 + 1, n + 1)
    logits, g = draft_forward(w, shape, st.dcache, st.pend_feats, st.pend_tokens, pos, list(pos),
                              [list(range(1, p + 1)) for p in pos], **_kw(st))
    st.g_root = g[-1]
    lp = log_softmax(logits[-1]).astype(np.float32)
    pool_tok: List[int] = []
    pool_par: List[int] = []      # pool index of the parent, -1 = root
    pool_dep: List[int] = []
    pool_sc: List[np.float32] = []
    for v in top_k(lp, topk):
        pool_tok.append(int(v)); pool_par.append(-1); pool_dep.append(1); pool_sc.append(lp[v])
    frontier = list(range(len(pool_tok)))
    g_of = {}                     # pool idx -> predicted feature of an expanded node
    slot_of = {}                  # pool idx -> scratch slot of an expanded node
    next_slot = n + 1
    # -- expansion steps 2..D: one draft forward per depth over the frontier
    for t in range(2, depth + 1):
        rows = len(frontier)
        feats = np.stack([st.g_root if pool_par[c] < 0 else g_of[pool_par[c]] for c in frontier])
        toks = np.array([pool_tok[c] for c in frontier])
        slots, vis = [], []
        for c in frontier:
            slot_of[c] = next_slot; next_slot += 1
            anc, a = [], c
            while a >= 0:
                anc.append(slot_of[a]); a = pool_par[a]
            slots.append(slot_of[c]); vis.append(list(range(1, n + 1)) + anc[::-1])
        logits, g = draft_forward(w, shape, st.dcache, feats, toks, np.full(rows, n + t - 1), slots, vis, **_kw(st))
        lp = log_softmax(logits).astype(np.float32)
        first_child = len(pool_tok)
        for r, c in enumerate(frontier):
            g_of[c] = g[r]
            for v in top_k(lp[r], topk):
                pool_tok.append(int(v)); pool_par.append(c); pool_dep.append(t)
                pool_sc.append(np.float32(pool_sc[c] + lp[r, v]))
        if t < depth:
            new = np.array(pool_sc[first_child:], dtype=np.float32)
            frontier = [first_child + int(i) for i in top_k(new, topk)]   # reading: K nodes expanded per depth
    # -- rerank: best (total - 1) of the pool by cumulative score, ties to the lower pool index
    sc = np.array(pool_sc, dtype=np.float32)
    keep = sorted(int(i) for i in top_k(sc, min(total - 1, len(sc))))
    node_of = {-1: 0}
    for j, c in enumerate(keep):
        node_of[c] = j + 1
    token = np.array([st.root] + [pool_tok[c] for c in keep], dtype=np.int32)
    parent = np.array([-1] + [node_of[pool_par[c]] for c in keep], dtype=np.int32)
    dep = np.array([0] + [pool_dep[c] for c in keep], dtype=np.int32)
    score = np.array([0.0] + [pool_sc[c] for c in keep], dtype=np.float32)
    return Tree(token, parent, dep, score)


def verify_tree(st: SpecState, tree: Tree):
    """One target forward over all tree nodes; row j sees the cache and its own root-to-j path."""
    n = st.n
    rows = tree.n_nodes
    vis = [list(range(n)) + [n + a for a in tree.path(j)] for j in range(rows)]
    return target_forward(st.w, st.shape, st.tcache, tree.token, n + tree.depth, [n + j for j in range(rows)], vis, **_kw(st))


def accept_greedy(tree: Tree, logits: np.ndarray) -> Tuple[List[int], int]:
    """T = 0: follow the child that carries the target's argmax while one exists."""
    l32 = logits.astype(np.float32)
    cur, acc = 0, []
    while True:
        best = argmax_low(l32[cur])
        nxt = [c for c in tree.children(cur) if int(tree.token[c]) == best]
        if not nxt:
            return acc, best
        cur = nxt[0]
        acc.append(cur)


def accept_sample(tree: Tree, logits: np.ndarray, temperature: float, seed: int, cycle: int) -> Tuple[List[int], int]:
    """T > 0: multi-round rejection sampling over each node's children.

    reading: the children were chosen deterministically (top-K), so each is a
    point-mass proposal: accept child c with probability p(c); on rejection the
    target distribution is replaced by the residual (p with c removed,
    renormalised); when every child is rejected the bonus token is drawn from
    the residual.  The bonus draw uses the Gumbel-max form of sampling."""
    l32 = logits.astype(np.float32)
    t = np.float32(temperature)
    cur, acc = 0, []
    while True:
        x = l32[cur] / t
        p = np.exp(x - x.max())
        p = p / p.sum()
        removed = np.zeros(p.shape[0], dtype=bool)
        moved = False
        for i, c in enumerate(tree.children(cur)):
            tok = int(tree.token[c])
            u = _rng.uniform01(seed, cycle, cur, i)
            if u < p[tok]:
                moved = True
            else:
                p[tok] = 0.0
                removed[tok] = True
                s = p.sum()
                if s > 0:
                    p = p / s
                else:
                    moved = True       # reading: residual has no mass left, c was certain
            if moved:
                cur = c
                acc.append(c)
                break
        if not moved:
            z = x + _rng.gumbel(seed, cycle, cur, p.shape[0])
            z[removed] = -np.inf
            return acc, argmax_low(z)


def commit(st: SpecState, tree: Tree, feats: np.ndarray, accepted: Sequence[int], bonus: int) -> List[int]:
    """KV compaction and hand-off: accepted node of depth d moves from slot n+j to slot n+d."""
    n = st.n
    for d, j in enumerate(accepted, start=1):
        st.tcache.k[:, n + d] = st.tcache.k[:, n + j]
        st.tcache.v[:, n + d] = st.tcache.v[:, n + j]
    rows = [0] + list(accepted)
    st.pend_feats = feats[rows].copy()
    st.pend_tokens = np.array([int(tree.token[j]) for j in accepted] + [bonus], dtype=np.int32)
    st.n = n + 1 + len(accepted)
    st.root = bonus
    return [int(tree.token[j]) for j in accepted] + [bonus]


def spec_decode(w: Weights, shape, prompt: np.ndarray, gen: int, *, depth=None, topk=None, total=None,
                temperature: float = 0.0, seed: int = 0, dtype=np.float64, store=None,
                tree_hook: Optional[Callable[[SpecState, Tree], Tree]] = None, record: Optional[list] = None):
    """Whole run: prefill, then draft / verify / accept cycles until `gen` tokens.

    Returns (tokens[:gen], emitted-per-cycle list)."""
    depth = shape.tree_depth if depth is None else depth
    topk = shape.tree_topk if topk is None else topk
    total = shape.tree_total if total is None else total
    max_seq = len(prompt) + gen + total + depth * topk + depth + 4
    st, first = prefill(w, shape, prompt, max_seq, temperature, seed, dtype, store)
    out, taus = [first], []
    while len(out) < gen:
        st.cycle += 1
        tree = draft_tree(st, depth, topk, total)
        if tree_hook is not None:
            tree = tree_hook(st, tree)
        logits, feats = verify_tree(st, tree)
        if temperature > 0:
            acc, bonus = accept_sample(tree, logits, temperature, seed, st.cycle)
        else:
            acc, bonus = accept_greedy(tree, logits)
        if record is not None:
            record.append(dict(n=st.n, tree=tree, logits=logits, feats=feats, accepted=list(acc), bonus=bonus))
        emitted = commit(st, tree, feats, acc, bonus)
        out += emitted
        taus.append(len(emitted))
    return out[:gen], taus
