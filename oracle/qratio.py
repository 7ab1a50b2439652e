"""Speculative sampling with SAMPLED draft tokens: the ratio acceptance rule (test infrastructure; nothing
on the product path imports this).

Sec. 2, Preliminary: the draft model proposes tokens by its own (sampled) decoding, the target scores them,
and a modified rejection sampling scheme keeps a prefix that retains the target distribution; the analysis
carries over to several draft sequences (the static-tree comparison systems of Sec. 4.1).  The paper names
the scheme and cites it; what is written out here is that cited textbook rule.  At a node with target
distribution p and draft distribution q, children x_1, x_2, ... drawn from q without replacement:

    accept x_j with probability min(1, p_j(x_j) / q_j(x_j));
    on rejection  p_{j+1} = normalise(max(p_j - q_j, 0)),   q_{j+1} = q_j with x_j removed, renormalised;
    when every child is rejected (or there is none) the next token is drawn from the current p.

The dynamic-tree path of the product uses the special case of deterministic children (q a point mass,
oracle/spec.py: accept_sample); this module is the general rule for sampled children.

reading: a residual with no mass left (p_j <= q_j everywhere, which needs p_j = q_j up to rounding, so the
child was certain to be accepted) accepts the child.
Random numbers: the counter-based generator of oracle/rng.py; the drafting noise of node i uses stream
(cycle, DRAFT_NODE_BASE + i) so that it is independent of the acceptance draws of stream (cycle, i).
"""
from __future__ import annotations

from typing import List, Sequence, Tuple

import numpy as np

from . import rng as _rng

DRAFT_NODE_BASE = 1 << 16


def _softmax64(x: np.ndarray) -> np.ndarray:
    x = x.astype(np.float64)
    e = np.exp(x - x.max())
    return e / e.sum()


def sample_children(q_logits_row: np.ndarray, temperature: float, m: int, seed: int, cycle: int, node: int) -> List[int]:
    """m distinct tokens drawn from softmax(q_logits / T) without replacement, in draw order: the m largest of
    logits / T + standard Gumbel noise (largest first, lower token id on exact ties)."""
    z = q_logits_row.astype(np.float32) / np.float32(temperature)
    z = z + _rng.gumbel(seed, cycle, DRAFT_NODE_BASE + node, z.shape[0])
    return [int(i) for i in np.argsort(-z, kind="stable")[:m]]


def accept_qratio(token: Sequence[int], parent: Sequence[int], p_logits: np.ndarray, q_logits: np.ndarray, temperature: float,
                  seed: int, cycle: int, max_depth: int = None) -> Tuple[List[int], int, float]:
    """Walk the tree from the root (node 0; parents precede children; the children of a node are tried in node
    order, which must be their draw order).  p_logits[i], q_logits[i]: target / draft logits AT node i (they
    score node i's children).  -> (accepted nodes, next token, margin): margin is the smallest relative distance
    |u q - p| / p of any accept/reject decision taken, so that a caller comparing against an fp32 evaluation
    can set aside the draws that rounding could flip.  max_depth: a caller that caps the tokens accepted per cycle
    passes its cap (the walk then stops at that depth and draws the next token there); None = no cap."""
    n = len(token)
    cur, acc, margin = 0, [], np.inf
    while True:
        p = _softmax64(p_logits[cur] / temperature)
        q = _softmax64(q_logits[cur] / temperature)
        kids = [c for c in range(cur + 1, n) if parent[c] == cur] if max_depth is None or len(acc) < max_depth else []
        moved = False
        for j, c in enumerate(kids):
            x = int(token[c])
            u = float(_rng.uniform01(seed, cycle, cur, j))
            if p[x] > 0:
                margin = min(margin, abs(u * q[x] - p[x]) / p[x])
            if u * q[x] < p[x]:
                moved = True
            else:
                p = np.maximum(p - q, 0.0)
                s = p.sum()
                if s > 0:
                    p = p / s
                else:
                    moved = True
                q = q.copy()
                q[x] = 0.0
                sq = q.sum()
                if sq > 0:
                    q = q / sq
            if moved:
                cur = c
                acc.append(c)
                break
        if not moved:
            with np.errstate(divide="ignore"):
                z = np.log(p).astype(np.float32) + _rng.gumbel(seed, cycle, cur, p.shape[0])
            return acc, int(np.argmax(z)), float(margin)
