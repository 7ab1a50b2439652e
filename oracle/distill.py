"""Harmonized objective distillation: the Top-K loss (test infrastructure; nothing on the product path
imports this).

Sec. 3.1, Eq. (1): with q the target LLM's next-token distribution, p the draft model's, and Omega-hat the
K tokens of highest target probability,  L = - sum over x in Omega-hat of q(x) log p(x).  Both distributions
come from the shared LM head: q = softmax(Head(target feature)), p = softmax(Head(draft feature)) (Sec. 3.1,
last paragraph; Sec. 3.2, P^(s) = Head(f)).  K = 10 and the loss enters EAGLE's objective with weight 1
(Sec. 4.1, Implementation).

reading: tokens of equal target probability at the K-th place are taken by lower token id (the paper does not
say; the product takes the same order).  The loss is reported per position; the mean over positions and the
weight w are the trainer's business.
"""
from __future__ import annotations

import numpy as np

from .llama import _identity


def _log_softmax(z: np.ndarray) -> np.ndarray:
    m = z.max(axis=-1, keepdims=True)
    return z - m - np.log(np.exp(z - m).sum(axis=-1, keepdims=True))


def topk_set(zq_row: np.ndarray, k: int) -> np.ndarray:
    """Omega-hat of one position: the k token ids of largest target logit (= largest q), lower id on ties."""
    return np.argsort(-zq_row, kind="stable")[:k]


def topk_distill_loss(zq: np.ndarray, zp: np.ndarray, k: int) -> np.ndarray:
    """Eq. (1) per position.  zq, zp: [rows, V] target / draft logits.  -> [rows]."""
    logq = _log_softmax(zq)
    logp = _log_softmax(zp)
    out = np.zeros(zq.shape[0], dtype=zq.dtype)
    for r in range(zq.shape[0]):
        om = topk_set(zq[r], k)
        out[r] = -(np.exp(logq[r, om]) * logp[r, om]).sum()
    return out


def soft_cross_entropy(zq: np.ndarray, zp: np.ndarray) -> np.ndarray:
    """- sum over the whole vocabulary of q log p: the cross-entropy term of the Sec. 3.2 objective, which is
    what Eq. (1) becomes when Omega-hat is the whole vocabulary."""
    return -(np.exp(_log_softmax(zq)) * _log_softmax(zp)).sum(axis=-1)


def head_losses(feat_target: np.ndarray, feat_draft: np.ndarray, lm_head: np.ndarray, k: int, store=_identity):
    """Both losses from features: logits through the shared LM head [V, d] first.
    -> (top-k loss [rows], cross-entropy [rows])."""
    zq = store(feat_target) @ lm_head.T
    zp = store(feat_draft) @ lm_head.T
    return topk_distill_loss(zq, zp, k), soft_cross_entropy(zq, zp)
