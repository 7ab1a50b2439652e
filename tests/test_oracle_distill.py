"""Pins of the Top-K distillation loss oracle (oracle/distill.py): a value worked out by hand from Eq. (1),
brute force in plain Python, library routines for the special cases (whole vocabulary = cross-entropy with
soft targets; identical distributions = entropy), and properties that follow from the definition."""
import math

import numpy as np
import pytest
import scipy.stats
import torch

from oracle import distill


def test_hand_worked_example():
    # q = (0.5, 0.3, 0.2), p = (0.25, 0.25, 0.5), K = 2: Omega-hat = {0, 1},
    # L = -(0.5 ln 0.25 + 0.3 ln 0.25) = 0.8 * ln 4
    zq = np.log(np.array([[0.5, 0.3, 0.2]]))
    zp = np.log(np.array([[0.25, 0.25, 0.5]]))
    np.testing.assert_allclose(distill.topk_distill_loss(zq, zp, 2), [0.8 * math.log(4.0)], rtol=1e-14)
    # K = 1 keeps the target's best token only; K = 3 is the whole sum
    np.testing.assert_allclose(distill.topk_distill_loss(zq, zp, 1), [0.5 * math.log(4.0)], rtol=1e-14)
    np.testing.assert_allclose(distill.topk_distill_loss(zq, zp, 3), [0.8 * math.log(4.0) + 0.2 * math.log(2.0)], rtol=1e-14)


def _brute(zq_row, zp_row, k):
    v = len(zq_row)
    sq = sum(math.exp(x) for x in zq_row)
    sp = sum(math.exp(x) for x in zp_row)
    order = sorted(range(v), key=lambda i: (-zq_row[i], i))
    return -sum(math.exp(zq_row[i]) / sq * (zp_row[i] - math.log(sp)) for i in order[:k])


@pytest.mark.parametrize("k", [1, 3, 10, 17])
def test_brute_force_small(k):
    g = np.random.default_rng(k)
    zq, zp = g.standard_normal((6, 17)) * 2, g.standard_normal((6, 17)) * 2
    want = [_brute(list(zq[r]), list(zp[r]), k) for r in range(6)]
    np.testing.assert_allclose(distill.topk_distill_loss(zq, zp, k), want, rtol=1e-12)


def test_whole_vocabulary_is_cross_entropy_with_soft_targets():
    g = np.random.default_rng(2)
    zq, zp = g.standard_normal((5, 40)) * 3, g.standard_normal((5, 40)) * 3
    q = torch.softmax(torch.from_numpy(zq), dim=-1)
    want = torch.nn.functional.cross_entropy(torch.from_numpy(zp), q, reduction="none").numpy()
    np.testing.assert_allclose(distill.topk_distill_loss(zq, zp, 40), want, rtol=1e-12)
    np.testing.assert_allclose(distill.soft_cross_entropy(zq, zp), want, rtol=1e-12)


def test_identical_distributions_give_the_entropy():
    g = np.random.default_rng(3)
    z = g.standard_normal((4, 25)) * 2
    q = np.exp(z) / np.exp(z).sum(axis=-1, keepdims=True)
    want = [scipy.stats.entropy(q[r]) for r in range(4)]
    np.testing.assert_allclose(distill.soft_cross_entropy(z, z + 1.5), want, rtol=1e-12)


def test_properties():
    g = np.random.default_rng(4)
    zq, zp = g.standard_normal((8, 50)) * 2, g.standard_normal((8, 50)) * 2
    base = distill.topk_distill_loss(zq, zp, 10)
    # softmax ignores a per-position shift of either logit row
    np.testing.assert_allclose(distill.topk_distill_loss(zq + 3.0, zp - 7.0, 10), base, rtol=1e-12)
    # the same relabelling of the vocabulary on both sides changes nothing (no ties in random data)
    perm = g.permutation(50)
    np.testing.assert_allclose(distill.topk_distill_loss(zq[:, perm], zp[:, perm], 10), base, rtol=1e-12)
    # every term is non-negative, so the loss grows with K and ends at the full cross-entropy
    prev = np.zeros(8)
    for k in (1, 2, 5, 10, 25, 50):
        cur = distill.topk_distill_loss(zq, zp, k)
        assert (cur >= prev - 1e-15).all()
        prev = cur
    np.testing.assert_allclose(prev, distill.soft_cross_entropy(zq, zp), rtol=1e-12)
    # only the draft's probabilities ON Omega-hat matter: moving draft mass among tokens outside it, with the
    # normaliser kept, leaves the loss unchanged
    r = 0
    om = set(distill.topk_set(zq[r], 10).tolist())
    outside = [i for i in range(50) if i not in om][:2]
    zp2 = zp.copy()
    a, b = np.exp(zp[r, outside[0]]), np.exp(zp[r, outside[1]])
    zp2[r, outside[0]], zp2[r, outside[1]] = np.log(0.25 * (a + b)), np.log(0.75 * (a + b))
    np.testing.assert_allclose(distill.topk_distill_loss(zq, zp2, 10)[r], base[r], rtol=1e-12)


def test_ties_at_the_boundary_take_the_lower_token_id():
    zq = np.array([[1.0, 2.0, 2.0, 2.0, 0.0]])
    assert distill.topk_set(zq[0], 2).tolist() == [1, 2]
    zp = np.log(np.array([[0.1, 0.2, 0.3, 0.15, 0.25]]))
    q = np.exp(zq[0]) / np.exp(zq[0]).sum()
    want = -(q[1] * math.log(0.2) + q[2] * math.log(0.3))
    np.testing.assert_allclose(distill.topk_distill_loss(zq, zp, 2), [want], rtol=1e-13)


def test_head_losses_use_the_shared_head():
    g = np.random.default_rng(5)
    ft, fd, w = g.standard_normal((3, 8)), g.standard_normal((3, 8)), g.standard_normal((20, 8))
    tk, ce = distill.head_losses(ft, fd, w, 4)
    zq = np.einsum("rd,vd->rv", ft, w)
    zp = np.einsum("rd,vd->rv", fd, w)
    np.testing.assert_allclose(tk, [_brute(list(zq[r]), list(zp[r]), 4) for r in range(3)], rtol=1e-12)
    np.testing.assert_allclose(ce, [_brute(list(zq[r]), list(zp[r]), 20) for r in range(3)], rtol=1e-12)
