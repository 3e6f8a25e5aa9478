"""Pins for the oracle of the ETS selection step: REBASE weights against hand-worked
values and invariants, the cost model against closed forms on small trees.  CPU only."""
import math

import numpy as np
import pytest

from oracle import selector as sel


def test_rebase_weights_hand_worked():
    # equal rewards, budget 4, three trajectories: ceil(4/3) = 2, then ceil(2/2) = 1, then 1
    assert sel.rebase_weights([0.5, 0.5, 0.5], 4, 0.2).tolist() == [2, 1, 1]
    # visited from the highest reward: index 2 first.  e = exp(r / 1) with r = ln 1, ln 2, ln 5
    r = [math.log(1.0), math.log(2.0), math.log(5.0)]
    # N = 8: W_2 = ceil(8 * 5/8) = 5; N = 3: W_1 = ceil(3 * 2/3) = 2; N = 1: W_0 = ceil(1 * 1/1) = 1
    assert sel.rebase_weights(r, 8, 1.0).tolist() == [1, 2, 5]
    # the budget runs out before the list does: the rest get nothing
    assert sel.rebase_weights([3.0, 2.0, 1.0, 0.0], 1, 1.0).tolist() == [1, 0, 0, 0]
    # a low temperature concentrates everything on the best trajectory
    assert sel.rebase_weights([0.9, 0.1], 16, 0.01).tolist() == [16, 0]


@pytest.mark.parametrize("seed", range(6))
def test_rebase_weights_invariants(seed):
    r = np.random.default_rng(seed)
    n, budget = int(r.integers(1, 40)), int(r.integers(1, 300))
    rew = r.random(n)
    w = sel.rebase_weights(rew, budget, 0.2)
    assert w.sum() == budget and (w >= 0).all()          # ceil hands out exactly the budget
    order = np.argsort(-rew, kind="stable")
    assert (np.diff(w[order]) <= 0).all()                # better reward, no fewer continuations
    # shifting every reward leaves the softmax, hence the weights, unchanged
    assert np.array_equal(sel.rebase_weights(rew + 3.0, budget, 0.2), w)


def _tree_two_pairs():
    #        0
    #      /   \
    #     1     2
    #    / \   / \
    #   3   4 5   6        leaves 3 4 5 6; live nodes 7: L = 4, P = 3
    return np.array([-1, 0, 0, 1, 1, 2, 2], np.int32), np.array([3, 4, 5, 6], np.int32)


def test_objective_closed_forms():
    parent, leaves = _tree_two_pairs()
    w = np.array([4, 3, 2, 1])
    assert sel.live_nodes(parent, leaves)[1:] == (4, 3)
    # everything kept: 1 - lam_b * 7/7 (+ lam_d)
    assert sel.objective(parent, leaves, w, None, 0.5, 0.0, [1, 1, 1, 1]) == pytest.approx(0.5)
    assert sel.objective(parent, leaves, w, [0, 0, 1, 2], 0.5, 0.3, [1, 1, 1, 1]) == pytest.approx(0.8)
    # leaves 3 and 4: weight 7/10, nodes {3, 4, 1, 0} = 4 of 7, clusters {0} = 1 of 3
    assert sel.objective(parent, leaves, w, [0, 0, 1, 2], 0.7, 0.3, [1, 1, 0, 0]) == \
        pytest.approx(0.7 - 0.7 * 4 / 7 + 0.3 / 3)
    # leaves 3 and 5 share only the root: 5 nodes
    assert sel.objective(parent, leaves, w, None, 0.7, 0.0, [1, 0, 1, 0]) == \
        pytest.approx(0.6 - 0.7 * 5 / 7)


def test_selection_closed_forms():
    parent, leaves = _tree_two_pairs()
    w = np.array([4, 3, 2, 1])
    # no budget term: everything with a weight is kept
    v, arg = sel.select_bruteforce(parent, leaves, w, None, 0.0, 0.0)
    assert v == pytest.approx(1.0) and len(arg) == 1 and arg[0].all()
    # lam_b = 1: a leaf costs 1/7 and brings W/10; the pair {3, 4} under node 1:
    # 0.7 - 4/7 = 0.1286; adding leaf 5 (+0.2, two more nodes: -2/7) loses; {3} alone:
    # 0.4 - 3/7 < 0.1286
    v, arg = sel.select_bruteforce(parent, leaves, w, None, 1.0, 0.0)
    assert v == pytest.approx(0.7 - 4 / 7) and [a.tolist() for a in arg] == [[True, True, False, False]]
    # a large budget weight still keeps one leaf: the heaviest one (every single leaf costs 3 nodes)
    v, arg = sel.select_bruteforce(parent, leaves, w, None, 50.0, 0.0)
    assert [a.tolist() for a in arg] == [[True, False, False, False]]
    assert v == pytest.approx(0.4 - 50.0 * 3 / 7)
    # coverage term: three clusters {3, 4}, {5}, {6}; with lam_d = 0.9 a leaf of a new
    # cluster under node 2 is worth 0.3: {3, 4, 5}: 0.9 - 6/7 + 0.6 beats {3, 4}: 0.7 - 4/7 + 0.3
    v, arg = sel.select_bruteforce(parent, leaves, w, [0, 0, 1, 2], 1.0, 0.9)
    assert v == pytest.approx(1.0 - 1.0 + 0.9) and arg[0].all()
    v, arg = sel.select_bruteforce(parent, leaves, w, [0, 0, 1, 2], 1.0, 0.5)
    # {3,4}: 0.7-4/7+1/6=0.2952; {3,4,5}: 0.9-6/7+2/6=0.3762; all: 1-1+0.5=0.5
    assert v == pytest.approx(0.5) and arg[0].all()
    v, arg = sel.select_bruteforce(parent, leaves, w, [0, 0, 1, 2], 2.0, 0.5)
    # {3,4}: 0.7-8/7+1/6=-0.276; {3}: 0.4-6/7+1/6=-0.290; all: 1-2+0.5=-0.5
    assert v == pytest.approx(0.7 - 8 / 7 + 1 / 6) and arg[0].tolist() == [True, True, False, False]


def test_any_reading_of_the_cluster_constraint():
    # one cluster of two leaves: keeping one of them already covers it
    parent = np.array([-1, 0, 0], np.int32)
    leaves = np.array([1, 2], np.int32)
    a = sel.objective(parent, leaves, [1, 1], [0, 0], 0.0, 1.0, [1, 0])
    assert a == pytest.approx(0.5 + 1.0)
