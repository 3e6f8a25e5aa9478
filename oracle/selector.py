"""CPU oracle of the ETS selection step (ETS paper Sec. 4.1-4.2, App. B): REBASE weights
(Eq. 1 / Eq. 3) and the retained set that maximises the cost model (Eq. 2 / Eq. 4, as the
ILPs of App. B, Eq. 6 / Eq. 7), found by trying every non-empty set of leaves.

TEST INFRASTRUCTURE ONLY: imported by tests/ and by the benchmark's check; the product
package never imports it and this module imports nothing from the product package.

Readings of the paper (it leaves these open or prints them inconsistently):
  * Eq. 1 visits the trajectories from the highest reward to the lowest; the number of
    continuations still to be sampled shrinks by what was handed out, N_{i+1} = N_i - W_i
    (implied by "still need to be sampled"), and A_i holds trajectory i and every one
    after it in that order.  Equal rewards keep their input order.
  * V_A is the set of live nodes (nodes with a leaf at or beneath them), L of them leaves
    and P of them not; a leaf is a node named in leaf_node, leaves are distinct and no
    leaf lies beneath another.
  * The cluster constraint is printed as z_k <= x_i for every i in C_k, which would make
    z_k = 1 only when ALL of a cluster's leaves are kept; the text says z_k is 1 when ANY
    of them is kept.  The text is followed: z_k = 1 iff some leaf of cluster k is kept.
"""
from __future__ import annotations

import itertools
import math

import numpy as np


def rebase_weights(rewards, budget, temperature):
    """Eq. 1: W (int64 [n]) for rewards [n], `budget` continuations, temperature T_R."""
    r = np.asarray(rewards, dtype=np.float64)
    n = r.shape[0]
    order = sorted(range(n), key=lambda i: (-r[i], i))
    e = [math.exp(r[i] / temperature) for i in order]
    # sum over A_i: this trajectory and all later ones, added from the last one backwards
    tail = [0.0] * (n + 1)
    for p in range(n - 1, -1, -1):
        tail[p] = tail[p + 1] + e[p]
    w = np.zeros(n, dtype=np.int64)
    left = int(budget)
    for p, i in enumerate(order):
        if left <= 0:
            break
        w[i] = min(left, int(math.ceil(left * (e[p] / tail[p]))))
        left -= int(w[i])
    return w


def live_nodes(parent, leaf_node):
    """(is_live bool [N], n_leaves L, n_internal P) of the tree spanned by the leaves."""
    parent = np.asarray(parent)
    live = np.zeros(parent.shape[0], dtype=bool)
    for v in np.asarray(leaf_node).tolist():
        while v >= 0 and not live[v]:
            live[v] = True
            v = int(parent[v])
    L = len(set(np.asarray(leaf_node).tolist()))
    return live, L, int(live.sum()) - L


def objective(parent, leaf_node, weights, cluster, lam_b, lam_d, keep):
    """Eq. 7 for the set of leaves keep (bool [L]); Eq. 6 when cluster is None or lam_d = 0."""
    parent = np.asarray(parent)
    leaf_node = np.asarray(leaf_node)
    w = np.asarray(weights, dtype=np.float64)
    keep = np.asarray(keep, dtype=bool)
    _, L, P = live_nodes(parent, leaf_node)
    kept = set()
    for v in leaf_node[keep].tolist():
        while v >= 0 and v not in kept:
            kept.add(v)
            v = int(parent[v])
    val = float(w[keep].sum() / w.sum()) - lam_b * len(kept) / (P + L)
    if cluster is not None and lam_d != 0.0:
        cluster = np.asarray(cluster)
        val += lam_d * len(set(cluster[keep].tolist())) / len(set(cluster.tolist()))
    return val


def select_bruteforce(parent, leaf_node, weights, cluster, lam_b, lam_d):
    """Best objective over all non-empty sets of leaves and every set that reaches it
    (within 1e-12): (value, [keep arrays])."""
    L = len(leaf_node)
    best, arg = -math.inf, []
    for bits in itertools.product([False, True], repeat=L):
        if not any(bits):
            continue
        v = objective(parent, leaf_node, weights, cluster, lam_b, lam_d, bits)
        if v > best + 1e-12:
            best, arg = v, [np.array(bits)]
        elif abs(v - best) <= 1e-12:
            arg.append(np.array(bits))
    return best, arg
