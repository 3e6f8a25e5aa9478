"""A synthetic PRM-guided tree search that uses the library's selection step, for the
time-summed KV-size accounting of the ETS paper (Sec. 3: the KV cache size of a search is
summed over its steps).  Rewards and cluster labels are drawn at random (they stand in
for the process reward model and for the sentence-embedding clusters); nothing here
computes attention.

Per search step: every kept leaf i receives W_i continuations (REBASE weights, Eq. 1);
the new nodes get a step length, a reward near their parent's and a cluster label (a few
"phrasings" per parent: siblings are often redundant).  Policy "rebase" continues from
every leaf with a weight; policy "ets" first keeps the set that maximises the cost model
(Eq. 4; App. B, Eq. 7) and re-weights the kept leaves (Eq. 3).
"""
from __future__ import annotations

import numpy as np

from .trees import Tree, _rng


def simulate_search(policy, width, steps, prompt, step_lo, step_hi, seed, lambda_b=1.5,
                    lambda_d=1.0, temperature=0.2, phrasings=3, select=None, rebase=None,
                    node_limit=20000):
    """Runs one search; `rebase(rewards, budget, T)` and `select(parent, leaf_node, w, cluster,
    lambda_b, lambda_d, node_limit)` are the library's entry points (passed in, so that this
    module stays free of the product).  Returns a dict with the per-step unique-token counts
    ("kv_tokens": the rows a decode step of that search step attends over, each shared node
    once), their sum, and the final Tree (leaves = the nodes of the last step)."""
    r = _rng(seed, 77)
    parent = [-1]
    n_tokens = [int(prompt)]
    reward = [0.5]
    frontier = np.array([0], dtype=np.int32)
    weights = np.array([width], dtype=np.int64)
    kv_tokens, kept_leaves = [], []
    for _ in range(steps):
        # expand: W_i children per kept leaf
        kids, kid_par = [], []
        for leaf, w in zip(frontier.tolist(), weights.tolist()):
            for _c in range(int(w)):
                kids.append(len(parent))
                kid_par.append(leaf)
                parent.append(leaf)
                n_tokens.append(int(r.integers(step_lo, step_hi + 1)))
                reward.append(float(np.clip(reward[leaf] + 0.15 * r.standard_normal(), 0.0, 1.0)))
        kids = np.array(kids, dtype=np.int32)
        cluster = np.array(kid_par, dtype=np.int64) * phrasings + r.integers(0, phrasings, len(kids))
        par_arr = np.array(parent, dtype=np.int32)
        rew = np.array([reward[k] for k in kids.tolist()])
        # the KV a decode step of this search step reads: ancestors once, every new step
        live = np.zeros(len(parent), dtype=bool)
        for k in kids.tolist():
            v = k
            while v >= 0 and not live[v]:
                live[v] = True
                v = int(par_arr[v])
        kv_tokens.append(int(np.asarray(n_tokens)[live].sum()))
        # choose what continues
        w = np.asarray(rebase(rew, width, temperature), dtype=np.int64)
        if policy == "ets":
            has_w = w > 0
            keep, _ = select(par_arr, kids[has_w], w[has_w].astype(np.int32), cluster[has_w],
                             lambda_b, lambda_d, node_limit)
            chosen = kids[has_w][keep]
            w2 = np.asarray(rebase(rew[has_w][keep], width, temperature), dtype=np.int64)
            frontier, weights = chosen[w2 > 0], w2[w2 > 0]
        elif policy == "rebase":
            frontier, weights = kids[w > 0], w[w > 0]
        else:
            raise ValueError(policy)
        kept_leaves.append(int(len(frontier)))
    # the last step's nodes as a Tree for the attention library (pool rows in node order)
    n_tok = np.array(n_tokens, dtype=np.int32)
    off = np.concatenate([[0], np.cumsum(n_tok[:-1], dtype=np.int64)]).astype(np.int64)
    tree = Tree(np.array(parent, dtype=np.int32), off, n_tok, kids, int(n_tok.sum()),
                np.zeros(len(parent), dtype=np.int32))
    return {"kv_tokens": kv_tokens, "kv_tokens_sum": int(sum(kv_tokens)),
            "kept_leaves": kept_leaves, "tree": tree}
