"""The seeded input generators: structure of the synthetic search trees."""
from dataclasses import replace

import numpy as np

from workload import CONFIGS, make_tree, random_tree, with_growth_room


def _live(t):
    live = np.zeros(t.n_nodes, dtype=bool)
    live[t.leaf_node] = True
    for i in range(t.n_nodes - 1, 0, -1):
        if live[i] and t.parent[i] >= 0:
            live[t.parent[i]] = True
    return live


def test_configs_have_the_stated_shape():
    for name, cfg in CONFIGS.items():
        t = make_tree(cfg)
        assert t.n_leaves == cfg.trees * (cfg.width if cfg.alpha is not None else
                                          cfg.branch ** cfg.steps), name
        assert np.all(t.parent[1:] < np.arange(1, t.n_nodes)) and np.all(t.parent >= -1)
        assert int((t.parent < 0).sum()) == cfg.trees
        roots = np.flatnonzero(t.parent < 0)
        assert np.all(t.n_tokens[roots] == cfg.prompt)
        inner = np.ones(t.n_nodes, dtype=bool)
        inner[roots] = False
        assert t.n_tokens[inner].min() >= cfg.step_lo and t.n_tokens[inner].max() <= cfg.step_hi
        # stored nodes own disjoint runs of pool rows that tile the pool
        live = _live(t)
        stored = np.ones(t.n_nodes, dtype=bool) if cfg.store_dead else live
        order = np.argsort(t.tok_offset[stored], kind="stable")
        off = t.tok_offset[stored][order]
        ln = t.n_tokens[stored][order]
        assert off[0] == 0 and np.all(off[1:] == off[:-1] + ln[:-1])
        assert off[-1] + ln[-1] == t.pool_tokens
        # same seed, same tree
        t2 = make_tree(cfg)
        assert np.array_equal(t.parent, t2.parent) and np.array_equal(t.n_tokens, t2.n_tokens)


def test_forest_is_a_concatenation_of_independent_searches():
    cfg = CONFIGS["c6_batch16"]
    f = make_tree(cfg)
    one = replace(cfg, trees=1)
    node0, row0, leaf0 = 0, 0, 0
    for k in range(cfg.trees):
        t = make_tree(one, cfg.seed + 7919 * k)
        sl = slice(node0, node0 + t.n_nodes)
        assert np.array_equal(np.where(t.parent < 0, -1, t.parent + node0), f.parent[sl])
        assert np.array_equal(t.n_tokens, f.n_tokens[sl])
        assert np.array_equal(t.tok_offset + row0, f.tok_offset[sl])
        assert np.array_equal(t.leaf_node + node0, f.leaf_node[leaf0:leaf0 + t.n_leaves])
        node0 += t.n_nodes
        row0 += t.pool_tokens
        leaf0 += t.n_leaves
    assert (node0, row0, leaf0) == (f.n_nodes, f.pool_tokens, f.n_leaves)
    # the searches differ from each other
    a, b = make_tree(one, cfg.seed), make_tree(one, cfg.seed + 7919)
    assert not np.array_equal(a.parent, b.parent)


def test_growth_room_keeps_the_tree_and_frees_rows_behind_leaf_nodes():
    t = random_tree(5, 40, 12, 50)
    g = with_growth_room(t, 7)
    assert np.array_equal(g.parent, t.parent) and np.array_equal(g.n_tokens, t.n_tokens)
    is_leaf = np.zeros(t.n_nodes, dtype=bool)
    is_leaf[t.leaf_node] = True
    owns = (t.n_tokens > 0) | is_leaf          # nodes without rows and room own nothing
    idx = np.flatnonzero(owns)
    order = idx[np.argsort(g.tok_offset[idx], kind="stable")]
    end = g.tok_offset[order] + g.n_tokens[order] + np.where(is_leaf[order], 7, 0)
    assert np.all(g.tok_offset[order][1:] >= end[:-1]) and end[-1] <= g.pool_tokens
