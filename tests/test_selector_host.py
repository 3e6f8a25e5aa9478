"""The library's ETS selection step (host C++) against the oracle: REBASE weights equal
bit for bit, the selected set reaches the best objective found by enumeration and is
itself valid.  Where several sets are optimal any of them is accepted.  CPU only."""
import math

import numpy as np
import pytest

import paper_2502_13575_amd as ets
from oracle import selector as osel
from workload import CONFIGS, make_tree, random_tree


@pytest.mark.parametrize("seed", range(10))
def test_rebase_weights_equal_the_oracle(seed):
    r = np.random.default_rng(seed)
    n, budget = int(r.integers(1, 300)), int(r.integers(0, 600))
    rew = r.random(n)
    if seed % 3 == 0:
        rew = np.round(rew, 1)          # ties keep their input order
    for temp in (0.2, 1.0, 0.03):
        got = ets.ets_rebase_weights(rew, budget, temp)
        assert np.array_equal(got, osel.rebase_weights(rew, budget, temp))


def _frontier_tree(seed, n_nodes, n_leaves):
    """A random forest and leaves that are distinct and not beneath each other."""
    t = random_tree(seed, n_nodes=n_nodes, n_leaves=1, max_tokens=3)
    has_child = np.zeros(n_nodes, bool)
    has_child[t.parent[t.parent >= 0]] = True
    cand = np.flatnonzero(~has_child)
    r = np.random.default_rng(seed + 1000)
    leaves = r.choice(cand, size=min(n_leaves, len(cand)), replace=False).astype(np.int32)
    return t.parent, leaves


@pytest.mark.parametrize("seed", range(40))
def test_selection_reaches_the_enumerated_optimum(seed):
    r = np.random.default_rng(seed)
    parent, leaves = _frontier_tree(seed, n_nodes=int(r.integers(6, 30)), n_leaves=int(r.integers(1, 12)))
    L = len(leaves)
    w = osel.rebase_weights(r.random(L), int(r.integers(L, 4 * L + 1)), 0.2)
    if w.sum() == 0:
        w[0] = 1
    cluster = None if seed % 4 == 0 else r.integers(0, max(1, L // 2) + 1, size=L)
    lam_b = [0.0, 0.5, 1.0, 1.5, 2.0, 6.0][seed % 6]
    lam_d = [0.0, 0.3, 1.0, 2.5][(seed // 2) % 4]
    keep, info = ets.ets_select_leaves(parent, leaves, w, cluster, lam_b, lam_d)
    best, arg = osel.select_bruteforce(parent, leaves, w, cluster, lam_b, lam_d)
    assert info.optimal == 1 and keep.any()
    val = osel.objective(parent, leaves, w, cluster, lam_b, lam_d, keep)
    assert abs(val - best) <= 1e-12, (val, best)
    assert abs(info.objective - best) <= 1e-9
    assert any(np.array_equal(keep, a) for a in arg)
    live, Lc, P = osel.live_nodes(parent, leaves)
    assert info.live_nodes == Lc + P


def test_selection_closed_forms_and_errors():
    parent = np.array([-1, 0, 0, 1, 1, 2, 2], np.int32)
    leaves = np.array([3, 4, 5, 6], np.int32)
    w = np.array([4, 3, 2, 1], np.int32)
    keep, info = ets.ets_select_leaves(parent, leaves, w, None, 1.0, 0.0)
    assert keep.tolist() == [True, True, False, False]
    assert info.objective == pytest.approx(0.7 - 4 / 7) and info.kept_nodes == 4 and info.live_nodes == 7
    keep, info = ets.ets_select_leaves(parent, leaves, w, [0, 0, 1, 2], 2.0, 0.5)
    assert keep.tolist() == [True, True, False, False] and info.kept_clusters == 1 and info.clusters == 3
    keep, _ = ets.ets_select_leaves(parent, leaves, w, None, 50.0, 0.0)
    assert keep.tolist() == [True, False, False, False]      # at least one leaf stays
    keep, _ = ets.ets_select_leaves(parent, leaves, w, None, 0.0, 0.0)
    assert keep.all()
    for bad_leaves, status in (([3, 3], 3), ([1, 3], 3), ([9], 3)):
        with pytest.raises(ets.EtsError) as e:
            ets.ets_select_leaves(parent, np.array(bad_leaves, np.int32),
                                  np.ones(len(bad_leaves), np.int32))
        assert e.value.status == status
    with pytest.raises(ets.EtsError) as e:
        ets.ets_select_leaves(parent, leaves, np.zeros(4, np.int32))
    assert e.value.status == 1
    with pytest.raises(ets.EtsError) as e:
        ets.ets_select_leaves(parent, leaves, w, None, -1.0, 0.0)
    assert e.value.status == 1
    with pytest.raises(ets.EtsError) as e:
        ets.ets_rebase_weights([0.1, 0.2], 4, 0.0)
    assert e.value.status == 1


def test_selection_at_search_width_256():
    """The last step of config 4's tree (256 leaves), synthetic rewards and cluster labels:
    the exact solver finishes, a larger lambda_b keeps fewer nodes, and the coverage term
    keeps more clusters."""
    cfg = CONFIGS["c4_34b"]
    t = make_tree(cfg)
    r = np.random.default_rng(4)
    w = ets.ets_rebase_weights(r.random(t.n_leaves), t.n_leaves, 0.2)
    cluster = r.integers(0, 40, size=t.n_leaves)
    kept = []
    for lam_b in (1.0, 1.5, 2.0):
        keep, info = ets.ets_select_leaves(t.parent, t.leaf_node, w, None, lam_b, 0.0)
        assert info.optimal == 1 and keep.any()
        assert info.objective == pytest.approx(
            osel.objective(t.parent, t.leaf_node, w, None, lam_b, 0.0, keep), abs=1e-9)
        kept.append(info.kept_nodes)
    assert kept[0] >= kept[1] >= kept[2] and kept[0] < info.live_nodes
    k0, i0 = ets.ets_select_leaves(t.parent, t.leaf_node, w, cluster, 1.5, 0.0)
    k1, i1 = ets.ets_select_leaves(t.parent, t.leaf_node, w, cluster, 1.5, 1.0, node_limit=200000)
    assert len(set(cluster[k1])) >= len(set(cluster[k0]))
    assert i1.objective == pytest.approx(
        osel.objective(t.parent, t.leaf_node, w, cluster, 1.5, 1.0, k1), abs=1e-9)
    assert i1.objective >= osel.objective(t.parent, t.leaf_node, w, cluster, 1.5, 1.0, k0) - 1e-12


def test_simulated_search_kv_accounting():
    """The synthetic search of workload/search_sim.py with the library's selection step:
    deterministic, its trees are well formed (oracle's check), the per-step KV counts equal
    the oracle's unique-token count of the final tree at the last step, and keeping the
    cost model's set shrinks the time-summed KV size relative to continuing from every
    weighted leaf."""
    import oracle
    from workload import simulate_search

    def sel(p, l, w, c, lb, ld, nl):
        return ets.ets_select_leaves(p, l, w, c, lb, ld, nl)

    sums = {"rebase": [], "ets": []}
    for seed in range(3):
        for pol in sums:
            r = simulate_search(pol, 32, 8, 256, 16, 64, seed, lambda_b=1.5, lambda_d=1.0,
                                select=sel, rebase=ets.ets_rebase_weights, node_limit=5000)
            r2 = simulate_search(pol, 32, 8, 256, 16, 64, seed, lambda_b=1.5, lambda_d=1.0,
                                 select=sel, rebase=ets.ets_rebase_weights, node_limit=5000)
            assert r["kv_tokens"] == r2["kv_tokens"]
            t = r["tree"]
            assert oracle.check_tree(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, t.pool_tokens) == 0
            assert t.n_leaves == 32          # the width is handed out in full at every step
            ost = oracle.tree_stats(t.parent, t.n_tokens, t.leaf_node)
            assert ost["unique_tokens"] == r["kv_tokens"][-1]
            sums[pol].append(r["kv_tokens_sum"])
    assert np.mean(sums["ets"]) < np.mean(sums["rebase"])
