"""Pins for the oracle's step-prefill attention (every token of a leaf query's node is a
query; it sees the strict ancestors in full and its own node causally).  The checks do
not re-type the oracle's formula path: a library routine on a special case, closed
forms, brute force, the link to the separately pinned decode oracle, and causality.
CPU only.
"""
import math

import numpy as np
import pytest
import torch

import oracle
from workload import CONFIGS, Tree, make_tree, random_tree, to_bf16_bits, bf16_bits_to_f32


def _prefill(t, k, v, q, hkv, hq, d, scale=0.0, rows=None):
    return oracle.tree_prefill_attn(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, k, v, q,
                                    hkv, hq, d, scale, rows)


def _vals(r, t, hkv, hq, d):
    nq = int(oracle.prefill_q_ptr(t.n_tokens, t.leaf_node)[-1])
    k = r.standard_normal((t.pool_tokens, hkv, d)).astype(np.float32)
    v = r.standard_normal((t.pool_tokens, hkv, d)).astype(np.float32)
    q = r.standard_normal((nq, hq, d)).astype(np.float32)
    return k, v, q


def _py_chain(t, node):
    c = []
    while node >= 0:
        c.append(int(node))
        node = int(t.parent[node])
    return c[::-1]


def test_query_rows_are_numbered_leaf_by_leaf():
    # c1: 8 leaf queries on nodes of 16 tokens each => rows 16 l .. 16 l + 15
    t = make_tree(CONFIGS["c1_tiny"])
    assert np.array_equal(oracle.prefill_q_ptr(t.n_tokens, t.leaf_node), 16 * np.arange(9))
    # duplicates and an empty node
    n_tok = np.array([3, 0, 5], np.int32)
    assert np.array_equal(oracle.prefill_q_ptr(n_tok, np.array([2, 1, 2, 0])), [0, 5, 5, 10, 13])


def test_visible_rows_closed_form():
    # chain 0 -> 1 -> 2 with lengths 4, 0, 3 at pool rows 10.., -, 2..
    parent = np.array([-1, 0, 1], np.int32)
    off = np.array([10, 0, 2], np.int64)
    n_tok = np.array([4, 0, 3], np.int32)
    assert oracle.visible_rows(parent, off, n_tok, 2).tolist() == [10, 11, 12, 13, 2, 3, 4]
    assert oracle.visible_rows(parent, off, n_tok, 2, 1).tolist() == [10, 11, 12, 13, 2]
    assert oracle.visible_rows(parent, off, n_tok, 0, 2).tolist() == [10, 11]
    assert oracle.visible_rows(parent, off, n_tok, 1).tolist() == [10, 11, 12, 13]


@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_root_only_node_is_plain_causal_self_attention(dtype):
    # One node, one leaf query on it: torch's causal scaled-dot-product attention in fp64.
    r = np.random.default_rng(31)
    n, hkv, hq, d = 23, 2, 4, 16
    t = Tree(np.array([-1], np.int32), np.array([0], np.int64), np.array([n], np.int32),
             np.array([0], np.int32), n)
    k, v, q = _vals(r, t, hkv, hq, d)
    args = (k, v, q)
    if dtype == "bf16":
        args = tuple(to_bf16_bits(x) for x in (k, v, q))
        k, v, q = (bf16_bits_to_f32(x) for x in args)
    out, lse = _prefill(t, *args, hkv, hq, d)
    G = hq // hkv
    Q = torch.from_numpy(q).double().permute(1, 0, 2)                      # [Hq, n, D]
    K = torch.from_numpy(k).double().permute(1, 0, 2).repeat_interleave(G, 0)
    V = torch.from_numpy(v).double().permute(1, 0, 2).repeat_interleave(G, 0)
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V, is_causal=True)
    assert torch.allclose(torch.from_numpy(out).permute(1, 0, 2), want, rtol=0, atol=1e-12)


def test_chain_with_cached_ancestors_equals_masked_dense_attention():
    # root (9 rows) -> mid (4) -> leaf (11), rows scattered; the leaf's 11 queries see the
    # 13 ancestor rows in full and the leaf's rows causally: dense attention with a mask.
    r = np.random.default_rng(32)
    n_tok = np.array([9, 4, 11], np.int32)
    off = np.array([15, 0, 4], np.int64)
    t = Tree(np.array([-1, 0, 1], np.int32), off, n_tok, np.array([2], np.int32), 24)
    hkv, hq, d = 2, 6, 8
    k, v, q = _vals(r, t, hkv, hq, d)
    out, lse = _prefill(t, k, v, q, hkv, hq, d, 0.3)
    rows = np.concatenate([np.arange(off[i], off[i] + n_tok[i]) for i in range(3)])
    mask = torch.ones(11, 24, dtype=torch.bool)
    mask[:, 13:] = torch.tril(torch.ones(11, 11, dtype=torch.bool))
    G = hq // hkv
    Q = torch.from_numpy(q).double().permute(1, 0, 2)
    K = torch.from_numpy(k[rows]).double().permute(1, 0, 2).repeat_interleave(G, 0)
    V = torch.from_numpy(v[rows]).double().permute(1, 0, 2).repeat_interleave(G, 0)
    want = torch.nn.functional.scaled_dot_product_attention(Q, K, V, attn_mask=mask, scale=0.3)
    assert torch.allclose(torch.from_numpy(out).permute(1, 0, 2), want, rtol=0, atol=1e-12)
    s = torch.einsum("hqd,hkd->hqk", Q, K) * 0.3
    s = s.masked_fill(~mask, float("-inf"))
    assert torch.allclose(torch.from_numpy(lse).permute(1, 0), torch.logsumexp(s, -1),
                          rtol=0, atol=1e-12)


def test_zero_queries_give_running_means_and_log_counts():
    # q = 0: every visible row weighs the same => LSE = ln(#visible), O = their mean V.
    r = np.random.default_rng(33)
    t = random_tree(41, n_nodes=14, n_leaves=6, max_tokens=6, p_empty=0.2)
    hkv, hq, d = 2, 4, 8
    k, v, q = _vals(r, t, hkv, hq, d)
    q[:] = 0
    out, lse = _prefill(t, k, v, q, hkv, hq, d)
    row = 0
    for l in range(t.n_leaves):
        node = int(t.leaf_node[l])
        anc = [x for n in _py_chain(t, node)[:-1]
               for x in range(int(t.tok_offset[n]), int(t.tok_offset[n] + t.n_tokens[n]))]
        for i in range(int(t.n_tokens[node])):
            vis = anc + list(range(int(t.tok_offset[node]), int(t.tok_offset[node]) + i + 1))
            assert np.allclose(lse[row], math.log(len(vis)), rtol=0, atol=1e-13)
            for j in range(hq):
                want = v[vis, j // 2, :].astype(np.float64).mean(axis=0)
                assert np.allclose(out[row, j], want, rtol=0, atol=1e-13)
            row += 1
    assert row == q.shape[0]


def test_each_row_equals_decode_on_the_truncated_node():
    # Token i of a node, as a prefill query, is the decode query of the tree whose leaf
    # node has been cut to its first i + 1 tokens (the decode oracle has its own pins).
    r = np.random.default_rng(34)
    t = random_tree(42, n_nodes=12, n_leaves=5, max_tokens=5, p_empty=0.1)
    hkv, hq, d = 1, 2, 8
    k, v, q = _vals(r, t, hkv, hq, d)
    out, lse = _prefill(t, k, v, q, hkv, hq, d)
    q_ptr = oracle.prefill_q_ptr(t.n_tokens, t.leaf_node)
    for l in range(t.n_leaves):
        node = int(t.leaf_node[l])
        for i in range(int(t.n_tokens[node])):
            cut = t.n_tokens.copy()
            cut[node] = i + 1
            # children of `node` are no leaf queries' business here: one leaf query only
            o1, l1 = oracle.tree_decode_attn(t.parent, t.tok_offset, cut,
                                             np.array([node], np.int32), k, v,
                                             q[q_ptr[l] + i][None], hkv, hq, d)
            assert np.array_equal(o1[0], out[q_ptr[l] + i])
            assert np.array_equal(l1[0], lse[q_ptr[l] + i])


def test_causality_inside_the_new_step():
    r = np.random.default_rng(35)
    n_tok = np.array([5, 8], np.int32)
    t = Tree(np.array([-1, 0], np.int32), np.array([0, 5], np.int64), n_tok,
             np.array([1], np.int32), 13)
    hkv, hq, d = 1, 2, 8
    k, v, q = _vals(r, t, hkv, hq, d)
    out0, lse0 = _prefill(t, k, v, q, hkv, hq, d)
    k2, v2 = k.copy(), v.copy()
    k2[5 + 4] += 1.0          # own token 4 of the leaf node
    v2[5 + 4] -= 2.0
    out1, lse1 = _prefill(t, k2, v2, q, hkv, hq, d)
    assert np.array_equal(out0[:4], out1[:4]) and np.array_equal(lse0[:4], lse1[:4])
    for i in range(4, 8):      # token 4 and every later token see the change
        assert not np.array_equal(out0[i], out1[i]) and not np.array_equal(lse0[i], lse1[i])
    k3 = k.copy()
    k3[2] += 1.0              # an ancestor row is seen by every query
    _, lse3 = _prefill(t, k3, v, q, hkv, hq, d)
    assert np.all(lse3 != lse0)


@pytest.mark.parametrize("seed", range(4))
def test_prefill_brute_force_tiny_trees(seed):
    t = random_tree(200 + seed, n_nodes=7, n_leaves=4, max_tokens=4)
    r = np.random.default_rng(seed)
    hkv, hq, d = 2, 4, 4
    k, v, q = _vals(r, t, hkv, hq, d)
    scale = 0.7
    out, lse = _prefill(t, k, v, q, hkv, hq, d, scale)
    row = 0
    for l in range(t.n_leaves):
        node = int(t.leaf_node[l])
        chain = _py_chain(t, node)
        for i in range(int(t.n_tokens[node])):
            vis = [x for n in chain[:-1]
                   for x in range(int(t.tok_offset[n]), int(t.tok_offset[n] + t.n_tokens[n]))]
            vis += list(range(int(t.tok_offset[node]), int(t.tok_offset[node]) + i + 1))
            for j in range(hq):
                h = j // 2
                e = [math.exp(scale * math.fsum(float(q[row, j, x]) * float(k[t_, h, x])
                                                for x in range(d))) for t_ in vis]
                z = math.fsum(e)
                assert abs(lse[row, j] - math.log(z)) < 1e-12
                for x in range(d):
                    o = math.fsum(e[a] * float(v[vis[a], h, x]) for a in range(len(vis))) / z
                    assert abs(out[row, j, x] - o) < 1e-12
            row += 1
    assert row == q.shape[0]


def test_duplicate_entries_and_selected_rows():
    # two leaf queries on one node own separate query rows; selected triples equal the
    # same entries of the full result
    r = np.random.default_rng(36)
    n_tok = np.array([6, 4, 0], np.int32)
    t = Tree(np.array([-1, 0, 0], np.int32), np.array([0, 6, 10], np.int64), n_tok,
             np.array([1, 1, 2, 0], np.int32), 10)
    hkv, hq, d = 2, 2, 8
    k, v, q = _vals(r, t, hkv, hq, d)
    assert q.shape[0] == 4 + 4 + 0 + 6
    q[4:8] = q[0:4]
    out, lse = _prefill(t, k, v, q, hkv, hq, d)
    assert np.array_equal(out[0:4], out[4:8]) and np.array_equal(lse[0:4], lse[4:8])
    q[4:8] += 1
    out2, _ = _prefill(t, k, v, q, hkv, hq, d)
    assert np.array_equal(out2[0:4], out[0:4]) and not np.array_equal(out2[4:8], out[4:8])
    sl = np.array([3, 1, 0], np.int32)
    st = np.array([5, 2, 3], np.int32)
    sh = np.array([1, 0, 1], np.int32)
    o_s, l_s = _prefill(t, k, v, q, hkv, hq, d, rows=(sl, st, sh))
    q_ptr = oracle.prefill_q_ptr(t.n_tokens, t.leaf_node)
    for a in range(3):
        assert np.array_equal(o_s[a], out2[q_ptr[sl[a]] + st[a], sh[a]])
    with pytest.raises(RuntimeError):
        _prefill(t, k, v, q, hkv, hq, d, rows=(np.array([2]), np.array([0]), np.array([0])))
