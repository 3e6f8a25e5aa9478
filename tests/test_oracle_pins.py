"""Pins for the CPU oracle: closed forms, library special cases, brute force,
merge invariance and sharing semantics.  None of these re-types the oracle's
own formula path; each would fail for a plausible mistake (dropped scale, wrong
log base, excluded leaf node, transposed head/stride, wrong GQA map, ...).
CPU only.
"""
import math
import os

import numpy as np
import pytest
import torch

import oracle
from workload import (CONFIGS, bf16_bits_to_f32, make_tree, make_values_host,
                      random_tree, to_bf16_bits, Tree)

GOLD = os.path.join(os.path.dirname(__file__), "golden", "closed_forms.txt")


def _golden():
    vals = {}
    with open(GOLD) as f:
        for line in f:
            line = line.strip()
            if line and not line.startswith("#"):
                k, v = line.split()
                vals[k] = float(v)
    return vals


def _run(tree, k, v, q, hkv, hq, d, scale=0.0, rows=None):
    return oracle.tree_decode_attn(tree.parent, tree.tok_offset, tree.n_tokens,
                                   tree.leaf_node, k, v, q, hkv, hq, d, scale, rows)


def _py_path(tree, v):
    p = []
    while v >= 0:
        p.append(int(v))
        v = int(tree.parent[v])
    return p[::-1]


def _py_rows(tree, leaf):
    rows = []
    for n in _py_path(tree, int(tree.leaf_node[leaf])):
        rows.extend(range(int(tree.tok_offset[n]), int(tree.tok_offset[n] + tree.n_tokens[n])))
    return rows


# ------------------------------------------------------------------ indexing
def test_c1_counts_match_closed_form():
    g = _golden()
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    assert t.n_nodes == g["n_nodes"] and t.n_leaves == g["n_leaves"]
    st = oracle.tree_stats(t.parent, t.n_tokens, t.leaf_node)
    assert st["unique_tokens"] == g["unique_tokens"]
    assert st["flat_tokens"] == g["flat_tokens"]
    assert st["live_nodes"] == g["n_nodes"]
    ptr, nodes = oracle.paths(t.parent, t.leaf_node)
    for l in range(t.n_leaves):
        p = nodes[ptr[l]:ptr[l + 1]]
        assert len(p) == 4 and p[0] == 0 and p[-1] == t.leaf_node[l]
        assert sum(int(t.n_tokens[n]) for n in p) == g["path_tokens"]


@pytest.mark.parametrize("seed", range(6))
def test_paths_and_stats_vs_python_walk(seed):
    t = random_tree(seed, n_nodes=40, n_leaves=17, max_tokens=5)
    ptr, nodes = oracle.paths(t.parent, t.leaf_node)
    cnt = np.zeros(t.n_nodes, dtype=np.int64)
    flat = 0
    for l in range(t.n_leaves):
        p = _py_path(t, int(t.leaf_node[l]))
        assert list(nodes[ptr[l]:ptr[l + 1]]) == p
        for n in p:
            cnt[n] += 1
            flat += int(t.n_tokens[n])
    st = oracle.tree_stats(t.parent, t.n_tokens, t.leaf_node)
    assert np.array_equal(st["leaf_count"], cnt)
    assert st["flat_tokens"] == flat
    assert st["unique_tokens"] == int(t.n_tokens[cnt > 0].sum())
    assert st["live_nodes"] == int((cnt > 0).sum())


def test_check_tree_rejects_malformed():
    t = make_tree(CONFIGS["c1_tiny"])
    ok = oracle.check_tree(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, t.pool_tokens)
    assert ok == 0
    bad = t.parent.copy(); bad[3] = 3
    assert oracle.check_tree(bad, t.tok_offset, t.n_tokens, t.leaf_node, t.pool_tokens) != 0
    bad = t.parent.copy(); bad[2] = 5
    assert oracle.check_tree(bad, t.tok_offset, t.n_tokens, t.leaf_node, t.pool_tokens) != 0
    assert oracle.check_tree(t.parent, t.tok_offset, t.n_tokens, t.leaf_node,
                             t.pool_tokens - 1) != 0
    lf = t.leaf_node.copy(); lf[0] = t.n_nodes
    assert oracle.check_tree(t.parent, t.tok_offset, t.n_tokens, lf, t.pool_tokens) != 0


# ------------------------------------------------------------- closed forms
def test_q_zero_gives_mean_of_path_values_and_ln_n():
    g = _golden()
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    q = np.zeros_like(q)
    out, lse = _run(t, k, v, q, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim)
    assert np.allclose(lse, g["lse_q0"], rtol=0, atol=1e-13)
    for l in range(t.n_leaves):
        rows = _py_rows(t, l)
        mean = v[rows, 0, :].astype(np.float64).mean(axis=0)
        for j in range(cfg.n_q_heads):
            assert np.allclose(out[l, j], mean, rtol=0, atol=1e-13)


def test_equal_keys_give_scaled_dot_plus_ln_n():
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    kvec = k[0, 0].copy()
    k[:] = kvec
    for scale in (0.0, 0.37):
        out, lse = _run(t, k, v, q, 1, 2, 64, scale)
        s = (1 / math.sqrt(64)) if scale == 0.0 else scale
        want = s * (q.astype(np.float64) @ kvec.astype(np.float64)) + math.log(80)
        assert np.allclose(lse, want, rtol=0, atol=1e-12)


def test_constant_values_and_gqa_head_map():
    # V of kv head h is the constant h => O[l, j, :] = j // G exactly.
    r = np.random.default_rng(5)
    t = random_tree(11, n_nodes=20, n_leaves=6, max_tokens=7, p_empty=0.0)
    hkv, hq, d = 3, 12, 8
    k = r.standard_normal((t.pool_tokens, hkv, d)).astype(np.float32)
    v = np.broadcast_to(np.arange(hkv, dtype=np.float32)[None, :, None],
                        (t.pool_tokens, hkv, d)).copy()
    q = r.standard_normal((t.n_leaves, hq, d)).astype(np.float32)
    out, _ = _run(t, k, v, q, hkv, hq, d)
    want = (np.arange(hq) // (hq // hkv)).astype(np.float64)
    assert np.allclose(out, want[None, :, None], rtol=0, atol=1e-13)


def test_key_shift_moves_lse_only():
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    u = np.random.default_rng(1).standard_normal(64).astype(np.float32)
    # keep the shifted keys exactly representable: use small dyadic shifts
    u = np.round(u * 8) / 8
    k0 = np.round(k * 64) / 64
    out0, lse0 = _run(t, k0.astype(np.float32), v, q, 1, 2, 64)
    out1, lse1 = _run(t, (k0 + u).astype(np.float32), v, q, 1, 2, 64)
    assert np.allclose(out0, out1, rtol=0, atol=1e-12)
    shift = (q.astype(np.float64) @ u.astype(np.float64)) / 8.0
    assert np.allclose(lse1 - lse0, shift, rtol=0, atol=1e-11)


def test_dominant_key_selects_its_value_row():
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    k *= 0.01
    leaf = 5
    rows = _py_rows(t, leaf)
    star = rows[37]                       # a row inside the path of `leaf`
    qv = q[leaf, 1].astype(np.float64)
    k[star, 0] = (qv / (qv @ qv) * 60.0 * 8.0).astype(np.float32)   # score ~ +60
    out, lse = _run(t, k, v, q, 1, 2, 64)
    # every other key scores ~0, so their total weight is ~79 e^-60
    assert np.max(np.abs(out[leaf, 1] - v[star, 0].astype(np.float64))) < 1e-12
    assert abs(lse[leaf, 1] - 60.0) < 1e-3


# ------------------------------------------- special case = library routine
@pytest.mark.parametrize("dtype", ["f32", "bf16"])
def test_single_leaf_chain_equals_dense_softmax_attention(dtype):
    r = np.random.default_rng(3)
    # a chain of 5 nodes whose pool rows are scattered (reverse order in the pool)
    n_tok = np.array([7, 1, 12, 3, 9], dtype=np.int32)
    parent = np.array([-1, 0, 1, 2, 3], dtype=np.int32)
    off = np.zeros(5, dtype=np.int64)
    pos = 0
    for i in (4, 2, 0, 3, 1):
        off[i] = pos
        pos += n_tok[i]
    hkv, hq, d = 2, 6, 16
    k = r.standard_normal((pos, hkv, d)).astype(np.float32)
    v = r.standard_normal((pos, hkv, d)).astype(np.float32)
    q = r.standard_normal((1, hq, d)).astype(np.float32)
    if dtype == "bf16":
        kb, vb, qb = to_bf16_bits(k), to_bf16_bits(v), to_bf16_bits(q)
        k, v, q = bf16_bits_to_f32(kb), bf16_bits_to_f32(vb), bf16_bits_to_f32(qb)
        args = (kb, vb, qb)
    else:
        args = (k, v, q)
    out, lse = oracle.tree_decode_attn(parent, off, n_tok, np.array([4], np.int32), *args,
                                       hkv, hq, d, 0.0)
    rows = np.concatenate([np.arange(off[i], off[i] + n_tok[i]) for i in range(5)])
    K = torch.from_numpy(k[rows]).double()      # [T, Hkv, D]
    V = torch.from_numpy(v[rows]).double()
    Q = torch.from_numpy(q[0]).double()         # [Hq, D]
    G = hq // hkv
    for j in range(hq):
        s = (K[:, j // G, :] @ Q[j]) / math.sqrt(d)
        w = torch.softmax(s, dim=0)
        o = w @ V[:, j // G, :]
        assert torch.allclose(torch.from_numpy(out[0, j]), o, rtol=0, atol=1e-12)
        assert abs(lse[0, j] - torch.logsumexp(s, 0).item()) < 1e-12


# -------------------------------------------------------------- brute force
@pytest.mark.parametrize("seed", range(5))
def test_brute_force_tiny_trees(seed):
    t = random_tree(100 + seed, n_nodes=8, n_leaves=5, max_tokens=4)
    r = np.random.default_rng(seed)
    hkv, hq, d = 2, 4, 4
    k = r.standard_normal((t.pool_tokens, hkv, d)).astype(np.float32)
    v = r.standard_normal((t.pool_tokens, hkv, d)).astype(np.float32)
    q = r.standard_normal((t.n_leaves, hq, d)).astype(np.float32)
    scale = 0.5
    out, lse = _run(t, k, v, q, hkv, hq, d, scale)
    for l in range(t.n_leaves):
        rows = _py_rows(t, l)
        for j in range(hq):
            h = j // 2
            if not rows:
                assert np.all(out[l, j] == 0) and lse[l, j] == -np.inf
                continue
            e = [math.exp(scale * math.fsum(float(q[l, j, x]) * float(k[t_, h, x])
                                            for x in range(d))) for t_ in rows]
            z = math.fsum(e)
            assert abs(lse[l, j] - math.log(z)) < 1e-12
            for x in range(d):
                o = math.fsum(e[i] * float(v[rows[i], h, x]) for i in range(len(rows))) / z
                assert abs(out[l, j, x] - o) < 1e-12


def test_empty_path_and_zero_length_nodes():
    parent = np.array([-1, 0, -1], dtype=np.int32)
    n_tok = np.array([0, 3, 0], dtype=np.int32)
    off = np.array([0, 0, 0], dtype=np.int64)
    r = np.random.default_rng(0)
    k = r.standard_normal((3, 1, 4)).astype(np.float32)
    v = r.standard_normal((3, 1, 4)).astype(np.float32)
    q = r.standard_normal((3, 1, 4)).astype(np.float32)
    out, lse = oracle.tree_decode_attn(parent, off, n_tok, np.array([2, 1, 0], np.int32),
                                       k, v, q, 1, 1, 4)
    assert np.all(out[0] == 0) and lse[0, 0] == -np.inf     # root with no tokens
    assert np.all(out[2] == 0) and lse[2, 0] == -np.inf
    assert np.isfinite(lse[1, 0])                           # zero-length ancestor skipped
    s = (k[:3, 0].astype(np.float64) @ q[1, 0].astype(np.float64)) / 2.0
    assert abs(lse[1, 0] - (np.log(np.exp(s).sum()))) < 1e-12


# ------------------------------------------------------------- LSE merging
def test_merge_of_any_split_equals_unsplit():
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    out, lse = _run(t, k, v, q, 1, 2, 64)
    leaf, j = 3, 1
    rows = np.array(_py_rows(t, leaf), dtype=np.int64)
    qv = q[leaf, j].astype(np.float64)
    for cut in range(0, len(rows) + 1):              # includes both empty splits
        parts = [rows[:cut], rows[cut:]]
        ps = [oracle.partial(k, v, qv, 0, p) for p in parts]
        o, l_ = oracle.merge(np.stack([p[0] for p in ps]), [p[1] for p in ps],
                             [p[2] for p in ps])
        assert np.allclose(o, out[leaf, j], rtol=0, atol=1e-12)
        assert abs(l_ - lse[leaf, j]) < 1e-12
    r = np.random.default_rng(9)
    for trial in range(10):                          # random k-way splits, random order
        kparts = int(r.integers(2, 9))
        cuts = np.sort(r.integers(0, len(rows) + 1, size=kparts - 1))
        perm = r.permutation(len(rows))              # token order inside the path is free
        parts = np.split(rows[perm], cuts)
        order = r.permutation(len(parts))
        ps = [oracle.partial(k, v, qv, 0, parts[i]) for i in order]
        o, l_ = oracle.merge(np.stack([p[0] for p in ps]), [p[1] for p in ps],
                             [p[2] for p in ps])
        assert np.allclose(o, out[leaf, j], rtol=0, atol=1e-12)
        assert abs(l_ - lse[leaf, j]) < 1e-12


def test_merge_matches_textbook_formula_on_hand_values():
    # two partials with one token each: scores 0 and ln 3, values 1 and 5
    # => weights 1/4 and 3/4 => out = 4, lse = ln 4.
    o, lse = oracle.merge(np.array([[1.0], [5.0]]), [0.0, math.log(3.0)], [1.0, 1.0])
    assert abs(o[0] - 4.0) < 1e-15 and abs(lse - math.log(4.0)) < 1e-15


# ------------------------------------------------------- sharing semantics
def test_tree_equals_private_deep_copies_bitwise():
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    out, lse = _run(t, k, v, q, 1, 2, 64)
    # flat copy: every leaf becomes a single root node holding its whole path
    rows = [np.array(_py_rows(t, l)) for l in range(t.n_leaves)]
    off = np.cumsum([0] + [len(r) for r in rows])
    kk = np.concatenate([k[r] for r in rows])
    vv = np.concatenate([v[r] for r in rows])
    out2, lse2 = oracle.tree_decode_attn(
        np.full(t.n_leaves, -1, np.int32), off[:-1].astype(np.int64),
        np.array([len(r) for r in rows], np.int32), np.arange(t.n_leaves, dtype=np.int32),
        kk, vv, q, 1, 2, 64)
    assert np.array_equal(out, out2) and np.array_equal(lse, lse2)


def test_duplicate_and_interior_leaf_entries():
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    leaf_node = np.array([7, 7, 3, 7], dtype=np.int32)     # node 3 is interior
    qq = q[:4].copy()
    qq[1] = qq[0]                                          # same node, same query
    out, lse = oracle.tree_decode_attn(t.parent, t.tok_offset, t.n_tokens, leaf_node, k, v, qq,
                                       1, 2, 64)
    assert np.array_equal(out[0], out[1]) and np.array_equal(lse[0], lse[1])
    assert not np.array_equal(out[0], out[3])              # same node, different query
    # interior entry sees root + step1 + its own node only: 32 + 16 + 16 tokens
    z = np.zeros_like(qq)
    _, lse0 = oracle.tree_decode_attn(t.parent, t.tok_offset, t.n_tokens, leaf_node, k, v, z,
                                      1, 2, 64)
    assert abs(lse0[2, 0] - math.log(64)) < 1e-13 and abs(lse0[0, 0] - math.log(80)) < 1e-13


def test_rows_subset_equals_full():
    cfg = CONFIGS["c2_w16"]
    t = make_tree(cfg)
    k, v, q = make_values_host(cfg, t)
    sl = np.array([0, 5, 15, 9], np.int32)
    sh = np.array([0, 31, 7, 16], np.int32)
    out_s, lse_s = _run(t, k, v, q, 8, 32, 128, rows=(sl, sh))
    # full oracle only on a sub-tree of leaves to keep it quick
    out_f, lse_f = _run(t, k, v, q, 8, 32, 128)
    for i in range(4):
        assert np.array_equal(out_s[i], out_f[sl[i], sh[i]])
        assert lse_s[i] == lse_f[sl[i], sh[i]]


def test_memory_order_of_the_pool_does_not_matter():
    # The same K[t, h, :] values held head-major in memory and handed over as a strided
    # view give bit-identical results; with V of kv head h = constant h the view must
    # still resolve heads by its second axis (a swapped stride would mix the constants).
    r = np.random.default_rng(12)
    t = random_tree(21, n_nodes=16, n_leaves=5, max_tokens=9, p_empty=0.0)
    hkv, hq, d = 3, 6, 8
    k = r.standard_normal((t.pool_tokens, hkv, d)).astype(np.float32)
    v = r.standard_normal((t.pool_tokens, hkv, d)).astype(np.float32)
    q = r.standard_normal((t.n_leaves, hq, d)).astype(np.float32)
    out0, lse0 = _run(t, k, v, q, hkv, hq, d)
    k_hm = np.ascontiguousarray(k.transpose(1, 0, 2))   # memory: [head][row][d]
    v_hm = np.ascontiguousarray(v.transpose(1, 0, 2))
    out1, lse1 = _run(t, k_hm.transpose(1, 0, 2), v_hm.transpose(1, 0, 2), q, hkv, hq, d)
    assert np.array_equal(out0, out1) and np.array_equal(lse0, lse1)
    vc = np.ascontiguousarray(np.broadcast_to(
        np.arange(hkv, dtype=np.float32)[:, None, None], (hkv, t.pool_tokens, d)))
    out2, _ = _run(t, k_hm.transpose(1, 0, 2), vc.transpose(1, 0, 2), q, hkv, hq, d)
    want = (np.arange(hq) // (hq // hkv)).astype(np.float64)
    assert np.allclose(out2, want[None, :, None], rtol=0, atol=1e-13)
    o_p, m_p, l_p = oracle.partial(k_hm.transpose(1, 0, 2), v_hm.transpose(1, 0, 2),
                                   q[0, 3].astype(np.float64), 1, np.arange(4))
    o_c, m_c, l_c = oracle.partial(k, v, q[0, 3].astype(np.float64), 1, np.arange(4))
    assert np.array_equal(o_p, o_c) and m_p == m_c and l_p == l_c


# --------------------------------------------------------------- generator
def test_bf16_bits_roundtrip_and_rne():
    x = np.array([1.0, 1.00390625, 1.005859375, -2.5, 3.140625, 1e-3], dtype=np.float32)
    b = to_bf16_bits(x)
    assert np.array_equal(bf16_bits_to_f32(b),
                          torch.from_numpy(x).to(torch.bfloat16).float().numpy())
    # 1 + 2^-8 is a tie between 1.0 and 1 + 2^-7: ties go to even (1.0)
    assert bf16_bits_to_f32(to_bf16_bits(np.array([1.00390625], np.float32)))[0] == 1.0


def test_generator_is_deterministic_and_variants_share_lengths():
    a, b = make_tree(CONFIGS["c3_div"]), make_tree(CONFIGS["c3_div"])
    assert np.array_equal(a.parent, b.parent) and np.array_equal(a.tok_offset, b.tok_offset)
    p = make_tree(CONFIGS["c3_pruned"])
    assert np.array_equal(a.n_tokens, p.n_tokens)
    sa = oracle.tree_stats(a.parent, a.n_tokens, a.leaf_node)
    sp = oracle.tree_stats(p.parent, p.n_tokens, p.leaf_node)
    assert sa["flat_tokens"] == sp["flat_tokens"] == 64 * (1024 + 16 * 128)
    ratio = sa["unique_tokens"] / sp["unique_tokens"]
    assert 1.4 < ratio < 2.6          # the pruned variant holds about half the unique KV
    k1 = make_values_host(CONFIGS["c2_w16"], make_tree(CONFIGS["c2_w16"]))[0]
    k2 = make_values_host(CONFIGS["c2_w16"], make_tree(CONFIGS["c2_w16"]))[0]
    assert np.array_equal(k1, k2)


# ------------------------------------------------------- decode-step advance
def test_append_kv_closed_forms():
    """After t appended tokens with q = 0 every LSE is ln(n_path + t); a dominant
    appended key turns the output into exactly that token's V row (GQA-mapped)."""
    from workload import with_growth_room, make_new_tokens_host
    cfg = CONFIGS["c1_tiny"]
    t = with_growth_room(make_tree(cfg), 4)
    k, v, q = make_values_host(cfg, t)
    base = [len(_py_rows(t, l)) for l in range(t.n_leaves)]
    n_tokens = t.n_tokens
    for step in range(3):
        kn, vn = make_new_tokens_host(cfg, t, step)
        n_tokens = oracle.append_kv(t.tok_offset, n_tokens, t.leaf_node, k, v, kn, vn)
    grown = Tree(t.parent, t.tok_offset, n_tokens, t.leaf_node, t.pool_tokens)
    out, lse = _run(grown, k, v, np.zeros_like(q), cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim)
    for l in range(t.n_leaves):
        assert np.allclose(lse[l], math.log(base[l] + 3), rtol=0, atol=1e-13)
    # a fourth token whose key is 200 q / |q|^2-aligned dominates every other score
    kn, vn = make_new_tokens_host(cfg, t, 3)
    G = cfg.n_q_heads // cfg.n_kv_heads
    for l in range(t.n_leaves):
        kn[l, :, :] = 0
        for h in range(cfg.n_kv_heads):
            kn[l, h, :] = 60.0 * q[l, h * G, :] / np.dot(q[l, h * G], q[l, h * G]) * math.sqrt(cfg.head_dim)
    n_tokens = oracle.append_kv(t.tok_offset, n_tokens, t.leaf_node, k, v, kn, vn)
    grown = Tree(t.parent, t.tok_offset, n_tokens, t.leaf_node, t.pool_tokens)
    out, lse = _run(grown, k, v, q, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim)
    for l in range(t.n_leaves):
        for h in range(cfg.n_kv_heads):
            assert np.allclose(out[l, h * G], vn[l, h].astype(np.float64), rtol=0, atol=1e-9)
    # rows written: exactly the first free row of every leaf node, nothing else moved
    k2, v2, _ = make_values_host(cfg, t)
    changed = np.nonzero((k2 != k).any(axis=(1, 2)))[0]
    want = np.sort(np.concatenate([t.tok_offset[n] + t.n_tokens[n] + np.arange(4)
                                   for n in np.unique(t.leaf_node)]))
    assert np.array_equal(changed, want)
