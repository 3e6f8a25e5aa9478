"""Parity of step-prefill attention (HIP library through its C ABI) with the CPU oracle:
element by element on small trees that span several blocks, tiles and ragged tails, on
sampled rows at the benchmark's full size, on the degenerate cases, and bitwise
reproducibility.  Tolerance: the bf16 bar of the decode path (max-abs 2e-3, per-row
relative 1e-2)."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_13575_amd as ets
from workload import (CONFIGS, Tree, TreeConfig, make_prefill_queries_host, make_tree,
                      make_values_device, make_values_host, random_tree)

from _gpu_util import (compare, gpu_prefill, make_ctx, oracle_prefill, pool_to_device,
                       pool_to_host, to_device, to_host_bits)

pytestmark = pytest.mark.gpu


def _full_parity(cfg, tree, what, seed=None):
    k, v, _ = make_values_host(cfg, tree, seed)
    q = make_prefill_queries_host(cfg, tree, seed)
    d = cfg.head_dim
    print("case", what, "rows", q.shape[0], flush=True)
    with make_ctx(cfg) as ctx:
        out, lse, st = gpu_prefill(ctx, tree, pool_to_device(k), pool_to_device(v), to_device(q))
    oo, ol = oracle_prefill(cfg, tree, k, v, q)
    assert out.shape[0] == oo.shape[0] == st.n_q_rows
    if st.n_q_rows:
        compare(out.cpu().numpy().reshape(-1, d), lse.cpu().numpy().reshape(-1),
                oo.reshape(-1, d), ol.reshape(-1), "bf16", what)
    return st


@pytest.mark.parametrize("seed", range(8))
def test_prefill_fuzz_irregular_forests(seed):
    hkv, hq = [(2, 8), (1, 1), (2, 16), (4, 8), (1, 2), (8, 32), (3, 12), (2, 2)][seed]
    cfg = TreeConfig("fuzz", hkv, hq, 128, "bf16", 0, 0, 0, 0, 0, None, seed=700 + seed)
    tree = random_tree(40 + seed, n_nodes=30, n_leaves=7, max_tokens=[70, 150, 20][seed % 3],
                       p_empty=0.15)
    _full_parity(cfg, tree, "prefill fuzz %d" % seed)


@pytest.mark.parametrize("n", [1, 15, 16, 17, 31, 32, 33, 63, 64, 65, 127, 128, 129, 200])
def test_prefill_node_lengths_around_block_and_tile_edges(n):
    # root of 45 rows (a ragged second run), one child of n rows carrying the queries,
    # plus a leaf query on the root itself (no ancestors: pure causal self-attention)
    cfg = TreeConfig("edge", 2, 8, 128, "bf16", 0, 0, 0, 0, 0, None, seed=800 + n)
    tree = Tree(np.array([-1, 0], np.int32), np.array([n, 0], np.int64),
                np.array([45, n], np.int32), np.array([1, 0], np.int32), n + 45)
    _full_parity(cfg, tree, "prefill edge n=%d" % n)


def test_prefill_long_paths_refill_the_descriptor_ring():
    # 700 scattered one-token ancestors (more than 256 runs, nothing merges), and a node
    # of 9000 contiguous rows below which a leaf step of 40 tokens hangs
    cfg = TreeConfig("long", 1, 4, 128, "bf16", 0, 0, 0, 0, 0, None, seed=31)
    n = 700
    parent = np.arange(-1, n - 1, dtype=np.int32)
    n_tok = np.ones(n, np.int32)
    n_tok[-1] = 37
    off = (np.arange(n, dtype=np.int64) * 7919) % n * 40
    tree = Tree(parent, off, n_tok, np.array([n - 1, 350], np.int32), int(off.max()) + 40)
    _full_parity(cfg, tree, "prefill 700 one-token ancestors")
    tree = Tree(np.array([-1, 0], np.int32), np.array([0, 9000], np.int64),
                np.array([9000, 40], np.int32), np.array([1], np.int32), 9040)
    _full_parity(cfg, tree, "prefill 9000-row ancestor")


def test_prefill_duplicates_empty_nodes_and_no_queries():
    cfg = TreeConfig("dup", 2, 8, 128, "bf16", 0, 0, 0, 0, 0, None, seed=33)
    tree = Tree(np.array([-1, 0, 0, 2], np.int32), np.array([0, 20, 0, 60], np.int64),
                np.array([20, 40, 0, 9], np.int32), np.array([1, 2, 1, 3, 0], np.int32), 69)
    st = _full_parity(cfg, tree, "prefill duplicates")
    assert st.n_q_rows == 40 + 0 + 40 + 9 + 20
    k, v, _ = make_values_host(cfg, tree)
    with make_ctx(cfg) as ctx:
        # leaf queries only on an empty node: nothing to do, nothing touched
        ctx.plan_prefill(tree.parent, tree.tok_offset, tree.n_tokens, np.array([2], np.int32))
        ctx.prefill(pool_to_device(k), pool_to_device(v), 69, None, None, None)
        torch.cuda.synchronize()


def test_prefill_c2_sampled_and_bitwise_reproducible():
    cfg = CONFIGS["c2_w16"]
    tree = make_tree(cfg)
    k, v, _ = make_values_host(cfg, tree)
    q = make_prefill_queries_host(cfg, tree)
    kd, vd, qd = pool_to_device(k), pool_to_device(v), to_device(q)
    with make_ctx(cfg) as ctx:
        o1, l1, st = gpu_prefill(ctx, tree, kd, vd, qd)
        o2, l2, _ = gpu_prefill(ctx, tree, kd, vd, qd)
    assert torch.equal(o1, o2) and torch.equal(l1, l2)
    r = np.random.default_rng(8)
    n = 256
    sl = r.integers(0, tree.n_leaves, size=n).astype(np.int32)
    stok = (r.random(n) * tree.n_tokens[tree.leaf_node[sl]]).astype(np.int32)
    sh = r.integers(0, cfg.n_q_heads, size=n).astype(np.int32)
    oo, ol = oracle_prefill(cfg, tree, k, v, q, rows=(sl, stok, sh))
    rows = oracle.prefill_q_ptr(tree.n_tokens, tree.leaf_node)[sl] + stok
    compare(o1.cpu().numpy()[rows, sh], l1.cpu().numpy()[rows, sh], oo, ol, "bf16", "prefill c2")


def test_prefill_c5_sampled_parity_at_full_size():
    """The benchmark's configuration: 512 leaf steps of the stress tree, inputs drawn on
    the device; sampled (leaf, token, head) triples against the oracle."""
    cfg = CONFIGS["c5_stress"]
    tree = make_tree(cfg)
    print("case prefill c5", flush=True)
    kd, vd, _ = make_values_device(cfg, tree, "cuda:0", layers=1)
    n_rows = int(oracle.prefill_q_ptr(tree.n_tokens, tree.leaf_node)[-1])
    g = torch.Generator(device="cuda:0")
    g.manual_seed(99)
    qd = torch.empty((n_rows, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16, device="cuda:0")
    qd.normal_(generator=g)
    with make_ctx(cfg) as ctx:
        out, lse, st = gpu_prefill(ctx, tree, kd[0], vd[0], qd)
    r = np.random.default_rng(9)
    n = 64
    sl = r.integers(0, tree.n_leaves, size=n).astype(np.int32)
    lens = tree.n_tokens[tree.leaf_node[sl]]
    stok = (r.random(n) * lens).astype(np.int32)
    stok[:8] = 0
    stok[8:16] = lens[8:16] - 1
    sh = r.integers(0, cfg.n_q_heads, size=n).astype(np.int32)
    rows = oracle.prefill_q_ptr(tree.n_tokens, tree.leaf_node)[sl] + stok
    idx = torch.from_numpy(rows).to("cuda:0")
    hidx = torch.from_numpy(sh.astype(np.int64)).to("cuda:0")
    og = out[idx, hidx].cpu().numpy()
    lg = lse[idx, hidx].cpu().numpy()
    assert torch.isfinite(lse).all()
    k, v = pool_to_host(kd[0]), pool_to_host(vd[0])
    q = to_host_bits(qd)
    oo, ol = oracle_prefill(cfg, tree, k, v, q, rows=(sl, stok, sh))
    compare(og, lg, oo, ol, "bf16", "prefill c5")


def test_prefill_device_error_paths():
    cfg = CONFIGS["c2_w16"]
    tree = make_tree(cfg)
    k, v, _ = make_values_host(cfg, tree)
    q = make_prefill_queries_host(cfg, tree)
    kd, vd, qd = pool_to_device(k), pool_to_device(v), to_device(q)
    with make_ctx(cfg) as ctx:
        out = torch.zeros((q.shape[0], cfg.n_q_heads, 128), device="cuda:0")
        lse = torch.zeros((q.shape[0], cfg.n_q_heads), device="cuda:0")
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill(kd, vd, tree.pool_tokens, qd, out, lse)
        assert e.value.status == 6                      # no prefill plan
        ctx.plan_prefill(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node)
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill(kd, vd, tree.pool_tokens - 1, qd, out, lse)
        assert e.value.status == 2                      # node rows outside the pool
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill(kd, vd, tree.pool_tokens, qd.data_ptr() + 2, out, lse)
        assert e.value.status == 1                      # misaligned q
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill(kd, None, tree.pool_tokens, qd, out, lse)
        assert e.value.status == 1
        assert torch.all(out == 0) and torch.all(lse == 0)


def test_prefill_custom_scale_larger_pool_and_side_stream():
    """sm_scale given explicitly, pools with more rows per head plane than the tree needs
    (pool_tokens is the plane stride), launch on a non-default stream."""
    cfg = TreeConfig("misc", 2, 8, 128, "bf16", 0, 0, 0, 0, 0, None, seed=41)
    tree = random_tree(77, n_nodes=24, n_leaves=6, max_tokens=90, p_empty=0.1)
    k, v, _ = make_values_host(cfg, tree)
    q = make_prefill_queries_host(cfg, tree)
    pad = 37
    kp = np.concatenate([k, np.zeros((pad,) + k.shape[1:], k.dtype)], axis=0)
    vp = np.concatenate([v, np.full((pad,) + v.shape[1:], 0x7FC0, v.dtype)], axis=0)  # NaN rows, never read
    scale = 0.05
    oo, ol = oracle.tree_prefill_attn(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                      k, v, q, 2, 8, 128, scale)
    side = torch.cuda.Stream()
    with ets.Context(2, 8, 128, ets.ETS_BF16, 0, scale) as ctx:
        kd, vd, qd = pool_to_device(kp), pool_to_device(vp), to_device(q)
        st = ctx.plan_prefill(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node)
        out = torch.full((st.n_q_rows, 8, 128), float("nan"), device="cuda:0")
        lse = torch.full((st.n_q_rows, 8), float("nan"), device="cuda:0")
        torch.cuda.synchronize()
        ctx.prefill(kd, vd, tree.pool_tokens + pad, qd, out, lse, side.cuda_stream)
        side.synchronize()
    compare(out.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1), oo.reshape(-1, 128),
            ol.reshape(-1), "bf16", "prefill scale/pad/stream")
