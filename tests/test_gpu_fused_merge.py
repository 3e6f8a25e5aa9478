"""GPU: the merge run inside the attention launch ("fuse_merge") against the separate merge
launch and against the CPU oracle.  Both run the same arithmetic on the same partial
results in the same order, so their outputs are compared bit by bit; the parity bar itself
is checked against the oracle."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_13575_amd as ets
from workload import CONFIGS, TreeConfig, make_tree, make_values_host, random_tree

from _gpu_util import (compare, gpu_attn, make_ctx, oracle_full, pool_to_device, to_device)

pytestmark = pytest.mark.gpu


def _both(cfg, tree, k, v, q, options=None, calls=2):
    """(out, lse) of the separate merge launch and of `calls` calls with the merge inside
    the attention launch, on one context each."""
    kd, vd, qd = pool_to_device(k), pool_to_device(v), to_device(q)
    base = dict(options or {})
    with make_ctx(cfg, dict(base, fuse_merge=0, wide_rows=0)) as ctx:
        out0, lse0, st0 = gpu_attn(ctx, tree, kd, vd, qd)
    assert st0.merge_fused == 0
    fused = []
    with make_ctx(cfg, dict(base, fuse_merge=1)) as ctx:
        st = ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node, ets.ETS_PLAN_TREE)
        assert ctx.check().violations == 0
        ws = torch.empty(max(st.workspace_bytes, 16), dtype=torch.uint8, device="cuda:0")
        for _ in range(calls):
            out = torch.full_like(out0, float("nan"))
            lse = torch.full_like(lse0, float("nan"))
            ctx.decode(kd, vd, kd.shape[1], qd, out, lse, ws, ws.numel())
            torch.cuda.synchronize()
            fused.append((out, lse))
    return (out0, lse0), fused, st


@pytest.mark.parametrize("name", ["c2_w16", "c3_div", "c3_pruned"])
def test_fused_merge_equals_merge_launch_bitwise_and_oracle(name):
    cfg = CONFIGS[name]
    tree = make_tree(cfg)
    k, v, q = make_values_host(cfg, tree)
    print("case fused", name, flush=True)
    (out0, lse0), fused, st = _both(cfg, tree, k, v, q)
    assert st.merge_fused == 1 and st.n_wide_items == 0 and st.n_stream_items == 0
    for out, lse in fused:  # the second call finds the counters the first one put back
        assert torch.equal(out, out0) and torch.equal(lse, lse0)
    oo, ol = oracle_full(cfg, tree, k, v, q)
    d = cfg.head_dim
    compare(fused[-1][0].cpu().numpy().reshape(-1, d), fused[-1][1].cpu().numpy().reshape(-1),
            oo.reshape(-1, d), ol.reshape(-1), cfg.dtype, name + "/fused")


def _chain_tokens(tree):
    tot = np.zeros(tree.n_leaves, dtype=np.int64)
    for l, n in enumerate(tree.leaf_node):
        while n >= 0:
            tot[l] += tree.n_tokens[n]
            n = tree.parent[n]
    return tot


@pytest.mark.parametrize("heads", [(4, 4), (4, 8), (2, 8), (2, 16), (8, 64), (2, 8, 64), (1, 8, 64),
                                   (4, 4, 64)])
@pytest.mark.parametrize("seed", [0, 1, 2])
def test_fused_merge_every_head_grouping_on_irregular_forests(heads, seed):
    """1, 2, 4 and 8 query heads per kv head (the merging wave's lane layout differs for
    each) and both head sizes, forests with interior leaf queries, duplicates, ragged, empty and one-token
    nodes.  A leaf query whose chain holds no token gets its result (out = 0, lse = -inf)
    from the merge launch and nothing arrives for it, so such a plan keeps the launch."""
    hkv, hq = heads[:2]
    d = heads[2] if len(heads) > 2 else 128
    cfg = TreeConfig("fz", hkv, hq, d, "bf16", 0, 0, 0, 0, 0, None, seed=700 + seed)
    tree = random_tree(40 + 7 * seed + hq, n_nodes=[30, 90, 160][seed], n_leaves=[9, 40, 70][seed],
                       max_tokens=[90, 40, 12][seed], p_empty=[0.0, 0.05, 0.15][seed])
    k, v, q = make_values_host(cfg, tree)
    print("case fused forest", heads, seed, flush=True)
    (out0, lse0), fused, st = _both(cfg, tree, k, v, q)
    assert st.merge_fused == int((_chain_tokens(tree) > 0).all())
    for out, lse in fused:
        assert torch.equal(out, out0) and torch.equal(lse, lse0)
    oo, ol = oracle_full(cfg, tree, k, v, q)
    compare(out0.cpu().numpy().reshape(-1, d), lse0.cpu().numpy().reshape(-1),
            oo.reshape(-1, d), ol.reshape(-1), "bf16", "forest")


def test_fused_merge_with_bf16_output_and_e4m3_pools():
    """The merging wave applies the V scale of its kv head and rounds to bf16 the way the
    merge launch does."""
    from workload import make_values_fp8_host
    cfg = CONFIGS["c3_pruned"]
    tree = make_tree(cfg)
    ks, vs = 0.0123, 0.0217
    kc, vc, q = make_values_fp8_host(cfg, tree, ks, vs)
    kd, vd, qd = pool_to_device(kc), pool_to_device(vc), to_device(q)
    L, hq, d = tree.n_leaves, cfg.n_q_heads, cfg.head_dim
    res = {}
    for fuse in (0, 1):
        for bf in (0, 1):
            print("case fused e4m3", fuse, bf, flush=True)
            with make_ctx(cfg, {"fuse_merge": fuse, "wide_rows": 0, "out_bf16": bf}) as ctx:
                ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, ks, vs)
                st = ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node, 0)
                assert st.merge_fused == fuse
                out = torch.zeros((L, hq, d), dtype=torch.bfloat16 if bf else torch.float32,
                                  device="cuda:0")
                lse = torch.zeros((L, hq), dtype=torch.float32, device="cuda:0")
                ws = torch.empty(st.workspace_bytes, dtype=torch.uint8, device="cuda:0")
                ctx.decode(kd, vd, kd.shape[1], qd, out, lse, ws, ws.numel())
                torch.cuda.synchronize()
                res[fuse, bf] = (out, lse)
    assert torch.equal(res[0, 0][0], res[1, 0][0]) and torch.equal(res[0, 0][1], res[1, 0][1])
    assert torch.equal(res[0, 1][0].view(torch.int16), res[1, 1][0].view(torch.int16))
    assert torch.equal(res[1, 1][0], res[1, 0][0].to(torch.bfloat16))   # nearest even, as torch rounds
    oo, ol = oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                           tree.leaf_node, kc, vc, ks, vs, q, cfg.n_kv_heads,
                                           cfg.n_q_heads, cfg.head_dim)
    compare(res[1, 0][0].cpu().numpy().reshape(-1, d), res[1, 0][1].cpu().numpy().reshape(-1),
            oo.reshape(-1, d), ol.reshape(-1), "bf16", "fused e4m3")


def test_fused_merge_under_graph_capture():
    """Counters go back to zero at the end of every call and nothing is cleared with a
    memset: replays of a captured call, with eager calls between them, reproduce the result
    of the merge launch bit for bit."""
    cfg = CONFIGS["c3_div"]
    tree = make_tree(cfg)
    k, v, q = make_values_host(cfg, tree)
    kd, vd, qd = pool_to_device(k), pool_to_device(v), to_device(q)
    L, hq, d = tree.n_leaves, cfg.n_q_heads, cfg.head_dim
    with make_ctx(cfg, {"fuse_merge": 0, "wide_rows": 0}) as ctx:
        ref_out, ref_lse, _ = gpu_attn(ctx, tree, kd, vd, qd)
    with make_ctx(cfg, {"fuse_merge": 1}) as ctx:
        st = ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node, 0)
        assert st.merge_fused == 1
        ws = torch.empty(st.workspace_bytes, dtype=torch.uint8, device="cuda:0")
        out = torch.zeros((L, hq, d), device="cuda:0")
        lse = torch.zeros((L, hq), device="cuda:0")
        s = torch.cuda.Stream()
        with torch.cuda.stream(s):
            ctx.decode(kd, vd, tree.pool_tokens, qd, out, lse, ws, ws.numel(), s.cuda_stream)
        torch.cuda.synchronize()
        assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse)
        print("case fused graph capture", flush=True)
        g = torch.cuda.CUDAGraph()
        with torch.cuda.graph(g, stream=s):
            ctx.decode(kd, vd, tree.pool_tokens, qd, out, lse, ws, ws.numel(), s.cuda_stream)
        torch.cuda.synchronize()
        for rep in range(3):
            out.fill_(float("nan"))
            lse.fill_(float("nan"))
            ws.zero_()
            torch.cuda.synchronize()
            g.replay()
            torch.cuda.synchronize()
            assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse), rep
            with torch.cuda.stream(s):
                ctx.decode(kd, vd, tree.pool_tokens, qd, out, lse, ws, ws.numel(), s.cuda_stream)
            torch.cuda.synchronize()
            assert torch.equal(out, ref_out) and torch.equal(lse, ref_lse), rep
        del g
