"""ets_tree_decode_attn_static (partial results in the library's own device buffer, no
allocation in the call) against ets_tree_decode_attn on the same inputs, through the C ABI."""
import numpy as np
import pytest
import torch

import paper_2502_13575_amd as ets
from workload import CONFIGS, make_tree, make_values_host

from _gpu_util import compare, make_ctx, oracle_rows, pool_to_device, to_device

pytestmark = pytest.mark.gpu


def _both_entry_points(ctx, cfg, tree, seed_note):
    k, v, q = make_values_host(cfg, tree)
    kd, vd, qd = pool_to_device(k), pool_to_device(v), to_device(q)
    st = ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node)
    assert 0 < st.workspace_bytes <= ets.ETS_STATIC_SCRATCH_BYTES, seed_note
    shape = (tree.n_leaves, cfg.n_q_heads, cfg.head_dim)
    out_a = torch.full(shape, float("nan"), dtype=torch.float32, device="cuda:0")
    lse_a = torch.full(shape[:2], float("nan"), dtype=torch.float32, device="cuda:0")
    out_b, lse_b = out_a.clone(), lse_a.clone()
    ws = torch.empty(st.workspace_bytes, dtype=torch.uint8, device="cuda:0")
    ctx.decode(kd, vd, tree.pool_tokens, qd, out_a, lse_a, ws, ws.numel())
    torch.cuda.synchronize()
    ctx.decode_static(kd, vd, tree.pool_tokens, qd, out_b, lse_b)
    torch.cuda.synchronize()
    # same kernels, same partial slots: the two entry points agree bit for bit
    assert torch.equal(out_a, out_b), seed_note
    assert torch.equal(lse_a, lse_b), seed_note
    # and the static call stands against the oracle by itself
    r = np.random.default_rng(11)
    n = min(96, tree.n_leaves * cfg.n_q_heads)
    leaves = r.integers(0, tree.n_leaves, size=n).astype(np.int32)
    heads = r.integers(0, cfg.n_q_heads, size=n).astype(np.int32)
    oo, ol = oracle_rows(cfg, tree, k, v, q, leaves, heads)
    compare(out_b.cpu().numpy()[leaves, heads], lse_b.cpu().numpy()[leaves, heads], oo, ol,
            cfg.dtype, "static " + seed_note)


def test_static_scratch_decode_matches_workspace_decode_two_calls():
    """Two calls in a row on one context, the second on a smaller tree: the buffer keeps
    the first call's partial rows, and none of them may leak into the second result."""
    big, small = CONFIGS["c3_pruned"], CONFIGS["c2_w16"]
    assert (big.n_kv_heads, big.n_q_heads, big.head_dim) == (small.n_kv_heads, small.n_q_heads,
                                                            small.head_dim)
    with make_ctx(big) as ctx:
        print("case static c3_pruned", flush=True)
        _both_entry_points(ctx, big, make_tree(big), "c3_pruned")
        print("case static c2_w16", flush=True)
        _both_entry_points(ctx, small, make_tree(small), "c2_w16")


def test_static_scratch_decode_refuses_a_plan_that_needs_more():
    cfg = CONFIGS["c4_34b"]
    tree = make_tree(cfg)
    with make_ctx(cfg) as ctx:
        st = ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node)
        assert st.workspace_bytes > ets.ETS_STATIC_SCRATCH_BYTES
        out = torch.zeros((tree.n_leaves, cfg.n_q_heads, cfg.head_dim), device="cuda:0")
        lse = torch.zeros((tree.n_leaves, cfg.n_q_heads), device="cuda:0")
        kv = torch.zeros((cfg.n_kv_heads, tree.pool_tokens, cfg.head_dim), dtype=torch.bfloat16,
                         device="cuda:0")
        q = torch.zeros((tree.n_leaves, cfg.n_q_heads, cfg.head_dim), dtype=torch.bfloat16,
                        device="cuda:0")
        with pytest.raises(ets.EtsError) as e:
            ctx.decode_static(kv, kv, tree.pool_tokens, q, out, lse)
        assert e.value.status == 5                      # ETS_ERR_WORKSPACE
        torch.cuda.synchronize()
        assert float(out.abs().max()) == 0.0            # nothing was enqueued
