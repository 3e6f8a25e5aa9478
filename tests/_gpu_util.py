"""Shared helpers of the GPU parity tests: run the library through its C ABI on
torch-owned device buffers and compare with the CPU oracle."""
import numpy as np
import torch

import oracle
import paper_2502_13575_amd as ets

# bf16 inputs, fp32 accumulation: bound on |gpu - oracle| for out and lse, and on
# the per-row error relative to the row's largest magnitude
TOL = {"bf16": dict(abs=2e-3, rel=1e-2), "f32": dict(abs=2e-5, rel=1e-4)}


def to_device(arr, device="cuda:0"):
    """numpy float32 -> torch float32; numpy uint16 (bf16 bits) -> torch bfloat16."""
    if arr.dtype == np.uint16:
        return torch.from_numpy(arr.view(np.int16)).to(device).view(torch.bfloat16)
    return torch.from_numpy(arr).to(device)


def pool_to_device(arr, device="cuda:0"):
    """K or V as the tests and the oracle index it, [pool row, kv head, D], laid out in
    device memory the way the library reads it: [kv head][pool row][D]."""
    return to_device(np.ascontiguousarray(arr.transpose(1, 0, 2)), device)


def pool_to_host(t):
    """Device pool [kv head][pool row][D] -> numpy view indexed [pool row, kv head, D]
    (not copied again: the oracle takes the strides as they are)."""
    return to_host_bits(t).transpose(1, 0, 2)


def to_host_bits(t):
    """torch tensor -> numpy in the oracle's input convention."""
    if t.dtype == torch.bfloat16:
        return t.contiguous().view(torch.int16).cpu().numpy().view(np.uint16)
    return t.contiguous().cpu().numpy()


def make_ctx(cfg, options=None, device=0):
    dt = ets.ETS_F32 if cfg.dtype == "f32" else ets.ETS_BF16
    ctx = ets.Context(cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim, dt, device)
    for k, v in (options or {}).items():
        ctx.set_option(k, v)
    return ctx


def gpu_attn(ctx, tree, k_dev, v_dev, q_dev, mode=ets.ETS_PLAN_TREE, stream=None):
    """Plans `tree`, runs one layer on device pools [Hkv][pool_tokens][D], returns (out [L,Hq,D], lse [L,Hq]) as torch tensors."""
    st = ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node, mode)
    L, hq, d = tree.n_leaves, ctx.shape.n_q_heads, ctx.shape.head_dim
    dev = q_dev.device
    out = torch.full((L, hq, d), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((L, hq), float("nan"), dtype=torch.float32, device=dev)
    ws = torch.empty(max(st.workspace_bytes, 16), dtype=torch.uint8, device=dev)
    ctx.decode(k_dev, v_dev, k_dev.shape[1], q_dev, out, lse, ws, ws.numel(),
               None if stream is None else stream.cuda_stream)
    torch.cuda.synchronize()
    return out, lse, st


def compare(out_g, lse_g, out_o, lse_o, dtype, what=""):
    """Parity bar: max-abs on out and lse; per-row inf-norm relative error on out;
    relative error on lse.  out_*: [n, D], lse_*: [n] (numpy)."""
    tol = TOL[dtype]
    out_g = np.asarray(out_g, dtype=np.float64)
    lse_g = np.asarray(lse_g, dtype=np.float64)
    assert np.all(np.isfinite(out_g)), what + ": non-finite out"
    fin = np.isfinite(lse_o)
    assert np.array_equal(np.isfinite(lse_g), fin), what + ": lse finiteness differs"
    assert np.all(lse_g[~fin] == lse_o[~fin]), what + ": empty-chain lse"
    err_o = np.abs(out_g - out_o)
    err_l = np.abs(lse_g[fin] - lse_o[fin])
    max_abs_o = float(err_o.max()) if err_o.size else 0.0
    max_abs_l = float(err_l.max()) if err_l.size else 0.0
    row_scale = np.maximum(np.abs(out_o).max(axis=-1), 1e-30)
    rel_o = float((err_o.max(axis=-1) / row_scale)[fin].max()) if fin.any() else 0.0
    # lse is a logarithm and passes through zero (a sum of weights near one): its error is
    # measured relative to max(|lse|, 1), i.e. absolutely where |lse| is small
    rel_l = float((err_l / np.maximum(np.abs(lse_o[fin]), 1.0)).max()) if fin.any() else 0.0
    msg = "%s: out max-abs %.3g row-rel %.3g; lse max-abs %.3g rel %.3g" % (
        what, max_abs_o, rel_o, max_abs_l, rel_l)
    assert max_abs_o <= tol["abs"] and max_abs_l <= tol["abs"], msg
    assert rel_o <= tol["rel"] and rel_l <= tol["rel"], msg
    return dict(out_abs=max_abs_o, out_rel=rel_o, lse_abs=max_abs_l, lse_rel=rel_l)


def oracle_full(cfg, tree, k, v, q):
    return oracle.tree_decode_attn(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                   k, v, q, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim)


def oracle_rows(cfg, tree, k, v, q, leaves, heads):
    return oracle.tree_decode_attn(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                   k, v, q, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim,
                                   rows=(leaves, heads))


def gpu_prefill(ctx, tree, k_dev, v_dev, q_dev, stream=None):
    """Plans step prefill for `tree`, runs one layer on device pools [Hkv][pool_tokens][D];
    returns (out [n_q_rows, Hq, D], lse [n_q_rows, Hq]) as torch tensors and the stats."""
    st = ctx.plan_prefill(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node)
    hq, d = ctx.shape.n_q_heads, ctx.shape.head_dim
    dev = q_dev.device
    out = torch.full((st.n_q_rows, hq, d), float("nan"), dtype=torch.float32, device=dev)
    lse = torch.full((st.n_q_rows, hq), float("nan"), dtype=torch.float32, device=dev)
    ctx.prefill(k_dev, v_dev, k_dev.shape[1], q_dev, out, lse,
                None if stream is None else stream.cuda_stream)
    torch.cuda.synchronize()
    return out, lse, st


def oracle_prefill(cfg, tree, k, v, q, rows=None):
    return oracle.tree_prefill_attn(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node,
                                    k, v, q, cfg.n_kv_heads, cfg.n_q_heads, cfg.head_dim,
                                    rows=rows)
