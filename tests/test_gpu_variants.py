"""GPU parity of the decode-path variants: K/V pools stored as E4M3 codes, bfloat16
output, and both together, against the CPU oracle through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
import paper_2502_13575_amd as ets
from workload import (CONFIGS, TreeConfig, make_tree, make_values_fp8_device, make_values_fp8_host,
                      make_values_host, random_tree, with_growth_room)

from _gpu_util import (compare, gpu_prefill, make_ctx, oracle_full, pool_to_device, pool_to_host,
                       to_device, to_host_bits)

pytestmark = pytest.mark.gpu

KS, VS = 0.0123, 0.0217      # pool scales: N(0,1) values land on codes of magnitude ~80


def oracle_fp8(cfg, tree, kc, vc, q, ks=KS, vs=VS, rows=None, sm_scale=0.0):
    return oracle.tree_decode_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                         tree.leaf_node, kc, vc, ks, vs, q, cfg.n_kv_heads,
                                         cfg.n_q_heads, cfg.head_dim, sm_scale=sm_scale, rows=rows)


def run(ctx, tree, kd, vd, qd, mode=ets.ETS_PLAN_TREE, out_dtype=torch.float32, plan=True,
        pool_tokens=None):
    st = (ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node, mode)
          if plan else ctx.stats())
    L, hq, d = tree.n_leaves, ctx.shape.n_q_heads, ctx.shape.head_dim
    out = torch.full((L, hq, d), float("nan"), dtype=out_dtype, device="cuda:0")
    lse = torch.full((L, hq), float("nan"), dtype=torch.float32, device="cuda:0")
    ws = torch.empty(max(st.workspace_bytes, 16), dtype=torch.uint8, device="cuda:0")
    ctx.decode(kd, vd, kd.shape[1] if pool_tokens is None else pool_tokens, qd, out, lse, ws,
               ws.numel())
    torch.cuda.synchronize()
    return out, lse, st


@pytest.mark.parametrize("name", ["c2_w16", "c3_div", "c3_pruned"])
@pytest.mark.parametrize("mode", [ets.ETS_PLAN_TREE, ets.ETS_PLAN_FLAT])
def test_fp8kv_full_parity(name, mode):
    cfg = CONFIGS[name]
    tree = make_tree(cfg)
    kc, vc, q = make_values_fp8_host(cfg, tree, KS, VS)
    print("case fp8", name, mode, flush=True)
    with make_ctx(cfg) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        out, lse, st = run(ctx, tree, pool_to_device(kc), pool_to_device(vc), to_device(q), mode)
    assert st.unique_kv_bytes == st.unique_tokens * 2 * cfg.n_kv_heads * cfg.head_dim
    oo, ol = oracle_fp8(cfg, tree, kc, vc, q)
    compare(out.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1),
            oo.reshape(-1, 128), ol.reshape(-1), "bf16", "fp8 %s/mode%d" % (name, mode))


@pytest.mark.parametrize("name,heads,options", [("c3_div", (8, 32), {}), ("c3_pruned", (4, 32), {"fuse_merge": 1}),
                                                ("c2_w16", (2, 2), {"wave_items": 0}),
                                                ("c2_w16", (4, 8), {"cascade_rows": 16})])
def test_fp8kv_head_dim_64_full_parity(name, heads, options):
    """Pools of E4M3 codes with head_dim 64 (rows of 64 bytes, 8-byte pieces) through the
    shared-node kernel's instantiation for that head size, with per-head scales."""
    import dataclasses
    cfg = dataclasses.replace(CONFIGS[name], n_kv_heads=heads[0], n_q_heads=heads[1], head_dim=64)
    tree = make_tree(cfg)
    kc, vc, q = make_values_fp8_host(cfg, tree, KS, VS)
    print("case fp8 d64", name, heads, options, flush=True)
    with make_ctx(cfg, options) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        out, lse, st = run(ctx, tree, pool_to_device(kc), pool_to_device(vc), to_device(q))
        assert ctx.check().violations == 0
    assert st.shares_nodes == 1 and st.n_stream_items == 0
    assert st.unique_kv_bytes == st.unique_tokens * 2 * cfg.n_kv_heads * 64
    oo, ol = oracle_fp8(cfg, tree, kc, vc, q)
    compare(out.cpu().numpy().reshape(-1, 64), lse.cpu().numpy().reshape(-1),
            oo.reshape(-1, 64), ol.reshape(-1), "bf16", "fp8 d64 " + name)


@pytest.mark.parametrize("seed", range(8))
def test_fp8kv_fuzz_irregular_forests(seed):
    """Ragged steps, empty nodes, several roots, duplicated and interior leaf queries, every
    group size, all item kinds (planner knobs), every E4M3 code that is a number."""
    hkv, hq = [(2, 8), (4, 4), (1, 8), (3, 6), (2, 2), (1, 4), (2, 16), (8, 8)][seed]
    cfg = TreeConfig("fuzz8", hkv, hq, 128, "bf16", 0, 0, 0, 0, 0, None, seed=700 + seed)
    tree = random_tree(300 + seed, n_nodes=50, n_leaves=21, max_tokens=90)
    options = {"stream_chunk": [0, 32, 64][seed % 3], "cascade_chunk": [0, 32, 96][(seed // 3) % 3],
               "cascade_rows": [64, 16, 32][(seed // 2) % 3],
               "wave_items": [512, 0, 48, 100000][seed % 4]}
    ks, vs = [(1.0, 1.0), (KS, VS), (0.5, 3.0), (2.0 ** -8, 7.5)][seed % 4]
    if seed < 4:
        kc, vc, q = make_values_fp8_host(cfg, tree, ks, vs)
    else:
        # uniformly drawn codes: all magnitudes from 2^-9 to 448 next to each other; scales
        # that keep the scores moderate
        r = np.random.default_rng(seed)
        finite = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
        kc = finite[r.integers(0, finite.size, size=(tree.pool_tokens, hkv, 128))]
        vc = finite[r.integers(0, finite.size, size=(tree.pool_tokens, hkv, 128))]
        q = make_values_host(cfg, tree)[2]
        ks, vs = 1.0 / 64, 1.0 / 128
    oo, ol = oracle_fp8(cfg, tree, kc, vc, q, ks, vs)
    for mode in (ets.ETS_PLAN_TREE, ets.ETS_PLAN_FLAT):
        print("case fp8 fuzz", seed, mode, flush=True)
        with make_ctx(cfg, options) as ctx:
            ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, ks, vs)
            out, lse, _ = run(ctx, tree, pool_to_device(kc), pool_to_device(vc), to_device(q), mode)
        compare(out.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1),
                oo.reshape(-1, 128), ol.reshape(-1), "bf16", "fp8 fuzz%d/mode%d" % (seed, mode))


def test_fp8kv_c5_sampled_parity_at_full_size():
    cfg = CONFIGS["c5_stress"]
    tree = make_tree(cfg)
    print("case fp8 c5", flush=True)
    kd, vd, qd = make_values_fp8_device(cfg, tree, "cuda:0", KS, VS, layers=1)
    with make_ctx(cfg) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        out, lse, st = run(ctx, tree, kd[0], vd[0], qd[0])
    assert torch.isfinite(lse).all()
    r = np.random.default_rng(58)
    leaves = r.integers(0, tree.n_leaves, size=48).astype(np.int32)
    heads = r.integers(0, cfg.n_q_heads, size=48).astype(np.int32)
    oo, ol = oracle_fp8(cfg, tree, pool_to_host(kd[0]), pool_to_host(vd[0]), to_host_bits(qd[0]),
                        rows=(leaves, heads))
    compare(out.cpu().numpy()[leaves, heads], lse.cpu().numpy()[leaves, heads], oo, ol, "bf16",
            "fp8 c5")


def test_fp8kv_decode_loop_appends_codes():
    """Decode steps on E4M3 pools: the appended rows are 128-byte rows of codes; outputs
    equal the oracle on the grown tree and the pools end up bytewise equal to the oracle's."""
    cfg = CONFIGS["c2_w16"]
    steps = 40
    tree = with_growth_room(make_tree(cfg), steps + 2)
    kc, vc, q = make_values_fp8_host(cfg, tree, KS, VS)
    kd, vd, qd = pool_to_device(kc), pool_to_device(vc), to_device(q)
    n_tokens = tree.n_tokens.copy()
    r = np.random.default_rng(12)
    finite = np.array([c for c in range(256) if c & 0x7F != 0x7F], dtype=np.uint8)
    with make_ctx(cfg) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        ctx.plan(tree.parent, tree.tok_offset, tree.n_tokens, tree.leaf_node)
        for step in range(steps):
            kn = finite[r.integers(0, finite.size, size=(tree.n_leaves, cfg.n_kv_heads, 128))]
            vn = finite[r.integers(0, finite.size, size=(tree.n_leaves, cfg.n_kv_heads, 128))]
            n_tokens = oracle.append_kv(tree.tok_offset, n_tokens, tree.leaf_node, kc, vc, kn, vn)
            ctx.plan_advance()
            ctx.kv_append(kd, vd, tree.pool_tokens, to_device(kn), to_device(vn))
            out, lse, _ = run(ctx, tree, kd, vd, qd, plan=False)
            if step % 7 == 0 or step >= steps - 2:
                grown = type(tree)(tree.parent, tree.tok_offset, n_tokens, tree.leaf_node,
                                   tree.pool_tokens)
                oo, ol = oracle_fp8(cfg, grown, kc, vc, q)
                compare(out.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1),
                        oo.reshape(-1, 128), ol.reshape(-1), "bf16", "fp8 step %d" % step)
    assert np.array_equal(pool_to_host(kd), kc) and np.array_equal(pool_to_host(vd), vc)


def test_fp8kv_needs_the_matrix_core_kernel():
    cfg = CONFIGS["c2_w16"]
    tree = make_tree(cfg)
    kc, vc, q = make_values_fp8_host(cfg, tree, KS, VS)
    with make_ctx(cfg, {"mfma": 0}) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        with pytest.raises(ets.EtsError) as e:
            run(ctx, tree, pool_to_device(kc), pool_to_device(vc), to_device(q))
        assert e.value.status == 4


@pytest.mark.parametrize("name,opts", [("c3_div", {}), ("c2_w16", {"mfma": 0}), ("c1_tiny", {})])
def test_bf16_output_is_the_rounded_fp32_output(name, opts):
    """With "out_bf16" the result is the fp32 result rounded to nearest even (bit for bit
    against torch's conversion of the fp32 run), and it meets the oracle within the
    parity bar plus half a bf16 unit in the last place."""
    cfg = CONFIGS[name]
    tree = make_tree(cfg)
    k, v, q = make_values_host(cfg, tree)
    kd, vd, qd = pool_to_device(k), pool_to_device(v), to_device(q)
    d = cfg.head_dim
    with make_ctx(cfg, opts) as ctx:
        o32, l32, _ = run(ctx, tree, kd, vd, qd)
        ctx.set_option("out_bf16", 1)
        o16, l16, _ = run(ctx, tree, kd, vd, qd, out_dtype=torch.bfloat16)
        ctx.set_option("out_bf16", 0)
        o32b, _, _ = run(ctx, tree, kd, vd, qd)
    assert torch.equal(l16, l32) and torch.equal(o32b, o32)
    assert torch.equal(o16.view(torch.int16), o32.to(torch.bfloat16).view(torch.int16))
    oo, ol = oracle_full(cfg, tree, k, v, q)
    tol = 2e-3 if cfg.dtype == "bf16" else 2e-5
    err = np.abs(o16.float().cpu().numpy().astype(np.float64) - oo)
    assert np.all(err <= tol + 2.0 ** -8 * np.abs(oo)), err.max()


def test_fp8kv_with_bf16_output():
    cfg = CONFIGS["c3_pruned"]
    tree = make_tree(cfg)
    kc, vc, q = make_values_fp8_host(cfg, tree, KS, VS)
    kd, vd, qd = pool_to_device(kc), pool_to_device(vc), to_device(q)
    with make_ctx(cfg, {"out_bf16": 1}) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        o16, lse, _ = run(ctx, tree, kd, vd, qd, out_dtype=torch.bfloat16)
    oo, ol = oracle_fp8(cfg, tree, kc, vc, q)
    err = np.abs(o16.float().cpu().numpy().astype(np.float64) - oo)
    assert np.all(err <= 2e-3 + 2.0 ** -8 * np.abs(oo)), err.max()
    assert np.abs(lse.cpu().numpy() - ol).max() <= 2e-3


def oracle_prefill_fp8(cfg, tree, kc, vc, q, ks, vs, rows=None):
    return oracle.tree_prefill_attn_fp8kv(tree.parent, tree.tok_offset, tree.n_tokens,
                                          tree.leaf_node, kc, vc, ks, vs, q, cfg.n_kv_heads,
                                          cfg.n_q_heads, cfg.head_dim, rows=rows)


@pytest.mark.parametrize("seed", range(6))
def test_fp8kv_prefill_fuzz_irregular_forests(seed):
    """Step prefill over E4M3 pools on irregular forests (ragged runs, empty nodes, duplicate
    and interior leaf queries), every row against the oracle."""
    from workload import make_prefill_queries_host
    hkv, hq = [(2, 8), (1, 8), (4, 4), (2, 4), (1, 2), (2, 16)][seed]
    cfg = TreeConfig("pfuzz8", hkv, hq, 128, "bf16", 0, 0, 0, 0, 0, None, seed=800 + seed)
    tree = random_tree(500 + seed, n_nodes=40, n_leaves=9, max_tokens=[70, 150, 40][seed % 3])
    ks, vs = [(KS, VS), (1.0, 1.0), (0.5, 3.0)][seed % 3]
    kc, vc, _ = make_values_fp8_host(cfg, tree, ks, vs)
    q = make_prefill_queries_host(cfg, tree)
    print("case fp8 prefill fuzz", seed, flush=True)
    with make_ctx(cfg) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, ks, vs)
        out, lse, st = gpu_prefill(ctx, tree, pool_to_device(kc), pool_to_device(vc), to_device(q))
    assert st.unique_kv_bytes == st.unique_tokens * 2 * hkv * 128
    if st.n_q_rows == 0:
        return
    oo, ol = oracle_prefill_fp8(cfg, tree, kc, vc, q, ks, vs)
    compare(out.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1),
            oo.reshape(-1, 128), ol.reshape(-1), "bf16", "fp8 prefill fuzz%d" % seed)


def test_fp8kv_prefill_c3_sampled_and_decode_on_one_context():
    """One context with E4M3 pools serves decode attention and step prefill of the same tree."""
    from workload import make_prefill_queries_host
    cfg = CONFIGS["c3_pruned"]
    tree = make_tree(cfg)
    kc, vc, q = make_values_fp8_host(cfg, tree, KS, VS)
    qs = make_prefill_queries_host(cfg, tree)
    kd, vd = pool_to_device(kc), pool_to_device(vc)
    with make_ctx(cfg) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        outp, lsep, _ = gpu_prefill(ctx, tree, kd, vd, to_device(qs))
        out, lse, _ = run(ctx, tree, kd, vd, to_device(q))
    r = np.random.default_rng(31)
    n = 96
    sl = r.integers(0, tree.n_leaves, size=n).astype(np.int32)
    lens = tree.n_tokens[tree.leaf_node[sl]]
    stok = (r.random(n) * lens).astype(np.int32)
    stok[:6] = 0
    stok[6:12] = lens[6:12] - 1
    sh = r.integers(0, cfg.n_q_heads, size=n).astype(np.int32)
    rows = oracle.prefill_q_ptr(tree.n_tokens, tree.leaf_node)[sl] + stok
    oo, ol = oracle_prefill_fp8(cfg, tree, kc, vc, qs, KS, VS, rows=(sl, stok, sh))
    compare(outp.cpu().numpy()[rows, sh], lsep.cpu().numpy()[rows, sh], oo, ol, "bf16",
            "fp8 prefill c3")
    do, dl = oracle_fp8(cfg, tree, kc, vc, q)
    compare(out.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1),
            do.reshape(-1, 128), dl.reshape(-1), "bf16", "fp8 decode c3")


def test_wide_random_sweep():
    """Two hundred random forests (1..160 nodes, 1..100 leaf queries, every group size, both
    head sizes, random planner knobs incl. the merge inside the attention launch, both pool
    formats; every third one of head_dim 128 also step prefill), every output row against
    the oracle.  Cheap on the GPU, and wide enough to hit layouts the
    hand-made cases miss (it found the entry-table padding and the append room check)."""
    from workload import make_prefill_queries_host
    shapes = [(2, 8), (1, 1), (2, 16), (4, 8), (1, 2), (8, 32), (3, 12), (2, 2), (1, 8), (4, 4)]
    for seed in range(5000, 5200):
        r = np.random.default_rng(seed)
        hkv, hq = shapes[seed % len(shapes)]
        d = 64 if (seed // 10) % 2 else 128
        cfg = TreeConfig("sweep", hkv, hq, d, "bf16", 0, 0, 0, 0, 0, None, seed=seed)
        tree = random_tree(seed, n_nodes=int(r.integers(2, 160)), n_leaves=int(r.integers(1, 100)),
                           max_tokens=int(r.choice([5, 20, 40, 90, 200, 500])),
                           p_root=float(r.choice([0.02, 0.1, 0.3])),
                           p_empty=float(r.choice([0.0, 0.15, 0.4])))
        options = {"stream_chunk": int(r.choice([0, 32, 64])),
                   "cascade_chunk": int(r.choice([0, 32, 96])),
                   "cascade_rows": int(r.choice([64, 16, 32])),
                   "wave_items": int(r.choice([512, 0, 48, 100000])),
                   "cascade_min_leaves": int(r.choice([2, 2, 0, 3])),
                   "wide_rows": int(r.choice([128, 16, 4, 40, 0])),
                   "interleave": int(r.choice([1, 1, 0])),
                   "fuse_merge": int(r.choice([0, 0, 1]))}
        mode = int(r.choice([ets.ETS_PLAN_TREE, ets.ETS_PLAN_TREE, ets.ETS_PLAN_FLAT]))
        print("case sweep", seed, (hkv, hq), tree.n_nodes, tree.n_leaves, options, mode, flush=True)
        k, v, q = make_values_host(cfg, tree)
        oo, ol = oracle_full(cfg, tree, k, v, q)
        with make_ctx(cfg, options) as ctx:
            out, lse, _ = run(ctx, tree, pool_to_device(k), pool_to_device(v), to_device(q), mode)
        compare(out.cpu().numpy().reshape(-1, d), lse.cpu().numpy().reshape(-1),
                oo.reshape(-1, d), ol.reshape(-1), "bf16", "sweep %d" % seed)
        ks, vs = float(r.choice([1.0, KS, 0.5])), float(r.choice([1.0, VS, 3.0]))
        kc, vc, q8 = make_values_fp8_host(cfg, tree, ks, vs)
        fo, fl = oracle_fp8(cfg, tree, kc, vc, q8, ks, vs)
        with make_ctx(cfg, options) as ctx:
            ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, ks, vs)
            out, lse, _ = run(ctx, tree, pool_to_device(kc), pool_to_device(vc), to_device(q8), mode)
        compare(out.cpu().numpy().reshape(-1, d), lse.cpu().numpy().reshape(-1),
                fo.reshape(-1, d), fl.reshape(-1), "bf16", "sweep e4m3 %d" % seed)
        if d == 128 and seed % 3 == 0 and 0 < int(tree.n_tokens[tree.leaf_node].sum()) < 3000:
            qs = make_prefill_queries_host(cfg, tree)
            with make_ctx(cfg) as ctx:
                po, pl, st = gpu_prefill(ctx, tree, pool_to_device(k), pool_to_device(v), to_device(qs))
            eo, el = oracle.tree_prefill_attn(tree.parent, tree.tok_offset, tree.n_tokens,
                                              tree.leaf_node, k, v, qs, hkv, hq, 128)
            compare(po.cpu().numpy().reshape(-1, 128), pl.cpu().numpy().reshape(-1),
                    eo.reshape(-1, 128), el.reshape(-1), "bf16", "sweep prefill %d" % seed)


def test_fp8kv_one_scale_per_kv_head():
    """ets_set_kv_head_scales: decode attention and step prefill with a scale of its own for
    every kv head and pool, against the oracle; a later ets_set_kv_format returns every
    head to the per-pool scales; bad arguments change nothing."""
    from workload import make_prefill_queries_host
    cfg = CONFIGS["c3_pruned"]
    tree = make_tree(cfg)
    r = np.random.default_rng(4)
    # (scales at most those the codes were made with: V stays of unit size, for which the
    # absolute bar is meant)
    ks = r.uniform(0.3 * KS, KS, size=cfg.n_kv_heads).astype(np.float32)
    vs = r.uniform(0.3 * VS, VS, size=cfg.n_kv_heads).astype(np.float32)
    kc, vc, q = make_values_fp8_host(cfg, tree, KS, VS)
    qs = make_prefill_queries_host(cfg, tree)
    kd, vd = pool_to_device(kc), pool_to_device(vc)
    with make_ctx(cfg) as ctx:
        with pytest.raises(ets.EtsError) as e:
            ctx.set_kv_head_scales(ks, vs)               # native pools have no scales
        assert e.value.status == 1
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        ctx.set_kv_head_scales(ks, vs)
        bad = ks.copy()
        bad[3] = 0.0
        with pytest.raises(ets.EtsError) as e:
            ctx.set_kv_head_scales(bad, vs)
        assert e.value.status == 1
        out, lse, _ = run(ctx, tree, kd, vd, to_device(q))
        outp, lsep, _ = gpu_prefill(ctx, tree, kd, vd, to_device(qs))
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, KS, VS)
        out1, lse1, _ = run(ctx, tree, kd, vd, to_device(q))
    oo, ol = oracle_fp8(cfg, tree, kc, vc, q, ks.astype(np.float64), vs.astype(np.float64))
    compare(out.cpu().numpy().reshape(-1, 128), lse.cpu().numpy().reshape(-1),
            oo.reshape(-1, 128), ol.reshape(-1), "bf16", "per-head scales decode")
    n = 80
    sl = r.integers(0, tree.n_leaves, size=n).astype(np.int32)
    stok = (r.random(n) * tree.n_tokens[tree.leaf_node[sl]]).astype(np.int32)
    sh = r.integers(0, cfg.n_q_heads, size=n).astype(np.int32)
    rows = oracle.prefill_q_ptr(tree.n_tokens, tree.leaf_node)[sl] + stok
    po, pl = oracle_prefill_fp8(cfg, tree, kc, vc, qs, ks.astype(np.float64),
                                vs.astype(np.float64), rows=(sl, stok, sh))
    compare(outp.cpu().numpy()[rows, sh], lsep.cpu().numpy()[rows, sh], po, pl, "bf16",
            "per-head scales prefill")
    o1, l1 = oracle_fp8(cfg, tree, kc, vc, q)
    compare(out1.cpu().numpy().reshape(-1, 128), lse1.cpu().numpy().reshape(-1),
            o1.reshape(-1, 128), l1.reshape(-1), "bf16", "back to per-pool scales")
