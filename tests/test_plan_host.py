"""Host logic of libetsattn, no GPU needed: the library loads and exports what
the header declares; the planner's indexing equals the oracle's walk bit for
bit; the work items tile every leaf's chain exactly once; every error path
reports its status code."""
import ctypes as C
import os
import re

import numpy as np
import pytest

import oracle
import paper_2502_13575_amd as ets
from workload import CONFIGS, make_tree, random_tree

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))


def _ctx(cfg_or_shape, device=-1):
    if isinstance(cfg_or_shape, tuple):
        hkv, hq, d, dt = cfg_or_shape
    else:
        c = cfg_or_shape
        hkv, hq, d = c.n_kv_heads, c.n_q_heads, c.head_dim
        dt = ets.ETS_F32 if c.dtype == "f32" else ets.ETS_BF16
    return ets.Context(hkv, hq, d, dt, device)


def _chain_rows(t, optr, onodes, l):
    nodes = onodes[optr[l]:optr[l + 1]]
    if len(nodes) == 0:
        return np.zeros(0, dtype=np.int64)
    return np.concatenate([np.arange(t.tok_offset[n], t.tok_offset[n] + t.n_tokens[n])
                           for n in nodes]).astype(np.int64)


def _check_plan_against_oracle(ctx, t, mode, leaves=None, esz=None):
    st = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, mode)
    ost = oracle.tree_stats(t.parent, t.n_tokens, t.leaf_node)
    assert st.unique_tokens == ost["unique_tokens"]
    assert st.flat_tokens == ost["flat_tokens"]
    assert st.live_nodes == ost["live_nodes"]
    assert np.array_equal(ctx.leaf_counts(), ost["leaf_count"])
    optr, onodes = oracle.paths(t.parent, t.leaf_node)
    ptr, nodes = ctx.paths()
    assert np.array_equal(ptr, optr) and np.array_equal(nodes, onodes)
    total_partials = 0
    for l in (range(t.n_leaves) if leaves is None else leaves):
        rows, npart = ctx.leaf_cover(l)
        want = _chain_rows(t, optr, onodes, l)
        assert np.array_equal(np.sort(rows), np.sort(want)), (mode, l)
        total_partials += npart
    if leaves is None:
        assert total_partials == st.n_partials
    esz = esz or (4 if ctx.shape.dtype == ets.ETS_F32 else 2)
    assert st.unique_kv_bytes == st.unique_tokens * 2 * ctx.shape.n_kv_heads * ctx.shape.head_dim * esz
    assert st.workspace_bytes == st.n_partials * ctx.shape.n_q_heads * (ctx.shape.head_dim + 2) * 4
    return st


def test_library_exports_every_declared_symbol():
    hdr = open(os.path.join(ROOT, "include", "etsattn.h")).read()
    hdr = re.sub(r"/\*.*?\*/", "", hdr, flags=re.S)
    names = sorted(set(re.findall(r"\b(ets_[a-z_]+)\s*\(", hdr)))
    assert "ets_tree_decode_attn" in names and "ets_plan" in names and len(names) >= 10
    lib = C.CDLL(ets.library_path())
    for n in names:
        assert hasattr(lib, n), "missing export: " + n


@pytest.mark.parametrize("name", list(CONFIGS))
@pytest.mark.parametrize("mode", [ets.ETS_PLAN_TREE, ets.ETS_PLAN_FLAT])
def test_plan_indexing_matches_oracle_on_configs(name, mode):
    cfg = CONFIGS[name]
    t = make_tree(cfg)
    with _ctx(cfg) as ctx:
        ctx.set_option("cascade_min_leaves", 2)
        leaves = None if t.n_leaves <= 64 else list(range(0, t.n_leaves, t.n_leaves // 32))
        st = _check_plan_against_oracle(ctx, t, mode, leaves)
        if mode == ets.ETS_PLAN_FLAT:
            assert st.cascade_tokens == 0           # nothing is shared in the flat baseline
            assert st.stream_tokens == st.flat_tokens
        elif cfg.dtype == "bf16":
            assert st.cascade_tokens > 0
        else:
            assert st.n_cascade_items == 0          # fp32 pools take the streaming kernel


def test_c1_closed_form_counts():
    cfg = CONFIGS["c1_tiny"]
    t = make_tree(cfg)
    with _ctx(cfg) as ctx:
        st = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        assert (st.n_nodes, st.live_nodes, st.n_leaves) == (15, 15, 8)
        assert (st.unique_tokens, st.flat_tokens) == (256, 640)
        assert st.n_segments == 15 and st.min_pool_tokens == 256


@pytest.mark.parametrize("seed", range(12))
def test_plan_fuzz_irregular_forests(seed):
    t = random_tree(seed, n_nodes=60, n_leaves=25, max_tokens=70)
    shapes = [(2, 8, 128, ets.ETS_BF16), (1, 8, 64, ets.ETS_BF16), (2, 2, 64, ets.ETS_F32)]
    with _ctx(shapes[seed % 3]) as ctx:
        ctx.set_option("cascade_min_leaves", 2)
        ctx.set_option("stream_chunk", [0, 32, 64][seed % 3])
        ctx.set_option("cascade_chunk", [0, 32, 96][(seed // 3) % 3])
        ctx.set_option("mfma", 0 if seed % 4 == 3 else 1)
        for mode in (ets.ETS_PLAN_TREE, ets.ETS_PLAN_FLAT):
            _check_plan_against_oracle(ctx, t, mode)


def test_chain_compaction_merges_single_child_chains():
    # root(4) - a(3) - b(5) with two leaves under b: one segment for root,a,b + 2 leaf segments
    parent = np.array([-1, 0, 1, 2, 2], np.int32)
    n_tok = np.array([4, 3, 5, 2, 6], np.int32)
    off = np.array([0, 4, 7, 12, 14], np.int64)
    with _ctx((1, 4, 128, ets.ETS_BF16)) as ctx:
        st = ctx.plan(parent, off, n_tok, np.array([3, 4], np.int32))
        assert st.n_segments == 3 and st.live_nodes == 5
        assert st.unique_tokens == 20 and st.flat_tokens == 12 * 2 + 8


def test_empty_tree_and_empty_chains():
    with _ctx((1, 1, 64, ets.ETS_F32)) as ctx:
        z32, z64 = np.zeros(0, np.int32), np.zeros(0, np.int64)
        st = ctx.plan(z32, z64, z32, z32)
        assert st.n_leaves == 0 and st.n_partials == 0 and st.workspace_bytes == 0
        st = ctx.plan(np.array([-1], np.int32), np.array([0], np.int64), np.array([0], np.int32),
                      np.array([0, 0], np.int32))
        assert st.n_leaves == 2 and st.n_partials == 0 and st.unique_tokens == 0
        rows, npart = ctx.leaf_cover(1)
        assert rows.size == 0 and npart == 0


def _status(fn):
    with pytest.raises(ets.EtsError) as e:
        fn()
    return e.value.status


def test_error_paths():
    assert _status(lambda: ets.Context(8, 32, 96, ets.ETS_BF16, -1)) == 4      # head_dim
    assert _status(lambda: ets.Context(8, 30, 128, ets.ETS_BF16, -1)) == 4     # Hq % Hkv
    assert _status(lambda: ets.Context(2, 32, 128, ets.ETS_BF16, -1)) == 4     # G = 16
    assert _status(lambda: ets.Context(8, 32, 128, 7, -1)) == 4                # dtype
    t = make_tree(CONFIGS["c1_tiny"])
    with _ctx(CONFIGS["c1_tiny"]) as ctx:
        assert _status(ctx.stats) == 6                                          # no plan yet
        bad = t.parent.copy(); bad[4] = 4
        assert _status(lambda: ctx.plan(bad, t.tok_offset, t.n_tokens, t.leaf_node)) == 2
        bad = t.parent.copy(); bad[2] = 9
        assert _status(lambda: ctx.plan(bad, t.tok_offset, t.n_tokens, t.leaf_node)) == 2
        bad = t.parent.copy(); bad[0] = -2
        assert _status(lambda: ctx.plan(bad, t.tok_offset, t.n_tokens, t.leaf_node)) == 2
        nt = t.n_tokens.copy(); nt[3] = -1
        assert _status(lambda: ctx.plan(t.parent, t.tok_offset, nt, t.leaf_node)) == 2
        lf = t.leaf_node.copy(); lf[1] = 15
        assert _status(lambda: ctx.plan(t.parent, t.tok_offset, t.n_tokens, lf)) == 3
        assert _status(ctx.stats) == 6                                          # failed plan dropped
        assert _status(lambda: ctx.set_option("no_such_knob", 1)) == 1
        assert _status(lambda: ctx.set_option("stream_chunk", -5)) == 1
        ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        assert _status(lambda: ctx.leaf_cover(8)) == 3
        # a host-only context cannot launch
        assert _status(lambda: ctx.decode(16, 16, 256, 16, 16, 16, 16, 1 << 20)) == 7
    lib = ets.load_library()
    assert lib.ets_create(None, None, -1) == 1
    assert lib.ets_plan(None, None, 0) == 1
    assert lib.ets_plan_stats(None, None) == 1
    assert lib.ets_tree_decode_attn(None, None, None, 0, None, None, None, None, 0, None) == 1
    lib.ets_destroy(None)
    assert ets.ets_strerror(0) == "ok" and "tree" in ets.ets_strerror(2)


def test_sharing_reduces_partials_and_flat_is_per_leaf():
    cfg = CONFIGS["c3_pruned"]
    t = make_tree(cfg)
    with _ctx(cfg) as ctx:
        ctx.set_option("cascade_min_leaves", 2)
        tree = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, ets.ETS_PLAN_TREE).as_dict()
        flat = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, ets.ETS_PLAN_FLAT).as_dict()
    assert tree["unique_tokens"] == flat["unique_tokens"]
    assert flat["cascade_tokens"] == 0
    assert flat["n_cascade_items"] + flat["n_stream_items"] >= t.n_leaves
    assert tree["cascade_tokens"] > 0 and tree["n_partials"] > flat["n_partials"]


def test_long_chain_of_one_token_nodes_is_cut_into_bounded_step_lists():
    # 1500 single-token nodes scattered in the pool: every node is its own step,
    # more than one work item can list
    n = 1500
    parent = np.arange(-1, n - 1, dtype=np.int32)
    n_tok = np.ones(n, np.int32)
    off = (np.arange(n, dtype=np.int64) * 7919) % n            # a permutation of the rows
    leaf = np.array([n - 1, n - 1, 700], np.int32)
    with _ctx((2, 8, 128, ets.ETS_BF16)) as ctx:
        st = ctx.plan(parent, off, n_tok, leaf)
        assert st.n_partials >= 3 + 2                          # the chain had to be chunked
        for l in range(3):
            rows, _ = ctx.leaf_cover(l)
            want = off[:leaf[l] + 1]
            assert np.array_equal(np.sort(rows), np.sort(want))


# ------------------------------------------------------- decode-step advance
def _check_cover(ctx, t, n_tokens):
    grown = type(t)(t.parent, t.tok_offset, n_tokens, t.leaf_node, t.pool_tokens)
    st = ctx.stats()
    ost = oracle.tree_stats(grown.parent, grown.n_tokens, grown.leaf_node)
    assert st.unique_tokens == ost["unique_tokens"] and st.flat_tokens == ost["flat_tokens"]
    holds = (ost["leaf_count"] > 0) & (grown.n_tokens > 0)       # live nodes that own rows
    assert st.min_pool_tokens == max(int((grown.tok_offset + grown.n_tokens)[holds].max(initial=0)), 0)
    optr, onodes = oracle.paths(grown.parent, grown.leaf_node)
    total = 0
    for l in range(grown.n_leaves):
        rows, npart = ctx.leaf_cover(l)
        assert np.array_equal(np.sort(rows), np.sort(_chain_rows(grown, optr, onodes, l))), l
        total += npart
    assert total == st.n_partials


@pytest.mark.parametrize("name,opts", [("c2_w16", {}), ("c2_w16", {"mfma": 0}),
                                       ("c1_tiny", {}), ("c3_pruned", {"cascade_min_leaves": 0})])
def test_plan_advance_tracks_oracle_walk(name, opts):
    """Every advance makes every distinct leaf node one token longer: rows read per leaf
    and the statistics equal the oracle's walk of the grown tree, through in-place
    advances and through the re-plan that follows when the step lists are full."""
    from workload import with_growth_room
    cfg = CONFIGS[name]
    t = with_growth_room(make_tree(cfg), 80)
    with _ctx(cfg) as ctx:
        for k, v in opts.items():
            ctx.set_option(k, v)
        ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        n_tokens = t.n_tokens.copy()
        replans = 0
        for step in range(75):
            replans += int(ctx.plan_advance())
            n_tokens[np.unique(t.leaf_node)] += 1
            if step % 6 == 0 or step > 70:
                _check_cover(ctx, t, n_tokens)
        limited = cfg.dtype == "bf16" and cfg.head_dim == 128 and opts.get("mfma", 1) != 0
        assert (replans >= 1) if limited else (replans == 0)
        assert replans <= 3


def test_plan_advance_fuzz_and_duplicates():
    from workload import with_growth_room
    for seed in range(6):
        t = with_growth_room(random_tree(100 + seed, 40, 12, 70), 40)
        with _ctx((2, 8, 128, ets.ETS_BF16)) as ctx:
            ctx.set_option("stream_chunk", [0, 32, 64][seed % 3])
            ctx.set_option("wave_items", [512, 0][seed % 2])
            ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
            n_tokens = t.n_tokens.copy()
            for step in range(36):
                ctx.plan_advance()
                n_tokens[np.unique(t.leaf_node)] += 1
                if step % 5 == 0 or step >= 33:
                    _check_cover(ctx, t, n_tokens)


_CHECK_SHAPES = [(2, 8, 128, ets.ETS_BF16), (4, 4, 128, ets.ETS_BF16), (2, 4, 128, ets.ETS_BF16),
                 (1, 1, 128, ets.ETS_BF16), (2, 16, 128, ets.ETS_BF16), (1, 8, 64, ets.ETS_BF16),
                 (2, 2, 64, ets.ETS_F32)]


def test_plan_check_replays_kernel_accesses_on_configs():
    """ets_plan_check walks the tables the kernels read: on every configuration every step
    stays inside the pool, every partial row inside the workspace, and no wavefront loads
    an entry further than 15 past its item's last one (one 16-entry scalar load), which the
    tables' padding covers."""
    for name, cfg in CONFIGS.items():
        t = make_tree(cfg)
        with _ctx(cfg) as ctx:
            st = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
            if cfg.dtype == "bf16" and cfg.head_dim == 128:
                ctx.plan_prefill(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
            rep = ctx.check()
            assert rep.violations == 0, name
            assert rep.decode_items == st.n_cascade_items + st.n_stream_items + st.n_wide_items
            assert rep.max_pool_row == st.min_pool_tokens - 1
            assert rep.max_partial_row == st.n_partials * cfg.n_q_heads - 1
            assert rep.max_entry_overreach <= 15
            assert rep.max_entry_index < rep.entry_table_entries
            assert rep.entry_table_entries >= t.n_leaves + 16


def test_merge_inside_the_attention_launch_only_when_every_partial_arrives_there():
    """"fuse_merge" = 1: the plan says so (merge_fused) only when the matrix-core kernel writes
    every partial result (bf16, head_dim 128, no wide items) and every leaf query has one;
    in every other case the merge launch stays.  The default is the merge launch."""
    cfg = CONFIGS["c3_div"]
    t = make_tree(cfg)
    for opts, want in (({}, 0), ({"fuse_merge": 1}, 1), ({"fuse_merge": 1, "wide_rows": 16}, 0),
                       ({"fuse_merge": 1, "mfma": 0}, 0), ({"fuse_merge": 0}, 0),
                       ({"fuse_merge": 1, "cascade_min_leaves": 0}, 1)):
        with _ctx(cfg) as ctx:
            for k, v in opts.items():
                ctx.set_option(k, v)
            for mode in (0, 1):
                st = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, mode)
                # (a flat plan has no shared segments, hence no wide items)
                assert st.merge_fused == (want if mode == 0 or "wide_rows" not in opts else 1), (opts, mode)
                assert ctx.check().violations == 0
    # a leaf query without a token gets its result from the merge launch
    parent = np.array([-1, 0, -1], dtype=np.int32)
    n_tokens = np.array([9, 3, 0], dtype=np.int32)
    tok_offset = np.array([0, 9, 12], dtype=np.int64)
    with _ctx(cfg) as ctx:
        ctx.set_option("fuse_merge", 1)
        st = ctx.plan(parent, tok_offset, n_tokens, np.array([1, 1, 0], dtype=np.int32))
        assert st.merge_fused == 1
        st = ctx.plan(parent, tok_offset, n_tokens, np.array([1, 2, 0], dtype=np.int32))
        assert st.merge_fused == 0 and ctx.check().violations == 0
    # head_dim 64 is served by the matrix-core kernel as well, fp32 pools are not
    with _ctx((2, 4, 64, ets.ETS_BF16)) as ctx:
        ctx.set_option("fuse_merge", 1)
        assert ctx.plan(parent, tok_offset, n_tokens, np.array([1, 0], dtype=np.int32)).merge_fused == 1
    with _ctx((2, 4, 64, ets.ETS_F32)) as ctx:
        ctx.set_option("fuse_merge", 1)
        assert ctx.plan(parent, tok_offset, n_tokens, np.array([1, 0], dtype=np.int32)).merge_fused == 0
    # the 8-heads-per-kv-head configurations plan no wide items unless asked to
    t4 = make_tree(CONFIGS["c4_34b"])
    with _ctx(CONFIGS["c4_34b"]) as ctx:
        assert ctx.plan(t4.parent, t4.tok_offset, t4.n_tokens, t4.leaf_node).n_wide_items == 0
        ctx.set_option("wide_rows", 64)
        assert ctx.plan(t4.parent, t4.tok_offset, t4.n_tokens, t4.leaf_node).n_wide_items > 0


def test_plan_check_sweep_of_random_forests():
    """The sweep that once found a wavefront reading entries of the next table (one query
    head per kv head, row blocks past an item's last row): 3000 random forests over the
    head geometries, planner knobs, both plan modes, decode-step advances and the prefill
    plan; every replay stays in bounds with at most 15 entries of overreach."""
    from workload import with_growth_room
    worst = 0
    for seed in range(20000, 23000):
        r = np.random.default_rng(seed)
        t = random_tree(seed, n_nodes=int(r.integers(1, 140)), n_leaves=int(r.integers(1, 90)),
                        max_tokens=int(r.choice([1, 5, 33, 70, 300, 2000])),
                        p_root=float(r.choice([0.02, 0.1, 0.5])),
                        p_empty=float(r.choice([0.0, 0.15, 0.6])))
        shape = _CHECK_SHAPES[seed % len(_CHECK_SHAPES)]
        opts = {"stream_chunk": int(r.choice([0, 32, 64, 1000])),
                "cascade_chunk": int(r.choice([0, 32, 96, 1000])),
                "cascade_rows": int(r.choice([64, 16, 32])),
                "wave_items": int(r.choice([512, 0, 48, 100000])),
                "cascade_min_leaves": int(r.choice([2, 0, 3, 9])),
                "mfma": int(r.choice([1, 1, 0])),
                "wide_rows": int(r.choice([128, 0, 16, 40, 300])),
                "fuse_merge": int(r.choice([0, 1, 1])),
                "interleave": int(r.choice([1, 0]))}
        mode = int(r.choice([0, 0, 1]))
        if seed % 3 == 0:
            t = with_growth_room(t, 40)
        with _ctx(shape) as ctx:
            for k, v in opts.items():
                ctx.set_option(k, v)
            ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, mode)
            if seed % 4 == 0 and shape[2] == 128 and shape[3] == ets.ETS_BF16:
                ctx.plan_prefill(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
            rep = ctx.check()
            assert rep.violations == 0 and rep.max_entry_overreach <= 15, (seed, rep.as_dict())
            worst = max(worst, rep.max_entry_overreach)
            if seed % 3 == 0:
                for step in range(int(r.choice([1, 34]))):
                    ctx.plan_advance()
                rep = ctx.check()
                assert rep.violations == 0 and rep.max_entry_overreach <= 15, (seed, rep.as_dict())
    assert worst == 15  # the sweep does reach the furthest load the kernel makes


def test_shapes_without_node_sharing_say_so_or_refuse():
    """Shared nodes are read once for bf16 pools (head_dim 128 or 64).  fp32 pools fall back
    to per-leaf reads and report it (shares_nodes 0, nothing on the shared-node kernel);
    with "require_sharing" the tree-mode plan is refused instead."""
    t = make_tree(CONFIGS["c2_w16"])
    for shape, shares in [((8, 32, 128, ets.ETS_BF16), 1), ((8, 32, 64, ets.ETS_BF16), 1),
                          ((8, 32, 128, ets.ETS_F32), 0), ((1, 2, 64, ets.ETS_F32), 0)]:
        with _ctx(shape) as ctx:
            st = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
            assert st.shares_nodes == shares
            assert (st.cascade_tokens > 0) == bool(shares)
            if not shares:
                assert st.stream_tokens == st.flat_tokens
            assert ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node,
                            ets.ETS_PLAN_FLAT).shares_nodes == 0
            ctx.set_option("require_sharing", 1)
            if shares:
                assert ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node).shares_nodes == 1
            else:
                with pytest.raises(ets.EtsError) as e:
                    ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
                assert e.value.status == 4  # ETS_ERR_UNSUPPORTED
            # the flat baseline is a per-leaf plan by definition and stays available
            ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, ets.ETS_PLAN_FLAT)
    with _ctx((8, 32, 128, ets.ETS_BF16)) as ctx:
        ctx.set_option("require_sharing", 1)
        ctx.set_option("mfma", 0)
        with pytest.raises(ets.EtsError) as e:
            ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        assert e.value.status == 4


def test_append_rows_follow_the_grown_tree_whatever_the_layer_count():
    """ets_kv_append writes the newest row of every distinct leaf node as the plan counts it:
    after a advances that is row tok_offset + n_tokens0 + a - 1, the row the oracle's
    append_kv (the definition) fills on its a-th call -- through the in-place advances and
    through the re-plan, for the first leaf query of every node only."""
    import oracle
    from workload import with_growth_room
    for seed in range(4):
        t = with_growth_room(random_tree(300 + seed, 30, 10, 40), 45)
        first = {}
        for l, n in enumerate(t.leaf_node.tolist()):
            first.setdefault(n, l)
        with _ctx((2, 8, 128, ets.ETS_BF16)) as ctx:
            ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
            # a plan that was just built: the last row the tree names (none for an empty node)
            rows = ctx.append_rows()
            for l, n in enumerate(t.leaf_node.tolist()):
                want = t.tok_offset[n] + t.n_tokens[n] - 1 if first[n] == l and t.n_tokens[n] > 0 else -1
                assert rows[l] == want, (seed, l)
            # the oracle's append marks, in a pool of zeros, the row every call fills
            n_tokens = t.n_tokens.copy()
            pool = np.zeros((t.pool_tokens + 64, 1, 1), dtype=np.int64)
            for a in range(1, 41):
                ctx.plan_advance()
                marks = np.arange(1, t.n_leaves + 1, dtype=np.int64).reshape(-1, 1, 1) + 1000 * a
                n_tokens = oracle.append_kv(t.tok_offset, n_tokens, t.leaf_node, pool, pool.copy(),
                                            marks, marks)
                rows = ctx.append_rows()
                assert np.array_equal(rows, ctx.append_rows())  # asking twice changes nothing
                for l, n in enumerate(t.leaf_node.tolist()):
                    if first[n] == l:
                        assert pool[rows[l], 0, 0] == 1000 * a + l + 1, (seed, a, l)
                    else:
                        assert rows[l] == -1


def test_advance_and_append_error_paths():
    with _ctx((2, 8, 128, ets.ETS_BF16)) as ctx:
        with pytest.raises(ets.EtsError) as e:
            ctx.plan_advance()
        assert e.value.status == 6  # ETS_ERR_NO_PLAN
        with pytest.raises(ets.EtsError) as e:
            ctx.kv_append(None, None, 0, None, None)
        assert e.value.status == 6


def test_kv_format_host_logic():
    """E4M3 pools: accepted only where the matrix-core kernel runs, the plans are dropped,
    byte statistics follow the 1-byte elements (of the prefill plan too), the indexing does
    not change."""
    cfg = CONFIGS["c3_pruned"]
    t = make_tree(cfg)
    with _ctx(cfg) as ctx:
        st2 = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        for bad in [(ets.ETS_KV_FP8_E4M3, 0.0, 1.0), (ets.ETS_KV_FP8_E4M3, 1.0, -2.0),
                    (ets.ETS_KV_FP8_E4M3, float("inf"), 1.0), (ets.ETS_KV_FP8_E4M3, float("nan"), 1.0),
                    (7, 1.0, 1.0)]:
            with pytest.raises(ets.EtsError) as e:
                ctx.set_kv_format(*bad)
            assert e.value.status == 1
        assert ctx.stats().unique_kv_bytes == st2.unique_kv_bytes      # nothing changed so far
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, 0.02, 0.03)
        with pytest.raises(ets.EtsError) as e:
            ctx.stats()
        assert e.value.status == 6                                     # plan dropped
        pf1 = ctx.plan_prefill(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        st1 = _check_plan_against_oracle(ctx, t, ets.ETS_PLAN_TREE,
                                         list(range(0, t.n_leaves, 4)), esz=1)
        assert st1.unique_tokens == st2.unique_tokens
        assert 2 * st1.unique_kv_bytes == st2.unique_kv_bytes
        assert 2 * st1.flat_kv_bytes == st2.flat_kv_bytes
        assert st1.unique_kv_bytes == st1.unique_tokens * 2 * cfg.n_kv_heads * cfg.head_dim
        ctx.set_kv_format(ets.ETS_KV_NATIVE)
        st3 = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        assert st3.unique_kv_bytes == st2.unique_kv_bytes
        pf2 = ctx.plan_prefill(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        assert 2 * pf1.unique_kv_bytes == pf2.unique_kv_bytes
        assert 2 * pf1.streamed_kv_bytes == pf2.streamed_kv_bytes
        assert (pf1.n_items, pf1.n_runs, pf1.flops) == (pf2.n_items, pf2.n_runs, pf2.flops)
    for shape in [(2, 4, 64, ets.ETS_F32), (2, 4, 128, ets.ETS_F32)]:
        with _ctx(shape) as ctx:
            with pytest.raises(ets.EtsError) as e:
                ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, 1.0, 1.0)
            assert e.value.status == 4
            ctx.set_kv_format(ets.ETS_KV_NATIVE)
            ctx.set_option("out_bf16", 1)
    # bf16 contexts of either head size take pools of codes (step prefill: head_dim 128 only)
    with _ctx((2, 4, 64, ets.ETS_BF16)) as ctx:
        ctx.set_kv_format(ets.ETS_KV_FP8_E4M3, 1.0, 1.0)
        st64 = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        assert st64.unique_kv_bytes == st64.unique_tokens * 2 * 2 * 64 and st64.shares_nodes == 1
        with pytest.raises(ets.EtsError) as e:
            ctx.plan_prefill(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
        assert e.value.status == 4
