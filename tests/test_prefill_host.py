"""Host logic of step prefill, no GPU needed: query-row numbering, the rows every query
token sees according to the work items and their masks, and the statistics equal the
oracle's walk bit for bit; error paths report their status codes."""
import numpy as np
import pytest

import oracle
import paper_2502_13575_amd as ets
from workload import CONFIGS, Tree, make_tree, random_tree


def _ctx(hkv, hq, d=128, dt=ets.ETS_BF16):
    return ets.Context(hkv, hq, d, dt, -1)


def _check(ctx, t, tokens=None):
    st = ctx.plan_prefill(t.parent, t.tok_offset, t.n_tokens, t.leaf_node)
    q_ptr = ctx.prefill_q_ptr()
    assert np.array_equal(q_ptr, oracle.prefill_q_ptr(t.n_tokens, t.leaf_node))
    assert st.n_q_rows == q_ptr[-1] and st.n_leaves == t.n_leaves
    pairs = 0
    for l in range(t.n_leaves):
        v = int(t.leaf_node[l])
        n = int(t.n_tokens[v])
        for i in (range(n) if tokens is None else [x for x in tokens if x < n]):
            got = ctx.prefill_cover(l, i)
            want = oracle.visible_rows(t.parent, t.tok_offset, t.n_tokens, v, i + 1)
            assert np.array_equal(got, want), (l, i)
            pairs += len(want)
    if tokens is None:
        assert pairs == st.visible_pairs
        assert st.flops == 4 * ctx.shape.head_dim * ctx.shape.n_q_heads * pairs
    return st


@pytest.mark.parametrize("seed", range(8))
def test_prefill_plan_fuzz_matches_oracle_walk(seed):
    t = random_tree(300 + seed, n_nodes=40, n_leaves=11, max_tokens=[5, 40, 140][seed % 3],
                    p_empty=0.15)
    hkv, hq = [(2, 8), (1, 1), (2, 16), (4, 8)][seed % 4]
    with _ctx(hkv, hq) as ctx:
        st = _check(ctx, t)
        # a block holds rows_per_item / G query tokens
        G = hq // hkv
        lens = t.n_tokens[t.leaf_node]
        assert st.rows_per_item % 64 == 0
        assert st.n_items == int(sum(-(-int(n) // (st.rows_per_item // G)) for n in lens))


@pytest.mark.parametrize("name", ["c2_w16", "c3_pruned", "c4_34b"])
def test_prefill_plan_on_configs(name):
    cfg = CONFIGS[name]
    t = make_tree(cfg)
    with _ctx(cfg.n_kv_heads, cfg.n_q_heads) as ctx:
        st = _check(ctx, t, tokens=[0, 1, 31, 32, 33, 63, 64, 100, 127, 128, 200])
        ost = oracle.tree_stats(t.parent, t.n_tokens, t.leaf_node)
        # every live node lies on a leaf query's chain
        assert st.unique_tokens == ost["unique_tokens"]
        assert st.unique_kv_bytes == st.unique_tokens * 2 * cfg.n_kv_heads * 128 * 2


def test_prefill_closed_form_counts():
    # root of 40 rows, two children of 70 and 5 rows, leaf queries on both children and
    # on the root itself
    t = Tree(np.array([-1, 0, 0], np.int32), np.array([0, 40, 110], np.int64),
             np.array([40, 70, 5], np.int32), np.array([1, 2, 0], np.int32), 115)
    with _ctx(2, 8) as ctx:
        st = _check(ctx, t)
        tq = st.rows_per_item // 4
        assert st.n_q_rows == 115 and st.n_items == -(-70 // tq) + 1 + -(-40 // tq)
        # pairs: child 1: 70 * 40 + 70 * 71 / 2; child 2: 5 * 40 + 15; root: 40 * 41 / 2
        assert st.visible_pairs == 70 * 40 + 70 * 71 // 2 + 5 * 40 + 15 + 40 * 41 // 2
        assert st.unique_tokens == 115 and st.min_pool_tokens == 115


def test_prefill_long_paths_and_scattered_one_token_nodes():
    # more than 256 runs per work item (the kernel's descriptor ring is refilled)
    n = 700
    parent = np.arange(-1, n - 1, dtype=np.int32)
    n_tok = np.ones(n, np.int32)
    n_tok[-1] = 37
    off = (np.arange(n, dtype=np.int64) * 7919) % n * 40   # scattered: nothing merges
    t = Tree(parent, off, n_tok, np.array([n - 1, 350], np.int32), int(off.max()) + 40)
    with _ctx(1, 8) as ctx:
        st = _check(ctx, t)
        assert st.n_runs >= 699 + 2 + 350 + 1


def test_prefill_empty_cases_and_errors():
    z32, z64 = np.zeros(0, np.int32), np.zeros(0, np.int64)
    with _ctx(2, 8) as ctx:
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill_stats()
        assert e.value.status == 6                               # no plan yet
        st = ctx.plan_prefill(z32, z64, z32, z32)
        assert st.n_q_rows == 0 and st.n_items == 0
        # leaf queries on empty nodes own no rows
        st = ctx.plan_prefill(np.array([-1, 0], np.int32), np.array([0, 4], np.int64),
                              np.array([4, 0], np.int32), np.array([1, 1], np.int32))
        assert st.n_q_rows == 0 and st.n_items == 0
        assert ctx.prefill_q_ptr().tolist() == [0, 0, 0]
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill_cover(0, 0)
        assert e.value.status == 1                               # token outside the node
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill_cover(2, 0)
        assert e.value.status == 3                               # leaf out of range
        with pytest.raises(ets.EtsError) as e:
            ctx.plan_prefill(np.array([0], np.int32), np.array([0], np.int64),
                             np.array([1], np.int32), np.array([0], np.int32))
        assert e.value.status == 2                               # parent >= own index
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill_stats()
        assert e.value.status == 6                               # failed plan leaves none
        with pytest.raises(ets.EtsError) as e:
            ctx.plan_prefill(np.array([-1], np.int32), np.array([0], np.int64),
                             np.array([1], np.int32), np.array([1], np.int32))
        assert e.value.status == 3
        ctx.plan_prefill(np.array([-1], np.int32), np.array([0], np.int64),
                         np.array([3], np.int32), np.array([0], np.int32))
        with pytest.raises(ets.EtsError) as e:
            ctx.prefill(None, None, 3, None, None, None)
        assert e.value.status == 7                               # host-only context
    for shape in [(2, 8, 64, ets.ETS_BF16), (2, 8, 128, ets.ETS_F32)]:
        with ets.Context(*shape, -1) as ctx:
            with pytest.raises(ets.EtsError) as e:
                ctx.plan_prefill(np.array([-1], np.int32), np.array([0], np.int64),
                                 np.array([3], np.int32), np.array([0], np.int32))
            assert e.value.status == 4                           # built for bf16, head_dim 128


def test_prefill_and_decode_plans_do_not_disturb_each_other():
    cfg = CONFIGS["c2_w16"]
    t = make_tree(cfg)
    with _ctx(cfg.n_kv_heads, cfg.n_q_heads) as ctx:
        s1 = ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node).as_dict()
        ctx.plan_prefill(t.parent[:3], t.tok_offset[:3], t.n_tokens[:3], np.array([2], np.int32))
        assert ctx.stats().as_dict() == s1
        p1 = ctx.prefill_stats().as_dict()
        ctx.plan(t.parent, t.tok_offset, t.n_tokens, t.leaf_node, ets.ETS_PLAN_FLAT)
        assert ctx.prefill_stats().as_dict() == p1
