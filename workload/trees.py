"""Seeded generators for search-tree topologies and K/V/Q values.

Topology recipe (stands in for a PRM-guided parallel tree search of width W):
node 0 is the shared prompt; search step 1 creates W children of the prompt;
at every later step a weight vector p ~ Dirichlet(alpha * 1_W) over the W nodes
of the previous step is drawn and the W new nodes pick their parents i.i.d.
from Categorical(p).  Small alpha concentrates the continuations on few parents
(heavy KV sharing, like a search that prunes for sharing), large alpha spreads
them (divergent trajectories).  The leaves are the W nodes of the last step;
nodes without a leaf beneath them are dead but stay in the parent array.

Step lengths, topology and values come from three independent Philox streams of
one seed, so two variants that differ only in alpha have identical node lengths.
"""
from __future__ import annotations

from dataclasses import dataclass, field
from typing import Optional

import numpy as np


# --------------------------------------------------------------------------
# configurations
# --------------------------------------------------------------------------
@dataclass(frozen=True)
class TreeConfig:
    name: str
    n_kv_heads: int
    n_q_heads: int
    head_dim: int
    dtype: str                  # "f32" | "bf16"
    prompt: int                 # tokens in the shared root
    steps: int                  # search steps below the root
    step_lo: int                # step length drawn uniformly in [lo, hi] per node
    step_hi: int
    width: int                  # leaves kept per step
    alpha: Optional[float]      # Dirichlet concentration; None => complete b-ary tree
    branch: int = 2             # used when alpha is None
    layers: int = 1
    store_dead: bool = True     # dead nodes own pool rows (False: they alias row 0)
    seed: int = 0
    trees: int = 1              # independent searches (problems) batched into one forest

    @property
    def group(self) -> int:
        return self.n_q_heads // self.n_kv_heads

    @property
    def elem_bytes(self) -> int:
        return 4 if self.dtype == "f32" else 2


CONFIGS = {
    # tiny fp32 tree: 1 + 2 + 4 + 8 nodes, 8 leaves, path = 32 + 3*16 = 80 tokens
    "c1_tiny": TreeConfig("c1_tiny", 1, 2, 64, "f32", 32, 3, 16, 16, 8, None, 2,
                          seed=1001),
    "c2_w16": TreeConfig("c2_w16", 8, 32, 128, "bf16", 512, 8, 64, 64, 16, 0.5,
                         seed=1002),
    "c3_div": TreeConfig("c3_div", 8, 32, 128, "bf16", 1024, 16, 128, 128, 64, 5.0,
                         seed=1003),
    "c3_pruned": TreeConfig("c3_pruned", 8, 32, 128, "bf16", 1024, 16, 128, 128, 64,
                            0.2, seed=1003),
    "c4_34b": TreeConfig("c4_34b", 8, 64, 128, "bf16", 2048, 24, 32, 256, 256, 0.3,
                         store_dead=False, seed=1004),
    "c5_stress": TreeConfig("c5_stress", 8, 32, 128, "bf16", 4096, 32, 64, 512, 512,
                            0.3, layers=32, store_dead=False, seed=1005),
    # 16 searches of the c4 shape running side by side, as a serving system batches
    # the problems it works on: one forest, one pool, one call
    "c6_batch16": TreeConfig("c6_batch16", 8, 64, 128, "bf16", 2048, 24, 32, 256, 256, 0.3,
                             layers=4, store_dead=False, seed=1006, trees=16),
}


@dataclass
class Tree:
    parent: np.ndarray          # int32 [N], -1 for a root, parent[i] < i
    tok_offset: np.ndarray      # int64 [N], first pool row of the node
    n_tokens: np.ndarray        # int32 [N]
    leaf_node: np.ndarray       # int32 [L], node id of every leaf query
    pool_tokens: int            # rows in the K/V pool
    step: np.ndarray = field(default=None)  # int32 [N], search step of the node

    @property
    def n_nodes(self) -> int:
        return int(self.parent.shape[0])

    @property
    def n_leaves(self) -> int:
        return int(self.leaf_node.shape[0])


def _rng(seed: int, stream: int) -> np.random.Generator:
    return np.random.Generator(np.random.Philox(key=[int(seed), int(stream)]))


def make_tree(cfg: TreeConfig, seed: Optional[int] = None) -> Tree:
    """Build the topology of `cfg` (see the module docstring for the recipe).  With
    cfg.trees > 1 the result is a forest of that many independent searches (search t
    drawn with seed + 7919 t), nodes and pool rows of one search after the other."""
    seed = cfg.seed if seed is None else seed
    if cfg.trees > 1:
        from dataclasses import replace
        one = replace(cfg, trees=1)
        parts = [make_tree(one, seed + 7919 * t) for t in range(cfg.trees)]
        node0 = np.cumsum([0] + [p.n_nodes for p in parts])
        row0 = np.cumsum([0] + [p.pool_tokens for p in parts])
        return Tree(
            np.concatenate([np.where(p.parent < 0, -1, p.parent + node0[t]).astype(np.int32)
                            for t, p in enumerate(parts)]),
            np.concatenate([p.tok_offset + row0[t] for t, p in enumerate(parts)]),
            np.concatenate([p.n_tokens for p in parts]),
            np.concatenate([(p.leaf_node + node0[t]).astype(np.int32)
                            for t, p in enumerate(parts)]),
            int(row0[-1]), np.concatenate([p.step for p in parts]))
    topo = _rng(seed, 0)
    lens = _rng(seed, 1)

    parent = [-1]
    step = [0]
    prev = np.array([0], dtype=np.int64)
    for s in range(1, cfg.steps + 1):
        if cfg.alpha is None:
            par = np.repeat(prev, cfg.branch)
        elif s == 1:
            par = np.zeros(cfg.width, dtype=np.int64)
        else:
            p = topo.dirichlet(np.full(prev.shape[0], cfg.alpha, dtype=np.float64))
            # guard against underflow to an all-zero vector for tiny alpha
            p = np.maximum(p, 0.0)
            p = p / p.sum() if p.sum() > 0 else np.full(p.shape, 1.0 / p.shape[0])
            par = np.sort(prev[topo.choice(prev.shape[0], size=cfg.width, p=p)])
        first = len(parent)
        parent.extend(int(x) for x in par)
        step.extend([s] * len(par))
        prev = np.arange(first, first + len(par), dtype=np.int64)
    parent = np.asarray(parent, dtype=np.int32)
    step = np.asarray(step, dtype=np.int32)
    n = parent.shape[0]

    n_tokens = lens.integers(cfg.step_lo, cfg.step_hi + 1, size=n).astype(np.int32)
    n_tokens[0] = cfg.prompt
    leaf_node = prev.astype(np.int32)

    live = np.zeros(n, dtype=bool)
    live[leaf_node] = True
    for i in range(n - 1, 0, -1):
        if live[i]:
            live[parent[i]] = True

    stored = np.ones(n, dtype=bool) if cfg.store_dead else live
    tok_offset = np.zeros(n, dtype=np.int64)
    sizes = np.where(stored, n_tokens, 0).astype(np.int64)
    tok_offset[:] = np.cumsum(sizes) - sizes
    tok_offset[~stored] = 0
    pool_tokens = int(sizes.sum())
    return Tree(parent, tok_offset, n_tokens, leaf_node, pool_tokens, step)


def random_tree(seed: int, n_nodes: int, n_leaves: int, max_tokens: int,
                p_root: float = 0.1, p_empty: float = 0.15,
                shuffle_pool: bool = True) -> Tree:
    """Irregular forest for fuzzing: random parents (parent[i] < i), several
    roots, zero-length nodes, leaf entries on interior nodes and duplicated."""
    r = _rng(seed, 7)
    parent = np.full(n_nodes, -1, dtype=np.int32)
    for i in range(1, n_nodes):
        if r.random() >= p_root:
            parent[i] = int(r.integers(0, i))
    n_tokens = r.integers(1, max_tokens + 1, size=n_nodes).astype(np.int32)
    n_tokens[r.random(n_nodes) < p_empty] = 0
    order = r.permutation(n_nodes) if shuffle_pool else np.arange(n_nodes)
    tok_offset = np.zeros(n_nodes, dtype=np.int64)
    pos = 0
    for i in order:
        tok_offset[i] = pos
        pos += int(n_tokens[i])
    leaf_node = r.integers(0, n_nodes, size=n_leaves).astype(np.int32)
    return Tree(parent, tok_offset, n_tokens, leaf_node, max(pos, 1),
                np.zeros(n_nodes, dtype=np.int32))


# --------------------------------------------------------------------------
# values
# --------------------------------------------------------------------------
def to_bf16_bits(x: np.ndarray) -> np.ndarray:
    """Round float32 to bfloat16 (round-to-nearest-even); returns uint16 bits."""
    b = np.ascontiguousarray(x, dtype=np.float32).view(np.uint32)
    b = b + (np.uint32(0x7FFF) + ((b >> np.uint32(16)) & np.uint32(1)))
    return (b >> np.uint32(16)).astype(np.uint16)


def bf16_bits_to_f32(b: np.ndarray) -> np.ndarray:
    return (b.astype(np.uint32) << np.uint32(16)).view(np.float32)


def make_values_host(cfg: TreeConfig, tree: Tree, seed: Optional[int] = None,
                     layer: int = 0):
    """K, V indexed [pool row, kv head, D] (the device library wants them laid out
    [kv head][pool row][D]: transpose before uploading); Q: [L, Hq, D]; i.i.d. N(0,1).
    float32 arrays for dtype "f32", uint16 bfloat16 bit patterns for "bf16"."""
    seed = cfg.seed if seed is None else seed
    r = _rng(seed, 2 + layer)
    k = r.standard_normal((tree.pool_tokens, cfg.n_kv_heads, cfg.head_dim),
                          dtype=np.float32)
    v = r.standard_normal((tree.pool_tokens, cfg.n_kv_heads, cfg.head_dim),
                          dtype=np.float32)
    q = r.standard_normal((tree.n_leaves, cfg.n_q_heads, cfg.head_dim),
                          dtype=np.float32)
    if cfg.dtype == "bf16":
        return to_bf16_bits(k), to_bf16_bits(v), to_bf16_bits(q)
    return k, v, q


def make_values_device(cfg: TreeConfig, tree: Tree, device, seed: Optional[int] = None,
                       layers: Optional[int] = None):
    """Device-side generation for pools too large to draw on the host.
    Returns torch tensors K, V: [layers, Hkv, pool_tokens, D] (the library's memory
    layout of a pool), Q: [layers, L, Hq, D]
    in cfg.dtype, drawn N(0,1) by torch's seeded device generator."""
    import torch
    seed = cfg.seed if seed is None else seed
    layers = cfg.layers if layers is None else layers
    dt = torch.float32 if cfg.dtype == "f32" else torch.bfloat16
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    k = torch.empty((layers, cfg.n_kv_heads, tree.pool_tokens, cfg.head_dim),
                    dtype=dt, device=device)
    v = torch.empty_like(k)
    q = torch.empty((layers, tree.n_leaves, cfg.n_q_heads, cfg.head_dim),
                    dtype=dt, device=device)
    for l in range(layers):
        k[l].normal_(generator=g)
        v[l].normal_(generator=g)
        q[l].normal_(generator=g)
    return k, v, q


def quantize_e4m3(x, scale: float):
    """torch tensor (any float dtype) -> E4M3 codes (torch.uint8, same shape and device) of
    x / scale: torch's own round-to-nearest conversion to float8_e4m3fn, so this module
    holds no arithmetic of the format; magnitudes beyond 448 are clamped first (the
    format has no infinity)."""
    import torch
    y = (x.to(torch.float32) / float(scale)).clamp_(-448.0, 448.0)
    return y.to(torch.float8_e4m3fn).view(torch.uint8)


def make_values_fp8_host(cfg: TreeConfig, tree: Tree, k_scale: float, v_scale: float,
                         seed: Optional[int] = None, layer: int = 0):
    """The values of make_values_host with K and V stored as E4M3 codes of K / k_scale and
    V / v_scale: (k_codes, v_codes) uint8 [pool row, kv head, D], q bfloat16 bits."""
    import torch
    assert cfg.dtype == "bf16"
    seed = cfg.seed if seed is None else seed
    r = _rng(seed, 2 + layer)
    shape = (tree.pool_tokens, cfg.n_kv_heads, cfg.head_dim)
    k = r.standard_normal(shape, dtype=np.float32)
    v = r.standard_normal(shape, dtype=np.float32)
    q = r.standard_normal((tree.n_leaves, cfg.n_q_heads, cfg.head_dim), dtype=np.float32)
    return (quantize_e4m3(torch.from_numpy(k), k_scale).numpy(),
            quantize_e4m3(torch.from_numpy(v), v_scale).numpy(), to_bf16_bits(q))


def make_values_fp8_device(cfg: TreeConfig, tree: Tree, device, k_scale: float, v_scale: float,
                           seed: Optional[int] = None, layers: Optional[int] = None):
    """Device-side generation: K, V uint8 E4M3 codes [layers, Hkv, pool_tokens, D] (the
    library's layout) of N(0,1) draws divided by the scales, Q bfloat16 [layers, L, Hq, D]."""
    import torch
    seed = cfg.seed if seed is None else seed
    layers = cfg.layers if layers is None else layers
    g = torch.Generator(device=device)
    g.manual_seed(int(seed))
    shape = (cfg.n_kv_heads, tree.pool_tokens, cfg.head_dim)
    k = torch.empty((layers,) + shape, dtype=torch.uint8, device=device)
    v = torch.empty_like(k)
    q = torch.empty((layers, tree.n_leaves, cfg.n_q_heads, cfg.head_dim),
                    dtype=torch.bfloat16, device=device)
    tmp = torch.empty(shape[1:], dtype=torch.float32, device=device)
    for l in range(layers):
        for dst, sc in ((k, k_scale), (v, v_scale)):
            for h in range(cfg.n_kv_heads):
                tmp.normal_(generator=g)
                dst[l, h] = quantize_e4m3(tmp, sc)
        q[l].normal_(generator=g)
    return k, v, q


def with_growth_room(tree: Tree, room: int) -> Tree:
    """The same tree laid out with `room` free pool rows after every node that holds a
    leaf query (as a cache reserves space for the step being generated), so that decode
    steps can append tokens to those nodes.  Nodes keep their order in the pool."""
    is_leaf = np.zeros(tree.n_nodes, dtype=bool)
    is_leaf[tree.leaf_node] = True
    order = np.argsort(tree.tok_offset, kind="stable")
    new_off = np.zeros(tree.n_nodes, dtype=np.int64)
    cur = 0
    for n in order:
        new_off[n] = cur
        cur += int(tree.n_tokens[n]) + (room if is_leaf[n] else 0)
    return Tree(tree.parent.copy(), new_off, tree.n_tokens.copy(), tree.leaf_node.copy(),
                max(cur, 1), tree.step)


def make_new_tokens_host(cfg: TreeConfig, tree: Tree, step: int, seed: Optional[int] = None):
    """K and V rows of the token every leaf query generates at decode step `step`:
    [L, Hkv, D] each, i.i.d. N(0,1), in the pool's dtype convention."""
    seed = cfg.seed if seed is None else seed
    r = _rng(seed, 1000 + step)
    k = r.standard_normal((tree.n_leaves, cfg.n_kv_heads, cfg.head_dim), dtype=np.float32)
    v = r.standard_normal((tree.n_leaves, cfg.n_kv_heads, cfg.head_dim), dtype=np.float32)
    if cfg.dtype == "bf16":
        return to_bf16_bits(k), to_bf16_bits(v)
    return k, v


def make_prefill_queries_host(cfg: TreeConfig, tree: Tree, seed: Optional[int] = None):
    """Query vectors for step prefill: one row per token of every leaf query's node,
    leaf query by leaf query, [sum of those node lengths, Hq, D], i.i.d. N(0,1), in the
    pool's dtype convention."""
    seed = cfg.seed if seed is None else seed
    r = _rng(seed, 500)
    n_rows = int(tree.n_tokens[tree.leaf_node].sum()) if tree.n_leaves else 0
    q = r.standard_normal((n_rows, cfg.n_q_heads, cfg.head_dim), dtype=np.float32)
    if cfg.dtype == "bf16":
        return to_bf16_bits(q)
    return q
