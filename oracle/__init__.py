"""ctypes front end of the CPU oracle (oracle/tree_attn_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by the smoke check and by the
benchmark's cpu_baseline leg.  The product package never imports it, and this
module imports nothing from the product package.

All array arguments are numpy arrays; bfloat16 data travels as uint16 bit
patterns, fp32 data as float32.  Results are float64.
"""
from __future__ import annotations

import ctypes as C
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_SRC = os.path.join(_HERE, "tree_attn_oracle.c")
_LIB = os.path.join(_HERE, "libets_oracle.so")

F32, BF16, F64 = 0, 1, 2


def build(force: bool = False) -> str:
    """Compile the oracle with gcc (fp64, OpenMP over (leaf, head) only)."""
    if force or not os.path.exists(_LIB) or os.path.getmtime(_LIB) < os.path.getmtime(_SRC):
        cmd = ["gcc", "-O2", "-std=c11", "-fopenmp", "-fPIC", "-shared", "-Wall", "-Wextra",
               "-ffp-contract=off", _SRC, "-o", _LIB, "-lm"]
        subprocess.run(cmd, check=True)
    return _LIB


_lib = None


def _load():
    global _lib
    if _lib is None:
        build()
        lib = C.CDLL(_LIB)
        i32p, i64p, f64p = (C.POINTER(C.c_int32), C.POINTER(C.c_int64),
                            C.POINTER(C.c_double))
        lib.ets_oracle_threads.restype = C.c_int
        lib.ets_oracle_check_tree.restype = C.c_int
        lib.ets_oracle_check_tree.argtypes = [C.c_int32, i32p, i64p, i32p, C.c_int32, i32p,
                                              C.c_int64]
        lib.ets_oracle_paths.restype = C.c_int64
        lib.ets_oracle_paths.argtypes = [C.c_int32, i32p, C.c_int32, i32p, i64p, i32p,
                                         C.c_int64]
        lib.ets_oracle_tree_stats.restype = None
        lib.ets_oracle_tree_stats.argtypes = [C.c_int32, i32p, i32p, C.c_int32, i32p, i64p,
                                              i64p, i64p, i64p]
        common = [C.c_int32, i32p, i64p, i32p, C.c_int32, i32p, C.c_int32, C.c_int32,
                  C.c_int32, C.c_int, C.c_double, C.c_void_p, C.c_void_p, C.c_int64,
                  C.c_int64, C.c_void_p]
        lib.ets_oracle_attn.restype = C.c_int
        lib.ets_oracle_attn.argtypes = common + [f64p, f64p]
        lib.ets_oracle_attn_rows.restype = C.c_int
        lib.ets_oracle_attn_rows.argtypes = common + [C.c_int64, i32p, i32p, f64p, f64p]
        lib.ets_oracle_prefill_rows.restype = C.c_int
        lib.ets_oracle_prefill_rows.argtypes = common + [C.c_int64, i32p, i32p, i32p, f64p, f64p]
        lib.ets_oracle_partial.restype = None
        lib.ets_oracle_partial.argtypes = [C.c_int32, C.c_int, C.c_double,
                                           C.c_void_p, C.c_void_p, C.c_int64, C.c_int64,
                                           f64p, C.c_int32, C.c_int64, i64p, f64p, f64p,
                                           f64p]
        lib.ets_oracle_merge.restype = None
        lib.ets_oracle_merge.argtypes = [C.c_int32, C.c_int64, f64p, f64p, f64p, f64p, f64p]
        _lib = lib
    return _lib


def _p(a, ct):
    return a.ctypes.data_as(C.POINTER(ct))


def _i32(a):
    return np.ascontiguousarray(a, dtype=np.int32)


def _i64(a):
    return np.ascontiguousarray(a, dtype=np.int64)


def _vals(a):
    a = np.ascontiguousarray(a)
    if a.dtype == np.float32:
        return a, F32
    if a.dtype == np.uint16:
        return a, BF16
    if a.dtype == np.float64:
        return a, F64
    raise TypeError("values must be float32, float64 or uint16 (bfloat16 bits), got %s" % a.dtype)


def _pool(a):
    """A pool K[t, h, :] as (array, dtype code, row stride, head stride), strides in
    elements.  Any memory order of the first two axes is taken as it is (no copy), so a
    head-major buffer can be handed over as the transposed view buf.transpose(1, 0, 2);
    only the last axis has to be contiguous."""
    a = np.asarray(a)
    if a.ndim != 3:
        raise ValueError("a pool has three axes: [pool row, kv head, head_dim]")
    if a.dtype == np.float32:
        dt = F32
    elif a.dtype == np.uint16:
        dt = BF16
    elif a.dtype == np.float64:
        dt = F64
    else:
        raise TypeError("values must be float32, float64 or uint16 (bfloat16 bits), got %s" % a.dtype)
    sz = a.dtype.itemsize
    if a.shape[2] > 1 and a.strides[2] != sz or a.strides[0] % sz or a.strides[1] % sz \
            or a.strides[0] < 0 or a.strides[1] < 0:
        a = np.ascontiguousarray(a)
    return a, dt, a.strides[0] // sz, a.strides[1] // sz


def threads() -> int:
    return int(_load().ets_oracle_threads())


def check_tree(parent, tok_offset, n_tokens, leaf_node, pool_tokens) -> int:
    parent, tok_offset, n_tokens, leaf_node = (_i32(parent), _i64(tok_offset),
                                               _i32(n_tokens), _i32(leaf_node))
    return int(_load().ets_oracle_check_tree(
        parent.shape[0], _p(parent, C.c_int32), _p(tok_offset, C.c_int64),
        _p(n_tokens, C.c_int32), leaf_node.shape[0], _p(leaf_node, C.c_int32),
        int(pool_tokens)))


def paths(parent, leaf_node):
    """(path_ptr int64 [L+1], path_nodes int32) with each path in root->leaf order."""
    parent, leaf_node = _i32(parent), _i32(leaf_node)
    n, L = parent.shape[0], leaf_node.shape[0]
    cap = max(1, n * max(L, 1))
    ptr = np.zeros(L + 1, dtype=np.int64)
    while True:
        nodes = np.zeros(cap, dtype=np.int32)
        tot = _load().ets_oracle_paths(n, _p(parent, C.c_int32), L, _p(leaf_node, C.c_int32),
                                       _p(ptr, C.c_int64), _p(nodes, C.c_int32), cap)
        if tot >= 0:
            return ptr, nodes[:tot].copy()
        cap *= 2


def tree_stats(parent, n_tokens, leaf_node):
    """dict(leaf_count[N], unique_tokens, flat_tokens, live_nodes)."""
    parent, n_tokens, leaf_node = _i32(parent), _i32(n_tokens), _i32(leaf_node)
    n = parent.shape[0]
    cnt = np.zeros(n, dtype=np.int64)
    u, f, lv = C.c_int64(0), C.c_int64(0), C.c_int64(0)
    _load().ets_oracle_tree_stats(n, _p(parent, C.c_int32), _p(n_tokens, C.c_int32),
                                  leaf_node.shape[0], _p(leaf_node, C.c_int32),
                                  _p(cnt, C.c_int64), C.byref(u), C.byref(f), C.byref(lv))
    return dict(leaf_count=cnt, unique_tokens=u.value, flat_tokens=f.value,
                live_nodes=lv.value)


def _tree_args(parent, tok_offset, n_tokens, leaf_node):
    parent, tok_offset, n_tokens, leaf_node = (_i32(parent), _i64(tok_offset),
                                               _i32(n_tokens), _i32(leaf_node))
    keep = (parent, tok_offset, n_tokens, leaf_node)
    args = [parent.shape[0], _p(parent, C.c_int32), _p(tok_offset, C.c_int64),
            _p(n_tokens, C.c_int32), leaf_node.shape[0], _p(leaf_node, C.c_int32)]
    return keep, args


def tree_decode_attn(parent, tok_offset, n_tokens, leaf_node, k_pool, v_pool, q,
                     n_kv_heads, n_q_heads, head_dim, sm_scale=0.0, rows=None):
    """Oracle attention.  k_pool/v_pool: K[t, h, :] as arrays of shape [pool_tokens, Hkv, D]
    (their strides say how the pool lies in memory); q: [L, Hq, D].

    rows=None: every (leaf, head) -> out float64 [L, Hq, D], lse float64 [L, Hq].
    rows=(leaf_idx, head_idx): only those pairs -> out [n, D], lse [n].
    """
    k_pool, dt, ts, hs = _pool(k_pool)
    v_pool, dt2, ts2, hs2 = _pool(v_pool)
    if k_pool.shape != v_pool.shape or (ts2, hs2) != (ts, hs):
        v_pool = np.ascontiguousarray(v_pool)
        k_pool = np.ascontiguousarray(k_pool)
        k_pool, dt, ts, hs = _pool(k_pool)
        v_pool, dt2, ts2, hs2 = _pool(v_pool)
    q, dt3 = _vals(q)
    if not (dt == dt2 == dt3):
        raise TypeError("k, v, q must share one dtype")
    keep, targs = _tree_args(parent, tok_offset, n_tokens, leaf_node)
    L = keep[3].shape[0]
    pool_tokens = k_pool.shape[0]
    rc = check_tree(*keep, pool_tokens)
    if rc:
        raise ValueError("oracle: malformed tree (code %d)" % rc)
    assert k_pool.shape == v_pool.shape == (pool_tokens, n_kv_heads, head_dim)
    assert q.shape == (L, n_q_heads, head_dim)
    common = targs + [n_kv_heads, n_q_heads, head_dim, dt, float(sm_scale),
                      k_pool.ctypes.data_as(C.c_void_p), v_pool.ctypes.data_as(C.c_void_p),
                      ts, hs, q.ctypes.data_as(C.c_void_p)]
    if rows is None:
        out = np.zeros((L, n_q_heads, head_dim), dtype=np.float64)
        lse = np.zeros((L, n_q_heads), dtype=np.float64)
        rc = _load().ets_oracle_attn(*common, _p(out, C.c_double), _p(lse, C.c_double))
    else:
        sl, sh = _i32(rows[0]), _i32(rows[1])
        out = np.zeros((sl.shape[0], head_dim), dtype=np.float64)
        lse = np.zeros((sl.shape[0],), dtype=np.float64)
        rc = _load().ets_oracle_attn_rows(*common, sl.shape[0], _p(sl, C.c_int32),
                                          _p(sh, C.c_int32), _p(out, C.c_double),
                                          _p(lse, C.c_double))
    if rc:
        raise RuntimeError("oracle failed (code %d)" % rc)
    return out, lse


def dequantise_e4m3(codes, scale):
    """fp64 pool [pool row, kv head, D] from E4M3 codes (uint8, same shape) and one scale per
    pool or per kv head: value(code) * scale[h], the product taken in fp64."""
    from .fp8 import E4M3_TABLE
    codes = np.asarray(codes)
    if codes.dtype != np.uint8 or codes.ndim != 3:
        raise TypeError("E4M3 pools travel as uint8 [pool row, kv head, head_dim]")
    s = np.broadcast_to(np.asarray(scale, dtype=np.float64), (codes.shape[1],))
    return E4M3_TABLE[codes] * s[None, :, None]


def _fp8kv(fn, parent, tok_offset, n_tokens, leaf_node, k_codes, v_codes, k_scale, v_scale,
           q, n_kv_heads, n_q_heads, head_dim, sm_scale, rows):
    """Attention `fn` (decode or step prefill) over pools of E4M3 codes, by the definition:
    the pools are dequantised to fp64 first (K = k_scale[h] * value(code), V likewise), then
    `fn` runs once on them with the caller's sm_scale.  q (bfloat16 bits or float32) is
    widened to fp64 exactly."""
    q = np.asarray(q)
    if q.dtype == np.uint16:
        q = (q.astype(np.uint32) << np.uint32(16)).view(np.float32)
    q = np.asarray(q, dtype=np.float64)
    k64 = dequantise_e4m3(k_codes, k_scale)
    v64 = dequantise_e4m3(v_codes, v_scale)
    return fn(parent, tok_offset, n_tokens, leaf_node, k64, v64, q, n_kv_heads, n_q_heads,
              head_dim, sm_scale=sm_scale, rows=rows)


def tree_decode_attn_fp8kv(parent, tok_offset, n_tokens, leaf_node, k_codes, v_codes, k_scale,
                           v_scale, q, n_kv_heads, n_q_heads, head_dim, sm_scale=0.0, rows=None):
    """Decode attention over pools stored as E4M3 codes:
    K[t, h, :] = k_scale[h] * value(k_codes[t, h, :]), V likewise with v_scale (a scalar
    stands for the same scale on every kv head); q as bfloat16 bit patterns (uint16) or
    float32.  The definition is tree_decode_attn's on those K and V."""
    return _fp8kv(tree_decode_attn, parent, tok_offset, n_tokens,
                  leaf_node, k_codes, v_codes, k_scale, v_scale, q, n_kv_heads, n_q_heads, head_dim,
                  sm_scale, rows)


def prefill_q_ptr(n_tokens, leaf_node):
    """First query row of every leaf query in step prefill: int64 [L + 1], the prefix
    sums of the leaf nodes' lengths (every token of a leaf query's node is a query)."""
    lens = np.asarray(n_tokens, dtype=np.int64)[np.asarray(leaf_node, dtype=np.int64)]
    return np.concatenate([np.zeros(1, np.int64), np.cumsum(lens, dtype=np.int64)])


def tree_prefill_attn(parent, tok_offset, n_tokens, leaf_node, k_pool, v_pool, q,
                      n_kv_heads, n_q_heads, head_dim, sm_scale=0.0, rows=None):
    """Oracle step-prefill attention: token i of leaf query l's node sees every row of the
    node's strict ancestors and rows 0..i of the node.  k_pool/v_pool as in
    tree_decode_attn; q: [n_q_rows, Hq, D], rows ordered as prefill_q_ptr says.

    rows=None: everything -> out float64 [n_q_rows, Hq, D], lse [n_q_rows, Hq].
    rows=(leaf_idx, tok_idx, head_idx): only those triples -> out [n, D], lse [n].
    """
    k_pool, dt, ts, hs = _pool(k_pool)
    v_pool, dt2, ts2, hs2 = _pool(v_pool)
    if k_pool.shape != v_pool.shape or (ts2, hs2) != (ts, hs):
        k_pool, dt, ts, hs = _pool(np.ascontiguousarray(k_pool))
        v_pool, dt2, ts2, hs2 = _pool(np.ascontiguousarray(v_pool))
    q, dt3 = _vals(q)
    if not (dt == dt2 == dt3):
        raise TypeError("k, v, q must share one dtype")
    keep, targs = _tree_args(parent, tok_offset, n_tokens, leaf_node)
    rc = check_tree(*keep, k_pool.shape[0])
    if rc:
        raise ValueError("oracle: malformed tree (code %d)" % rc)
    q_ptr = prefill_q_ptr(keep[2], keep[3])
    n_rows = int(q_ptr[-1])
    assert k_pool.shape == v_pool.shape == (k_pool.shape[0], n_kv_heads, head_dim)
    assert q.shape == (n_rows, n_q_heads, head_dim)
    full = rows is None
    if full:
        L = keep[3].shape[0]
        lens = np.diff(q_ptr)
        sl = np.repeat(np.repeat(np.arange(L, dtype=np.int32), lens), n_q_heads)
        st = np.repeat(np.concatenate([np.arange(n, dtype=np.int32) for n in lens] +
                                      [np.zeros(0, np.int32)]), n_q_heads)
        sh = np.tile(np.arange(n_q_heads, dtype=np.int32), n_rows)
    else:
        sl, st, sh = _i32(rows[0]), _i32(rows[1]), _i32(rows[2])
    sl, st, sh = _i32(sl), _i32(st), _i32(sh)
    n = sl.shape[0]
    out = np.zeros((n, head_dim), dtype=np.float64)
    lse = np.zeros((n,), dtype=np.float64)
    common = targs + [n_kv_heads, n_q_heads, head_dim, dt, float(sm_scale),
                      k_pool.ctypes.data_as(C.c_void_p), v_pool.ctypes.data_as(C.c_void_p),
                      ts, hs, q.ctypes.data_as(C.c_void_p)]
    rc = _load().ets_oracle_prefill_rows(*common, n, _p(sl, C.c_int32), _p(st, C.c_int32),
                                         _p(sh, C.c_int32), _p(out, C.c_double),
                                         _p(lse, C.c_double))
    if rc:
        raise RuntimeError("oracle failed (code %d)" % rc)
    if full:
        return out.reshape(n_rows, n_q_heads, head_dim), lse.reshape(n_rows, n_q_heads)
    return out, lse


def tree_prefill_attn_fp8kv(parent, tok_offset, n_tokens, leaf_node, k_codes, v_codes, k_scale,
                            v_scale, q, n_kv_heads, n_q_heads, head_dim, sm_scale=0.0, rows=None):
    """Step-prefill attention over pools stored as E4M3 codes with one scale per pool or
    per kv head: the definition of tree_prefill_attn on K = k_scale[h] * value(k_codes),
    V = v_scale[h] * value(v_codes)."""
    return _fp8kv(tree_prefill_attn, parent, tok_offset, n_tokens, leaf_node, k_codes,
                  v_codes, k_scale, v_scale, q, n_kv_heads, n_q_heads, head_dim, sm_scale, rows)


def visible_rows(parent, tok_offset, n_tokens, node, own_rows=None):
    """Pool rows a query on `node` sees, in path order: all rows of the strict ancestors,
    then the first `own_rows` rows of the node (None: all of them)."""
    chain = []
    x = int(node)
    while x >= 0:
        chain.append(x)
        x = int(parent[x])
    chain.reverse()
    rows = []
    for n in chain[:-1]:
        rows.extend(range(int(tok_offset[n]), int(tok_offset[n]) + int(n_tokens[n])))
    own = int(n_tokens[node]) if own_rows is None else min(int(own_rows), int(n_tokens[node]))
    rows.extend(range(int(tok_offset[node]), int(tok_offset[node]) + own))
    return np.asarray(rows, dtype=np.int64)


def partial(k_pool, v_pool, qvec, kv_head, rows, sm_scale=0.0):
    """Unnormalised partial (o[D], m, l) of one query vector over pool rows `rows`."""
    k_pool, dt, ts, hs = _pool(np.ascontiguousarray(k_pool))
    v_pool, _, _, _ = _pool(np.ascontiguousarray(v_pool))
    assert k_pool.shape == v_pool.shape
    qvec = np.ascontiguousarray(qvec, dtype=np.float64)
    rows = _i64(rows)
    _, hkv, d = k_pool.shape
    o = np.zeros(d, dtype=np.float64)
    m, l = C.c_double(0), C.c_double(0)
    _load().ets_oracle_partial(d, dt, float(sm_scale), k_pool.ctypes.data_as(C.c_void_p),
                               v_pool.ctypes.data_as(C.c_void_p), ts, hs, _p(qvec, C.c_double),
                               int(kv_head), rows.shape[0], _p(rows, C.c_int64),
                               _p(o, C.c_double), C.byref(m), C.byref(l))
    return o, m.value, l.value


def merge(o, m, l):
    """LSE merge of partials o [n, D], m [n], l [n] -> (out [D], lse)."""
    o = np.ascontiguousarray(o, dtype=np.float64)
    m = np.ascontiguousarray(m, dtype=np.float64)
    l = np.ascontiguousarray(l, dtype=np.float64)
    n, d = o.shape
    out = np.zeros(d, dtype=np.float64)
    lse = C.c_double(0)
    _load().ets_oracle_merge(d, n, _p(o, C.c_double), _p(m, C.c_double), _p(l, C.c_double),
                             _p(out, C.c_double), C.byref(lse))
    return out, lse.value


def append_kv(tok_offset, n_tokens, leaf_node, k_pool, v_pool, k_new, v_new):
    """Decode-step advance, written out (ETS paper Sec. 4.1: within a search step the
    topology is fixed; App. B: the leaves are the latest steps, which are the ones being
    generated).  Every distinct node of `leaf_node` receives one token: the K and V row
    of the first leaf query that sits on it goes to pool row tok_offset + n_tokens of
    that node, and the node becomes one token longer.  Pools are modified in place;
    returns the new n_tokens array."""
    n_tokens = np.array(n_tokens, dtype=np.int32, copy=True)
    seen = set()
    for l, n in enumerate(np.asarray(leaf_node).tolist()):
        if n in seen:
            continue
        seen.add(n)
        row = int(tok_offset[n]) + int(n_tokens[n])
        k_pool[row] = k_new[l]
        v_pool[row] = v_new[l]
    for n in seen:
        n_tokens[n] += 1
    return n_tokens
