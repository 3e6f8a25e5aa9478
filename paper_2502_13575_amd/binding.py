"""ctypes binding of include/etsattn.h.  Same names, same order of arguments;
numpy arrays stand for host pointers, torch tensors (or integer addresses) for
device pointers."""
from __future__ import annotations

import ctypes as C
import os

import numpy as np

ETS_F32, ETS_BF16 = 0, 1
ETS_PLAN_TREE, ETS_PLAN_FLAT = 0, 1
ETS_KV_NATIVE, ETS_KV_FP8_E4M3 = 0, 1
ETS_STATIC_SCRATCH_BYTES = 32 << 20

_HERE = os.path.dirname(os.path.abspath(__file__))
_LIB_PATH = os.path.join(_HERE, "libetsattn.so")
_lib = None


class EtsError(RuntimeError):
    def __init__(self, status: int, where: str):
        self.status = int(status)
        super().__init__("%s: %s (status %d)" % (where, ets_strerror(status), status))


class EtsShape(C.Structure):
    _fields_ = [("n_kv_heads", C.c_int32), ("n_q_heads", C.c_int32), ("head_dim", C.c_int32),
                ("dtype", C.c_int32), ("sm_scale", C.c_float)]


class _EtsTree(C.Structure):
    _fields_ = [("n_nodes", C.c_int32), ("parent", C.POINTER(C.c_int32)),
                ("tok_offset", C.POINTER(C.c_int64)), ("n_tokens", C.POINTER(C.c_int32)),
                ("n_leaves", C.c_int32), ("leaf_node", C.POINTER(C.c_int32))]


class EtsStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "n_nodes", "live_nodes", "n_leaves", "unique_tokens", "flat_tokens", "unique_kv_bytes",
        "flat_kv_bytes", "n_segments", "n_partials", "n_stream_items", "n_cascade_items",
        "min_pool_tokens", "workspace_bytes", "cascade_tokens", "stream_tokens", "shares_nodes",
        "n_wide_items", "wide_tokens", "merge_fused")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class EtsPrefillStats(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "n_leaves", "n_q_rows", "n_items", "n_runs", "rows_per_item", "unique_tokens",
        "unique_kv_bytes", "streamed_tokens", "streamed_kv_bytes", "visible_pairs", "flops",
        "min_pool_tokens")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class EtsSelectInfo(C.Structure):
    _fields_ = [("objective", C.c_double), ("kept_nodes", C.c_int64), ("live_nodes", C.c_int64),
                ("kept_clusters", C.c_int64), ("clusters", C.c_int64), ("bb_nodes", C.c_int64),
                ("optimal", C.c_int32), ("pad", C.c_int32)]


class EtsPlanCheckReport(C.Structure):
    _fields_ = [(n, C.c_int64) for n in (
        "decode_items", "prefill_items", "entry_table_entries", "max_entry_index",
        "max_entry_overreach", "max_pool_row", "max_partial_row", "violations")]

    def as_dict(self):
        return {n: int(getattr(self, n)) for n, _ in self._fields_}


class EtsProfile(C.Structure):
    _fields_ = [("calls", C.c_int64), ("stream_ms", C.c_double), ("cascade_ms", C.c_double),
                ("merge_ms", C.c_double), ("wide_ms", C.c_double)]


def library_path() -> str:
    return _LIB_PATH


def load_library():
    """Loads libetsattn.so; raises if it has not been built (no fallback exists)."""
    global _lib
    if _lib is not None:
        return _lib
    if not os.path.exists(_LIB_PATH):
        raise ImportError(
            "libetsattn.so is not built: run `python -m paper_2502_13575_amd.build` "
            "(there is no CPU fallback for the attention path)")
    try:
        # device buffers come from PyTorch: load it first, so that this library binds to
        # the HIP runtime torch brings along instead of loading a second one
        import torch  # noqa: F401
    except ImportError:
        pass
    lib = C.CDLL(_LIB_PATH)
    vp = C.c_void_p
    i32p, i64p = C.POINTER(C.c_int32), C.POINTER(C.c_int64)
    lib.ets_create.restype = C.c_int
    lib.ets_create.argtypes = [C.POINTER(vp), C.POINTER(EtsShape), C.c_int]
    lib.ets_destroy.restype = None
    lib.ets_destroy.argtypes = [vp]
    lib.ets_plan.restype = C.c_int
    lib.ets_plan.argtypes = [vp, C.POINTER(_EtsTree), C.c_int]
    lib.ets_plan_stats.restype = C.c_int
    lib.ets_plan_stats.argtypes = [vp, C.POINTER(EtsStats)]
    lib.ets_plan_paths.restype = C.c_int
    lib.ets_plan_paths.argtypes = [vp, i64p, i32p, C.c_int64, i64p]
    lib.ets_plan_leaf_counts.restype = C.c_int
    lib.ets_plan_leaf_counts.argtypes = [vp, i64p]
    lib.ets_plan_leaf_cover.restype = C.c_int
    lib.ets_plan_leaf_cover.argtypes = [vp, C.c_int32, i64p, C.c_int64, i64p, i32p]
    lib.ets_set_option.restype = C.c_int
    lib.ets_set_option.argtypes = [vp, C.c_char_p, C.c_int64]
    lib.ets_tree_decode_attn.restype = C.c_int
    lib.ets_tree_decode_attn.argtypes = [vp, vp, vp, C.c_int64, vp, vp, vp, vp, C.c_int64, vp]
    lib.ets_tree_decode_attn_static.restype = C.c_int
    lib.ets_tree_decode_attn_static.argtypes = [vp, vp, vp, C.c_int64, vp, vp, vp, vp]
    lib.ets_set_kv_format.restype = C.c_int
    lib.ets_set_kv_format.argtypes = [vp, C.c_int, C.c_float, C.c_float]
    lib.ets_set_kv_head_scales.restype = C.c_int
    lib.ets_set_kv_head_scales.argtypes = [vp, C.POINTER(C.c_float), C.POINTER(C.c_float)]
    lib.ets_kv_append.restype = C.c_int
    lib.ets_kv_append.argtypes = [vp, vp, vp, C.c_int64, vp, vp, vp]
    lib.ets_plan_advance.restype = C.c_int
    lib.ets_plan_advance.argtypes = [vp, vp, i32p]
    lib.ets_plan_check.restype = C.c_int
    lib.ets_plan_check.argtypes = [vp, C.POINTER(EtsPlanCheckReport)]
    lib.ets_plan_append_rows.restype = C.c_int
    lib.ets_plan_append_rows.argtypes = [vp, i64p]
    lib.ets_plan_prefill.restype = C.c_int
    lib.ets_plan_prefill.argtypes = [vp, C.POINTER(_EtsTree)]
    lib.ets_prefill_plan_stats.restype = C.c_int
    lib.ets_prefill_plan_stats.argtypes = [vp, C.POINTER(EtsPrefillStats)]
    lib.ets_prefill_q_ptr.restype = C.c_int
    lib.ets_prefill_q_ptr.argtypes = [vp, i64p]
    lib.ets_prefill_cover.restype = C.c_int
    lib.ets_prefill_cover.argtypes = [vp, C.c_int32, C.c_int32, i64p, C.c_int64, i64p]
    lib.ets_tree_prefill_attn.restype = C.c_int
    lib.ets_tree_prefill_attn.argtypes = [vp, vp, vp, C.c_int64, vp, vp, vp, vp]
    lib.ets_rebase_weights.restype = C.c_int
    lib.ets_rebase_weights.argtypes = [C.c_int32, C.POINTER(C.c_double), C.c_int32, C.c_double, i32p]
    lib.ets_select_leaves.restype = C.c_int
    lib.ets_select_leaves.argtypes = [C.POINTER(_EtsTree), i32p, i32p, C.c_double, C.c_double,
                                      C.c_int64, C.POINTER(C.c_uint8), C.POINTER(EtsSelectInfo)]
    lib.ets_bench_read_stream.restype = C.c_int
    lib.ets_bench_read_stream.argtypes = [C.c_int, vp, C.c_int64, C.c_int, vp, C.c_int64, vp]
    lib.ets_profile_read.restype = C.c_int
    lib.ets_profile_read.argtypes = [vp, C.POINTER(EtsProfile)]
    lib.ets_strerror.restype = C.c_char_p
    lib.ets_strerror.argtypes = [C.c_int]
    _lib = lib
    return lib


def _check(status: int, where: str):
    if status != 0:
        raise EtsError(status, where)


def _dev_ptr(x):
    """Device address of a torch tensor, or an integer address, or None."""
    if x is None:
        return None
    if isinstance(x, int):
        return C.c_void_p(x)
    return C.c_void_p(x.data_ptr())


def ets_strerror(status: int) -> str:
    return load_library().ets_strerror(int(status)).decode()


def ets_create(shape: EtsShape, hip_device: int):
    ctx = C.c_void_p()
    _check(load_library().ets_create(C.byref(ctx), C.byref(shape), int(hip_device)), "ets_create")
    return ctx


def ets_destroy(ctx):
    load_library().ets_destroy(ctx)


def ets_set_option(ctx, key: str, value: int):
    _check(load_library().ets_set_option(ctx, key.encode(), int(value)), "ets_set_option")


def ets_set_kv_format(ctx, kv_format: int, k_scale: float = 1.0, v_scale: float = 1.0):
    _check(load_library().ets_set_kv_format(ctx, int(kv_format), float(k_scale), float(v_scale)),
           "ets_set_kv_format")


def ets_set_kv_head_scales(ctx, k_scales, v_scales):
    k = np.ascontiguousarray(k_scales, dtype=np.float32)
    v = np.ascontiguousarray(v_scales, dtype=np.float32)
    if k.ndim != 1 or k.shape != v.shape:
        raise ValueError("one scale per kv head for each pool")
    _check(load_library().ets_set_kv_head_scales(ctx, k.ctypes.data_as(C.POINTER(C.c_float)),
                                                 v.ctypes.data_as(C.POINTER(C.c_float))),
           "ets_set_kv_head_scales")


def _tree_struct(parent, tok_offset, n_tokens, leaf_node):
    """(_EtsTree, arrays to keep alive) from host arrays."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    tok_offset = np.ascontiguousarray(tok_offset, dtype=np.int64)
    n_tokens = np.ascontiguousarray(n_tokens, dtype=np.int32)
    leaf_node = np.ascontiguousarray(leaf_node, dtype=np.int32)
    if not (parent.shape == tok_offset.shape == n_tokens.shape):
        raise ValueError("parent, tok_offset and n_tokens must have one length")
    t = _EtsTree(parent.shape[0], parent.ctypes.data_as(C.POINTER(C.c_int32)),
                 tok_offset.ctypes.data_as(C.POINTER(C.c_int64)),
                 n_tokens.ctypes.data_as(C.POINTER(C.c_int32)), leaf_node.shape[0],
                 leaf_node.ctypes.data_as(C.POINTER(C.c_int32)))
    return t, (parent, tok_offset, n_tokens, leaf_node)


def ets_plan(ctx, parent, tok_offset, n_tokens, leaf_node, mode: int = ETS_PLAN_TREE):
    t, keep = _tree_struct(parent, tok_offset, n_tokens, leaf_node)
    _check(load_library().ets_plan(ctx, C.byref(t), int(mode)), "ets_plan")
    del keep


def ets_plan_prefill(ctx, parent, tok_offset, n_tokens, leaf_node):
    t, keep = _tree_struct(parent, tok_offset, n_tokens, leaf_node)
    _check(load_library().ets_plan_prefill(ctx, C.byref(t)), "ets_plan_prefill")
    del keep


def ets_prefill_plan_stats(ctx) -> EtsPrefillStats:
    st = EtsPrefillStats()
    _check(load_library().ets_prefill_plan_stats(ctx, C.byref(st)), "ets_prefill_plan_stats")
    return st


def ets_prefill_q_ptr(ctx):
    """int64 [L + 1]: first query row of every leaf query."""
    st = ets_prefill_plan_stats(ctx)
    q_ptr = np.zeros(st.n_leaves + 1, dtype=np.int64)
    _check(load_library().ets_prefill_q_ptr(ctx, q_ptr.ctypes.data_as(C.POINTER(C.c_int64))),
           "ets_prefill_q_ptr")
    return q_ptr


def ets_prefill_cover(ctx, leaf: int, tok: int):
    """Pool rows (int64 [n]) that query token `tok` of leaf query `leaf` sees, in reading order."""
    lib = load_library()
    n = C.c_int64(0)
    rc = lib.ets_prefill_cover(ctx, int(leaf), int(tok), None, 0, C.byref(n))
    if rc != 0 and not (rc == 1 and n.value > 0):
        _check(rc, "ets_prefill_cover")
    rows = np.zeros(max(n.value, 1), dtype=np.int64)
    _check(lib.ets_prefill_cover(ctx, int(leaf), int(tok),
                                 rows.ctypes.data_as(C.POINTER(C.c_int64)), rows.shape[0],
                                 C.byref(n)), "ets_prefill_cover")
    return rows[:n.value].copy()


def ets_tree_prefill_attn(ctx, k_pool, v_pool, pool_tokens: int, q, out, lse, hip_stream=None):
    stream = None if hip_stream is None else C.c_void_p(int(hip_stream))
    _check(load_library().ets_tree_prefill_attn(
        ctx, _dev_ptr(k_pool), _dev_ptr(v_pool), int(pool_tokens), _dev_ptr(q), _dev_ptr(out),
        _dev_ptr(lse), stream), "ets_tree_prefill_attn")


def ets_plan_stats(ctx) -> EtsStats:
    st = EtsStats()
    _check(load_library().ets_plan_stats(ctx, C.byref(st)), "ets_plan_stats")
    return st


def ets_plan_paths(ctx):
    """(path_ptr int64 [L+1], path_nodes int32 [total]) in root->leaf order."""
    lib = load_library()
    st = ets_plan_stats(ctx)
    ptr = np.zeros(st.n_leaves + 1, dtype=np.int64)
    total = C.c_int64(0)
    rc = lib.ets_plan_paths(ctx, ptr.ctypes.data_as(C.POINTER(C.c_int64)), None, 0,
                            C.byref(total))
    if rc != 0 and total.value == 0:
        _check(rc, "ets_plan_paths")
    nodes = np.zeros(max(total.value, 1), dtype=np.int32)
    _check(lib.ets_plan_paths(ctx, ptr.ctypes.data_as(C.POINTER(C.c_int64)),
                              nodes.ctypes.data_as(C.POINTER(C.c_int32)), nodes.shape[0],
                              C.byref(total)), "ets_plan_paths")
    return ptr, nodes[:total.value].copy()


def ets_plan_leaf_counts(ctx):
    st = ets_plan_stats(ctx)
    cnt = np.zeros(max(st.n_nodes, 1), dtype=np.int64)
    _check(load_library().ets_plan_leaf_counts(ctx, cnt.ctypes.data_as(C.POINTER(C.c_int64))),
           "ets_plan_leaf_counts")
    return cnt[:st.n_nodes].copy()


def ets_plan_leaf_cover(ctx, leaf: int):
    """(rows int64 [n], n_partials) read for one leaf query, in partial order."""
    lib = load_library()
    n, npart = C.c_int64(0), C.c_int32(0)
    rc = lib.ets_plan_leaf_cover(ctx, int(leaf), None, 0, C.byref(n), C.byref(npart))
    if rc != 0 and not (rc == 1 and n.value > 0):
        _check(rc, "ets_plan_leaf_cover")
    rows = np.zeros(max(n.value, 1), dtype=np.int64)
    _check(lib.ets_plan_leaf_cover(ctx, int(leaf), rows.ctypes.data_as(C.POINTER(C.c_int64)),
                                   rows.shape[0], C.byref(n), C.byref(npart)),
           "ets_plan_leaf_cover")
    return rows[:n.value].copy(), int(npart.value)


def ets_tree_decode_attn(ctx, k_pool, v_pool, pool_tokens: int, q, out, lse, workspace,
                         workspace_bytes: int, hip_stream=None):
    stream = None if hip_stream is None else C.c_void_p(int(hip_stream))
    _check(load_library().ets_tree_decode_attn(
        ctx, _dev_ptr(k_pool), _dev_ptr(v_pool), int(pool_tokens), _dev_ptr(q), _dev_ptr(out),
        _dev_ptr(lse), _dev_ptr(workspace), int(workspace_bytes), stream),
        "ets_tree_decode_attn")


def ets_tree_decode_attn_static(ctx, k_pool, v_pool, pool_tokens: int, q, out, lse,
                                hip_stream=None):
    stream = None if hip_stream is None else C.c_void_p(int(hip_stream))
    _check(load_library().ets_tree_decode_attn_static(
        ctx, _dev_ptr(k_pool), _dev_ptr(v_pool), int(pool_tokens), _dev_ptr(q), _dev_ptr(out),
        _dev_ptr(lse), stream), "ets_tree_decode_attn_static")


def ets_kv_append(ctx, k_pool, v_pool, pool_tokens: int, k_new, v_new, stream=None) -> None:
    st = None if stream is None else C.c_void_p(int(stream))
    _check(load_library().ets_kv_append(ctx, _dev_ptr(k_pool), _dev_ptr(v_pool), int(pool_tokens),
                                        _dev_ptr(k_new), _dev_ptr(v_new), st), "ets_kv_append")


def ets_plan_advance(ctx, stream=None) -> bool:
    """Returns True when the library had to plan again (read the statistics again then)."""
    flag = C.c_int32(0)
    st = None if stream is None else C.c_void_p(int(stream))
    _check(load_library().ets_plan_advance(ctx, st, C.byref(flag)), "ets_plan_advance")
    return bool(flag.value)


def ets_plan_check(ctx) -> EtsPlanCheckReport:
    """Raises EtsError when a kernel of the current plans would leave its tables."""
    rep = EtsPlanCheckReport()
    _check(load_library().ets_plan_check(ctx, C.byref(rep)), "ets_plan_check")
    return rep


def ets_plan_append_rows(ctx):
    """int64 [L]: pool row that ets_kv_append writes for every leaf query now (-1: none)."""
    st = ets_plan_stats(ctx)
    rows = np.zeros(max(st.n_leaves, 1), dtype=np.int64)
    _check(load_library().ets_plan_append_rows(ctx, rows.ctypes.data_as(C.POINTER(C.c_int64))),
           "ets_plan_append_rows")
    return rows[:st.n_leaves].copy()


def ets_rebase_weights(rewards, budget: int, temperature: float):
    """int32 [n]: continuations per trajectory (ETS paper Eq. 1)."""
    r = np.ascontiguousarray(rewards, dtype=np.float64)
    w = np.zeros(max(r.shape[0], 1), dtype=np.int32)
    _check(load_library().ets_rebase_weights(r.shape[0], r.ctypes.data_as(C.POINTER(C.c_double)),
                                             int(budget), float(temperature),
                                             w.ctypes.data_as(C.POINTER(C.c_int32))),
           "ets_rebase_weights")
    return w[:r.shape[0]].copy()


def ets_select_leaves(parent, leaf_node, weights, cluster=None, lambda_b=1.0, lambda_d=0.0,
                      node_limit=0):
    """(keep bool [L], EtsSelectInfo): the kept leaves that maximise the cost model."""
    parent = np.ascontiguousarray(parent, dtype=np.int32)
    leaf_node = np.ascontiguousarray(leaf_node, dtype=np.int32)
    weights = np.ascontiguousarray(weights, dtype=np.int32)
    if weights.shape != leaf_node.shape:
        raise ValueError("one weight per leaf")
    t = _EtsTree(parent.shape[0], parent.ctypes.data_as(C.POINTER(C.c_int32)), None, None,
                 leaf_node.shape[0], leaf_node.ctypes.data_as(C.POINTER(C.c_int32)))
    cl = None
    if cluster is not None:
        cl = np.ascontiguousarray(cluster, dtype=np.int32)
        if cl.shape != leaf_node.shape:
            raise ValueError("one cluster id per leaf")
    keep = np.zeros(max(leaf_node.shape[0], 1), dtype=np.uint8)
    info = EtsSelectInfo()
    _check(load_library().ets_select_leaves(
        C.byref(t), weights.ctypes.data_as(C.POINTER(C.c_int32)),
        None if cl is None else cl.ctypes.data_as(C.POINTER(C.c_int32)), float(lambda_b),
        float(lambda_d), int(node_limit), keep.ctypes.data_as(C.POINTER(C.c_uint8)),
        C.byref(info)), "ets_select_leaves")
    return keep[:leaf_node.shape[0]].astype(bool), info


def ets_bench_read_stream(hip_device: int, buf, nbytes: int, nontemporal: bool, sink,
                          sink_bytes: int, hip_stream=None):
    stream = None if hip_stream is None else C.c_void_p(int(hip_stream))
    _check(load_library().ets_bench_read_stream(int(hip_device), _dev_ptr(buf), int(nbytes),
                                                int(bool(nontemporal)), _dev_ptr(sink),
                                                int(sink_bytes), stream), "ets_bench_read_stream")


def ets_profile_read(ctx) -> EtsProfile:
    pr = EtsProfile()
    _check(load_library().ets_profile_read(ctx, C.byref(pr)), "ets_profile_read")
    return pr


class Context:
    """Owns one ets_ctx.  Thin convenience over the functions above."""

    def __init__(self, n_kv_heads: int, n_q_heads: int, head_dim: int, dtype: int,
                 hip_device: int, sm_scale: float = 0.0):
        self.shape = EtsShape(n_kv_heads, n_q_heads, head_dim, dtype, sm_scale)
        self._ctx = ets_create(self.shape, hip_device)

    def close(self):
        if self._ctx is not None:
            ets_destroy(self._ctx)
            self._ctx = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def __enter__(self):
        return self

    def __exit__(self, *exc):
        self.close()

    def set_option(self, key, value):
        ets_set_option(self._ctx, key, value)

    def set_kv_format(self, kv_format, k_scale=1.0, v_scale=1.0):
        ets_set_kv_format(self._ctx, kv_format, k_scale, v_scale)

    def set_kv_head_scales(self, k_scales, v_scales):
        if len(k_scales) != self.shape.n_kv_heads or len(v_scales) != self.shape.n_kv_heads:
            raise ValueError("one scale per kv head for each pool")
        ets_set_kv_head_scales(self._ctx, k_scales, v_scales)

    def plan(self, parent, tok_offset, n_tokens, leaf_node, mode=ETS_PLAN_TREE) -> EtsStats:
        ets_plan(self._ctx, parent, tok_offset, n_tokens, leaf_node, mode)
        return ets_plan_stats(self._ctx)

    def stats(self) -> EtsStats:
        return ets_plan_stats(self._ctx)

    def paths(self):
        return ets_plan_paths(self._ctx)

    def leaf_counts(self):
        return ets_plan_leaf_counts(self._ctx)

    def leaf_cover(self, leaf):
        return ets_plan_leaf_cover(self._ctx, leaf)

    def kv_append(self, k_pool, v_pool, pool_tokens, k_new, v_new, stream=None):
        ets_kv_append(self._ctx, k_pool, v_pool, pool_tokens, k_new, v_new, stream)

    def plan_advance(self, stream=None) -> bool:
        return ets_plan_advance(self._ctx, stream)

    def check(self) -> EtsPlanCheckReport:
        return ets_plan_check(self._ctx)

    def append_rows(self):
        return ets_plan_append_rows(self._ctx)

    def profile_read(self) -> EtsProfile:
        return ets_profile_read(self._ctx)

    def plan_prefill(self, parent, tok_offset, n_tokens, leaf_node) -> EtsPrefillStats:
        ets_plan_prefill(self._ctx, parent, tok_offset, n_tokens, leaf_node)
        return ets_prefill_plan_stats(self._ctx)

    def prefill_stats(self) -> EtsPrefillStats:
        return ets_prefill_plan_stats(self._ctx)

    def prefill_q_ptr(self):
        return ets_prefill_q_ptr(self._ctx)

    def prefill_cover(self, leaf, tok):
        return ets_prefill_cover(self._ctx, leaf, tok)

    def prefill(self, k_pool, v_pool, pool_tokens, q, out, lse, hip_stream=None):
        ets_tree_prefill_attn(self._ctx, k_pool, v_pool, pool_tokens, q, out, lse, hip_stream)

    def decode(self, k_pool, v_pool, pool_tokens, q, out, lse, workspace, workspace_bytes,
               hip_stream=None):
        ets_tree_decode_attn(self._ctx, k_pool, v_pool, pool_tokens, q, out, lse, workspace,
                             workspace_bytes, hip_stream)

    def decode_static(self, k_pool, v_pool, pool_tokens, q, out, lse, hip_stream=None):
        ets_tree_decode_attn_static(self._ctx, k_pool, v_pool, pool_tokens, q, out, lse,
                                    hip_stream)
