/*
 * libetsattn -- decode attention over a tree-structured KV cache (gfx950).
 *
 * The problem, as the ETS paper states it (Sec. 1; Sec. 3, factor 1; Sec. 4.1;
 * App. B): a PRM-guided parallel tree search keeps a tree whose nodes are
 * reasoning steps; a trajectory is the chain of step nodes from the root to a
 * leaf; every trajectory needs the KV state of all of its steps at every
 * generation step, and trajectories share the KV of their common ancestors.
 * The size of that shared state -- not FLOPs -- decides the run time because
 * decoding is memory-bandwidth bound.  This library is the kernel that turns
 * the sharing into fewer bytes moved: each live node's K/V is read from HBM
 * once per call for all the leaves beneath it.
 *
 * For every leaf query l (node v = leaf_node[l]) and query head j it returns
 *
 *     s_t      = sm_scale * <q[l,j,:], K[t,h,:]>   for every pool row t of every
 *                node on the root->v chain (v included), h = j / (Hq/Hkv)
 *     lse[l,j] = ln sum_t exp(s_t)                 (natural log)
 *     out[l,j] = sum_t exp(s_t - lse[l,j]) * V[t,h,:]
 *
 * (K[t,h,:] = row t of kv head h; in memory the pools are head-major, see
 * ets_tree_decode_attn) with no mask (the query is the newest position of its
 * trajectory).  A leaf
 * whose chain holds no tokens gets out = 0 and lse = -inf.
 *
 * Conventions
 *   - Plain C ABI.  "host" / "device" is stated for every pointer.
 *   - Status codes only; nothing throws or aborts across this boundary and on
 *     any error the outputs are left untouched.
 *   - A context is not thread safe; distinct contexts are independent.
 */
#ifndef ETSATTN_H
#define ETSATTN_H

#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct ets_ctx ets_ctx; /* opaque */

typedef enum {
    ETS_OK = 0,
    ETS_ERR_INVALID_ARG = 1, /* null pointer, negative size, misaligned buffer            */
    ETS_ERR_BAD_TREE = 2,    /* parent out of range or >= own index, negative length,      */
                             /* node rows outside the pool                                 */
    ETS_ERR_BAD_LEAF = 3,    /* leaf node id out of range                                  */
    ETS_ERR_UNSUPPORTED = 4, /* shape outside what the kernels are built for               */
    ETS_ERR_WORKSPACE = 5,   /* workspace smaller than ets_stats.workspace_bytes           */
    ETS_ERR_NO_PLAN = 6,     /* decode or query before a successful ets_plan               */
    ETS_ERR_HIP = 7,         /* a HIP runtime call failed, or the context has no device    */
    ETS_ERR_NOMEM = 8        /* host allocation failed                                     */
} ets_status;

typedef enum { ETS_F32 = 0, ETS_BF16 = 1 } ets_dtype;

/* Element type and head geometry of the pools and of q.
 * Supported: head_dim in {64, 128}; n_q_heads = G * n_kv_heads with G in
 * {1, 2, 4, 8} (query head j reads kv head j / G).  sm_scale <= 0 selects
 * 1/sqrt(head_dim).
 *
 * Which shapes get the method.  Reading every shared node once per call for all the
 * leaves beneath it is built for bfloat16 pools, head_dim 128 (the shapes of the paper's
 * models) and head_dim 64.  fp32 pools exist as a correctness path: they give the same
 * result through the per-leaf kernel, in which every leaf query reads its whole chain
 * itself (shared rows come out of the caches, not out of the plan), at the cost of the
 * flat baseline.  ets_stats.shares_nodes says which of the two a plan is, and with the
 * option "require_sharing" ets_plan refuses (ETS_ERR_UNSUPPORTED) a tree-mode plan that
 * would not share.  The wide kernel and step prefill are built for head_dim 128 only. */
typedef struct {
    int32_t n_kv_heads;
    int32_t n_q_heads;
    int32_t head_dim;
    int32_t dtype; /* ets_dtype of k_pool, v_pool and q */
    float sm_scale;
} ets_shape;

/* The search tree (ETS paper Sec. 4.1, App. B).  All arrays are HOST memory,
 * borrowed for the duration of ets_plan only.
 *   parent[i]     parent node of i, -1 for a root; parent[i] < i is required
 *                 (so cycles cannot be expressed); several roots are allowed.
 *   tok_offset[i] first pool row of node i; the node owns the n_tokens[i]
 *                 consecutive rows from there.  Nodes may be scattered in the
 *                 pool in any order; overlap is not checked.
 *   n_tokens[i]   >= 0; zero-length nodes contribute nothing.
 *   leaf_node[l]  node of leaf query l.  Any node may be named, interior ones
 *                 too, and a node may be named several times (a search samples
 *                 several continuations from one node); each entry has its own
 *                 query row. */
typedef struct {
    int32_t n_nodes;
    const int32_t* parent;
    const int64_t* tok_offset;
    const int32_t* n_tokens;
    int32_t n_leaves;
    const int32_t* leaf_node;
} ets_tree;

/* Statistics of the current plan.  unique_* counts the tokens of live nodes
 * (nodes with a leaf query at or beneath them) once; flat_* sums every leaf's
 * own chain -- what a kernel without tree awareness would read.  Bytes are K
 * plus V over all kv heads for ONE layer.  This is the per-tree analogue of
 * the paper's "KV size" proxy (Sec. 3), which sums it over the search steps. */
typedef struct {
    int64_t n_nodes;
    int64_t live_nodes;
    int64_t n_leaves;
    int64_t unique_tokens;
    int64_t flat_tokens;
    int64_t unique_kv_bytes;
    int64_t flat_kv_bytes;
    int64_t n_segments;      /* chains of live nodes with identical leaf sets            */
    int64_t n_partials;      /* partial results per query head, summed over the leaves   */
    int64_t n_stream_items;  /* work items of the per-leaf streaming kernel              */
    int64_t n_cascade_items; /* work items of the shared-node kernel                     */
    int64_t min_pool_tokens; /* pools must hold at least this many rows                  */
    int64_t workspace_bytes; /* device scratch ets_tree_decode_attn needs                */
    int64_t cascade_tokens;  /* unique tokens read (once) by the shared-node kernel      */
    int64_t stream_tokens;   /* tokens read by the streaming kernel, repeats included    */
    int64_t shares_nodes;    /* 1: shared nodes are read once per call (bf16 pools, tree */
                             /* mode); 0: every leaf reads its chain itself              */
    int64_t n_wide_items;    /* work items of the kernel for widely shared segments      */
    int64_t wide_tokens;     /* unique tokens of those segments (part of cascade_tokens) */
    int64_t merge_fused;     /* 1: the shared-node kernel merges the partials itself (no  */
                             /* merge launch); see the "fuse_merge" option                */
} ets_stats;

typedef enum {
    ETS_PLAN_TREE = 0, /* every live node is read once for all leaves beneath it        */
    ETS_PLAN_FLAT = 1  /* baseline: every leaf streams its whole chain by itself        */
} ets_plan_mode;

/* Creates a context for one head geometry on HIP device `hip_device`.
 * hip_device < 0 creates a host-only context: planning and the plan queries
 * work, ets_tree_decode_attn returns ETS_ERR_HIP.  *out is set only on ETS_OK
 * and is released with ets_destroy (NULL is accepted). */
ets_status ets_create(ets_ctx** out, const ets_shape* shape, int hip_device);
void ets_destroy(ets_ctx* ctx);

/* Integer planning, once per search step (the topology changes only when the
 * search prunes or expands: ETS paper Sec. 4.1).  Validates the tree, counts
 * the leaf queries beneath every node, merges chains of nodes with identical
 * leaf sets into segments, cuts the segments into work items and numbers the
 * partial results.  Copies what it needs: the caller's arrays are not
 * referenced after return.  On a device context the index arrays are uploaded
 * to device memory owned by the context; the call waits for the stream last
 * used with this context before it replaces them.  On error the previous plan
 * is dropped. */
ets_status ets_plan(ets_ctx* ctx, const ets_tree* tree, int mode /* ets_plan_mode */);

ets_status ets_plan_stats(const ets_ctx* ctx, ets_stats* out /* host */);

/* Root->leaf node chains of the planned tree in CSR form, for checking the
 * planner's indexing bit for bit: path_ptr[n_leaves + 1], path_nodes[cap]
 * (host).  *n_path_nodes (may be NULL) receives the total; if it exceeds cap
 * nothing is written to path_nodes and ETS_ERR_INVALID_ARG is returned. */
ets_status ets_plan_paths(const ets_ctx* ctx, int64_t* path_ptr, int32_t* path_nodes,
                          int64_t cap, int64_t* n_path_nodes);

/* leaf_count[n_nodes] (host): number of leaf queries at or beneath each node. */
ets_status ets_plan_leaf_counts(const ets_ctx* ctx, int64_t* leaf_count);

/* Pool rows the planned work items read on behalf of leaf query `leaf`, in
 * the order of its partial results: rows[cap] (host).  *n_rows and
 * *n_partials (either may be NULL) receive the counts.  With a correct plan
 * the rows are exactly the leaf's chain, root first, each row once. */
ets_status ets_plan_leaf_cover(const ets_ctx* ctx, int32_t leaf, int64_t* rows, int64_t cap,
                               int64_t* n_rows, int32_t* n_partials);

/* Replays on the host what the kernels of the current plans (decode and, when present,
 * step prefill) will read and write, from the same tables the kernels read: every step's
 * rows against min_pool_tokens, every index a wavefront loads from the per-leaf-query
 * tables against their padded size, the leaf queries whose q rows it fetches, the partial
 * rows it writes against the workspace.  ETS_OK when everything is in bounds;
 * ETS_ERR_BAD_TREE otherwise (a planner defect: the plan must not be launched).  *report
 * (HOST, may be NULL) is filled either way.  Works without a device. */
typedef struct {
    int64_t decode_items;         /* work items replayed (both kernels)                        */
    int64_t prefill_items;        /* 0 without a prefill plan                                  */
    int64_t entry_table_entries;  /* entries of each per-leaf-query table, padding included    */
    int64_t max_entry_index;      /* highest entry index any wavefront loads                   */
    int64_t max_entry_overreach;  /* entries loaded past an item's own last entry, at most     */
    int64_t max_pool_row;         /* highest pool row any step names                           */
    int64_t max_partial_row;      /* highest (partial, head) row written                       */
    int64_t violations;
} ets_plan_check_report;
ets_status ets_plan_check(const ets_ctx* ctx, ets_plan_check_report* report);

/* Decode-step advance.  Between two decode tokens of one search step the tree's
 * topology is fixed and only the nodes that hold leaf queries grow, by one token each
 * (ETS paper, Sec. 4.1: the tree changes once per step; App. B: leaves are the latest
 * steps).  Per decode token the caller runs, on one stream and in this order:
 *     ets_plan_advance                      once: the plan now counts the new token
 *     for every layer:  ets_kv_append       the new token's K/V rows into that layer's pools
 *                       ets_tree_decode_attn
 * (a layer's K/V of the new token depend on the previous layer's attention output, so the
 * appends cannot all precede the first attention call; this order serves one pool and
 * many alike).
 *
 * ets_plan_advance makes every distinct node of leaf_node one token longer in the plan
 * (the library's copy of the tree, statistics, and the step lists on the device, the
 * latter through a small kernel on hip_stream).  The step lists have room for at
 * least 32 advances; when it is used up the call plans again from its grown copy of
 * the tree (this waits for the context's previous work, like ets_plan) and sets
 * *replanned (may be NULL) to 1: n_partials and workspace_bytes may then have changed
 * and are to be read again with ets_plan_stats.  Works without a device too.
 *
 * ets_kv_append writes, for every distinct node of leaf_node, one row of K and V at the
 * node's NEWEST row as the plan counts it, tok_offset[node] + n_tokens[node] - 1: after an
 * ets_plan_advance that is the row of the token the advance added (which the caller must
 * have reserved behind the node); on a plan that was just built it is the last row the
 * caller's tree named.  The row does not depend on how many layers have been appended
 * before.  A node without rows is skipped.
 *   k_pool, v_pool  DEVICE, as in ets_tree_decode_attn (same element size), written
 *   pool_tokens     rows per head plane, as in ets_tree_decode_attn; must exceed
 *                   every written row, else ETS_ERR_INVALID_ARG and nothing is written
 *   k_new, v_new    DEVICE, [n_leaves][n_kv_heads][head_dim] of the pools' element type,
 *                   16-byte aligned: row l is the new token of leaf query l; when several leaf
 *                   queries sit on one node, the first of them supplies the row
 * Asynchronous on hip_stream; no allocation.
 *
 * ets_plan_append_rows reports where ets_kv_append would write now: rows[l] (HOST,
 * [n_leaves]) = the pool row that receives row l of k_new / v_new, or -1 when leaf query l
 * supplies none (a later leaf query of a node, or a node without rows). */
ets_status ets_kv_append(ets_ctx* ctx, void* k_pool, void* v_pool, int64_t pool_tokens,
                         const void* k_new, const void* v_new, void* hip_stream);
ets_status ets_plan_advance(ets_ctx* ctx, void* hip_stream, int32_t* replanned);
ets_status ets_plan_append_rows(const ets_ctx* ctx, int64_t* rows);

/* Planner knobs, effective from the next ets_plan.  Keys:
 *   "stream_chunk"   max tokens per work item of a single leaf query (0 = auto)
 *   "cascade_chunk"  max tokens per work item of a shared segment (0 = auto)
 *   "cascade_min_leaves"  a segment shared by at least this many leaf queries is
 *                    read once for all of them; below it every leaf reads the
 *                    segment itself (default 2; 0 = never share)
 *   "cascade_rows"   query rows (leaf queries x query heads per kv head) that one
 *                    work item of a shared segment serves: 16, 32 or 64
 *                    (default 64); a segment with more rows is read by several
 *                    items
 *   "wide_rows"      a shared segment with more query rows than this is read by the
 *                    wide kernel (256 query rows per work item, bound by the matrix
 *                    cores; head_dim 128) instead of by several items of "cascade_rows" rows each
 *                    (0 or -1 = never, the default: items of 64 rows in the merged launch
 *                    order measure 5-6 % faster on every configuration tried)
 *   "fuse_merge"     1 = the shared-node kernel also merges: the wavefront that stores a
 *                    leaf query's last partial result combines them, and no merge kernel
 *                    is launched.  Only for plans whose partial results all come from
 *                    that kernel (bf16 or E4M3 pools, no wide items),
 *                    in which every leaf query has a token, and whose workspace is below
 *                    2 GiB; other plans keep the merge launch (ets_stats.merge_fused
 *                    tells).  Same results bit for bit.  The arrival counters belong to
 *                    the context: calls of one context must then not overlap on the
 *                    device.  0 or -1 = separate merge launch, the default: it measures
 *                    faster (the device-scope round trips at the end of the last item
 *                    cost more than the launch they replace)
 *   "interleave"     1 (default) = the workgroups that hold small items are spread through
 *                    the launch order; 0 = they follow all the others
 *   "wave_items"     a work item of at most 16 query rows and at most this many
 *                    tokens is walked by a single wavefront, four such items to
 *                    a workgroup (default 512; 0 = every item gets a workgroup)
 *   "require_sharing"  1 = ets_plan in tree mode returns ETS_ERR_UNSUPPORTED when this
 *                    context cannot read shared nodes once (fp32 pools, or "mfma" /
 *                    "cascade_min_leaves" set to 0) instead
 *                    of falling back to per-leaf reads; 0 (default) = fall back
 *   "mfma"           1 (default) = matrix-core kernel for bf16 pools; 0 = vector-ALU
 *                    kernel for every shape (each leaf then reads its whole chain
 *                    itself)
 *   "out_bf16"       1 = ets_tree_decode_attn writes `out` as bfloat16 (the merged fp32
 *                    result rounded to nearest even), for a consumer that takes the next
 *                    projection's input in bf16; 0 (default) = fp32.  Effective from
 *                    the next decode call; lse stays fp32
 *   "profile"        1 = record kernel times (see ets_profile_read), 0 = off
 * Unknown key or negative value (other than -1 for wide_rows, fuse_merge): ETS_ERR_INVALID_ARG. */
ets_status ets_set_option(ets_ctx* ctx, const char* key, int64_t value);

/* Storage format of the K/V pools.  The search is bound by the bytes of KV state that
 * every generation step reads (ETS paper Sec. 1; Sec. 3, factor 1); a cache that stores
 * K and V in 8 bits halves them.
 *   ETS_KV_NATIVE    pools hold shape.dtype elements (default)
 *   ETS_KV_FP8_E4M3  pools hold one byte per element: codes of the OCP 8-bit floating
 *                    point format E4M3 (1 sign, 4 exponent bits with bias 7, 3 mantissa
 *                    bits; no infinities; S.1111.111 is NaN), and
 *                        K[t,h,d] = k_scale * value(k_code),  V[t,h,d] = v_scale * value(v_code)
 *                    with one positive finite scale per pool.  Layout, row numbering and
 *                    alignment are as for native pools with 1-byte elements; q stays
 *                    bf16.  Only for bf16 contexts (ETS_ERR_UNSUPPORTED
 *                    otherwise) and with the "mfma" option on (else ets_tree_decode_attn
 *                    returns ETS_ERR_UNSUPPORTED).  ets_kv_append then copies 1-byte
 *                    elements (k_new, v_new hold codes); step prefill reads such pools
 *                    as well (its q stays bf16, its output fp32).
 * The scales are ignored for ETS_KV_NATIVE.  The call drops the current plans: run
 * ets_plan again (byte statistics and work-item sizes follow the element size). */
typedef enum { ETS_KV_NATIVE = 0, ETS_KV_FP8_E4M3 = 1 } ets_kv_format;
ets_status ets_set_kv_format(ets_ctx* ctx, int kv_format /* ets_kv_format */, float k_scale,
                             float v_scale);
/* One scale per kv head instead of one per pool, for ETS_KV_FP8_E4M3 pools:
 *     K[t,h,d] = k_scales[h] * value(k_code),  V[t,h,d] = v_scales[h] * value(v_code).
 * k_scales, v_scales: HOST, [n_kv_heads], positive and finite (else ETS_ERR_INVALID_ARG and
 * nothing changes); copied.  Call after ets_set_kv_format(ctx, ETS_KV_FP8_E4M3, ...)
 * (ETS_ERR_INVALID_ARG for native pools; a later ets_set_kv_format sets all heads to its
 * two scales again).  At most 64 kv heads (ETS_ERR_UNSUPPORTED beyond).  The plans stay
 * valid; calls enqueued earlier keep the scales they were enqueued with. */
ets_status ets_set_kv_head_scales(ets_ctx* ctx, const float* k_scales, const float* v_scales);

/* One layer of decode attention for every leaf query of the planned tree.
 *   k_pool, v_pool  DEVICE, [n_kv_heads][pool_tokens][head_dim] of shape.dtype (of E4M3
 *                   codes after ets_set_kv_format), 16-byte aligned: one plane of pool_tokens rows per kv head, so
 *                   that the rows of a node are contiguous within a head (pool row
 *                   t of head h starts at element (h * pool_tokens + t) * head_dim)
 *   pool_tokens     rows per head plane of BOTH pools, i.e. the plane stride (not
 *                   merely a bound); >= stats.min_pool_tokens, else ETS_ERR_BAD_TREE
 *   q               DEVICE, [n_leaves][n_q_heads][head_dim] of shape.dtype, 16-byte aligned
 *   out             DEVICE, [n_leaves][n_q_heads][head_dim] float (bfloat16 with the
 *                   "out_bf16" option), 16-byte aligned
 *   lse             DEVICE, [n_leaves][n_q_heads] float
 *   workspace       DEVICE, >= stats.workspace_bytes, 16-byte aligned, contents
 *                   undefined before and after; may be NULL when that is 0
 *   hip_stream      hipStream_t (NULL = the default stream) of the context's device
 * The call only enqueues kernels on hip_stream: it does not synchronise and
 * does not allocate.  All buffers stay owned by the caller and must stay valid
 * until the stream has passed the call.  A plan may be reused for any number
 * of calls (layers, decode steps) while the tree is unchanged.  The result is
 * bitwise reproducible from run to run (no floating-point atomics). */
ets_status ets_tree_decode_attn(ets_ctx* ctx, const void* k_pool, const void* v_pool,
                                int64_t pool_tokens, const void* q, void* out, float* lse,
                                void* workspace, int64_t workspace_bytes, void* hip_stream);

/* The same call for callers that cannot allocate device memory or hand over a workspace:
 * code under HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.
 * The partial results go to a buffer of ETS_STATIC_SCRATCH_BYTES that is part of the
 * library's device image (one per GPU, held until the process ends; its address on the
 * context's device is looked up by ets_create).  Arguments and result are those of
 * ets_tree_decode_attn without `workspace`; same kernels, same bits.
 *   - a plan whose stats.workspace_bytes exceeds ETS_STATIC_SCRATCH_BYTES is refused with
 *     ETS_ERR_WORKSPACE (nothing is enqueued);
 *   - the call allocates nothing on host or device and records no profiling events
 *     (the "profile" option does not apply to it);
 *   - every call on one GPU uses that GPU's one buffer, whatever the context: calls that
 *     may overlap on a GPU (different streams without ordering between them) race.  Calls
 *     on one stream, or ordered by events, are safe; nothing has to be cleared between
 *     calls (every partial row is written before it is read). */
#define ETS_STATIC_SCRATCH_BYTES (32ll << 20)
ets_status ets_tree_decode_attn_static(ets_ctx* ctx, const void* k_pool, const void* v_pool,
                                       int64_t pool_tokens, const void* q, void* out, float* lse,
                                       void* hip_stream);

/* Kernel times for benchmarks.  After ets_set_option(ctx, "profile", 1) every
 * ets_tree_decode_attn call brackets its kernels with HIP events on the call's
 * stream (this mode may create events, i.e. allocate; at most 8192 calls are
 * kept between reads).  ets_profile_read waits for the last recorded call,
 * returns the summed kernel times since the previous read and clears them. */
typedef struct {
    int64_t calls;
    double stream_ms;  /* per-leaf streaming kernel                  */
    double cascade_ms; /* shared-node kernel                         */
    double merge_ms;   /* log-sum-exp merge kernel                   */
    double wide_ms;    /* kernel for widely shared segments          */
} ets_profile;
ets_status ets_profile_read(ets_ctx* ctx, ets_profile* out /* host */);

/* Benchmark hook: one plain streaming read of buf[0, bytes) on hip_device (16 bytes per
 * lane and load, consecutive lanes on consecutive addresses; bytes past the last multiple
 * of 16 are not read), so that a benchmark can state the attention kernels' unique-KV
 * GB/s also against the read rate this device sustains in the same run, not only against
 * the published HBM peak (the paper's premise, Sec. 1 and Sec. 3, is that these reads bound
 * the search).  nontemporal != 0 uses loads that bypass cache allocation, as the
 * attention kernel does for rows nobody re-reads.
 *   buf    DEVICE, 16-byte aligned
 *   sink   DEVICE, sink_bytes >= 16384, 4-byte aligned, zero or anything: one word per
 *          workgroup is XOR-ed into it (keeps the loads alive; contents meaningless)
 * Asynchronous on hip_stream; no allocation.  ETS_ERR_WORKSPACE when sink is too small. */
ets_status ets_bench_read_stream(int hip_device, const void* buf, int64_t bytes, int nontemporal,
                                 void* sink, int64_t sink_bytes, void* hip_stream);

/* ---- Step prefill: scoring a newly generated step with the reward model ----------
 *
 * The search scores every candidate step with a process reward model (ETS paper,
 * Abstract; Sec. 1; Sec. 5.1: the PRM score at each step is that step's reward).  The
 * reward model is a transformer over the same tree of cached steps, so scoring the
 * steps just generated is a prefill of their tokens: EVERY token i of the node
 * v = leaf_node[l] of leaf query l is a query; it sees all rows of v's strict
 * ancestors and rows 0..i of v itself (causal inside the new step, whose K/V rows the
 * caller has already written to the pools), and
 *
 *     lse[r,j] = ln sum_t exp(sm_scale * <q[r,j,:], K[t,h,:]>)     over the rows t it sees
 *     out[r,j] = sum_t exp(s_t - lse[r,j]) * V[t,h,:],   h = j / (Hq/Hkv)
 *
 * where r = q_ptr[l] + i numbers the query rows leaf query by leaf query:
 * q_ptr[l] = sum of n_tokens[leaf_node[l']] over l' < l (duplicate leaf queries on a
 * node own separate rows; a node without tokens owns none).
 *
 * Built for bf16 pools with head_dim 128 (ETS_ERR_UNSUPPORTED otherwise).  The plan is
 * separate from the decode plan of the same context; neither disturbs the other. */
typedef struct {
    int64_t n_leaves;
    int64_t n_q_rows;          /* query rows = sum of the leaf queries' node lengths      */
    int64_t n_items;           /* work items: blocks of rows_per_item / G query tokens    */
    int64_t n_runs;            /* entries of the run lists on the device                  */
    int64_t rows_per_item;     /* query rows (tokens x heads of a kv head) per work item  */
    int64_t unique_tokens;     /* rows of the nodes on some leaf query's chain, once      */
    int64_t unique_kv_bytes;   /* K plus V of those rows over all kv heads, one layer     */
    int64_t streamed_tokens;   /* rows walked, summed over the work items                 */
    int64_t streamed_kv_bytes; /* the same in bytes: what L2 and HBM serve together       */
    int64_t visible_pairs;     /* (query token, visible row) pairs                        */
    int64_t flops;             /* 4 * head_dim * n_q_heads * visible_pairs                */
    int64_t min_pool_tokens;   /* pools must hold at least this many rows per head        */
} ets_prefill_stats;

/* Plans step prefill for `tree` (host arrays, borrowed for the call; same rules and
 * errors as ets_plan).  Waits for the context's previous work before it replaces the
 * device tables. */
ets_status ets_plan_prefill(ets_ctx* ctx, const ets_tree* tree);
ets_status ets_prefill_plan_stats(const ets_ctx* ctx, ets_prefill_stats* out /* host */);
/* q_ptr: HOST, [n_leaves + 1], the first query row of every leaf query. */
ets_status ets_prefill_q_ptr(const ets_ctx* ctx, int64_t* q_ptr);
/* For checking the indexing bit for bit: the pool rows that query token `tok` of leaf
 * query `leaf` sees according to the work items and their masks, in reading order.
 * rows: HOST, capacity cap; *n_rows (may be NULL) receives the count; too small a cap
 * or tok outside the node gives ETS_ERR_INVALID_ARG. */
ets_status ets_prefill_cover(const ets_ctx* ctx, int32_t leaf, int32_t tok, int64_t* rows,
                             int64_t cap, int64_t* n_rows);
/* One layer of step-prefill attention.
 *   k_pool, v_pool, pool_tokens   as in ets_tree_decode_attn (E4M3 codes after
 *         ets_set_kv_format, which has to precede ets_plan_prefill)
 *   q     DEVICE, [n_q_rows][n_q_heads][head_dim] bf16, 16-byte aligned
 *   out   DEVICE, [n_q_rows][n_q_heads][head_dim] float, 16-byte aligned
 *   lse   DEVICE, [n_q_rows][n_q_heads] float
 * Enqueues one kernel per 65535 work items on hip_stream; no workspace, no allocation,
 * no synchronisation; bitwise reproducible.  ETS_ERR_NO_PLAN before ets_plan_prefill,
 * ETS_ERR_HIP on a host-only context. */
ets_status ets_tree_prefill_attn(ets_ctx* ctx, const void* k_pool, const void* v_pool,
                                 int64_t pool_tokens, const void* q, float* out, float* lse,
                                 void* hip_stream);

/* ---- The selection step that produces the tree (host only, no context) ---------------
 *
 * ETS decides at every search step which trajectories to keep (ETS paper Sec. 4.1-4.2;
 * App. B).  ets_rebase_weights is Eq. 1 (and Eq. 3 when called on the kept set): the
 * trajectories are visited from the highest reward to the lowest, equal rewards in input
 * order; trajectory i receives W_i = ceil(N_i e_i / sum_{k in A_i} e_k) continuations,
 * e = exp(R / temperature), A_i = i and everything after it, N_1 = budget and
 * N_{i+1} = N_i - W_i (the recurrence the paper implies); fp64.
 *   rewards  HOST [n];  weights  HOST [n], written;  budget >= 0, temperature > 0.
 *
 * ets_select_leaves maximises the cost model of Eq. 4 (Eq. 2 when cluster is NULL; the ILPs of App. B,
 * Eq. 7 and Eq. 6) exactly:
 *     sum_{i kept} W_i / sum_i W_i  -  lambda_b |V_S| / |V_A|  +  lambda_d |C_S| / |C_A|
 * V_A = the nodes with a leaf at or beneath them, V_S = those with a KEPT leaf at or
 * beneath them, C_A / C_S = the clusters present / with a kept leaf (the text's reading
 * of the cluster constraint: a cluster counts when ANY of its leaves is kept), at least
 * one leaf kept.
 *   tree      only parent and leaf_node are read; the leaves must be distinct nodes and
 *             none may lie beneath another (ETS_ERR_BAD_LEAF)
 *   weights   HOST [n_leaves], >= 0, not all zero
 *   cluster   HOST [n_leaves] arbitrary ids, or NULL for no coverage term
 *   node_limit  branch-and-bound nodes to spend (<= 0: 2^22); when it is reached the best
 *             set found so far is returned with info->optimal = 0
 *   keep      HOST [n_leaves], written: 1 = kept
 *   info      HOST, may be NULL */
typedef struct {
    double objective;
    int64_t kept_nodes;    /* |V_S| */
    int64_t live_nodes;    /* |V_A| */
    int64_t kept_clusters; /* |C_S| */
    int64_t clusters;      /* |C_A|, 0 without coverage term */
    int64_t bb_nodes;      /* branch-and-bound nodes visited */
    int32_t optimal;
    int32_t pad;
} ets_select_info;
ets_status ets_rebase_weights(int32_t n, const double* rewards, int32_t budget,
                              double temperature, int32_t* weights);
ets_status ets_select_leaves(const ets_tree* tree, const int32_t* weights, const int32_t* cluster,
                             double lambda_b, double lambda_d, int64_t node_limit, uint8_t* keep,
                             ets_select_info* info);

/* Static string for a status code. */
const char* ets_strerror(int status);

#ifdef __cplusplus
}
#endif
#endif /* ETSATTN_H */
