/*
 * CPU oracle for decode attention over a tree-structured KV cache.
 *
 * TEST INFRASTRUCTURE ONLY.  Nothing on the product path may call this file;
 * it exists so that the GPU library can be checked against a slow, plain,
 * independent statement of the result.  It shares no code with the library.
 *
 * What it computes (ETS paper, Sec. 1, Sec. 3 factor 1, Sec. 4.1 and App. B:
 * a search tree whose nodes are reasoning steps, a trajectory being the chain
 * of step nodes from the root down to a leaf, every trajectory needing the KV
 * state of all its steps and trajectories sharing the KV of common ancestors):
 * for every leaf query l (node v = leaf_node[l]) and query head j
 *
 *   path(l)  = nodes from the root down to v inclusive
 *   T(l)     = the pool rows of those nodes, concatenated in path order
 *   h        = j / G                       (G = Hq / Hkv, contiguous GQA groups)
 *   s_t      = scale * sum_d q[l,j,d] * K[t,h,d]              for t in T(l)
 *   LSE[l,j] = m + ln sum_t exp(s_t - m),  m = max_t s_t      (natural log)
 *   O[l,j,:] = sum_t exp(s_t - LSE) * V[t,h,:]
 *
 * all in fp64 after exact widening of the fp32 / bfloat16 inputs (fp64 inputs are taken
 * as they are).  K[t,h,:] and
 * V[t,h,:] are D consecutive elements starting at element t * tok_stride +
 * h * head_stride of their pool, so that any memory order of (row, head) can be
 * described.  An empty
 * path gives O = 0 and LSE = -inf.  The paper treats the model as a black box,
 * so the attention formula is the standard scaled-dot-product one; the paper
 * supplies the tree and sharing semantics.
 *
 * Step prefill (scoring a newly generated step with the reward model: the paper's
 * search scores every candidate step, Abstract, Sec. 1 and Sec. 5.1; the reward
 * model is a transformer with the same tree of cached steps): every token i of the
 * leaf node v of a leaf query carries a query vector of its own; it sees all rows of
 * v's strict ancestors and rows 0..i of v itself (causal inside the new step), and
 * the same three formulas apply to that row set.  Query rows are numbered leaf query
 * by leaf query: row q_ptr[l] + i with q_ptr[l] = sum of n_tokens[leaf_node[l']]
 * over l' < l.
 *
 * Also here, for pinning the identity the GPU path relies on: the partial
 * (unnormalised) result of an arbitrary token subset and the log-sum-exp merge
 * of several partials.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

/* element types of the inputs; ORACLE_F64 takes values that are already doubles (pools
 * that a test dequantised itself from an 8-bit code and a scale) */
enum { ORACLE_F32 = 0, ORACLE_BF16 = 1, ORACLE_F64 = 2 };

static double load_elem(const void* base, int dtype, int64_t idx) {
    if (dtype == ORACLE_F64) return ((const double*)base)[idx];
    if (dtype == ORACLE_F32) return (double)((const float*)base)[idx];
    uint32_t bits = (uint32_t)((const uint16_t*)base)[idx] << 16;
    float f;
    memcpy(&f, &bits, sizeof f);
    return (double)f;
}

int ets_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* Checks the tree arrays the way the paper's tree is defined: every node has
 * at most one parent that was created before it.  0 = fine. */
int ets_oracle_check_tree(int32_t n_nodes, const int32_t* parent, const int64_t* tok_offset,
                          const int32_t* n_tokens, int32_t n_leaves, const int32_t* leaf_node,
                          int64_t pool_tokens) {
    for (int32_t i = 0; i < n_nodes; ++i) {
        if (parent[i] < -1 || parent[i] >= i) return 1;
        if (n_tokens[i] < 0) return 2;
        if (tok_offset[i] < 0 || tok_offset[i] + n_tokens[i] > pool_tokens) return 3;
    }
    for (int32_t l = 0; l < n_leaves; ++l)
        if (leaf_node[l] < 0 || leaf_node[l] >= n_nodes) return 4;
    return 0;
}

/* Depth (number of nodes) of the root->node chain. */
static int64_t chain_len(const int32_t* parent, int32_t v) {
    int64_t n = 0;
    for (int32_t x = v; x >= 0; x = parent[x]) ++n;
    return n;
}

/* Root->leaf node lists in CSR form.  path_ptr has n_leaves + 1 entries.
 * Returns the total number of path nodes, or -1 when cap is too small. */
int64_t ets_oracle_paths(int32_t n_nodes, const int32_t* parent, int32_t n_leaves,
                         const int32_t* leaf_node, int64_t* path_ptr, int32_t* path_nodes,
                         int64_t cap) {
    (void)n_nodes;
    int64_t pos = 0;
    for (int32_t l = 0; l < n_leaves; ++l) {
        path_ptr[l] = pos;
        int64_t len = chain_len(parent, leaf_node[l]);
        if (pos + len > cap) return -1;
        int64_t k = len;
        for (int32_t x = leaf_node[l]; x >= 0; x = parent[x]) path_nodes[pos + --k] = x;
        pos += len;
    }
    path_ptr[n_leaves] = pos;
    return pos;
}

/* Per-node number of leaf queries at or beneath the node, and the totals the
 * paper's KV-size proxy is built from: tokens of live nodes counted once
 * (unique) and tokens summed over every leaf's own path (flat). */
void ets_oracle_tree_stats(int32_t n_nodes, const int32_t* parent, const int32_t* n_tokens,
                           int32_t n_leaves, const int32_t* leaf_node, int64_t* leaf_count,
                           int64_t* unique_tokens, int64_t* flat_tokens, int64_t* live_nodes) {
    for (int32_t i = 0; i < n_nodes; ++i) leaf_count[i] = 0;
    int64_t flat = 0;
    for (int32_t l = 0; l < n_leaves; ++l)
        for (int32_t x = leaf_node[l]; x >= 0; x = parent[x]) {
            leaf_count[x] += 1;
            flat += n_tokens[x];
        }
    int64_t uniq = 0, live = 0;
    for (int32_t i = 0; i < n_nodes; ++i)
        if (leaf_count[i] > 0) {
            uniq += n_tokens[i];
            live += 1;
        }
    *unique_tokens = uniq;
    *flat_tokens = flat;
    *live_nodes = live;
}

/* Attention of query row q_row, query head j, over the path of node v: every row of v's
 * strict ancestors and the first own_rows rows of v itself (own_rows < 0: all of them).
 * out has D entries. */
static int attn_one(const int32_t* parent, const int64_t* tok_offset, const int32_t* n_tokens,
                    int32_t v, int64_t own_rows, int32_t Hkv, int32_t Hq, int32_t D, int dtype,
                    double scale, const void* k_pool, const void* v_pool, int64_t tok_stride,
                    int64_t head_stride, const void* q, int64_t q_row, int32_t j, double* out,
                    double* lse) {
    const int32_t G = Hq / Hkv;
    const int32_t h = j / G;
    const int64_t depth = chain_len(parent, v);
    int32_t* path = (int32_t*)malloc(sizeof(int32_t) * (size_t)(depth > 0 ? depth : 1));
    if (!path) return 1;
    int64_t k = depth;
    for (int32_t x = v; x >= 0; x = parent[x]) path[--k] = x;

    if (own_rows < 0 || own_rows > n_tokens[v]) own_rows = n_tokens[v];
    int64_t n_p = own_rows;
    for (int64_t i = 0; i + 1 < depth; ++i) n_p += n_tokens[path[i]];
    for (int32_t d = 0; d < D; ++d) out[d] = 0.0;
    if (n_p == 0) {
        *lse = -INFINITY;
        free(path);
        return 0;
    }
    int64_t* rows = (int64_t*)malloc(sizeof(int64_t) * (size_t)n_p);
    double* s = (double*)malloc(sizeof(double) * (size_t)n_p);
    if (!rows || !s) {
        free(path); free(rows); free(s);
        return 1;
    }
    int64_t t = 0;
    for (int64_t i = 0; i < depth; ++i) {
        const int64_t n_vis = i + 1 < depth ? n_tokens[path[i]] : own_rows;
        for (int64_t r = 0; r < n_vis; ++r) rows[t++] = tok_offset[path[i]] + r;
    }

    const int64_t qbase = (q_row * Hq + j) * D;
    double m = -INFINITY;
    for (t = 0; t < n_p; ++t) {
        const int64_t kbase = rows[t] * tok_stride + h * head_stride;
        double acc = 0.0;
        for (int32_t d = 0; d < D; ++d)
            acc += load_elem(q, dtype, qbase + d) * load_elem(k_pool, dtype, kbase + d);
        s[t] = scale * acc;
        if (s[t] > m) m = s[t];
    }
    double sum = 0.0;
    for (t = 0; t < n_p; ++t) sum += exp(s[t] - m);
    *lse = m + log(sum);
    for (t = 0; t < n_p; ++t) {
        const double w = exp(s[t] - *lse);
        const int64_t vbase = rows[t] * tok_stride + h * head_stride;
        for (int32_t d = 0; d < D; ++d) out[d] += w * load_elem(v_pool, dtype, vbase + d);
    }
    free(path); free(rows); free(s);
    return 0;
}

/* Selected (leaf, head) rows: out [n_sel][D], lse [n_sel].  scale <= 0 means
 * 1/sqrt(D). */
int ets_oracle_attn_rows(int32_t n_nodes, const int32_t* parent, const int64_t* tok_offset,
                         const int32_t* n_tokens, int32_t n_leaves, const int32_t* leaf_node,
                         int32_t Hkv, int32_t Hq, int32_t D, int dtype, double scale,
                         const void* k_pool, const void* v_pool, int64_t tok_stride,
                         int64_t head_stride, const void* q, int64_t n_sel,
                         const int32_t* sel_leaf, const int32_t* sel_head, double* out,
                         double* lse) {
    (void)n_nodes;
    if (Hkv <= 0 || Hq % Hkv != 0 || D <= 0) return 2;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_sel; ++i) {
        const int32_t l = sel_leaf[i], j = sel_head[i];
        if (l < 0 || l >= n_leaves || j < 0 || j >= Hq) {
#pragma omp atomic write
            err = 3;
            continue;
        }
        int e = attn_one(parent, tok_offset, n_tokens, leaf_node[l], -1, Hkv, Hq, D, dtype, scale,
                         k_pool, v_pool, tok_stride, head_stride, q, l, j, out + i * D, lse + i);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

/* Every (leaf, head): out [L][Hq][D], lse [L][Hq]. */
int ets_oracle_attn(int32_t n_nodes, const int32_t* parent, const int64_t* tok_offset,
                    const int32_t* n_tokens, int32_t n_leaves, const int32_t* leaf_node,
                    int32_t Hkv, int32_t Hq, int32_t D, int dtype, double scale,
                    const void* k_pool, const void* v_pool, int64_t tok_stride,
                    int64_t head_stride, const void* q, double* out, double* lse) {
    (void)n_nodes;
    if (Hkv <= 0 || Hq % Hkv != 0 || D <= 0) return 2;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
    int err = 0;
    const int64_t n = (int64_t)n_leaves * Hq;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n; ++i) {
        const int32_t l = (int32_t)(i / Hq), j = (int32_t)(i % Hq);
        int e = attn_one(parent, tok_offset, n_tokens, leaf_node[l], -1, Hkv, Hq, D, dtype, scale,
                         k_pool, v_pool, tok_stride, head_stride, q, l, j, out + i * D, lse + i);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    return err;
}

/* Step prefill, selected (leaf query, token of its node, query head) triples:
 * out [n_sel][D], lse [n_sel].  q is [sum of leaf node lengths][Hq][D]. */
int ets_oracle_prefill_rows(int32_t n_nodes, const int32_t* parent, const int64_t* tok_offset,
                            const int32_t* n_tokens, int32_t n_leaves, const int32_t* leaf_node,
                            int32_t Hkv, int32_t Hq, int32_t D, int dtype, double scale,
                            const void* k_pool, const void* v_pool, int64_t tok_stride,
                            int64_t head_stride, const void* q, int64_t n_sel,
                            const int32_t* sel_leaf, const int32_t* sel_tok,
                            const int32_t* sel_head, double* out, double* lse) {
    (void)n_nodes;
    if (Hkv <= 0 || Hq % Hkv != 0 || D <= 0) return 2;
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
    int64_t* q_ptr = (int64_t*)malloc(sizeof(int64_t) * ((size_t)n_leaves + 1));
    if (!q_ptr) return 1;
    q_ptr[0] = 0;
    for (int32_t l = 0; l < n_leaves; ++l) q_ptr[l + 1] = q_ptr[l] + n_tokens[leaf_node[l]];
    int err = 0;
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t i = 0; i < n_sel; ++i) {
        const int32_t l = sel_leaf[i], tok = sel_tok[i], j = sel_head[i];
        if (l < 0 || l >= n_leaves || j < 0 || j >= Hq || tok < 0 ||
            tok >= n_tokens[leaf_node[l]]) {
#pragma omp atomic write
            err = 3;
            continue;
        }
        int e = attn_one(parent, tok_offset, n_tokens, leaf_node[l], (int64_t)tok + 1, Hkv, Hq, D,
                         dtype, scale, k_pool, v_pool, tok_stride, head_stride, q,
                         q_ptr[l] + tok, j, out + i * D, lse + i);
        if (e) {
#pragma omp atomic write
            err = e;
        }
    }
    free(q_ptr);
    return err;
}

/* Partial result of one query vector over an explicit list of pool rows:
 *   m = max_t s_t,  l = sum_t exp(s_t - m),  o[d] = sum_t exp(s_t - m) V[t,h,d]
 * (unnormalised).  n_rows == 0 gives m = -inf, l = 0, o = 0. */
void ets_oracle_partial(int32_t D, int dtype, double scale, const void* k_pool,
                        const void* v_pool, int64_t tok_stride, int64_t head_stride,
                        const double* qvec, int32_t h, int64_t n_rows,
                        const int64_t* rows, double* o, double* m_out, double* l_out) {
    if (scale <= 0.0) scale = 1.0 / sqrt((double)D);
    for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
    *m_out = -INFINITY;
    *l_out = 0.0;
    if (n_rows == 0) return;
    double* s = (double*)malloc(sizeof(double) * (size_t)n_rows);
    double m = -INFINITY;
    for (int64_t t = 0; t < n_rows; ++t) {
        const int64_t kbase = rows[t] * tok_stride + h * head_stride;
        double acc = 0.0;
        for (int32_t d = 0; d < D; ++d) acc += qvec[d] * load_elem(k_pool, dtype, kbase + d);
        s[t] = scale * acc;
        if (s[t] > m) m = s[t];
    }
    double l = 0.0;
    for (int64_t t = 0; t < n_rows; ++t) {
        const double p = exp(s[t] - m);
        l += p;
        const int64_t vbase = rows[t] * tok_stride + h * head_stride;
        for (int32_t d = 0; d < D; ++d) o[d] += p * load_elem(v_pool, dtype, vbase + d);
    }
    free(s);
    *m_out = m;
    *l_out = l;
}

/* Log-sum-exp merge of n partials (o [n][D], m [n], l [n]) in the given order:
 *   m* = max m_i, w_i = exp(m_i - m*), l* = sum l_i w_i,
 *   out = sum o_i w_i / l*,  lse = m* + ln l*.
 * Partials with l == 0 (empty subsets) contribute nothing. */
void ets_oracle_merge(int32_t D, int64_t n, const double* o, const double* m, const double* l,
                      double* out, double* lse) {
    double ms = -INFINITY;
    for (int64_t i = 0; i < n; ++i)
        if (l[i] > 0.0 && m[i] > ms) ms = m[i];
    for (int32_t d = 0; d < D; ++d) out[d] = 0.0;
    if (ms == -INFINITY) {
        *lse = -INFINITY;
        return;
    }
    double ls = 0.0;
    for (int64_t i = 0; i < n; ++i) {
        if (!(l[i] > 0.0)) continue;
        const double w = exp(m[i] - ms);
        ls += l[i] * w;
        for (int32_t d = 0; d < D; ++d) out[d] += o[i * D + d] * w;
    }
    for (int32_t d = 0; d < D; ++d) out[d] /= ls;
    *lse = ms + log(ls);
}
