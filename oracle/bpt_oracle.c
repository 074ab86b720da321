/*
 * bpt_oracle.c -- CPU oracle for BP-Transformer graph self-attention.
 *
 * THIS IS TEST INFRASTRUCTURE, NOT THE PRODUCT.  It is a plain, slow,
 * double-precision restatement of what the paper defines, used only to check
 * the GPU library and to time a CPU baseline.  It shares no code, header,
 * table or helper with the HIP path and must never be linked or called from
 * it.  Only the tests, the smoke check and the benchmark's cpu_baseline leg
 * may load this file.
 *
 * What is restated here (paper sections):
 *   - Sec. 3.2.1  node construction: a perfect binary tree over n tokens,
 *                 level 0 = tokens, node (l,m) covers tokens [m*2^l,(m+1)*2^l).
 *   - Sec. 3.2.2  affiliated edges: every token of a span -> that span node.
 *   - Sec. 3.2.2  contextual edges + Algorithm 1: per token, per side, per
 *                 level k nodes starting at p_l, p_0 = i+1, plus one extra
 *                 node when the run would not end on a parent boundary; the
 *                 next level starts at the parent of the node after the run.
 *   - Sec. 3.4    relative positions on the tree: r_self, r_left(j,i),
 *                 r_right(j,i), r_anc(j), packed as (level j, signed offset).
 *   - Sec. 3.1 eq. (6) with Sec. 3.4 eq. (8): per node u, softmax over its
 *                 predecessors v of q_u.(k_v + r_{v,u})*scale, times v_v.
 *   - the gradient of eq. (8) with respect to Q, K, V and the r table.
 *
 * Readings of points the paper leaves open (indices are 0-based here):
 *   - the extra ("alignment") node is added on the right side iff the last
 *     regular node is a left child (even index), on the left side iff it is a
 *     right child (odd index): the only choice under which the spans a token
 *     attends to do not overlap (Sec. 3 opening paragraph).
 *   - a side stops when its start index leaves the level; the run is clipped
 *     to the level's last (first) node.
 *   - token rows carry a self edge (Algorithm 1 starts from N = {u}); span
 *     rows have exactly their contained tokens as predecessors (Sec. 3.3) and
 *     no self edge.
 *   - causal graph: the right side of every token row is dropped.
 *   - i-th node to join at level j: nearest first, i = 1..k+1.
 *   - one table Rel[level][W][D], W = 2(k+1)+1, slot = offset + (k+1);
 *     (0,0) is r_self, (j,0) for j>=1 is r_anc(j).
 *   - edges of a row are stored in ascending packed id  level*W + slot.
 *
 * Sequences of any length (the bpto_*_len functions; the paper states the tree for
 * n a power of two only, Sec. 3.2.1): a sequence of len tokens, 1 <= len <= n,
 * keeps the nodes of the tree over n that hold at least one of its tokens --
 * level l keeps its first ceil(len / 2^l) nodes, the last one possibly cut short --
 * and Algorithm 1 walks these shorter levels: a run is clipped to the level's
 * last kept node and the side stops there.  Ids stay those of the tree over n, so
 * rows of nodes that are not kept are empty; their output is defined as zero.
 *
 * Dropout on the attention weights (p_a of the hyper-parameter tables; the paper gives no formula):
 * the usual inverted dropout after the softmax -- weight p_e becomes keep_e p_e / (1 - p_a) in the
 * weighted sum of values, lse is that of the full softmax -- with keep_e drawn from a counter-based
 * hash of (seed, batch*heads index, query node, x_e), x_e = relative-position id of the edge for a
 * token row and 2^31 + key node for a span row (both identify the edge within its row):
 *   mix(z): z ^= z>>16; z *= 0x7FEB352D; z ^= z>>15; z *= 0x846CA68B; z ^= z>>16   (32-bit)
 *   keep = mix(mix(mix(seed ^ (0x9E3779B9 * bh)) + u) + x) >= floor(p_a * 2^32).
 *
 * Node ids: level-major, id(l,m) = off(l) + m with off(l) = 2n - (2n >> l);
 * tokens are 0..n-1 and the root is 2n-2.
 *
 * All arithmetic on values is double; inputs arrive as float (already rounded
 * to the dtype of the configuration under test by the caller).
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>

#ifdef _OPENMP
#include <omp.h>
#endif

#define BPTO_MAX_LEVELS 40

static int is_pow2(int64_t n) { return n >= 2 && (n & (n - 1)) == 0; }

/* number of tree levels, tokens included: log2(n) + 1 */
int32_t bpto_num_levels(int32_t n)
{
    if (!is_pow2(n)) return -1;
    int32_t L = 0;
    while (((int64_t)1 << L) < n) ++L;
    return L + 1;
}

/* first node id of a level */
int64_t bpto_level_offset(int32_t n, int32_t level)
{
    return 2 * (int64_t)n - ((2 * (int64_t)n) >> level);
}

int32_t bpto_rel_width(int32_t k) { return 2 * (k + 1) + 1; }

/* One side's runs for token i: for level j the nodes first[j]..last[j]
 * (first = nearest to the token).  Returns the number of levels used. */
static int right_runs(int64_t n, int64_t k, int64_t i, int64_t *first, int64_t *last)
{
    int j = 0;
    int64_t p = i + 1, size = n;
    while (p < size) {
        int64_t e = p + k - 1;
        if (e > size - 1) e = size - 1;
        if ((e & 1) == 0) e += 1;          /* left child: take its sibling too */
        first[j] = p;
        last[j] = e;
        ++j;
        int64_t nxt = e + 1;
        if (nxt >= size) break;
        p = nxt >> 1;                      /* parent of the node after the run */
        size >>= 1;
    }
    return j;
}

static int left_runs(int64_t n, int64_t k, int64_t i, int64_t *first, int64_t *last)
{
    (void)n;
    int j = 0;
    int64_t q = i - 1;
    while (q >= 0) {
        int64_t e = q - k + 1;
        if (e < 0) e = 0;
        if ((e & 1) == 1) e -= 1;          /* right child: take its sibling too */
        first[j] = q;
        last[j] = e;
        ++j;
        int64_t nxt = e - 1;
        if (nxt < 0) break;
        q = nxt >> 1;
    }
    return j;
}

/* degree of every node; returns total edge count, or -1 on bad arguments */
int64_t bpto_count_edges(int32_t n, int32_t k, int32_t causal, int64_t *deg /* [2n-1] or NULL */)
{
    if (!is_pow2(n) || k < 1) return -1;
    int32_t levels = bpto_num_levels(n);
    int64_t total = 0;
    int64_t f[BPTO_MAX_LEVELS], l[BPTO_MAX_LEVELS];
    for (int64_t i = 0; i < n; ++i) {
        int64_t d = 1;                                    /* self */
        int nl = left_runs(n, k, i, f, l);
        for (int j = 0; j < nl; ++j) d += f[j] - l[j] + 1;
        if (!causal) {
            int nr = right_runs(n, k, i, f, l);
            for (int j = 0; j < nr; ++j) d += l[j] - f[j] + 1;
        }
        if (deg) deg[i] = d;
        total += d;
    }
    for (int32_t lev = 1; lev < levels; ++lev) {
        int64_t cnt = (int64_t)n >> lev, off = bpto_level_offset(n, lev);
        for (int64_t m = 0; m < cnt; ++m) {
            if (deg) deg[off + m] = (int64_t)1 << lev;
            total += (int64_t)1 << lev;
        }
    }
    return total;
}

/* CSR by query node: row_ptr[2n], col[E], rel[E] (caller allocates after
 * bpto_count_edges).  Returns 0, or -1 on bad arguments / int32 overflow. */
int32_t bpto_build_graph(int32_t n, int32_t k, int32_t causal,
                         int32_t *row_ptr, int32_t *col, int32_t *rel)
{
    int64_t E = bpto_count_edges(n, k, causal, NULL);
    if (E < 0 || E > INT32_MAX) return -1;
    int32_t levels = bpto_num_levels(n);
    int64_t W = bpto_rel_width(k), zero = k + 1;
    int64_t lf[BPTO_MAX_LEVELS], ll[BPTO_MAX_LEVELS], rf[BPTO_MAX_LEVELS], rl[BPTO_MAX_LEVELS];
    int64_t e = 0;
    for (int64_t i = 0; i < n; ++i) {
        row_ptr[i] = (int32_t)e;
        int nl = left_runs(n, k, i, lf, ll);
        int nr = causal ? 0 : right_runs(n, k, i, rf, rl);
        int top = nl > nr ? nl : nr;
        if (top < 1) top = 1;
        for (int j = 0; j < top; ++j) {
            int64_t off = bpto_level_offset(n, j);
            if (j < nl)                                   /* far -> near: offsets -(cnt)..-1 */
                for (int64_t x = ll[j]; x <= lf[j]; ++x) {
                    col[e] = (int32_t)(off + x);
                    rel[e] = (int32_t)(j * W + zero - (lf[j] - x + 1));
                    ++e;
                }
            if (j == 0) {                                 /* self, r_self */
                col[e] = (int32_t)i;
                rel[e] = (int32_t)zero;
                ++e;
            }
            if (j < nr)                                   /* near -> far: offsets +1..+cnt */
                for (int64_t x = rf[j]; x <= rl[j]; ++x) {
                    col[e] = (int32_t)(off + x);
                    rel[e] = (int32_t)(j * W + zero + (x - rf[j] + 1));
                    ++e;
                }
        }
    }
    for (int32_t lev = 1; lev < levels; ++lev) {
        int64_t cnt = (int64_t)n >> lev, off = bpto_level_offset(n, lev);
        for (int64_t m = 0; m < cnt; ++m) {
            row_ptr[off + m] = (int32_t)e;
            for (int64_t t = m << lev; t < ((m + 1) << lev); ++t) {   /* contained tokens */
                col[e] = (int32_t)t;
                rel[e] = (int32_t)(lev * W + zero);       /* r_anc(lev) */
                ++e;
            }
        }
    }
    row_ptr[2 * (int64_t)n - 1] = (int32_t)e;
    return e == E ? 0 : -1;
}

/* Transposed adjacency by its definition: for each key node v, all edges
 * (u -> v is "u attends to v") in ascending edge index.  t_ptr[N+1],
 * t_src[E] = query node of the edge, t_eid[E] = index of the edge in the CSR. */
void bpto_transpose(int32_t N, const int32_t *row_ptr, const int32_t *col,
                    int32_t *t_ptr, int32_t *t_src, int32_t *t_eid)
{
    int64_t E = row_ptr[N];
    memset(t_ptr, 0, sizeof(int32_t) * ((size_t)N + 1));
    for (int64_t e = 0; e < E; ++e) t_ptr[col[e] + 1] += 1;
    for (int32_t v = 0; v < N; ++v) t_ptr[v + 1] += t_ptr[v];
    int32_t *cursor = (int32_t *)malloc(sizeof(int32_t) * (size_t)(N > 0 ? N : 1));
    memcpy(cursor, t_ptr, sizeof(int32_t) * (size_t)N);
    for (int32_t u = 0; u < N; ++u)
        for (int32_t e = row_ptr[u]; e < row_ptr[u + 1]; ++e) {
            int32_t v = col[e], at = cursor[v]++;
            t_src[at] = u;
            t_eid[at] = e;
        }
    free(cursor);
}

/* ---- sequences of len <= n tokens on the tree over n (see the header) ------ */

/* nodes kept on a level */
static int64_t level_count(int64_t len, int level)
{
    return (len + (((int64_t)1 << level) - 1)) >> level;
}

/* right side of token i when level j holds level_count(len, j) nodes */
static int right_runs_len(int64_t len, int64_t k, int64_t i, int64_t *first, int64_t *last)
{
    int j = 0;
    int64_t p = i + 1;
    while (p < level_count(len, j)) {
        int64_t size = level_count(len, j);
        int64_t e = p + k - 1;
        if (e > size - 1) e = size - 1;
        if ((e & 1) == 0 && e + 1 < size) e += 1;   /* left child whose sibling is kept */
        first[j] = p;
        last[j] = e;
        ++j;
        if (e + 1 >= size) break;
        p = (e + 1) >> 1;
    }
    return j;
}

/* Edge count of the graph of a sequence of len tokens; deg[2n-1] optional. */
int64_t bpto_count_edges_len(int32_t n, int32_t len, int32_t k, int32_t causal, int64_t *deg)
{
    if (!is_pow2(n) || k < 1 || len < 1 || len > n) return -1;
    int32_t levels = bpto_num_levels(n);
    int64_t total = 0;
    int64_t f[BPTO_MAX_LEVELS], l[BPTO_MAX_LEVELS];
    if (deg) memset(deg, 0, sizeof(int64_t) * (size_t)(2 * (int64_t)n - 1));
    for (int64_t i = 0; i < len; ++i) {
        int64_t d = 1;
        int nl = left_runs(n, k, i, f, l);          /* everything left of a token is kept */
        for (int j = 0; j < nl; ++j) d += f[j] - l[j] + 1;
        if (!causal) {
            int nr = right_runs_len(len, k, i, f, l);
            for (int j = 0; j < nr; ++j) d += l[j] - f[j] + 1;
        }
        if (deg) deg[i] = d;
        total += d;
    }
    for (int32_t lev = 1; lev < levels; ++lev) {
        int64_t off = bpto_level_offset(n, lev);
        for (int64_t m = 0; m < level_count(len, lev); ++m) {
            int64_t hi = (m + 1) << lev;
            if (hi > len) hi = len;
            if (deg) deg[off + m] = hi - (m << lev);
            total += hi - (m << lev);
        }
    }
    return total;
}

/* CSR of that graph over the 2n-1 node ids of the tree over n: row_ptr[2n],
 * col[E], rel[E]; rows of nodes that are not kept are empty. */
int32_t bpto_build_graph_len(int32_t n, int32_t len, int32_t k, int32_t causal,
                             int32_t *row_ptr, int32_t *col, int32_t *rel)
{
    int64_t E = bpto_count_edges_len(n, len, k, causal, NULL);
    if (E < 0 || E > INT32_MAX) return -1;
    int32_t levels = bpto_num_levels(n);
    int64_t W = bpto_rel_width(k), zero = k + 1;
    int64_t lf[BPTO_MAX_LEVELS], ll[BPTO_MAX_LEVELS], rf[BPTO_MAX_LEVELS], rl[BPTO_MAX_LEVELS];
    int64_t e = 0;
    for (int64_t i = 0; i < n; ++i) {
        row_ptr[i] = (int32_t)e;
        if (i >= len) continue;
        int nl = left_runs(n, k, i, lf, ll);
        int nr = causal ? 0 : right_runs_len(len, k, i, rf, rl);
        int top = nl > nr ? nl : nr;
        if (top < 1) top = 1;
        for (int j = 0; j < top; ++j) {
            int64_t off = bpto_level_offset(n, j);
            if (j < nl)
                for (int64_t x = ll[j]; x <= lf[j]; ++x) {
                    col[e] = (int32_t)(off + x);
                    rel[e] = (int32_t)(j * W + zero - (lf[j] - x + 1));
                    ++e;
                }
            if (j == 0) {
                col[e] = (int32_t)i;
                rel[e] = (int32_t)zero;
                ++e;
            }
            if (j < nr)
                for (int64_t x = rf[j]; x <= rl[j]; ++x) {
                    col[e] = (int32_t)(off + x);
                    rel[e] = (int32_t)(j * W + zero + (x - rf[j] + 1));
                    ++e;
                }
        }
    }
    for (int32_t lev = 1; lev < levels; ++lev) {
        int64_t cnt = (int64_t)n >> lev, off = bpto_level_offset(n, lev);
        for (int64_t m = 0; m < cnt; ++m) {
            row_ptr[off + m] = (int32_t)e;
            for (int64_t t = m << lev; t < ((m + 1) << lev) && t < len; ++t) {
                col[e] = (int32_t)t;
                rel[e] = (int32_t)(lev * W + zero);
                ++e;
            }
        }
    }
    row_ptr[2 * (int64_t)n - 1] = (int32_t)e;
    return e == E ? 0 : -1;
}

/* ---- dropout mask ------------------------------------------------------------- */
static uint32_t mix32(uint32_t z)
{
    z ^= z >> 16; z *= 0x7FEB352Du; z ^= z >> 15; z *= 0x846CA68Bu; z ^= z >> 16;
    return z;
}
static uint32_t drop_threshold(double p)
{
    double t = floor(p * 4294967296.0);
    return t <= 0.0 ? 0u : (t >= 4294967295.0 ? 4294967295u : (uint32_t)t);
}
/* 1/(1-p) if the edge is kept, else 0; p <= 0 keeps everything */
static double keep_scale(double p, uint32_t thr, uint32_t seed, int64_t bh, int32_t n_tokens, int32_t u, int32_t v, int32_t rel)
{
    if (p <= 0.0) return 1.0;
    uint32_t x = u < n_tokens ? (uint32_t)rel : (0x80000000u + (uint32_t)v);
    uint32_t r = mix32(mix32(mix32(seed ^ (0x9E3779B9u * (uint32_t)bh)) + (uint32_t)u) + x);
    return r >= thr ? 1.0 / (1.0 - p) : 0.0;
}

/* ---- attention, eq. (6)/(8) -------------------------------------------- */

/* scores of one row into s[], returns lse */
static double row_scores(const float *q, const float *Kbh, const float *Rel, int32_t D,
                         const int32_t *col, const int32_t *rel, int32_t deg, double scale,
                         double *s)
{
    double mx = -INFINITY;
    for (int32_t e = 0; e < deg; ++e) {
        const float *kv = Kbh + (int64_t)col[e] * D;
        const float *r = Rel + (int64_t)rel[e] * D;
        double acc = 0.0;
        for (int32_t d = 0; d < D; ++d) acc += (double)q[d] * ((double)kv[d] + (double)r[d]);
        s[e] = acc * scale;
        if (s[e] > mx) mx = s[e];
    }
    double z = 0.0;
    for (int32_t e = 0; e < deg; ++e) z += exp(s[e] - mx);
    return mx + log(z);
}

static int32_t max_degree(int32_t N, const int32_t *row_ptr)
{
    int32_t m = 1;
    for (int32_t u = 0; u < N; ++u)
        if (row_ptr[u + 1] - row_ptr[u] > m) m = row_ptr[u + 1] - row_ptr[u];
    return m;
}

/* Q,K,V: [BH][N][D] contiguous floats; Rel: [ids][D]; out: [BH][N][D] double;
 * lse: [BH][N] double.  threads <= 0 means all cores. Returns threads used. */
int32_t bpto_attn_fwd(int32_t N, const int32_t *row_ptr, const int32_t *col, const int32_t *rel,
                      int32_t BH, int32_t D, const float *Q, const float *K, const float *V,
                      const float *Rel, double scale, double *out, double *lse, int32_t threads,
                      double p_drop, uint32_t seed, int32_t bh0)
{
    const uint32_t thr = drop_threshold(p_drop);
    const int32_t n_tokens = (N + 1) / 2;
    int32_t used = 1;
    int32_t md = max_degree(N, row_ptr);
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    used = threads;
#else
    (void)threads;
#endif
#pragma omp parallel num_threads(threads)
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)md);
#pragma omp for collapse(2) schedule(dynamic, 64)
        for (int32_t bh = 0; bh < BH; ++bh)
            for (int32_t u = 0; u < N; ++u) {
                const float *Qbh = Q + (int64_t)bh * N * D, *Kbh = K + (int64_t)bh * N * D;
                const float *Vbh = V + (int64_t)bh * N * D;
                int32_t b = row_ptr[u], deg = row_ptr[u + 1] - b;
                double l = row_scores(Qbh + (int64_t)u * D, Kbh, Rel, D, col + b, rel + b, deg,
                                      scale, s);
                double *o = out + ((int64_t)bh * N + u) * D;
                for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
                for (int32_t e = 0; e < deg; ++e) {
                    double p = exp(s[e] - l) * keep_scale(p_drop, thr, seed, (int64_t)bh0 + bh, n_tokens, u, col[b + e], rel[b + e]);
                    const float *vv = Vbh + (int64_t)col[b + e] * D;
                    for (int32_t d = 0; d < D; ++d) o[d] += p * (double)vv[d];
                }
                lse[(int64_t)bh * N + u] = deg > 0 ? l : 0.0;   /* a row without edges: zero by definition */
            }
        free(s);
    }
    return used;
}

/* Gradient of eq. (8).  With p_e the attention weight of edge e = (u <- v),
 *   dP_e = dO_u . v_v,   delta_u = dO_u . out_u = sum_e p_e dP_e,
 *   dS_e = p_e (dP_e - delta_u),
 *   dQ_u = scale * sum_e dS_e (k_v + r_e),   dK_v = scale * sum_{e->v} dS_e q_u,
 *   dV_v = sum_{e->v} p_e dO_u,              dRel[id] = scale * sum_{rel e = id} dS_e q_u
 * (dRel summed over batch and heads: the table is shared, Sec. 3.4).
 * The forward is recomputed here in double; nothing comes from the caller's
 * forward.  dQ,dK,dV: [BH][N][D] double; dRel: [ids][D] double. */
int32_t bpto_attn_bwd(int32_t N, const int32_t *row_ptr, const int32_t *col, const int32_t *rel,
                      int32_t BH, int32_t D, int32_t num_ids, const float *Q, const float *K,
                      const float *V, const float *Rel, const float *dO, double scale, double *dQ,
                      double *dK, double *dV, double *dRel, int32_t threads,
                      double p_drop, uint32_t seed, int32_t bh0)
{
    /* with dropout, out_u = sum_e m_e p_e v_v (m_e = keep/(1-p_a)): dP_e = m_e dO_u . v_v,
     * delta_u = sum_e p_e dP_e = dO_u . out_u, dV_v += m_e p_e dO_u; the rest is unchanged */
    const uint32_t thr = drop_threshold(p_drop);
    const int32_t n_tokens = (N + 1) / 2;
    int32_t used = 1;
    int32_t md = max_degree(N, row_ptr);
#ifdef _OPENMP
    if (threads <= 0) threads = omp_get_max_threads();
    if (threads > BH) threads = BH;
    used = threads;
#else
    (void)threads;
#endif
    size_t relsz = (size_t)num_ids * (size_t)D;
    double *dRel_bh = (double *)calloc((size_t)BH * relsz, sizeof(double));
    memset(dQ, 0, sizeof(double) * (size_t)BH * N * D);
    memset(dK, 0, sizeof(double) * (size_t)BH * N * D);
    memset(dV, 0, sizeof(double) * (size_t)BH * N * D);
#pragma omp parallel num_threads(threads)
    {
        double *s = (double *)malloc(sizeof(double) * (size_t)md);
        double *o = (double *)malloc(sizeof(double) * (size_t)D);
#pragma omp for schedule(dynamic, 1)
        for (int32_t bh = 0; bh < BH; ++bh) {
            const int64_t base = (int64_t)bh * N * D;
            double *dR = dRel_bh + (size_t)bh * relsz;
            for (int32_t u = 0; u < N; ++u) {
                const float *q = Q + base + (int64_t)u * D, *g = dO + base + (int64_t)u * D;
                int32_t b = row_ptr[u], deg = row_ptr[u + 1] - b;
                double l = row_scores(q, K + base, Rel, D, col + b, rel + b, deg, scale, s);
                for (int32_t d = 0; d < D; ++d) o[d] = 0.0;
                for (int32_t e = 0; e < deg; ++e) {
                    double p = exp(s[e] - l) * keep_scale(p_drop, thr, seed, (int64_t)bh0 + bh, n_tokens, u, col[b + e], rel[b + e]);
                    const float *vv = V + base + (int64_t)col[b + e] * D;
                    for (int32_t d = 0; d < D; ++d) o[d] += p * (double)vv[d];
                }
                double delta = 0.0;
                for (int32_t d = 0; d < D; ++d) delta += (double)g[d] * o[d];
                double *dq = dQ + base + (int64_t)u * D;
                for (int32_t e = 0; e < deg; ++e) {
                    int64_t v = col[b + e];
                    const float *kv = K + base + v * D, *vv = V + base + v * D;
                    const float *r = Rel + (int64_t)rel[b + e] * D;
                    double p = exp(s[e] - l), dP = 0.0;
                    const double m = keep_scale(p_drop, thr, seed, (int64_t)bh0 + bh, n_tokens, u, (int32_t)v, rel[b + e]);
                    for (int32_t d = 0; d < D; ++d) dP += (double)g[d] * (double)vv[d];
                    dP *= m;
                    double dS = p * (dP - delta);
                    double *dk = dK + base + v * D, *dv = dV + base + v * D;
                    double *dr = dR + (int64_t)rel[b + e] * D;
                    for (int32_t d = 0; d < D; ++d) {
                        dq[d] += scale * dS * ((double)kv[d] + (double)r[d]);
                        dk[d] += scale * dS * (double)q[d];
                        dv[d] += m * p * (double)g[d];
                        dr[d] += scale * dS * (double)q[d];
                    }
                }
            }
        }
        free(s);
        free(o);
    }
    for (size_t x = 0; x < relsz; ++x) {
        double acc = 0.0;
        for (int32_t bh = 0; bh < BH; ++bh) acc += dRel_bh[(size_t)bh * relsz + x];
        dRel[x] = acc;
    }
    free(dRel_bh);
    return used;
}
