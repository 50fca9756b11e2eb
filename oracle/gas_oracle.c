/*
 * CPU oracle for one Gather-Apply-Scatter GNN layer of full-graph inference.
 *
 * TEST INFRASTRUCTURE ONLY.  Plain per-vertex loops, fp64 accumulation, host
 * pointers everywhere.  It shares no code, header, table or helper with the
 * HIP library and must never be called from the product path.
 *
 * What it computes is the plain definition of the message-passing layer
 * (paper Sec. II-B, Eq. (1)): for every vertex v, reduce the messages of its
 * in-edges, then update v's state from its own former state and the reduced
 * message (Sec. IV-B: gather_nbrs/aggregate, apply_node; scatter = storing the
 * new state for the next layer).  The paper states that its optimisations
 * (partial-gather, shadow nodes; Sec. IV-D) never change the result, so the
 * oracle for features is the unsplit definition; the split variants below
 * exist to check that invariant on the CPU.
 *
 * Vertices are independent, so the outer loops may run under OpenMP; every
 * vertex is still evaluated by one thread in edge order, so results do not
 * depend on the thread count.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

enum { ORC_SUM = 0, ORC_MEAN = 1, ORC_GCN = 2, ORC_MAX = 4, ORC_MIN = 5 };
enum { ORC_ACT_NONE = 0, ORC_ACT_RELU = 1 };

int oracle_set_threads(int n)
{
#ifdef _OPENMP
    if (n > 0) omp_set_num_threads(n);
    return omp_get_max_threads();
#else
    (void)n;
    return 1;
#endif
}

/* ---------------------------------------------------------------------------
 * Threshold heuristic (Sec. IV-D, closing paragraph): a vertex counts as a hub
 * when its edge count exceeds the fraction lambda of the edges one worker
 * holds, threshold = lambda * total_edges / total_workers (lambda = 0.1 in the
 * paper's runs).  Degrees are integers, so "exceeds the real number t" is
 * "exceeds floor(t)"; the quotient is formed exactly in integers where
 * lambda is given as the rational num/den.
 * ------------------------------------------------------------------------- */
int oracle_hub_threshold(int64_t total_edges, int64_t total_workers, int64_t lambda_num, int64_t lambda_den,
                         int64_t *threshold)
{
    if (total_edges < 0 || total_workers <= 0 || lambda_num <= 0 || lambda_den <= 0 || !threshold) return -1;
    __int128 t = ((__int128)lambda_num * (__int128)total_edges) / ((__int128)lambda_den * (__int128)total_workers);
    if (t < 1) t = 1;
    *threshold = (int64_t)t;
    return 0;
}

/* ---------------------------------------------------------------------------
 * In-edge grouping (Sec. IV-B gather_nbrs: a vertex receives messages via its
 * in-edges; Sec. IV-C: the edge table is a list of (source, destination)).
 * rowptr[v+1]-rowptr[v] = in-degree of v; col holds, for each v, the sources of
 * its in-edges in the order those edges appear in the input list.
 * Multi-edges and self-loops are ordinary edges.  deg_out may be NULL.
 * Returns 0, or -3 if an endpoint is outside [0, n_nodes).
 * ------------------------------------------------------------------------- */
int oracle_build_csr(int64_t n_nodes, int64_t n_edges, const int32_t *src, const int32_t *dst,
                     int64_t *rowptr, int32_t *col, int32_t *deg_out)
{
    for (int64_t e = 0; e < n_edges; ++e)
        if (src[e] < 0 || src[e] >= n_nodes || dst[e] < 0 || dst[e] >= n_nodes) return -3;
    for (int64_t v = 0; v <= n_nodes; ++v) rowptr[v] = 0;
    if (deg_out) for (int64_t v = 0; v < n_nodes; ++v) deg_out[v] = 0;
    for (int64_t e = 0; e < n_edges; ++e) {
        rowptr[dst[e] + 1] += 1;
        if (deg_out) deg_out[src[e]] += 1;
    }
    for (int64_t v = 0; v < n_nodes; ++v) rowptr[v + 1] += rowptr[v];
    int64_t *cursor = (int64_t *)malloc(sizeof(int64_t) * (size_t)(n_nodes > 0 ? n_nodes : 1));
    if (!cursor) return -7;
    for (int64_t v = 0; v < n_nodes; ++v) cursor[v] = rowptr[v];
    for (int64_t e = 0; e < n_edges; ++e) col[cursor[dst[e]]++] = src[e];
    free(cursor);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Hub split (Sec. IV-D "Shadow Nodes": the edges of a hub are divided into n
 * groups evenly, one mirror per group, done in preprocessing; the strategy is
 * activated when the edge count *exceeds* the threshold).  Applied here to the
 * in-edge segment of every vertex whose in-degree d > T: n = ceil(d/T) groups,
 * group g = [floor(g*d/n), floor((g+1)*d/n)) relative to the row start.
 * Pass arrays as NULL to obtain the counts only.
 * ------------------------------------------------------------------------- */
int oracle_split_hubs(int64_t n_nodes, const int64_t *rowptr, int64_t threshold,
                      int64_t *n_hubs, int64_t *n_shadows,
                      int32_t *hub_ids, int64_t *hub_shadow_off,
                      int64_t *shadow_begin, int64_t *shadow_end, int32_t *shadow_owner)
{
    if (threshold <= 0) return -2;
    int64_t h = 0, s = 0;
    for (int64_t v = 0; v < n_nodes; ++v) {
        int64_t d = rowptr[v + 1] - rowptr[v];
        if (d > threshold) {
            int64_t n = (d + threshold - 1) / threshold;
            if (hub_ids) {
                hub_ids[h] = (int32_t)v;
                hub_shadow_off[h] = s;
                for (int64_t g = 0; g < n; ++g) {
                    /* g*d < 2^63 for every size used here (d < 2^31, n < 2^31) */
                    shadow_begin[s + g] = rowptr[v] + (g * d) / n;
                    shadow_end[s + g] = rowptr[v] + ((g + 1) * d) / n;
                    shadow_owner[s + g] = (int32_t)v;
                }
            }
            h += 1;
            s += n;
        }
    }
    if (hub_ids) hub_shadow_off[h] = s;
    *n_hubs = h;
    *n_shadows = s;
    return 0;
}

/* ---------------------------------------------------------------------------
 * Gather = gather_nbrs + aggregate (Sec. IV-B), the reduce R of Eq. (1) with
 * the message being the source's hidden state (Sec. II-B, last paragraph).
 *   sum : agg[v] = sum_{u in in(v)} h[u]
 *   mean: sum / in-degree (0 for an isolated vertex)
 *   gcn : sum_{u} h[u] / sqrt(max(deg_out(u),1) * max(deg_in(v),1))
 *   max / min: element-wise maximum / minimum over the in-neighbours' states
 *         (Sec. IV-B lists max and min pooling among the commutative and
 *         associative aggregates); 0 for an isolated vertex
 * h holds fp32 values (bf16 inputs are widened exactly by the caller).
 * verts == NULL: all vertices, out is [n_nodes x dim]; else out is
 * [n_verts x dim] for the listed vertices.
 * ------------------------------------------------------------------------- */
int oracle_gather(int agg, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                  int64_t dim, const float *h, const int32_t *deg_out,
                  const int64_t *verts, int64_t n_verts, double *out)
{
    if (agg == ORC_GCN && !deg_out) return -1;
    int64_t n_out = verts ? n_verts : n_nodes;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_out; ++i) {
        int64_t v = verts ? verts[i] : i;
        double *acc = out + i * dim;
        for (int64_t k = 0; k < dim; ++k) acc[k] = 0.0;
        int64_t b = rowptr[v], e = rowptr[v + 1], d = e - b;
        for (int64_t j = b; j < e; ++j) {
            int64_t u = col[j];
            const float *hu = h + u * dim;
            if (agg == ORC_MAX || agg == ORC_MIN) {
                for (int64_t k = 0; k < dim; ++k) {
                    double x = (double)hu[k];
                    if (j == b || (agg == ORC_MAX ? x > acc[k] : x < acc[k])) acc[k] = x;
                }
            } else if (agg == ORC_GCN) {
                double du = deg_out[u] > 1 ? (double)deg_out[u] : 1.0;
                double dv = d > 1 ? (double)d : 1.0;
                double c = 1.0 / sqrt(du * dv);
                for (int64_t k = 0; k < dim; ++k) acc[k] += c * (double)hu[k];
            } else {
                for (int64_t k = 0; k < dim; ++k) acc[k] += (double)hu[k];
            }
        }
        if (agg == ORC_MEAN && d > 0)
            for (int64_t k = 0; k < dim; ++k) acc[k] /= (double)d;
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Gather of edge-weighted messages (Sec. IV-B apply_edge: the message of an
 * edge is generated from the source's state and the edge's own feature; here
 * the feature is one scalar w_e per edge, stored in CSR order):
 *   sum : agg[v] = sum_{e in in(v)} w_e * h[col[e]]
 *   mean: that sum divided by the in-degree (the number of messages), 0 for an
 *         isolated vertex.
 * ------------------------------------------------------------------------- */
int oracle_gather_weighted(int agg, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                           int64_t dim, const float *h, const float *edge_w,
                           const int64_t *verts, int64_t n_verts, double *out)
{
    if ((agg != ORC_SUM && agg != ORC_MEAN) || !edge_w) return -1;
    int64_t n_out = verts ? n_verts : n_nodes;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_out; ++i) {
        int64_t v = verts ? verts[i] : i;
        double *acc = out + i * dim;
        for (int64_t k = 0; k < dim; ++k) acc[k] = 0.0;
        int64_t b = rowptr[v], e = rowptr[v + 1];
        for (int64_t j = b; j < e; ++j) {
            const float *hu = h + (int64_t)col[j] * dim;
            double w = (double)edge_w[j];
            for (int64_t k = 0; k < dim; ++k) acc[k] += w * (double)hu[k];
        }
        if (agg == ORC_MEAN && e > b)
            for (int64_t k = 0; k < dim; ++k) acc[k] /= (double)(e - b);
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Gather of messages built from the source's state AND a feature vector of
 * the edge (Sec. II-A: edges carry a feature matrix E; Sec. II-B: the message
 * function M takes the neighbour's state and the edge; Sec. IV-B apply_edge).
 * Reading taken: the message of edge e = (u -> v) is
 *     m_e = h[u] + ef[e] . W_e          (ef[e] in R^edge_dim, W_e [edge_dim x dim])
 * i.e. the edge feature is mapped linearly into the state space and added.
 * The reduce is the layer's aggregator over the messages, one message at a
 * time, exactly as for plain states:
 *   sum : agg[v] = sum_e m_e            mean: divided by the number of messages
 *   GCN : agg[v] = sum_e m_e / sqrt(max(deg_out(u),1) * max(deg_in(v),1))
 * Edge features are stored per in-edge in CSR order: ef[(rowptr[v] + j) * edge_dim ..].
 * ------------------------------------------------------------------------- */
int oracle_gather_edge_features(int agg, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                                int64_t dim, const float *h, const int32_t *deg_out,
                                int64_t edge_dim, const float *ef, const float *w_e,
                                const int64_t *verts, int64_t n_verts, double *out)
{
    if (agg != ORC_SUM && agg != ORC_MEAN && agg != ORC_GCN) return -1;
    if (agg == ORC_GCN && !deg_out) return -1;
    if (!ef || !w_e || edge_dim <= 0) return -1;
    int64_t n_out = verts ? n_verts : n_nodes;
    int failed = 0;
#pragma omp parallel for schedule(dynamic, 256)
    for (int64_t i = 0; i < n_out; ++i) {
        int64_t v = verts ? verts[i] : i;
        double *acc = out + i * dim;
        double *msg = (double *)malloc(sizeof(double) * (size_t)dim);
        if (!msg) { failed = 1; continue; }
        for (int64_t k = 0; k < dim; ++k) acc[k] = 0.0;
        int64_t b = rowptr[v], e = rowptr[v + 1], d = e - b;
        for (int64_t j = b; j < e; ++j) {
            int64_t u = col[j];
            /* the message of this edge */
            for (int64_t k = 0; k < dim; ++k) msg[k] = (double)h[u * dim + k];
            for (int64_t t = 0; t < edge_dim; ++t) {
                double f = (double)ef[j * edge_dim + t];
                for (int64_t k = 0; k < dim; ++k) msg[k] += f * (double)w_e[t * dim + k];
            }
            /* reduced like any message */
            double c = 1.0;
            if (agg == ORC_GCN) c = 1.0 / sqrt((deg_out[u] > 1 ? (double)deg_out[u] : 1.0) * (d > 1 ? (double)d : 1.0));
            for (int64_t k = 0; k < dim; ++k) acc[k] += c * msg[k];
        }
        if (agg == ORC_MEAN && d > 0)
            for (int64_t k = 0; k < dim; ++k) acc[k] /= (double)d;
        free(msg);
    }
    return failed ? -7 : 0;
}

/* ---------------------------------------------------------------------------
 * Partial-gather over shadow segments (Sec. IV-D "Partial-Gather": aggregate
 * runs on partially available messages, the receiver aggregates the partials;
 * exact because aggregate is commutative and associative).  Non-hub vertices
 * are gathered directly; each hub's segments produce (partial sum, count) and
 * are combined in ascending segment order; mean divides once by the combined
 * count.  edge_count (nullable, [n_nodes]) receives the number of messages
 * combined into every vertex.
 * ------------------------------------------------------------------------- */
int oracle_gather_split(int agg, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                        int64_t dim, const float *h, const int32_t *deg_out,
                        int64_t n_hubs, const int32_t *hub_ids, const int64_t *hub_shadow_off,
                        const int64_t *shadow_begin, const int64_t *shadow_end,
                        double *out, int64_t *edge_count)
{
    if (agg == ORC_GCN && !deg_out) return -1;
    char *is_hub = (char *)calloc((size_t)(n_nodes > 0 ? n_nodes : 1), 1);
    if (!is_hub) return -7;
    for (int64_t i = 0; i < n_hubs; ++i) is_hub[hub_ids[i]] = 1;
    double *part = (double *)malloc(sizeof(double) * (size_t)(dim > 0 ? dim : 1));
    for (int64_t v = 0; v < n_nodes; ++v) {
        if (is_hub[v]) continue;
        double *acc = out + v * dim;
        for (int64_t k = 0; k < dim; ++k) acc[k] = 0.0;
        int64_t d = rowptr[v + 1] - rowptr[v];
        for (int64_t j = rowptr[v]; j < rowptr[v + 1]; ++j) {
            int64_t u = col[j];
            double c = 1.0;
            if (agg == ORC_GCN) c = 1.0 / sqrt((deg_out[u] > 1 ? (double)deg_out[u] : 1.0) * (d > 1 ? (double)d : 1.0));
            if (agg == ORC_MAX || agg == ORC_MIN) {
                for (int64_t k = 0; k < dim; ++k) {
                    double x = (double)h[u * dim + k];
                    if (j == rowptr[v] || (agg == ORC_MAX ? x > acc[k] : x < acc[k])) acc[k] = x;
                }
            } else {
                for (int64_t k = 0; k < dim; ++k) acc[k] += c * (double)h[u * dim + k];
            }
        }
        if (agg == ORC_MEAN && d > 0) for (int64_t k = 0; k < dim; ++k) acc[k] /= (double)d;
        if (edge_count) edge_count[v] = d;
    }
    for (int64_t i = 0; i < n_hubs; ++i) {
        int64_t v = hub_ids[i];
        double *acc = out + v * dim;
        for (int64_t k = 0; k < dim; ++k) acc[k] = 0.0;
        int64_t count = 0;
        int64_t d = rowptr[v + 1] - rowptr[v];
        for (int64_t s = hub_shadow_off[i]; s < hub_shadow_off[i + 1]; ++s) {
            for (int64_t k = 0; k < dim; ++k) part[k] = 0.0;
            for (int64_t j = shadow_begin[s]; j < shadow_end[s]; ++j) {
                int64_t u = col[j];
                double c = 1.0;
                if (agg == ORC_GCN) c = 1.0 / sqrt((deg_out[u] > 1 ? (double)deg_out[u] : 1.0) * (d > 1 ? (double)d : 1.0));
                if (agg == ORC_MAX || agg == ORC_MIN) {
                    for (int64_t k = 0; k < dim; ++k) {
                        double x = (double)h[u * dim + k];
                        if (j == shadow_begin[s] || (agg == ORC_MAX ? x > part[k] : x < part[k])) part[k] = x;
                    }
                } else {
                    for (int64_t k = 0; k < dim; ++k) part[k] += c * (double)h[u * dim + k];
                }
            }
            if (agg == ORC_MAX || agg == ORC_MIN) {   /* the partials of the mirrors are reduced by the same operator */
                for (int64_t k = 0; k < dim; ++k)
                    if (count == 0 || (agg == ORC_MAX ? part[k] > acc[k] : part[k] < acc[k])) acc[k] = part[k];
            } else {
                for (int64_t k = 0; k < dim; ++k) acc[k] += part[k];
            }
            count += shadow_end[s] - shadow_begin[s];
        }
        if (agg == ORC_MEAN && count > 0) for (int64_t k = 0; k < dim; ++k) acc[k] /= (double)count;
        if (edge_count) edge_count[v] = count;
    }
    free(part);
    free(is_hub);
    return 0;
}

/* ---------------------------------------------------------------------------
 * Apply = apply_node (Sec. IV-B): the update U of Eq. (1) combining the
 * vertex's former state with the gathered message:
 *   y[v] = h_self[v] . W_self + agg[v] . W_nbr + bias ;  out = act(y)
 * W_* are [d_in x d_out] row-major.  h_self/w_self may be NULL together (no
 * self term); bias may be NULL.  Rows are [n x d_in] for the n vertices given.
 * ------------------------------------------------------------------------- */
int oracle_apply(int64_t n, int64_t d_in, int64_t d_out,
                 const float *h_self, const float *agg,
                 const float *w_self, const float *w_nbr, const float *bias,
                 int act, double *out)
{
    if ((h_self == NULL) != (w_self == NULL)) return -1;
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v) {
        for (int64_t c = 0; c < d_out; ++c) {
            double y = bias ? (double)bias[c] : 0.0;
            for (int64_t k = 0; k < d_in; ++k) {
                if (h_self) y += (double)h_self[v * d_in + k] * (double)w_self[k * d_out + c];
                y += (double)agg[v * d_in + k] * (double)w_nbr[k * d_out + c];
            }
            if (act == ORC_ACT_RELU && y < 0.0) y = 0.0;
            out[v * d_out + c] = y;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Attention scores for a GAT layer (Sec. II-B: GAT's reduce is an attention-
 * weighted sum of the messages): s[v,k] = sum_d a[k,d] * z[v,k,d].
 * z is [n x heads*dh] (double), a is [heads x dh].
 * ------------------------------------------------------------------------- */
int oracle_gat_scores(int64_t n, int64_t heads, int64_t dh, const double *z, const float *a, double *s)
{
#pragma omp parallel for schedule(static)
    for (int64_t v = 0; v < n; ++v)
        for (int64_t k = 0; k < heads; ++k) {
            double t = 0.0;
            for (int64_t d = 0; d < dh; ++d) t += (double)a[k * dh + d] * z[(v * heads + k) * dh + d];
            s[v * heads + k] = t;
        }
    return 0;
}

/* ---------------------------------------------------------------------------
 * GAT reduce (Sec. IV-B: attention is not commutative/associative, so the
 * aggregate stage only unions the messages and the reduce runs in apply_node).
 * For vertex v and head k, over the multiset in(v) plus v itself (implicit
 * self edge, not stored in the CSR):
 *   e_u = LeakyReLU_slope(s_src[u,k] + s_dst[v,k]);  alpha = softmax(e)
 *   out[v,k,:] = sum_u alpha_u z[u,k,:]
 * Two-pass softmax: maximum first, then the sums.  z, s_src, s_dst hold the
 * stored (already rounded) values as fp32.
 * ------------------------------------------------------------------------- */
int oracle_gat_gather(int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                      int64_t heads, int64_t dh, double slope,
                      const float *z, const float *s_src, const float *s_dst,
                      const int64_t *verts, int64_t n_verts, double *out)
{
    int64_t n_out = verts ? n_verts : n_nodes;
    int64_t dim = heads * dh;
#pragma omp parallel for schedule(dynamic, 64)
    for (int64_t i = 0; i < n_out; ++i) {
        int64_t v = verts ? verts[i] : i;
        int64_t b = rowptr[v], e = rowptr[v + 1];
        for (int64_t k = 0; k < heads; ++k) {
            double sd = (double)s_dst[v * heads + k];
            double t = (double)s_src[v * heads + k] + sd;
            double m = t > 0 ? t : slope * t;                 /* the self edge */
            for (int64_t j = b; j < e; ++j) {
                t = (double)s_src[(int64_t)col[j] * heads + k] + sd;
                t = t > 0 ? t : slope * t;
                if (t > m) m = t;
            }
            double *acc = out + i * dim + k * dh;
            for (int64_t d = 0; d < dh; ++d) acc[d] = 0.0;
            double denom = 0.0;
            for (int64_t j = b - 1; j < e; ++j) {
                int64_t u = (j < b) ? v : (int64_t)col[j];
                t = (double)s_src[u * heads + k] + sd;
                t = t > 0 ? t : slope * t;
                double p = exp(t - m);
                denom += p;
                const float *zu = z + u * dim + k * dh;
                for (int64_t d = 0; d < dh; ++d) acc[d] += p * (double)zu[d];
            }
            for (int64_t d = 0; d < dh; ++d) acc[d] /= denom;
        }
    }
    return 0;
}

/* ---------------------------------------------------------------------------
 * Storage rounding: fp64 -> nearest bf16 (ties to even), returned as the fp32
 * holding that value.  frexp gives x = m * 2^e with 0.5 <= |m| < 1; a bf16 has
 * 8 significant bits, so round m * 2^8 to an integer.  Normal range only
 * (|x| between 2^-126 and the bf16 maximum); zero, inf and nan pass through.
 * ------------------------------------------------------------------------- */
int oracle_round_bf16(int64_t n, const double *x, float *out)
{
    for (int64_t i = 0; i < n; ++i) {
        double v = x[i];
        if (v == 0.0 || isnan(v) || isinf(v)) { out[i] = (float)v; continue; }
        int e;
        double m = frexp(v, &e);
        double q = nearbyint(ldexp(m, 8));      /* default rounding mode: ties to even */
        out[i] = (float)ldexp(q, e - 8);
    }
    return 0;
}
