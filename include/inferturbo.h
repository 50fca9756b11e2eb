/*
 * inferturbo.h -- C ABI of the MI355X (gfx950) hot path of full-graph GNN
 * inference in the Gather-Apply-Scatter schema (InferTurbo, arXiv 2307.00228).
 *
 * One GNN layer is evaluated for EVERY vertex, layer by layer, with no
 * neighbour sampling (Sec. IV-B "Inference", Sec. IV-C: k supersteps for a
 * k-layer model).  The stages of the paper's abstraction (Sec. IV-B) map to
 * the calls below:
 *   gather_nbrs + aggregate  -> gather_layer   (pull over in-edges, CSR by destination)
 *   apply_node               -> apply_layer    (dense update of own state + gathered message)
 *   apply_edge + scatter_nbrs-> the store of the new state that the next layer's gather reads
 * and the strategies of Sec. IV-D to split_hubs (even split of a hub's edge
 * set into mirrors, done in preprocessing) and to the partial-gather passes
 * inside gather_layer (partials per mirror, then an ordered combine).
 *
 * Conventions for every call
 *  - Every pointer is a DEVICE pointer unless marked "host".  All buffers
 *    (inputs, outputs, workspace) are allocated, owned and freed by the
 *    caller; the library never modifies an input and keeps no pointer to a
 *    caller's buffer or handle after return.
 *  - What the library itself owns, per device, from the first call that needs
 *    it until itb_shutdown() or the end of the process: one helper stream
 *    (default priority, non-blocking) with two events, on which gather_layer
 *    runs the hub passes and build_csr_by_dst the out-degree branch; the
 *    launch attributes of its kernels; and the fixed scratch array of
 *    gather_layer_noalloc, which is part of the loaded code object.  Nothing
 *    else outlives a call.
 *  - Workspace protocol: if `workspace` is NULL the call only writes the
 *    number of bytes it needs for these sizes to *workspace_bytes (host) and
 *    returns ITB_OK.  Otherwise *workspace_bytes is the size provided;
 *    too small -> ITB_ERR_WORKSPACE.  Workspace must be 256-byte aligned.
 *  - `stream` is a hipStream_t passed as void* (NULL = the default stream).
 *    gather_layer, apply_layer, gcn_norm_scales and infer_full_graph only
 *    enqueue work and return without synchronising.  build_csr_by_dst
 *    synchronises the stream before returning (it reports range errors to
 *    the host); split_hubs synchronises once to read the two counts, the
 *    arrays it fills afterwards are ordered on the stream like any output.
 *    gather_layer (hub passes) and build_csr_by_dst (out-degrees) put part of
 *    their work on the helper stream and join it back into `stream` before
 *    returning, on error returns too; host threads calling on different
 *    streams are serialised around that fork and join.  Nothing the calls
 *    enqueue uses a memset node or a synchronisation, so infer_full_graph,
 *    gather_layer and apply_layer can be captured into a HIP graph (after one
 *    uncaptured call on the device, which creates the helper stream).
 *  - Return value: ITB_OK (0) or a negative itb_status.  Argument errors are
 *    detected on the host before any launch.  Nothing throws, aborts or prints.
 *  - Dense tensors are row-major and 16-byte aligned (they are moved as
 *    16-byte vectors; a misaligned feature tensor is ITB_ERR_UNSUPPORTED).
 *    ITB_BF16 tensors hold IEEE bfloat16 (round-to-nearest-even on store); all
 *    sums accumulate in fp32.  Feature data is expected to be finite: the
 *    attention gather feeds the tail of an edge chunk with weight zero, so an
 *    infinity in a source row can surface as NaN in a destination whose exact
 *    result is infinite.
 *  - Sizes: 0 <= n_nodes < 2^31, 0 <= n_edges < 2^31.
 *  - Results are bitwise reproducible run to run: no floating-point atomics,
 *    every summation order is fixed by the inputs and sizes (the paper's
 *    consistency requirement, Sec. IV-A).
 */
#ifndef INFERTURBO_H
#define INFERTURBO_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
    ITB_OK = 0,
    ITB_ERR_NULL = -1,        /* a required pointer is NULL */
    ITB_ERR_SIZE = -2,        /* negative or too large size, threshold <= 0 */
    ITB_ERR_RANGE = -3,       /* an edge endpoint is outside [0, n_nodes) */
    ITB_ERR_DTYPE = -4,       /* unknown dtype / aggregator / activation code */
    ITB_ERR_UNSUPPORTED = -5, /* a width the kernels do not cover (see each call) */
    ITB_ERR_WORKSPACE = -6,   /* workspace too small or misaligned */
    ITB_ERR_DEVICE = -7       /* a HIP call failed */
} itb_status;

enum { ITB_F32 = 0, ITB_BF16 = 1 };
enum {
    ITB_AGG_SUM = 0, ITB_AGG_MEAN = 1, ITB_AGG_GCN = 2, ITB_AGG_GAT = 3,
    ITB_AGG_MAX = 4, ITB_AGG_MIN = 5, /* element-wise extrema (Sec. IV-B lists max and min among the reduces that
                                         satisfy the commutative and associative laws) */
    ITB_AGG_NONE = 6                  /* infer_full_graph only: a layer without a gather (feature encoder before
                                         the first round, prediction head after the last, Sec. IV-C) */
};
enum { ITB_ACT_NONE = 0, ITB_ACT_RELU = 1 };

/* ---------------------------------------------------------------------------
 * build_csr_by_dst -- group the in-edges of every vertex (Sec. IV-B
 * gather_nbrs: a vertex receives the messages of its in-edges; Sec. IV-C: the
 * input is an edge table of (source, destination) pairs).
 *
 *   src, dst   [n_edges] int32, edge e goes src[e] -> dst[e]; multi-edges and
 *              self-loops are ordinary edges.
 *   rowptr     out [n_nodes+1] int64; rowptr[v+1]-rowptr[v] = in-degree of v.
 *   col        out [n_edges] int32; col[rowptr[v] + j] = source of the j-th
 *              in-edge of v in ORIGINAL edge order (stable).
 *   deg_out    out [n_nodes] int32 out-degree of every vertex; may be NULL.
 * n_nodes == 0 or n_edges == 0 are valid.  Returns ITB_ERR_RANGE (outputs
 * unspecified but in bounds) if any endpoint is outside [0, n_nodes).
 * ------------------------------------------------------------------------- */
int32_t build_csr_by_dst(int64_t n_nodes, int64_t n_edges,
                         const int32_t *src, const int32_t *dst,
                         int64_t *rowptr, int32_t *col, int32_t *deg_out,
                         void *workspace, size_t *workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * split_hubs -- mirror ("shadow") split of high-in-degree vertices (Sec. IV-D
 * "Shadow Nodes": a hub's edges are divided evenly into n groups, one mirror
 * per group, in preprocessing; activated when the edge count EXCEEDS the
 * threshold).  A vertex with in-degree d > threshold gets n = ceil(d/threshold)
 * contiguous segments of its CSR row, segment g covering
 * [rowptr[v] + floor(g*d/n), rowptr[v] + floor((g+1)*d/n)).
 *
 *   n_hubs, n_shadows  host out: number of hubs H and of segments S.
 *   hub_ids        out [H]   int32, ascending vertex ids.
 *   hub_shadow_off out [H+1] int64, segments of hub i are [off[i], off[i+1]).
 *   shadow_begin/shadow_end out [S] int64 edge offsets into col.
 *   shadow_owner   out [S]   int32 vertex id owning the segment.
 * Call once with all five arrays NULL to obtain H and S, allocate, call again.
 * ------------------------------------------------------------------------- */
int32_t split_hubs(int64_t n_nodes, const int64_t *rowptr, int64_t threshold,
                   int64_t *n_hubs, int64_t *n_shadows,
                   int32_t *hub_ids, int64_t *hub_shadow_off,
                   int64_t *shadow_begin, int64_t *shadow_end, int32_t *shadow_owner,
                   void *workspace, size_t *workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * hub_threshold_heuristic -- the paper's rule of thumb for the threshold
 * (Sec. IV-D, closing paragraph; Sec. V, strategy analysis: 1e9 edges on 1000
 * workers with lambda = 0.1 give 100,000): threshold = lambda * total_edges /
 * total_workers, returned as floor (degrees are integers), at least 1.  Host
 * only; `threshold` is a host pointer.  On one GPU a "worker" is a compute
 * unit; measured on two hub-dominated graphs the gather time is flat over
 * more than a decade of thresholds around the value this returns.
 * ------------------------------------------------------------------------- */
int32_t hub_threshold_heuristic(int64_t total_edges, int64_t total_workers, double lambda,
                                int64_t *threshold);

/* The split as consumed by gather_layer / infer_full_graph.  `threshold` must
 * be the value given to split_hubs: rows with in-degree > threshold are
 * skipped by the per-row pass and produced by the partial/combine passes. */
typedef struct {
    int64_t threshold;
    int64_t n_hubs, n_shadows;
    const int32_t *hub_ids;
    const int64_t *hub_shadow_off;
    const int64_t *shadow_begin, *shadow_end;
    const int32_t *shadow_owner;
} itb_split;

/* ---------------------------------------------------------------------------
 * gcn_norm_scales -- per-vertex factors of the symmetric degree normalisation:
 * src_scale[u] = max(deg_out[u],1)^-1/2, dst_scale[v] = max(deg_in[v],1)^-1/2,
 * so that the coefficient of edge u->v is src_scale[u]*dst_scale[v].
 * Outputs [n_nodes] fp32.
 * ------------------------------------------------------------------------- */
int32_t gcn_norm_scales(int64_t n_nodes, const int64_t *rowptr, const int32_t *deg_out,
                        float *src_scale, float *dst_scale, void *stream);

/* ---------------------------------------------------------------------------
 * gcn_edge_coefficients -- apply_edge of the degree normalisation (Sec. IV-B:
 * the message of an edge is generated from the source's state; here its
 * coefficient): coef[e] = src_scale[col[e]] for every in-edge e in CSR order.
 * Done once per graph; gather_layer then reads the coefficient sequentially
 * beside the column index instead of looking it up per edge.
 * ------------------------------------------------------------------------- */
int32_t gcn_edge_coefficients(int64_t n_edges, const int32_t *col, const float *src_scale,
                              float *coef, void *stream);

/* ---------------------------------------------------------------------------
 * gather_layer -- gather_nbrs + aggregate (Sec. IV-B), i.e. the reduce R of
 * Eq. (1) with the source's hidden state as the message (Sec. II-B).  The
 * aggregate is commutative and associative, which is what makes the hub
 * partials exact (Sec. IV-D "Partial-Gather").
 *
 *   ITB_AGG_SUM : agg[v] = sum over in-edges of h[col]
 *   ITB_AGG_MEAN: the sum divided by the in-degree; 0 for an isolated vertex
 *                 With desc->edge_coef ([n_edges] fp32, CSR order) both take
 *                 edge-weighted messages w_e * h[col[e]] (apply_edge with a
 *                 scalar edge feature, Sec. IV-B); the mean still divides by
 *                 the number of in-edges.
 *   ITB_AGG_GCN : dst_scale[v] * sum of c_e * h[col]; dst_scale is required.
 *                 The source coefficient c_e of an in-edge comes from
 *                 desc->edge_coef[e] ([n_edges] fp32 in CSR order, read beside
 *                 col: see gcn_edge_coefficients) if given, else from
 *                 src_scale[col[e]] ([n_nodes], one random look-up per edge);
 *                 both NULL means the rows of h_src already carry it (see
 *                 scale_rows / msg_out)
 *   ITB_AGG_MAX / ITB_AGG_MIN: element-wise maximum / minimum of h[col] over
 *                 the in-edges, exactly (no rounding: the result is one of
 *                 the stored values); 0 for an isolated vertex; hub partials
 *                 are merged by the same operator
 *   ITB_AGG_GAT : attention-weighted sum, see below.
 *
 *   rowptr/col the CSR by destination as build_csr_by_dst writes it (rowptr
 *              non-decreasing, rowptr[n_nodes] = number of edges, every col
 *              entry in [0, n_nodes)); trusted, not validated again.
 *   dim        feature width; dim * sizeof(element) must be a multiple of 16.
 *   h_src      [n_nodes x dim] dtype_in.
 *   agg_out    [n_nodes x dim] dtype_out (f32->f32, bf16->bf16, bf16->f32).
 *   split      NULL = every row in one pass; else hub rows go through
 *              per-segment partial sums (fp32, in workspace) that are combined
 *              in ascending segment order.
 *   edge_lo/edge_hi  only rows (and segments) whose first edge offset lies in
 *              [edge_lo, edge_hi) are produced by this call; pass 0 and
 *              INT64_MAX for the whole graph.  Rows with no in-edge belong to
 *              the range that contains their rowptr value.
 *
 * The update fused into the reduce (Sec. IV-B "Inference": the computation may
 * be reorganised around the aggregate): with desc->addend, desc->bias and
 * desc->act the stored row is act(agg[v] + addend[v] + bias) instead of agg[v].
 * A narrowing layer uses it: W_nbr and W_self are applied to h first (one
 * launch, apply_layer's second product), the gather runs over h.W_nbr with
 * addend = h.W_self, and no update launch follows.  Hub rows get the epilogue
 * in the combine pass.
 *
 * ITB_AGG_GAT (Sec. II-B: GAT's reduce is an attention-weighted sum; Sec. IV-B:
 * it runs after the messages are collected): h_src is the projected state z,
 * heads divides dim, src_scale = s_src [n_nodes x heads], dst_scale = s_dst
 * [n_nodes x heads] (fp32).  For vertex v and head k, over its in-edges plus an
 * implicit self edge: e = LeakyReLU_slope(s_src[u,k] + s_dst[v,k]),
 * alpha = softmax(e), agg[v,k,:] = sum alpha_u z[u,k,:]; then bias and the
 * activation of the layer (the update that follows GAT's reduce) are applied
 * before the row is stored.  dim/heads must be a multiple of the 16-byte
 * vector (4 fp32 / 8 bf16 elements); dtype_out == dtype_in.
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t agg;        /* ITB_AGG_* */
    int32_t dtype_in;   /* ITB_F32 | ITB_BF16 */
    int32_t dtype_out;
    int32_t dim;
    int32_t heads;      /* GAT only, else 1 */
    float leaky_slope;  /* GAT only */
    int32_t act;        /* activation of the update fused into the reduce (below); ITB_ACT_NONE for a plain aggregate */
    const float *bias;  /* [dim] fp32 added to the reduced row (16-byte aligned), or NULL */
    const float *edge_coef; /* SUM / MEAN / GCN, optional: [n_edges] fp32 scalar of every in-edge, CSR order */
    const void *addend; /* not GAT, optional: [n_nodes x dim] of dtype_out added to the reduced row before the bias */
} itb_gather_desc;

int32_t gather_layer(const itb_gather_desc *desc, int64_t n_nodes,
                     const int64_t *rowptr, const int32_t *col, const itb_split *split,
                     const void *h_src, const float *src_scale, const float *dst_scale,
                     void *agg_out, int64_t edge_lo, int64_t edge_hi,
                     void *workspace, size_t *workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * gather_layer_noalloc -- gather_layer for callers that cannot allocate or
 * size a workspace: code under HIP graph capture, tight serving loops,
 * harnesses that forbid hipMalloc.  Same arguments and results (bitwise) as
 * gather_layer without the workspace pair; the work list of long rows and the
 * hub partials live in a fixed scratch array inside the library's code object,
 * ITB_NOALLOC_SCRATCH_BYTES per GPU, held until the process ends.  The call
 * allocates nothing, creates no stream or event and runs every pass on
 * `stream`.  Sizes whose workspace (what gather_layer's size query reports)
 * exceeds the array return ITB_ERR_WORKSPACE before anything is enqueued:
 * roughly 4 * n_nodes + 4 * dim * n_shadows bytes must fit.  All calls on one
 * GPU share the array: calls that overlap in time on one GPU (different
 * streams, different host threads) race and must be serialised by the caller.
 * ------------------------------------------------------------------------- */
#define ITB_NOALLOC_SCRATCH_BYTES (16u << 20)
int32_t gather_layer_noalloc(const itb_gather_desc *desc, int64_t n_nodes,
                             const int64_t *rowptr, const int32_t *col, const itb_split *split,
                             const void *h_src, const float *src_scale, const float *dst_scale,
                             void *agg_out, int64_t edge_lo, int64_t edge_hi, void *stream);

/* ---------------------------------------------------------------------------
 * aggregate_edge_features -- the edge half of apply_edge + aggregate for
 * messages that carry a feature vector of the edge (Sec. II-A: edge feature
 * matrix E; Sec. II-B: the message function takes the neighbour's state and
 * the edge; Sec. IV-B apply_edge).  Reading: the message of e = (u -> v) is
 * h[u] + ef[e] . W_e with W_e [edge_dim x dim].  Sum, mean and the
 * degree-normalised sum are linear in the message, so
 *     aggregate(messages)[v] = aggregate(h)[v] + (reduced edge features)[v] . W_e
 * and the edge features, which do not change from layer to layer, are reduced
 * per destination ONCE per graph by this call; a layer then multiplies the
 * result by its W_e (apply_layer) and hands it to gather_layer as `addend`.
 *
 *   out[v] = sum over the in-edges e of v of ef[e]          (ITB_AGG_SUM)
 *            that sum / in-degree, 0 for an isolated vertex  (ITB_AGG_MEAN)
 *            dst_scale[v] * sum of edge_coef[e] * ef[e]      (ITB_AGG_GCN; both
 *            arrays required: gcn_norm_scales, gcn_edge_coefficients)
 *   edge_feat [n_edges x edge_dim] of `dtype`, in CSR order: the rows
 *             rowptr[v] .. rowptr[v+1]-1 belong to the in-edges of v, so the
 *             reduce streams the table once.  out [n_nodes x edge_dim], `dtype`.
 * Hub rows go through the same partial / combine passes as gather_layer
 * (`split` may be NULL); workspace protocol as everywhere.  Max / min are not
 * linear in the message and are refused (ITB_ERR_UNSUPPORTED).
 * ------------------------------------------------------------------------- */
int32_t aggregate_edge_features(int32_t agg, int32_t dtype, int64_t n_nodes, const int64_t *rowptr,
                                const itb_split *split, int32_t edge_dim, const void *edge_feat,
                                const float *edge_coef, const float *dst_scale, void *out,
                                void *workspace, size_t *workspace_bytes, void *stream);

/* ---------------------------------------------------------------------------
 * apply_layer -- apply_node (Sec. IV-B), the update U of Eq. (1): combine the
 * vertex's former state with the gathered message, then the activation; the
 * store of h_out is the scatter of the new state for the next layer.
 *
 *   h_out[v] = act( h_self[v] . W_self + agg[v] . W_nbr + bias )
 *
 *   h_self [n x d_in] or NULL together with w_self (no self term).
 *   agg    [n x d_in];  w_self, w_nbr [d_in x d_out];  all of `dtype`.
 *   bias   [d_out] fp32 or NULL.   h_out [n x d_out] of `dtype`.
 *   dtype ITB_F32: fp32 matrix-core path; dtype ITB_BF16: bf16 matrix-core
 *   path with fp32 accumulation.  Rows are read as 16-byte pieces: d_in must
 *   be a multiple of 4 (fp32) / 8 (bf16); any d_out >= 1.  The weights of one
 *   32-column tile over the whole k range (d_in, twice that with a self term,
 *   rounded up to 8 / 16 values) must fit the LDS next to the staging areas:
 *   about 1000 fp32 or 2000 bf16 values of k; beyond that ITB_ERR_UNSUPPORTED.
 *   att_src/att_dst/s_src/s_dst: optional attention-score epilogue for the GAT
 *   projection: s_src[v,k] = sum_d att_src[k,d] * y[v,k,d] (fp32, from the fp32
 *   accumulators before rounding), heads dividing d_out, heads <= 16, no self
 *   term; NULL/0 to skip.
 *   msg_scale/msg_out: optional second output, the message the vertex sends in
 *   the next round (apply_edge of the scatter stage, Sec. IV-B):
 *   msg_out[v] = h_out[v] * msg_scale[v] ([n] fp32, [n x d_out] of `dtype`);
 *   both NULL to skip.
 *   addend: optional [n x d_out] tensor of `dtype` added before the
 *   activation: h_out = act(... + addend + bias).  It carries the gathered
 *   projection when W_nbr was applied before the gather (sum, mean and the
 *   degree-normalised sum are linear, so a narrowing layer can gather d_out
 *   instead of d_in elements per edge); NULL to skip.
 *   w_second/out_second: optional second product of the same rows in the same
 *   launch: out_second[v] = agg[v] . w_second ([d_in x d_out] of `dtype`, no
 *   bias, no activation; bias, addend, activation and messages apply to h_out
 *   only).  A narrowing layer uses it for h . [W_nbr | W_self]: h is read once.
 *   Needs d_out to be a multiple of 4 (fp32) / 8 (bf16), no self term and no
 *   score epilogue; both NULL to skip.
 *   chain: optional chained projection (Sec. IV-B "Inference": the computation
 *   flow may be reorganised as long as every vertex gets the same function).
 *   The finished rows h_out[v], rounded to `dtype` exactly as they would be
 *   stored, are multiplied on the spot by two more matrices,
 *     chain->out_first[v]  = h_out[v] . chain->w_first,
 *     chain->out_second[v] = h_out[v] . chain->w_second   ([d_out x dc] each),
 *   which is the next layer's h . [W_nbr | W_self] when that layer applies
 *   W_nbr before its gather: the state between the two layers is then never
 *   written or read back, and h_out may be NULL.  Built for ITB_BF16,
 *   d_out == 64, d_in a multiple of 64, dc a multiple of 8 with 2 dc <= 64, no
 *   score epilogue, no second product, no message output; other shapes return
 *   ITB_ERR_UNSUPPORTED (infer_layer_plan tells which layers qualify).  NULL to
 *   skip.
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t dtype;
    int32_t d_in, d_out;
    int32_t act;        /* ITB_ACT_* */
    int32_t heads;      /* score epilogue only, else 0 */
} itb_apply_desc;

typedef struct {
    const void *w_first;   /* [d_out x dc] of the layer's dtype */
    const void *w_second;  /* [d_out x dc] */
    int32_t dc;
    void *out_first;       /* [n x dc] */
    void *out_second;      /* [n x dc] */
} itb_apply_chain;

int32_t apply_layer(const itb_apply_desc *desc, int64_t n_nodes,
                    const void *h_self, const void *agg,
                    const void *w_self, const void *w_nbr, const float *bias,
                    void *h_out,
                    const float *att_src, const float *att_dst, float *s_src, float *s_dst,
                    const float *msg_scale, void *msg_out,
                    const void *addend,
                    const void *w_second, void *out_second,
                    const itb_apply_chain *chain,
                    void *stream);

/* ---------------------------------------------------------------------------
 * scale_rows -- apply_edge for the first round (Sec. IV-B: a vertex generates
 * its messages from its state; Sec. IV-C: the first round turns the raw
 * features into what is sent): out[v][:] = x[v][:] * row_scale[v].
 * x, out [n_nodes x dim] of `dtype`; dim * sizeof(element) multiple of 16.
 * Later rounds get the same from apply_layer's msg_out.
 * ------------------------------------------------------------------------- */
int32_t scale_rows(int32_t dtype, int64_t n_nodes, int32_t dim, const void *x, const float *row_scale,
                   void *out, void *stream);

/* ---------------------------------------------------------------------------
 * infer_full_graph -- the layer loop (Sec. IV-C: after k rounds the result of
 * a k-layer model is available for every vertex; h^0 = x, Eq. (1)).
 * Layer l: gather_layer, then apply_layer (GAT: projection, attention gather,
 * bias, activation).  Intermediate states live in `workspace`.
 *
 *   layers     host array of n_layers descriptors; weight pointers are device.
 *   x          [n_nodes x layers[0].d_in], out [n_nodes x layers[last].d_out],
 *              both of `dtype` (all layers share it).
 *   deg_out    required when a layer uses ITB_AGG_GCN, else may be NULL.
 *   edge_chunk 0 = one gather launch set per layer; else each layer's gather is
 *              issued per range of `edge_chunk` edge offsets (see gather_layer).
 * A sum/mean/GCN layer with d_out < d_in and a self matrix is evaluated as
 * act(gather(h . W_nbr) + h . W_self + bias): one matrix launch with two
 * products, then the gather with the update fused into its row epilogue (see
 * gather_layer); infer_layer_plan reports which layers take that form.  The
 * products have whole 16-byte rows: a last layer of another width (47 classes,
 * say) runs on zero-padded copies of its matrices and bias made at the start
 * of the call (copy_columns), and the padding columns are dropped when `out` is
 * written; the form is taken when the padded width is still below d_in.
 * A gather -> update layer of 64 bf16 columns in front of such a
 * layer hands its rows to that layer's two products inside its own update
 * launch (apply_layer's `chain`), and its state is never stored.  GCN
 * layers share one array of per-edge source coefficients
 * (gcn_edge_coefficients) built at the start.  With edge_chunk > 0 there may be
 * at most 65536 ranges.
 * An ITB_AGG_NONE layer is h' = act(h . w_nbr + bias) per vertex, no edges
 * touched (w_self must be NULL).
 *   edge_feat  [n_edges x edge_dim] of `dtype`, the feature vector of every
 *              in-edge in CSR order (row rowptr[v] + j belongs to the j-th
 *              in-edge of v), or NULL when no layer has an edge matrix.  A
 *              layer with w_edge takes the messages h[u] + ef[e] . W_e (see
 *              aggregate_edge_features); edge_dim * sizeof(element) must be a
 *              multiple of 16.
 *   events     NULL, or a host struct naming a host array of hipEvent_t
 *              handles, four per layer: the call records events[4l + 0..3] on
 *              `stream` at layer l's begin, before its gather, after its
 *              gather and at its end (NULL entries and layers beyond n_events
 *              are skipped).  The handles are used during the call only.
 * ------------------------------------------------------------------------- */
typedef struct {
    int32_t agg;        /* ITB_AGG_* */
    int32_t d_in, d_out;
    int32_t act;
    int32_t heads;
    float leaky_slope;
    const void *w_self; /* [d_in x d_out], NULL for GAT */
    const void *w_nbr;  /* [d_in x d_out]; GAT: the projection */
    const float *bias;  /* [d_out] or NULL */
    const float *att_src, *att_dst; /* GAT: [heads x d_out/heads] */
    const void *w_edge; /* sum / mean / GCN, optional: [edge_dim x d_in] edge matrix W_e (messages h[u] + ef[e] . W_e) */
} itb_layer;

typedef struct {
    void **events;      /* host array of hipEvent_t */
    int32_t n_events;
} itb_stage_events;

int32_t infer_full_graph(int64_t n_nodes, int64_t n_edges, const int64_t *rowptr, const int32_t *col,
                         const int32_t *deg_out, const itb_split *split,
                         int32_t dtype, int32_t n_layers, const itb_layer *layers,
                         const void *x, void *out, int64_t edge_chunk,
                         const void *edge_feat, int32_t edge_dim,
                         void *workspace, size_t *workspace_bytes,
                         const itb_stage_events *events, void *stream);

/* ---------------------------------------------------------------------------
 * copy_columns -- out[r][c] = in[r][c] for c < min(cols_in, cols_out) and 0 for
 * the columns a wider `out` has beyond cols_in: pads a row-major matrix
 * [rows x cols_in] to [rows x cols_out] with zero columns, or keeps the first
 * cols_out columns of every row.  infer_full_graph uses it for a projected last
 * layer whose width is not whole 16-byte pieces (see there).  `in` and `out`
 * are device buffers of `dtype` elements and must not overlap.
 * ------------------------------------------------------------------------- */
int32_t copy_columns(int32_t dtype, int64_t rows, int32_t cols_in, int32_t cols_out, const void *in, void *out,
                     void *stream);

/* ---------------------------------------------------------------------------
 * infer_layer_plan -- the evaluation order infer_full_graph takes for every
 * layer of a model (host only; `layers` and `plan` are host arrays, the weight
 * pointers are not dereferenced): plan[l] is one of ITB_PLAN_*.
 * ------------------------------------------------------------------------- */
enum {
    ITB_PLAN_GATHER_UPDATE = 0,   /* gather_layer on the state, then apply_layer */
    ITB_PLAN_PROJECT_GATHER = 1,  /* apply_layer with two products, then gather_layer with the fused update */
    ITB_PLAN_ATTENTION = 2,       /* projection with scores, then the attention reduce */
    ITB_PLAN_UPDATE_ONLY = 3,     /* ITB_AGG_NONE: apply_layer alone */
    ITB_PLAN_GATHER_UPDATE_CHAINED = 4 /* gather_layer, then apply_layer whose chained projection is the next layer's
                                          (ITB_PLAN_PROJECT_GATHER) pair of products: that layer starts at its gather, and
                                          this layer's state is never stored */
};
int32_t infer_layer_plan(int32_t dtype, int32_t n_layers, const itb_layer *layers, int32_t *plan);

/* ---------------------------------------------------------------------------
 * itb_shutdown -- destroys what the library owns (the helper stream and its
 * events on every device that has them), after synchronising the helper
 * stream.  Call it when no call is in flight; a later call creates the state
 * again.  Optional: the objects are otherwise released with the process.
 * ------------------------------------------------------------------------- */
int32_t itb_shutdown(void);

#ifdef __cplusplus
}
#endif
#endif /* INFERTURBO_H */
