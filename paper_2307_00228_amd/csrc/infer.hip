// infer_full_graph: the layer loop.  Each layer is a gather over every vertex followed by the dense update;
// states ping-pong between two workspace buffers (the scatter of layer l is the store that layer l+1 reads).
// Only enqueues work on the caller's stream.
#include "common.h"

namespace itb {
bool apply_shape_supported(int32_t dtype, int32_t d_in, int32_t d_out, bool has_self, int32_t heads);
bool apply_chain_supported(int32_t dtype, int32_t d_in, int32_t d_out, bool has_self, int32_t dc);
int32_t gather_layer_impl(const itb_gather_desc *desc, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                          const itb_split *split, const void *h_src, const float *src_scale, const float *dst_scale,
                          void *agg_out, int64_t edge_lo, int64_t edge_hi, void *workspace, size_t *workspace_bytes,
                          const GatherOptions &opt, void *stream);
SideStream *side_stream();
int32_t enqueue_range_bounds(int64_t n_ranges, int64_t edge_step, int64_t edge_lo, int64_t edge_hi, int64_t n_nodes,
                             const int64_t *rowptr, const itb_split *split, int64_t *out, hipStream_t st);
}

namespace {
using namespace itb;

// Stage events of the caller (four per layer: layer begin, before the gather, after the gather, layer end), recorded
// on the launch stream so that the stages of the single call can be timed without issuing them one by one.
struct Marks {
    const itb_stage_events *ev;
    void *stream;
    int32_t operator()(int layer, int which) const {
        if (!ev || !ev->events) return ITB_OK;
        const int64_t k = (int64_t)layer * 4 + which;
        if (k >= ev->n_events || !ev->events[k]) return ITB_OK;
        return hipEventRecord(static_cast<hipEvent_t>(ev->events[k]), static_cast<hipStream_t>(stream)) == hipSuccess ? ITB_OK
                                                                                                                      : ITB_ERR_DEVICE;
    }
};

__global__ void gcn_scales_kernel(int64_t n, const int64_t *rowptr, const int32_t *deg_out, float *src_scale, float *dst_scale) {
    for (int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x) {
        const int64_t din = rowptr[v + 1] - rowptr[v];
        const int32_t dout = deg_out[v];
        dst_scale[v] = 1.0f / sqrtf((float)(din > 1 ? din : 1));
        src_scale[v] = 1.0f / sqrtf((float)(dout > 1 ? dout : 1));
    }
}

// coef[e] = src_scale[col[e]]: the per-source coefficient laid out per in-edge, in CSR order.
// Four edges per thread where the arrays allow 16-byte accesses: four independent look-ups in flight per lane.
__global__ void edge_coef_kernel(int64_t n_edges, const int32_t *col, const float *src_scale, float *coef) {
    const bool vec = ((reinterpret_cast<uintptr_t>(col) | reinterpret_cast<uintptr_t>(coef)) & 15u) == 0;
    const int64_t n4 = vec ? n_edges / 4 : 0;
    for (int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; q < n4; q += (int64_t)gridDim.x * blockDim.x) {
        const int4 c = reinterpret_cast<const int4 *>(col)[q];
        reinterpret_cast<float4 *>(coef)[q] = make_float4(src_scale[c.x], src_scale[c.y], src_scale[c.z], src_scale[c.w]);
    }
    for (int64_t e = 4 * n4 + blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n_edges; e += (int64_t)gridDim.x * blockDim.x)
        coef[e] = src_scale[col[e]];
}

// out[v][:] = x[v][:] * scale[v]; one 16-byte vector per thread.
template <bool BF16>
__global__ void scale_rows_kernel(const uint4 *x, const float *scale, uint4 *out, int64_t n_vec, int32_t row_vecs) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * blockDim.x) {
        const float s = scale[i / row_vecs];
        const uint4 v = x[i];
        uint4 o;
        if constexpr (BF16) {
            o.x = pack_bf16x2(bf16_lo(v.x) * s, bf16_hi(v.x) * s);
            o.y = pack_bf16x2(bf16_lo(v.y) * s, bf16_hi(v.y) * s);
            o.z = pack_bf16x2(bf16_lo(v.z) * s, bf16_hi(v.z) * s);
            o.w = pack_bf16x2(bf16_lo(v.w) * s, bf16_hi(v.w) * s);
        } else {
            o.x = __float_as_uint(__uint_as_float(v.x) * s);
            o.y = __float_as_uint(__uint_as_float(v.y) * s);
            o.z = __float_as_uint(__uint_as_float(v.z) * s);
            o.w = __float_as_uint(__uint_as_float(v.w) * s);
        }
        out[i] = o;
    }
}

// out[r][c] = in[r][c] for c < min(cols_in, cols_out), 0 for the columns a wider `out` has beyond cols_in.
template <typename T>
__global__ void copy_columns_kernel(const T *in, T *out, int64_t rows, int32_t cols_in, int32_t cols_out) {
    const int64_t total = rows * cols_out;
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < total; i += (int64_t)gridDim.x * blockDim.x) {
        const int64_t r = i / cols_out;
        const int32_t c = (int32_t)(i - r * cols_out);
        out[i] = c < cols_in ? in[r * cols_in + c] : T(0);
    }
}

}  // namespace

extern "C" int32_t copy_columns(int32_t dtype, int64_t rows, int32_t cols_in, int32_t cols_out, const void *in, void *out,
                                void *stream) {
    if (dtype != ITB_F32 && dtype != ITB_BF16) return ITB_ERR_DTYPE;
    if (rows < 0 || cols_in <= 0 || cols_out <= 0 || rows >= ((int64_t)1 << 40)) return ITB_ERR_SIZE;
    if (rows > 0 && (!in || !out)) return ITB_ERR_NULL;
    if (rows == 0) return ITB_OK;
    int64_t g = (rows * cols_out + 255) / 256;
    if (g > 65536) g = 65536;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == ITB_BF16)
        copy_columns_kernel<uint16_t><<<(unsigned)g, 256, 0, st>>>(static_cast<const uint16_t *>(in), static_cast<uint16_t *>(out), rows, cols_in, cols_out);
    else
        copy_columns_kernel<uint32_t><<<(unsigned)g, 256, 0, st>>>(static_cast<const uint32_t *>(in), static_cast<uint32_t *>(out), rows, cols_in, cols_out);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

extern "C" int32_t scale_rows(int32_t dtype, int64_t n_nodes, int32_t dim, const void *x, const float *row_scale, void *out,
                              void *stream) {
    if (dtype != ITB_F32 && dtype != ITB_BF16) return ITB_ERR_DTYPE;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31) || dim <= 0) return ITB_ERR_SIZE;
    const int elem = dtype == ITB_BF16 ? 2 : 4;
    if ((dim * elem) % 16 != 0) return ITB_ERR_UNSUPPORTED;
    if (n_nodes > 0 && (!x || !row_scale || !out)) return ITB_ERR_NULL;
    if (!aligned16(x) || !aligned16(out)) return ITB_ERR_UNSUPPORTED;
    if (n_nodes == 0) return ITB_OK;
    const int32_t row_vecs = dim * elem / 16;
    const int64_t n_vec = n_nodes * row_vecs;
    int64_t g = (n_vec + 255) / 256;
    if (g > 32768) g = 32768;
    hipStream_t st = static_cast<hipStream_t>(stream);
    if (dtype == ITB_BF16)
        scale_rows_kernel<true><<<(unsigned)g, 256, 0, st>>>(static_cast<const uint4 *>(x), row_scale, static_cast<uint4 *>(out), n_vec, row_vecs);
    else
        scale_rows_kernel<false><<<(unsigned)g, 256, 0, st>>>(static_cast<const uint4 *>(x), row_scale, static_cast<uint4 *>(out), n_vec, row_vecs);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

extern "C" int32_t gcn_edge_coefficients(int64_t n_edges, const int32_t *col, const float *src_scale, float *coef, void *stream) {
    if (n_edges < 0 || n_edges >= ((int64_t)1 << 31)) return ITB_ERR_SIZE;
    if (n_edges > 0 && (!col || !src_scale || !coef)) return ITB_ERR_NULL;
    if (n_edges == 0) return ITB_OK;
    int64_t g = (n_edges / 4 + 255) / 256 + 1;
    if (g > 65536) g = 65536;
    edge_coef_kernel<<<(unsigned)g, 256, 0, static_cast<hipStream_t>(stream)>>>(n_edges, col, src_scale, coef);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

extern "C" int32_t gcn_norm_scales(int64_t n_nodes, const int64_t *rowptr, const int32_t *deg_out, float *src_scale,
                                   float *dst_scale, void *stream) {
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31)) return ITB_ERR_SIZE;
    if (!rowptr || (n_nodes > 0 && (!deg_out || !src_scale || !dst_scale))) return ITB_ERR_NULL;
    if (n_nodes == 0) return ITB_OK;
    int64_t g = (n_nodes + 255) / 256;
    if (g > 16384) g = 16384;
    gcn_scales_kernel<<<(unsigned)g, 256, 0, static_cast<hipStream_t>(stream)>>>(n_nodes, rowptr, deg_out, src_scale, dst_scale);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

// Sum, mean and the degree-normalised sum are linear in the source rows, so W_nbr can be applied before the gather
// (the computation flow may be reorganised around the aggregate, Sec. IV-B "Inference"): when a layer narrows
// (d_out < d_in) the edges then carry d_out instead of d_in elements.  Such a layer is one matrix launch
// h . [W_nbr | W_self] (h is read once, two row-major outputs) followed by the gather of the first output, whose row
// epilogue adds the second output and the bias and applies the activation: no update launch, and the aggregate never
// makes a round trip through memory.
// (For a layer of equal width the split into projection + update was measured slower than the fused update, even
// where it would save the pass that writes the GCN message rows: both launches are bound by their memory traffic,
// not by the matrix cores.)
// Output width of a layer rounded up to whole 16-byte pieces.
static int32_t padded_width(const itb_layer &L, int32_t dtype) {
    const int ve = dtype == ITB_BF16 ? 8 : 4;
    return (L.d_out + ve - 1) / ve * ve;
}
// A width that is not whole 16-byte pieces (47 classes, say) is padded: the layer runs on zero-padded copies of its
// matrices and bias, and the padding columns are dropped when the result is stored.  Only the last layer can have such
// a width (the next layer could not read rows that are not whole pieces).
static bool project_before_gather(const itb_layer &L, int32_t dtype, bool is_last) {
    const bool linear = L.agg == ITB_AGG_SUM || L.agg == ITB_AGG_MEAN || L.agg == ITB_AGG_GCN;
    const int32_t dp = padded_width(L, dtype);
    if (dp != L.d_out && !is_last) return false;
    // (a layer whose messages carry edge features keeps gather -> update: its edge term is added in the state space)
    return linear && L.w_self != nullptr && !L.w_edge && dp < L.d_in;
}

// The update of layer l can hand its rows straight to the projection of a narrowing layer l+1 (one launch, the state
// between the two layers is never written or read back): layer l is gather -> update, layer l+1 takes W_nbr before its
// gather and needs nothing of h_l but h_l . [W_nbr | W_self].
static bool chain_into_next(const itb_layer *layers, int l, int n_layers, int32_t dtype) {
    if (l + 1 >= n_layers || !g_tuning.chain_updates.load()) return false;
    const itb_layer &L = layers[l], &N = layers[l + 1];
    const bool plain = L.agg != ITB_AGG_NONE && L.agg != ITB_AGG_GAT && !project_before_gather(L, dtype, false);
    return plain && project_before_gather(N, dtype, l + 2 == n_layers) &&
           apply_chain_supported(dtype, L.d_in, L.d_out, L.w_self != nullptr, padded_width(N, dtype));
}

extern "C" int32_t infer_layer_plan(int32_t dtype, int32_t n_layers, const itb_layer *layers, int32_t *plan) {
    if (!layers || !plan) return ITB_ERR_NULL;
    if (n_layers <= 0) return ITB_ERR_SIZE;
    if (dtype != ITB_F32 && dtype != ITB_BF16) return ITB_ERR_DTYPE;
    for (int l = 0; l < n_layers; ++l) {
        const itb_layer &L = layers[l];
        if (L.agg < ITB_AGG_SUM || L.agg > ITB_AGG_NONE) return ITB_ERR_DTYPE;
        plan[l] = L.agg == ITB_AGG_NONE  ? ITB_PLAN_UPDATE_ONLY
                  : L.agg == ITB_AGG_GAT ? ITB_PLAN_ATTENTION
                  : project_before_gather(L, dtype, l + 1 == n_layers) ? ITB_PLAN_PROJECT_GATHER
                                                    : ITB_PLAN_GATHER_UPDATE;
    }
    for (int l = 0; l + 1 < n_layers; ++l)
        if (layers[l + 1].agg >= ITB_AGG_SUM && layers[l + 1].agg <= ITB_AGG_NONE && chain_into_next(layers, l, n_layers, dtype))
            plan[l] = ITB_PLAN_GATHER_UPDATE_CHAINED;
    return ITB_OK;
}


extern "C" int32_t infer_full_graph(int64_t n_nodes, int64_t n_edges, const int64_t *rowptr, const int32_t *col,
                                    const int32_t *deg_out, const itb_split *split, int32_t dtype, int32_t n_layers,
                                    const itb_layer *layers, const void *x, void *out, int64_t edge_chunk,
                                    const void *edge_feat, int32_t edge_dim, void *workspace, size_t *workspace_bytes,
                                    const itb_stage_events *events, void *stream) {
    if (!workspace_bytes || !layers) return ITB_ERR_NULL;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31) || n_edges < 0 || n_edges >= ((int64_t)1 << 31) || n_layers <= 0 ||
        edge_chunk < 0)
        return ITB_ERR_SIZE;
    if (dtype != ITB_F32 && dtype != ITB_BF16) return ITB_ERR_DTYPE;
    const size_t elem = dtype == ITB_BF16 ? 2 : 4;
    int32_t max_d = 0;
    bool any_gcn = false, any_project = false;
    bool edge_kind[3] = {false, false, false};  // layers with an edge matrix, by aggregator (sum, mean, GCN)
    int32_t max_heads = 0;
    size_t gather_ws = 0;
    int pad_layer = -1;   // the (last) layer that runs on zero-padded matrices, if any
    for (int l = 0; l < n_layers; ++l) {
        const itb_layer &L = layers[l];
        if (L.agg < ITB_AGG_SUM || L.agg > ITB_AGG_NONE) return ITB_ERR_DTYPE;
        if (L.d_in <= 0 || L.d_out <= 0) return ITB_ERR_SIZE;
        if (l > 0 && L.d_in != layers[l - 1].d_out) return ITB_ERR_SIZE;
        if (L.d_in > max_d) max_d = L.d_in;
        if (L.d_out > max_d) max_d = L.d_out;
        if (L.agg == ITB_AGG_NONE) {  // per-vertex layer: no gather, no gather workspace
            if (L.w_self) return ITB_ERR_UNSUPPORTED;
            if (!apply_shape_supported(dtype, L.d_in, L.d_out, false, 0)) return ITB_ERR_UNSUPPORTED;
            continue;
        }
        any_gcn = any_gcn || L.agg == ITB_AGG_GCN;
        const bool gat = L.agg == ITB_AGG_GAT;
        if (L.w_edge) {
            // messages h[u] + ef[e] . W_e: the reduce is linear, so the edge term is (reduced edge features) . W_e
            if (L.agg != ITB_AGG_SUM && L.agg != ITB_AGG_MEAN && L.agg != ITB_AGG_GCN) return ITB_ERR_UNSUPPORTED;
            if (edge_dim <= 0 || (edge_dim * (int)elem) % 16 != 0) return ITB_ERR_UNSUPPORTED;
            if (!apply_shape_supported(dtype, edge_dim, L.d_in, false, 0)) return ITB_ERR_UNSUPPORTED;
            edge_kind[L.agg] = true;
            any_project = true;  // the edge term of the layer lives in the projection buffer
        }
        if (gat && L.heads > max_heads) max_heads = L.heads;
        const bool pf = project_before_gather(L, dtype, l + 1 == n_layers);
        any_project = any_project || pf;
        const int32_t dp = pf ? padded_width(L, dtype) : L.d_out;   // a projected layer runs at whole 16-byte rows
        if (dp != L.d_out) pad_layer = l;
        // every update launch of the layer must have a kernel configuration: refuse the model before enqueueing anything
        if (gat ? !apply_shape_supported(dtype, L.d_in, L.d_out, false, L.heads)
                : (pf ? !apply_shape_supported(dtype, L.d_in, dp, false, 0)
                      : !apply_shape_supported(dtype, L.d_in, L.d_out, L.w_self != nullptr, 0)))
            return ITB_ERR_UNSUPPORTED;
        itb_gather_desc gd{L.agg, dtype, dtype, gat ? L.d_out : (pf ? dp : L.d_in), gat ? L.heads : 1, L.leaky_slope, ITB_ACT_NONE, nullptr, nullptr, nullptr};
        size_t need = 0;
        int32_t rc = gather_layer(&gd, n_nodes, rowptr, col, split, nullptr, nullptr, nullptr, nullptr, 0, INT64_MAX, nullptr,
                                  &need, nullptr);
        if (rc != ITB_OK) return rc;
        if (need > gather_ws) gather_ws = need;
    }
    const int64_t n_chunks = (edge_chunk > 0 && n_edges > 0) ? (n_edges + edge_chunk - 1) / edge_chunk : 1;
    if (n_chunks > 65536) return ITB_ERR_SIZE;  // (the ranges' row bounds are kept in the workspace)
    Carver cv(workspace);
    const size_t state_bytes = (size_t)n_nodes * max_d * elem;
    char *state0 = cv.take<char>(n_layers > 1 ? state_bytes : 0);
    char *state1 = cv.take<char>(n_layers > 2 ? state_bytes : 0);
    char *aggbuf = cv.take<char>(state_bytes);
    float *edge_coef = cv.take<float>(any_gcn ? (size_t)n_edges : 0);  // source coefficient of every in-edge (GCN layers)
    char *projbuf = cv.take<char>(any_project ? state_bytes : 0);  // W_nbr-projected rows of a narrowing layer
    float *src_scale = cv.take<float>(any_gcn ? (size_t)n_nodes : 0);
    float *dst_scale = cv.take<float>(any_gcn ? (size_t)n_nodes : 0);
    float *att_s_src = cv.take<float>((size_t)n_nodes * max_heads);
    float *att_s_dst = cv.take<float>((size_t)n_nodes * max_heads);
    char *edge_sum[3];
    for (int k = 0; k < 3; ++k) edge_sum[k] = cv.take<char>(edge_kind[k] ? (size_t)n_nodes * edge_dim * elem : 0);
    size_t edge_ws = 0;
    if (edge_kind[0] || edge_kind[1] || edge_kind[2]) {
        const int32_t rc = aggregate_edge_features(ITB_AGG_SUM, dtype, n_nodes, nullptr, split, edge_dim, nullptr, nullptr, nullptr,
                                                   nullptr, nullptr, &edge_ws, nullptr);
        if (rc != ITB_OK) return rc;
        if (edge_ws > gather_ws) gather_ws = edge_ws;
    }
    // zero-padded copies of the matrices and the bias of a projected last layer whose width is not whole 16-byte pieces,
    // and its result at the padded width
    const int32_t pad_dp = pad_layer >= 0 ? padded_width(layers[pad_layer], dtype) : 0;
    char *pad_w_nbr = cv.take<char>(pad_layer >= 0 ? (size_t)layers[pad_layer].d_in * pad_dp * elem : 0);
    char *pad_w_self = cv.take<char>(pad_layer >= 0 ? (size_t)layers[pad_layer].d_in * pad_dp * elem : 0);
    float *pad_bias = cv.take<float>(pad_layer >= 0 ? (size_t)pad_dp : 0);
    char *pad_out = cv.take<char>(pad_layer >= 0 ? (size_t)n_nodes * pad_dp * elem : 0);
    char *gws = cv.take<char>(gather_ws);
    int64_t *range_bounds = cv.take<int64_t>(n_chunks > 1 ? 6 * (size_t)n_chunks : 0);
    if (!workspace) {
        *workspace_bytes = cv.off;
        return ITB_OK;
    }
    if (*workspace_bytes < cv.off || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return ITB_ERR_WORKSPACE;
    if (!rowptr || (n_nodes > 0 && (!x || !out)) || (n_edges > 0 && !col) || (any_gcn && n_nodes > 0 && !deg_out)) return ITB_ERR_NULL;
    if ((edge_kind[0] || edge_kind[1] || edge_kind[2]) && n_edges > 0 && !edge_feat) return ITB_ERR_NULL;
    if (n_nodes == 0) return ITB_OK;

    if (any_gcn) {
        // The coefficient of a GCN edge factors into a per-source and a per-destination part.  The source part is
        // laid out once per in-edge (apply_edge, done in preprocessing) so that every GCN gather reads it beside the
        // column index: a sequential 4 bytes per edge instead of a random look-up, and no scaled copy of the state.
        int32_t rc = gcn_norm_scales(n_nodes, rowptr, deg_out, src_scale, dst_scale, stream);
        if (rc != ITB_OK) return rc;
        rc = gcn_edge_coefficients(n_edges, col, src_scale, edge_coef, stream);
        if (rc != ITB_OK) return rc;
    }
    if (events && events->n_events < 0) return ITB_ERR_SIZE;
    if (n_chunks > 1) {
        // the rows, shadow segments and hubs of every edge range, once per call (they depend on the graph only)
        const int32_t rc = enqueue_range_bounds(n_chunks, edge_chunk, 0, 0, n_nodes, rowptr, split, range_bounds,
                                                static_cast<hipStream_t>(stream));
        if (rc != ITB_OK) return rc;
    }
    if (pad_layer >= 0) {
        const itb_layer &P = layers[pad_layer];
        if (!P.w_nbr || !P.w_self) return ITB_ERR_NULL;
        int32_t rc = copy_columns(dtype, P.d_in, P.d_out, pad_dp, P.w_nbr, pad_w_nbr, stream);
        if (rc == ITB_OK) rc = copy_columns(dtype, P.d_in, P.d_out, pad_dp, P.w_self, pad_w_self, stream);
        if (rc == ITB_OK && P.bias) rc = copy_columns(ITB_F32, 1, P.d_out, pad_dp, P.bias, pad_bias, stream);
        if (rc != ITB_OK) return rc;
    }
    const Marks mark{events, stream};
    // Edge features are static, so their reduce per destination is taken once per aggregator, before the layer loop
    // (Sec. IV-B: the computation flow may be reorganised as long as the result is the same function).
    for (int k = 0; k < 3; ++k) {
        if (!edge_kind[k]) continue;
        size_t ws = gather_ws;
        const int32_t rc = aggregate_edge_features(k, dtype, n_nodes, rowptr, split, edge_dim, edge_feat, edge_coef, dst_scale,
                                                   edge_sum[k], gws, &ws, stream);
        if (rc != ITB_OK) return rc;
    }
    char *state[2] = {state0, state1};
    const void *cur = x;
    bool projected_by_previous = false;   // this layer's h . [W_nbr | W_self] came out of the previous layer's update
    for (int l = 0; l < n_layers; ++l) {
        const itb_layer &L = layers[l];
        void *dst = (l == n_layers - 1) ? out : static_cast<void *>(state[l & 1]);
        const bool chain = chain_into_next(layers, l, n_layers, dtype);
        if (mark(l, 0) != ITB_OK) return ITB_ERR_DEVICE;
        if (L.agg == ITB_AGG_NONE) {
            if (mark(l, 1) != ITB_OK || mark(l, 2) != ITB_OK) return ITB_ERR_DEVICE;
            // encoder / prediction head (Sec. IV-C): the update alone, on the vertex's own state
            itb_apply_desc ad{dtype, L.d_in, L.d_out, L.act, 0};
            int32_t rc = apply_layer(&ad, n_nodes, nullptr, cur, nullptr, L.w_nbr, L.bias, dst, nullptr, nullptr, nullptr, nullptr,
                                     nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, stream);
            if (rc != ITB_OK) return rc;
            if (mark(l, 3) != ITB_OK) return ITB_ERR_DEVICE;
            cur = dst;
            continue;
        }
        const bool gat = L.agg == ITB_AGG_GAT;
        const bool gcn = L.agg == ITB_AGG_GCN;
        const void *gather_src = cur;
        const float *gs = nullptr, *gd_scale = gcn ? dst_scale : nullptr;
        void *gather_out = aggbuf;
        itb_gather_desc gd{L.agg, dtype, dtype, L.d_in, 1, 0.f, ITB_ACT_NONE, nullptr, gcn ? edge_coef : nullptr, nullptr};
        const bool pf = project_before_gather(L, dtype, l + 1 == n_layers);
        const bool padded = pf && l == pad_layer;
        const int32_t dp = padded ? pad_dp : L.d_out;
        const void *w_nbr = padded ? pad_w_nbr : L.w_nbr, *w_self = padded ? pad_w_self : L.w_self;
        const float *bias = padded ? (L.bias ? pad_bias : nullptr) : L.bias;
        if (gat) {
            // project first (z and the per-head scores), then the attention reduce writes the new state directly
            if (!L.w_nbr || !L.att_src || !L.att_dst) return ITB_ERR_NULL;
            itb_apply_desc pd{dtype, L.d_in, L.d_out, ITB_ACT_NONE, L.heads};
            int32_t rc = apply_layer(&pd, n_nodes, nullptr, cur, nullptr, L.w_nbr, nullptr, aggbuf, L.att_src, L.att_dst,
                                     att_s_src, att_s_dst, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, stream);
            if (rc != ITB_OK) return rc;
            gather_src = aggbuf;
            gs = att_s_src;
            gd_scale = att_s_dst;
            gather_out = dst;
            gd = itb_gather_desc{L.agg, dtype, dtype, L.d_out, L.heads, L.leaky_slope, L.act, L.bias, nullptr, nullptr};
        }
        if (pf) {
            // h . [W_nbr | W_self] in one launch; the gather of the first product finishes the layer in its row epilogue
            const void *self_product = aggbuf;
            if (projected_by_previous) {
                // both products left the previous layer's update: first in projbuf, second in that layer's state buffer
                self_product = state[(l - 1) & 1];
            } else {
                itb_apply_desc pd{dtype, L.d_in, dp, ITB_ACT_NONE, 0};
                int32_t rc = apply_layer(&pd, n_nodes, nullptr, gather_src, nullptr, w_nbr, nullptr, projbuf, nullptr, nullptr,
                                         nullptr, nullptr, nullptr, nullptr, nullptr, w_self, aggbuf, nullptr, stream);
                if (rc != ITB_OK) return rc;
            }
            gather_src = projbuf;
            gather_out = padded ? static_cast<void *>(pad_out) : dst;
            gd.dim = dp;
            gd.addend = self_product;
            gd.bias = bias;
            gd.act = L.act;
        }
        projected_by_previous = false;
        if (L.w_edge) {
            // the edge term of the aggregate, in the state space: (reduced edge features) . W_e, added in the gather's epilogue
            itb_apply_desc ed{dtype, edge_dim, L.d_in, ITB_ACT_NONE, 0};
            int32_t rc = apply_layer(&ed, n_nodes, nullptr, edge_sum[L.agg], nullptr, L.w_edge, nullptr, projbuf, nullptr, nullptr,
                                     nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, stream);
            if (rc != ITB_OK) return rc;
            gd.addend = projbuf;
        }
        if (mark(l, 1) != ITB_OK) return ITB_ERR_DEVICE;
        {
            // One fork of the helper stream for all edge ranges of the layer: the hub passes of the ranges queue up on the
            // helper stream, the row passes on the caller's, and the two streams meet once, after the last range
            // (ranges write disjoint rows; the partials buffer is reused in helper-stream order).
            SideFork layer_fork;
            GatherOptions opt;
            const bool hubs = split && split->n_hubs > 0;
            if (n_chunks > 1 && hubs && g_tuning.overlap_hubs.load()) {
                const int32_t rc = layer_fork.begin(side_stream(), static_cast<hipStream_t>(stream));
                if (rc != ITB_OK) return rc;
                opt.outer_fork = &layer_fork;
            }
            for (int64_t c = 0; c < n_chunks; ++c) {
                const int64_t lo = (n_chunks == 1) ? 0 : c * edge_chunk;
                const int64_t hi = (c == n_chunks - 1) ? INT64_MAX : (c + 1) * edge_chunk;
                size_t ws = gather_ws;
                opt.bounds = n_chunks > 1 ? range_bounds + 6 * c : nullptr;
                const int32_t rc = gather_layer_impl(&gd, n_nodes, rowptr, col, split, gather_src, gs, gd_scale, gather_out, lo, hi,
                                                     gws, &ws, opt, stream);
                if (rc != ITB_OK) return rc;   // (layer_fork joins in its destructor)
            }
            const int32_t rc = layer_fork.finish();
            if (rc != ITB_OK) return rc;
        }
        if (mark(l, 2) != ITB_OK) return ITB_ERR_DEVICE;
        if (!gat && !pf) {
            itb_apply_desc ad{dtype, L.d_in, L.d_out, L.act, 0};
            // chained: the new state goes straight into the next layer's projection and is never stored; the two products
            // take the projection buffer and this layer's (otherwise unused) state buffer
            const itb_layer &N = layers[chain ? l + 1 : l];
            const bool next_padded = chain && l + 1 == pad_layer;
            const itb_apply_chain ch{next_padded ? pad_w_nbr : N.w_nbr, next_padded ? pad_w_self : N.w_self,
                                     next_padded ? pad_dp : N.d_out, projbuf, dst};
            int32_t rc = apply_layer(&ad, n_nodes, L.w_self ? cur : nullptr, aggbuf, L.w_self, L.w_nbr, L.bias, chain ? nullptr : dst,
                                     nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr, nullptr,
                                     chain ? &ch : nullptr, stream);   // no self matrix: no self term
            if (rc != ITB_OK) return rc;
            projected_by_previous = chain;
        }
        if (padded) {   // drop the padding columns
            const int32_t rc = copy_columns(dtype, n_nodes, dp, L.d_out, pad_out, dst, stream);
            if (rc != ITB_OK) return rc;
        }
        if (mark(l, 3) != ITB_OK) return ITB_ERR_DEVICE;
        cur = dst;
    }
    return ITB_OK;
}
