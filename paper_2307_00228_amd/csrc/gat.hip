// Attention-weighted gather (the GAT reduce): for every destination v and head k, a softmax over the scores
// of its in-edges plus an implicit self edge, applied to the projected source rows.
//
// Same data movement as the plain gather (one 16-byte vector of the source row per lane per edge, plus the
// 4-byte source score of the lane's head), so the kernels keep its shape: lane groups of G lanes per row,
// 64 rows per wavefront, short rows one lane group per row, long rows by the whole wavefront, hub rows as
// one wavefront per shadow segment.  The softmax runs online: every lane carries (running max m, denominator
// l, weighted sum acc) for its head; partial states of lane groups, and of shadow segments, are merged by
//   M = max(m1, m2);  l = l1*exp(m1-M) + l2*exp(m2-M);  acc likewise,
// which is commutative and associative, so the hub partials satisfy the rule that makes partial aggregation
// exact.  The self edge starts the state (m = e_self, l = 1, acc = z[v]), so an isolated vertex returns z[v].
// Bias and activation of the layer are applied when the row is finished.
#include "common.h"

namespace itb {
size_t lds_for_occupancy(int waves, int lanes_per_row, bool beside_hub_passes);
int32_t enqueue_range_bounds(int64_t n_ranges, int64_t edge_step, int64_t edge_lo, int64_t edge_hi, int64_t n_nodes,
                             const int64_t *rowptr, const itb_split *split, int64_t *out, hipStream_t st);
}  // namespace itb

namespace {
using namespace itb;

struct GatArgs {
    int64_t n_nodes;
    const int64_t *rowptr;
    const int32_t *col;
    const uint4 *z;        // [n_nodes x row_vecs] 16-byte vectors
    const float *s_src;    // [n_nodes x heads]
    const float *s_dst;
    const float *bias;     // [dim] or nullptr
    void *out;
    int64_t threshold;
    int64_t edge_lo, edge_hi;
    const int64_t *bounds;   // nullable: {row_lo, row_hi, seg_lo, seg_hi, hub_lo, hub_hi} of the edge range (see gather_layer)
    int32_t row_vecs, heads, dh, act;
    int32_t stream_rows;   // rows of z and scores of the sources are read with non-temporal loads (table far beyond the caches)
    float slope;
    int32_t small_limit;
    int32_t long_limit;    // rows with more in-edges go to the work list and get a whole block
    int32_t *long_list;
    uint32_t *long_count;
    // hub passes
    int64_t n_shadows;
    const int64_t *shadow_begin, *shadow_end;
    const int32_t *shadow_owner;
    float *part_acc;       // [S x dim]
    float *part_m, *part_l;  // [S x heads]
};

template <bool BF16>
struct Elems {
    static constexpr int kPerVec = BF16 ? 8 : 4;
};

template <bool BF16>
__device__ __forceinline__ void unpack(float (&f)[Elems<BF16>::kPerVec], const uint4 &raw) {
    if constexpr (BF16) {
        f[0] = bf16_lo(raw.x); f[1] = bf16_hi(raw.x); f[2] = bf16_lo(raw.y); f[3] = bf16_hi(raw.y);
        f[4] = bf16_lo(raw.z); f[5] = bf16_hi(raw.z); f[6] = bf16_lo(raw.w); f[7] = bf16_hi(raw.w);
    } else {
        f[0] = __uint_as_float(raw.x); f[1] = __uint_as_float(raw.y); f[2] = __uint_as_float(raw.z); f[3] = __uint_as_float(raw.w);
    }
}

template <int VE>
struct SoftState {
    float m, l;
    float acc[VE];
};

__device__ __forceinline__ float leaky(float x, float slope) { return x > 0.f ? x : slope * x; }

// one edge into the running state; `on` false leaves the state unchanged
template <bool BF16>
__device__ __forceinline__ void absorb(SoftState<Elems<BF16>::kPerVec> &st, float e, const uint4 &raw, bool on) {
    constexpr int VE = Elems<BF16>::kPerVec;
    const float mn = on ? fmaxf(st.m, e) : st.m;
    const float sc = __expf(st.m - mn);
    const float p = on ? __expf(e - mn) : 0.f;
    float f[VE];
    unpack<BF16>(f, raw);
    st.l = fmaf(st.l, sc, p);
#pragma unroll
    for (int i = 0; i < VE; ++i) st.acc[i] = fmaf(st.acc[i], sc, p * f[i]);
    st.m = mn;
}

// A batch of U edges.  The running maximum settles after a few edges of a row (it changes about ln(degree)
// times), so the common case -- no lane of the wavefront sees a larger score -- skips the rescaling of the
// accumulators: one exponential and one fused multiply-add per element.
template <bool BF16, int U>
__device__ __forceinline__ void absorb_batch(SoftState<Elems<BF16>::kPerVec> &st, const float (&e)[U], const uint4 (&raw)[U],
                                             const bool (&on)[U]) {
    constexpr int VE = Elems<BF16>::kPerVec;
    bool grows = false;
#pragma unroll
    for (int q = 0; q < U; ++q) grows = grows || (on[q] && e[q] > st.m);
    if (__ballot(grows) == 0ull) {
#pragma unroll
        for (int q = 0; q < U; ++q) {
            const float p = on[q] ? __expf(e[q] - st.m) : 0.f;
            float f[VE];
            unpack<BF16>(f, raw[q]);
            st.l += p;
#pragma unroll
            for (int i = 0; i < VE; ++i) st.acc[i] = fmaf(p, f[i], st.acc[i]);
        }
    } else {
#pragma unroll
        for (int q = 0; q < U; ++q) absorb<BF16>(st, e[q], raw[q], on[q]);
    }
}

// merge the state held by the lane `off` lanes away (same head: off is a multiple of the lane-group size)
template <int VE>
__device__ __forceinline__ void merge_xor(SoftState<VE> &st, int off) {
    const float m2 = __shfl_xor(st.m, off, kWave);
    const float l2 = __shfl_xor(st.l, off, kWave);
    const float M = fmaxf(st.m, m2);
    const float s1 = __expf(st.m - M), s2 = __expf(m2 - M);
    st.l = st.l * s1 + l2 * s2;
#pragma unroll
    for (int i = 0; i < VE; ++i) st.acc[i] = st.acc[i] * s1 + __shfl_xor(st.acc[i], off, kWave) * s2;
    st.m = M;
}

constexpr float kNegInf = -3.0e38f;  // "no edge yet": exp(kNegInf - m) underflows to exactly 0

__device__ __forceinline__ int64_t shfl_i64(int64_t v, int src) {
    int lo = __shfl((int)(v & 0xffffffff), src, kWave);
    int hi = __shfl((int)(v >> 32), src, kWave);
    return ((int64_t)hi << 32) | (uint32_t)lo;
}

// Whole-wavefront pass over the edges [start, start+deg) of destination score sd; lane group g takes the
// edges congruent to g modulo 64/G in every 64-edge chunk; on return all lane groups hold the merged state.
template <bool BF16, int G>
__device__ __forceinline__ void wave_segment_softmax(SoftState<Elems<BF16>::kPerVec> &st, const GatArgs &a, int64_t start,
                                                     int64_t deg, float sd, int vec, int hk, bool lane_on,
                                                     int first_chunk = 0, int chunk_stride = 1) {
    constexpr int NG = kWave / G;
    constexpr int U = 4;   // (8 row loads in flight, which pays for the plain gather, measured no gain here)
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / G;
    const int vec_c = lane_on ? vec : 0;   // lanes beyond the row's width read its first vector (never used)
    for (int64_t c = (int64_t)first_chunk * kWave; c < deg; c += (int64_t)chunk_stride * kWave) {
        int myc = 0;
        if (c + lane < deg) myc = a.col[start + c + lane];
        const int cnt = (deg - c < kWave) ? (int)(deg - c) : kWave;
        const int steps = (cnt + NG - 1) / NG;
        for (int t = 0; t < steps; t += U) {
            uint4 raw[U];
            float e[U];
            bool on[U];
            auto issue = [&](auto stream_tag) {
                constexpr bool S = decltype(stream_tag)::value;
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    // A slot past the end of the chunk re-reads the chunk's last edge and enters with weight zero (its
                    // row is a row this segment sums anyway): the loads need no predicate and no select.
                    const int ei = (t + q) * NG + g;
                    const int eic = ei < cnt ? ei : cnt - 1;
                    const int u = __shfl(myc, eic, kWave);
                    on[q] = lane_on && ei < cnt;
                    raw[q] = load_row_piece<S>(a.z + ((int64_t)u * a.row_vecs + vec_c));
                    e[q] = load_row_scalar<S>(a.s_src + ((int64_t)u * a.heads + hk));
                }
            };
            if (a.stream_rows) issue(std::true_type{}); else issue(std::false_type{});  // kernel argument: wave-uniform
#pragma unroll
            for (int q = 0; q < U; ++q) e[q] = leaky(e[q] + sd, a.slope);
            absorb_batch<BF16, U>(st, e, raw, on);
        }
    }
#pragma unroll
    for (int off = G; off < kWave; off <<= 1) merge_xor(st, off);
}

// out = act(acc / l + bias): one reciprocal per lane and row, bias fetched as 16-byte vectors.
template <bool BF16, int VE>
__device__ __forceinline__ void finish_store(const GatArgs &a, int64_t row, int vec, const float (&acc)[VE], float l) {
    float y[VE];
    const float inv = 1.0f / l;
#pragma unroll
    for (int i = 0; i < VE; ++i) y[i] = acc[i] * inv;
    if (a.bias) {
        const float4 *b4 = reinterpret_cast<const float4 *>(a.bias + vec * VE);
#pragma unroll
        for (int k = 0; k < VE / 4; ++k) {
            const float4 b = b4[k];
            y[4 * k + 0] += b.x; y[4 * k + 1] += b.y; y[4 * k + 2] += b.z; y[4 * k + 3] += b.w;
        }
    }
    if (a.act == ITB_ACT_RELU) {
#pragma unroll
        for (int i = 0; i < VE; ++i) y[i] = fmaxf(y[i], 0.f);
    }
    const int64_t elem0 = (row * a.row_vecs + vec) * VE;
    if constexpr (BF16) {
        uint4 p;
        p.x = pack_bf16x2(y[0], y[1]); p.y = pack_bf16x2(y[2], y[3]);
        p.z = pack_bf16x2(y[4], y[5]); p.w = pack_bf16x2(y[6], y[7]);
        store_piece(static_cast<uint16_t *>(a.out) + elem0, p, a.stream_rows);   // non-temporal beside streamed row loads
    } else {
        store_piece(static_cast<float *>(a.out) + elem0,
                    make_uint4(__float_as_uint(y[0]), __float_as_uint(y[1]), __float_as_uint(y[2]), __float_as_uint(y[3])), a.stream_rows);
    }
}

template <bool BF16, int G>
__global__ __launch_bounds__(256) void gat_rows_kernel(GatArgs a) {
    constexpr int NG = kWave / G;
    constexpr int VE = Elems<BF16>::kPerVec;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / G;
    const int li = lane % G;
    const int64_t r0 = ((int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave)) * kWave;
    if (r0 >= a.n_nodes) return;
    if (a.bounds && (r0 + kWave <= a.bounds[0] || r0 >= a.bounds[1])) return;  // no row of this wavefront starts in the range
    const int vec = blockIdx.y * G + li;
    const bool lane_on = vec < a.row_vecs;
    const int hk = lane_on ? (vec * VE) / a.dh : 0;

    const int64_t my_row = r0 + lane;
    int64_t rs = 0, re = 0;
    if (my_row < a.n_nodes) {
        rs = a.rowptr[my_row];
        re = a.rowptr[my_row + 1];
    }
    const int64_t deg64 = re - rs;
    const bool mine = my_row < a.n_nodes && rs >= a.edge_lo && rs < a.edge_hi && deg64 <= a.threshold;
    const int deg = (int)deg64;
    // A vertex without in-edges attends to itself only: alpha = 1, the row is finish(z[v]).  Power-law
    // in-degrees leave most vertices in this state, so they get a streaming pass of their own: no scores, no
    // exponentials, four independent row copies in flight per lane group.
    const uint64_t iso_mask = __ballot(mine && deg == 0);
    if (iso_mask) {
        constexpr int Q = 4;
        constexpr int STEP = (NG * Q > kWave) ? kWave : NG * Q;
        for (int sub = 0; sub < kWave; sub += STEP) {
            const uint64_t sel = (STEP == kWave) ? iso_mask : ((iso_mask >> sub) & ((1ull << STEP) - 1ull));
            if (sel == 0) continue;
            uint4 raw[Q];
            bool on[Q];
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                const int rl = sub + q * NG + g;
                on[q] = lane_on && rl < kWave && ((iso_mask >> (rl & (kWave - 1))) & 1ull);
                raw[q] = on[q] ? a.z[(r0 + rl) * a.row_vecs + vec] : make_uint4(0, 0, 0, 0);
            }
#pragma unroll
            for (int q = 0; q < Q; ++q) {
                if (on[q]) {
                    float f[VE];
                    unpack<BF16>(f, raw[q]);
                    finish_store<BF16, VE>(a, r0 + sub + q * NG + g, vec, f, 1.f);
                }
            }
        }
    }
    const uint64_t small_mask = __ballot(mine && deg > 0 && deg <= a.small_limit);
    uint64_t large_mask = __ballot(mine && deg > a.small_limit && deg <= a.long_limit);
    const uint64_t long_mask = __ballot(mine && deg > a.long_limit);
    // hand the long rows to the block-per-row kernel (the list order enters no result); one entry per row: only the
    // first of the column blocks (blockIdx.y) that share these rows appends
    if (long_mask && blockIdx.y == 0) {
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(a.long_count, (uint32_t)__popcll(long_mask));
        base = __shfl(base, 0, kWave);
        if ((long_mask >> lane) & 1ull) {
            const uint64_t below = (lane == 0) ? 0ull : (long_mask & (~0ull >> (kWave - lane)));
            a.long_list[base + (uint32_t)__popcll(below)] = (int32_t)my_row;
        }
    }

    // Rows with few in-edges (most rows of a power-law graph, isolated ones included): one lane group per row and
    // R rows per lane group in flight, so that R independent row loads are outstanding per lane.
    if (small_mask) {
        constexpr int R = 2;
        constexpr int STEP = (NG * R > kWave) ? kWave : NG * R;
        for (int sub = 0; sub < kWave; sub += STEP) {
            const uint64_t sel = (STEP == kWave) ? small_mask : ((small_mask >> sub) & ((1ull << STEP) - 1ull));
            if (sel == 0) continue;
            int d[R];
            int64_t st0[R], v[R];
            bool on_v[R];
            float sd[R];
            SoftState<VE> st[R];
#pragma unroll
            for (int r = 0; r < R; ++r) {
                const int rl = sub + r * NG + g;
                const bool act = rl < kWave && ((small_mask >> (rl & (kWave - 1))) & 1ull);
                d[r] = __shfl(deg, rl & (kWave - 1), kWave);
                if (!act) d[r] = 0;
                st0[r] = shfl_i64(rs, rl & (kWave - 1));
                v[r] = (act && r0 + rl < a.n_nodes) ? r0 + rl : a.n_nodes - 1;
                on_v[r] = act && lane_on;
            }
#pragma unroll
            for (int r = 0; r < R; ++r) {   // the implicit self edge starts each state
                sd[r] = on_v[r] ? a.s_dst[v[r] * a.heads + hk] : 0.f;
                const uint4 raw = on_v[r] ? a.z[v[r] * a.row_vecs + vec] : make_uint4(0, 0, 0, 0);
                st[r].m = on_v[r] ? leaky(a.s_src[v[r] * a.heads + hk] + sd[r], a.slope) : 0.f;
                st[r].l = 1.f;
                unpack<BF16>(st[r].acc, raw);
            }
            for (int j = 0;; j += G) {
                bool more = false;
#pragma unroll
                for (int r = 0; r < R; ++r) more = more || j < d[r];
                if (__ballot(more) == 0ull) break;
                int myc[R];
#pragma unroll
                for (int r = 0; r < R; ++r) myc[r] = (j + li < d[r]) ? a.col[st0[r] + j + li] : 0;
                for (int t = 0; t < G; ++t) {
                    bool any = false;
#pragma unroll
                    for (int r = 0; r < R; ++r) any = any || (j + t) < d[r];
                    if (__ballot(any) == 0ull) break;
                    uint4 raw[R];
                    float e[R];
                    bool on[R];
                    auto issue = [&](auto stream_tag) {
                        constexpr bool S = decltype(stream_tag)::value;
#pragma unroll
                        for (int r = 0; r < R; ++r) {
                            const int u = __shfl(myc[r], g * G + t, kWave);
                            on[r] = lane_on && (j + t) < d[r];
                            raw[r] = on[r] ? load_row_piece<S>(a.z + ((int64_t)u * a.row_vecs + vec)) : make_uint4(0, 0, 0, 0);
                            e[r] = on[r] ? load_row_scalar<S>(a.s_src + ((int64_t)u * a.heads + hk)) : 0.f;
                        }
                    };
                    if (a.stream_rows) issue(std::true_type{}); else issue(std::false_type{});
#pragma unroll
                    for (int r = 0; r < R; ++r) absorb<BF16>(st[r], leaky(e[r] + sd[r], a.slope), raw[r], on[r]);
                }
            }
#pragma unroll
            for (int r = 0; r < R; ++r)
                if (on_v[r]) finish_store<BF16, VE>(a, v[r], vec, st[r].acc, st[r].l);
        }
    }

    while (large_mask) {
        const int rl = __ffsll((unsigned long long)large_mask) - 1;
        large_mask &= large_mask - 1;
        const int d = __shfl(deg, rl, kWave);
        const int64_t st0 = shfl_i64(rs, rl);
        const int64_t v = r0 + rl;
        const float sd = lane_on ? a.s_dst[v * a.heads + hk] : 0.f;
        SoftState<VE> st;
        if (g == 0) {   // lane group 0 carries the self edge, the others start empty
            const uint4 raw = lane_on ? a.z[v * a.row_vecs + vec] : make_uint4(0, 0, 0, 0);
            st.m = lane_on ? leaky(a.s_src[v * a.heads + hk] + sd, a.slope) : 0.f;
            st.l = 1.f;
            unpack<BF16>(st.acc, raw);
        } else {
            st.m = kNegInf;
            st.l = 0.f;
#pragma unroll
            for (int i = 0; i < VE; ++i) st.acc[i] = 0.f;
        }
        wave_segment_softmax<BF16, G>(st, a, st0, d, sd, vec, hk, lane_on);
        if (g == 0 && lane_on) finish_store<BF16, VE>(a, v, vec, st.acc, st.l);
    }
}

constexpr int kRangeWaves = 8;  // wavefronts that share one edge range (a shadow segment or a long row)

// Block-cooperative pass over one edge range: wave w takes the 64-edge chunks congruent to w modulo kRangeWaves,
// the wave states are merged in wave order.  `st` is the caller's starting state for wave 0's lane group 0
// (the self edge, or empty); every other lane group starts empty.  On return lane group 0 of wave 0 holds
// the merged state.
template <bool BF16, int G>
__device__ __forceinline__ void block_range_softmax(SoftState<Elems<BF16>::kPerVec> &st, const GatArgs &a, int64_t start,
                                                    int64_t deg, float sd, int vec, int hk, bool lane_on, float *sm) {
    constexpr int VE = Elems<BF16>::kPerVec;
    constexpr int SV = VE + 2;  // floats per lane state
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    if (!(w == 0 && lane < G)) {
        st.m = kNegInf;
        st.l = 0.f;
#pragma unroll
        for (int i = 0; i < VE; ++i) st.acc[i] = 0.f;
    }
    wave_segment_softmax<BF16, G>(st, a, start, deg, sd, vec, hk, lane_on, w, kRangeWaves);
    __syncthreads();  // the buffer may still be read from the previous range
    if (lane < G) {
        float *o = sm + (w * G + lane) * SV;
        o[0] = st.m;
        o[1] = st.l;
#pragma unroll
        for (int i = 0; i < VE; ++i) o[2 + i] = st.acc[i];
    }
    __syncthreads();
    if (w == 0 && lane < G) {
        for (int ww = 1; ww < kRangeWaves; ++ww) {
            const float *o = sm + (ww * G + lane) * SV;
            const float m2 = o[0], l2 = o[1];
            const float M = fmaxf(st.m, m2);
            const float s1 = __expf(st.m - M), s2 = __expf(m2 - M);
            st.l = st.l * s1 + l2 * s2;
#pragma unroll
            for (int i = 0; i < VE; ++i) st.acc[i] = st.acc[i] * s1 + o[2 + i] * s2;
            st.m = M;
        }
    }
}

// One block per shadow segment: the partial softmax state (without the self edge).
template <bool BF16, int G>
__global__ __launch_bounds__(kRangeWaves * kWave) void gat_segments_kernel(GatArgs a) {
    constexpr int VE = Elems<BF16>::kPerVec;
    __shared__ float sm[kRangeWaves * G * (VE + 2)];
    const int lane = threadIdx.x & (kWave - 1);
    const int li = lane % G;
    const int64_t s = blockIdx.x;
    if (a.bounds && (s < a.bounds[2] || s >= a.bounds[3])) return;
    const int64_t v = a.shadow_owner[s];
    const int64_t owner_start = a.rowptr[v];
    if (owner_start < a.edge_lo || owner_start >= a.edge_hi) return;
    const int vec = blockIdx.y * G + li;
    const bool lane_on = vec < a.row_vecs;
    const int hk = lane_on ? (vec * VE) / a.dh : 0;
    const float sd = lane_on ? a.s_dst[v * a.heads + hk] : 0.f;
    SoftState<VE> st;
    st.m = kNegInf;
    st.l = 0.f;
#pragma unroll
    for (int i = 0; i < VE; ++i) st.acc[i] = 0.f;
    const int64_t b = a.shadow_begin[s];
    block_range_softmax<BF16, G>(st, a, b, a.shadow_end[s] - b, sd, vec, hk, lane_on, sm);
    if (threadIdx.x < G && lane_on) {
        float4 *o = reinterpret_cast<float4 *>(a.part_acc + (s * a.row_vecs + vec) * VE);
        o[0] = make_float4(st.acc[0], st.acc[1], st.acc[2], st.acc[3]);
        if constexpr (VE == 8) o[1] = make_float4(st.acc[4], st.acc[5], st.acc[6], st.acc[7]);
        if ((vec * VE) % a.dh == 0) {   // one lane per head records the scalar state
            a.part_m[s * a.heads + hk] = st.m;
            a.part_l[s * a.heads + hk] = st.l;
        }
    }
}

// Long rows from the work list, one block per row at a time.
template <bool BF16, int G>
__global__ __launch_bounds__(kRangeWaves * kWave) void gat_long_rows_kernel(GatArgs a) {
    constexpr int VE = Elems<BF16>::kPerVec;
    __shared__ float sm[kRangeWaves * G * (VE + 2)];
    const int lane = threadIdx.x & (kWave - 1);
    const int li = lane % G;
    const int vec = blockIdx.y * G + li;
    const bool lane_on = vec < a.row_vecs;
    const int hk = lane_on ? (vec * VE) / a.dh : 0;
    const uint32_t count = *a.long_count;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const int64_t v = a.long_list[i];
        const int64_t b = a.rowptr[v];
        const int64_t d = a.rowptr[v + 1] - b;
        const float sd = lane_on ? a.s_dst[v * a.heads + hk] : 0.f;
        SoftState<VE> st;
        {   // the implicit self edge starts the state of wave 0's lane group 0
            const uint4 raw = lane_on ? a.z[v * a.row_vecs + vec] : make_uint4(0, 0, 0, 0);
            st.m = lane_on ? leaky(a.s_src[v * a.heads + hk] + sd, a.slope) : 0.f;
            st.l = 1.f;
            unpack<BF16>(st.acc, raw);
        }
        block_range_softmax<BF16, G>(st, a, b, d, sd, vec, hk, lane_on, sm);
        if (threadIdx.x < G && lane_on) finish_store<BF16, VE>(a, v, vec, st.acc, st.l);
    }
}

__global__ void zero_u32_kernel(uint32_t *p) { *p = 0u; }

// One block per hub.  Per head: M = max over the segment maxima and the self score (exact, order-free), then
// the rescaled partials are added in ascending segment order within interleaved chains and the chains in
// ascending order, the self edge last.
template <bool BF16>
__global__ __launch_bounds__(1024) void gat_combine_kernel(GatArgs a, int64_t n_hubs, const int32_t *hub_ids,
                                                           const int64_t *hub_shadow_off) {
    __shared__ float4 sm_acc[1024];
    __shared__ float sm_l[1024];
    __shared__ float sm_max[64];
    constexpr int VE = Elems<BF16>::kPerVec;
    if (a.bounds && ((int64_t)blockIdx.x < a.bounds[4] || (int64_t)blockIdx.x >= a.bounds[5])) return;
    const int64_t v = hub_ids[blockIdx.x];
    const int64_t rs = a.rowptr[v];
    if (rs < a.edge_lo || rs >= a.edge_hi) return;
    const int64_t s0 = hub_shadow_off[blockIdx.x], s1 = hub_shadow_off[blockIdx.x + 1];
    const int dim = a.row_vecs * VE;
    const int lanes_per_row = dim / 4;

    // per-head maximum (heads <= 64)
    for (int k = threadIdx.x / kWave; k < a.heads; k += blockDim.x / kWave) {
        const int lane = threadIdx.x & (kWave - 1);
        float m = leaky(a.s_src[v * a.heads + k] + a.s_dst[v * a.heads + k], a.slope);
        for (int64_t s = s0 + lane; s < s1; s += kWave) m = fmaxf(m, a.part_m[s * a.heads + k]);
#pragma unroll
        for (int off = 1; off < kWave; off <<= 1) m = fmaxf(m, __shfl_xor(m, off, kWave));
        if (lane == 0) sm_max[k] = m;
    }
    __syncthreads();

    for (int q0 = 0; q0 < lanes_per_row; q0 += 1024) {
        const int cols_here = (lanes_per_row - q0 < 1024) ? (lanes_per_row - q0) : 1024;
        const int slices = 1024 / cols_here;
        const int slice = threadIdx.x / cols_here;
        const int lv = threadIdx.x % cols_here;
        const int hk = ((q0 + lv) * 4) / a.dh;
        const float M = sm_max[hk];
        float4 acc = make_float4(0.f, 0.f, 0.f, 0.f);
        float l = 0.f;
        if (slice < slices) {
            const float4 *p = reinterpret_cast<const float4 *>(a.part_acc) + q0 + lv;
            int64_t s = s0 + slice;
            for (; s + 3 * (int64_t)slices < s1; s += 4 * (int64_t)slices) {   // four partials in flight, added in order
                float w[4], pl[4];
                float4 x[4];
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const int64_t su = s + u * (int64_t)slices;
                    w[u] = a.part_m[su * a.heads + hk];
                    pl[u] = a.part_l[su * a.heads + hk];
                    x[u] = p[su * lanes_per_row];
                }
#pragma unroll
                for (int u = 0; u < 4; ++u) {
                    const float wu = __expf(w[u] - M);
                    acc.x = fmaf(x[u].x, wu, acc.x); acc.y = fmaf(x[u].y, wu, acc.y);
                    acc.z = fmaf(x[u].z, wu, acc.z); acc.w = fmaf(x[u].w, wu, acc.w);
                    l = fmaf(pl[u], wu, l);
                }
            }
            for (; s < s1; s += slices) {
                const float w = __expf(a.part_m[s * a.heads + hk] - M);
                const float4 x = p[s * lanes_per_row];
                acc.x = fmaf(x.x, w, acc.x); acc.y = fmaf(x.y, w, acc.y); acc.z = fmaf(x.z, w, acc.z); acc.w = fmaf(x.w, w, acc.w);
                l = fmaf(a.part_l[s * a.heads + hk], w, l);
            }
        }
        __syncthreads();
        sm_acc[threadIdx.x] = acc;
        sm_l[threadIdx.x] = l;
        __syncthreads();
        if (slice == 0) {
            float r[4] = {0.f, 0.f, 0.f, 0.f};
            float lt = 0.f;
            for (int k = 0; k < slices; ++k) {
                const float4 x = sm_acc[k * cols_here + lv];
                r[0] += x.x; r[1] += x.y; r[2] += x.z; r[3] += x.w;
                lt += sm_l[k * cols_here + lv];
            }
            // the self edge
            const float ws = __expf(leaky(a.s_src[v * a.heads + hk] + a.s_dst[v * a.heads + hk], a.slope) - M);
            const int64_t elem0 = v * dim + (int64_t)(q0 + lv) * 4;
            float zs[4];
            if constexpr (BF16) {
                const uint2 raw = *reinterpret_cast<const uint2 *>(reinterpret_cast<const uint16_t *>(a.z) + elem0);
                zs[0] = bf16_lo(raw.x); zs[1] = bf16_hi(raw.x); zs[2] = bf16_lo(raw.y); zs[3] = bf16_hi(raw.y);
            } else {
                const float4 raw = *reinterpret_cast<const float4 *>(reinterpret_cast<const float *>(a.z) + elem0);
                zs[0] = raw.x; zs[1] = raw.y; zs[2] = raw.z; zs[3] = raw.w;
            }
            lt += ws;
            float y[4];
#pragma unroll
            for (int i = 0; i < 4; ++i) {
                y[i] = fmaf(zs[i], ws, r[i]) / lt;
                if (a.bias) y[i] += a.bias[(q0 + lv) * 4 + i];
                if (a.act == ITB_ACT_RELU) y[i] = fmaxf(y[i], 0.f);
            }
            if constexpr (BF16) {
                uint2 pk;
                pk.x = pack_bf16x2(y[0], y[1]);
                pk.y = pack_bf16x2(y[2], y[3]);
                *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.out) + elem0) = pk;
            } else {
                *reinterpret_cast<float4 *>(static_cast<float *>(a.out) + elem0) = make_float4(y[0], y[1], y[2], y[3]);
            }
        }
    }
}

template <bool BF16, int G>
int32_t launch_all(const GatArgs &a, bool hubs, int64_t n_hubs, const int32_t *hub_ids, const int64_t *hub_shadow_off,
                   const itb::GatherOptions &opt, hipStream_t st) {
    const int64_t waves = (a.n_nodes + kWave - 1) / kWave;
    const unsigned gy = (unsigned)((a.row_vecs + G - 1) / G);
    // hub passes first, on the helper stream when there is one (see gather_layer)
    itb::SideFork own_fork;
    itb::SideFork &fork = opt.outer_fork ? *opt.outer_fork : own_fork;
    if (!opt.outer_fork) {
        const int32_t rc = own_fork.begin((hubs && opt.allow_side && itb::g_tuning.overlap_hubs.load()) ? itb::side_stream() : nullptr, st);
        if (rc != ITB_OK) return rc;
    }
    if (hubs) {
        hipStream_t hst = fork.stream();
        gat_segments_kernel<BF16, G><<<dim3((unsigned)a.n_shadows, gy), kRangeWaves * kWave, 0, hst>>>(a);
        ITB_LAUNCH_CHECK();
        gat_combine_kernel<BF16><<<(unsigned)n_hubs, 1024, 0, hst>>>(a, n_hubs, hub_ids, hub_shadow_off);
        ITB_LAUNCH_CHECK();
        if (!opt.outer_fork) {
            const int32_t rc = own_fork.mark_done();
            if (rc != ITB_OK) return rc;
        }
    }
    zero_u32_kernel<<<1, 1, 0, st>>>(a.long_count);
    ITB_LAUNCH_CHECK();
    const int cap = itb::g_tuning.rows_waves_per_simd.load();
    gat_rows_kernel<BF16, G><<<dim3((unsigned)((waves + 3) / 4), gy), 256, itb::lds_for_occupancy(cap == -1 ? 0 : cap, G, hubs), st>>>(a);
    ITB_LAUNCH_CHECK();
    int64_t lg = waves > 2048 ? 2048 : waves;  // fixed grid over the device-side work list
    gat_long_rows_kernel<BF16, G><<<dim3((unsigned)lg, gy), kRangeWaves * kWave, 0, st>>>(a);
    ITB_LAUNCH_CHECK();
    return opt.outer_fork ? ITB_OK : own_fork.finish();
}

template <bool BF16>
int32_t dispatch(int G, const GatArgs &a, bool hubs, int64_t n_hubs, const int32_t *hub_ids, const int64_t *hub_shadow_off,
                 const itb::GatherOptions &opt, hipStream_t st) {
    switch (G) {
        case 1: return launch_all<BF16, 1>(a, hubs, n_hubs, hub_ids, hub_shadow_off, opt, st);
        case 2: return launch_all<BF16, 2>(a, hubs, n_hubs, hub_ids, hub_shadow_off, opt, st);
        case 4: return launch_all<BF16, 4>(a, hubs, n_hubs, hub_ids, hub_shadow_off, opt, st);
        case 8: return launch_all<BF16, 8>(a, hubs, n_hubs, hub_ids, hub_shadow_off, opt, st);
        case 16: return launch_all<BF16, 16>(a, hubs, n_hubs, hub_ids, hub_shadow_off, opt, st);
        case 32: return launch_all<BF16, 32>(a, hubs, n_hubs, hub_ids, hub_shadow_off, opt, st);
        default: return launch_all<BF16, 64>(a, hubs, n_hubs, hub_ids, hub_shadow_off, opt, st);
    }
}

}  // namespace

namespace itb {

int32_t gat_gather_impl(const itb_gather_desc *desc, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                        const itb_split *split, const void *z, const float *s_src, const float *s_dst, void *out,
                        int64_t edge_lo, int64_t edge_hi, void *workspace, size_t *workspace_bytes, const GatherOptions &opt,
                        hipStream_t st) {
    const int64_t *bounds = opt.bounds;
    const bool bf16 = desc->dtype_in == ITB_BF16;
    if (desc->dtype_out != desc->dtype_in) return ITB_ERR_UNSUPPORTED;
    if (desc->act != ITB_ACT_NONE && desc->act != ITB_ACT_RELU) return ITB_ERR_DTYPE;
    if (reinterpret_cast<uintptr_t>(desc->bias) & 15u) return ITB_ERR_UNSUPPORTED;  // bias is read as 16-byte vectors
    if (desc->heads <= 0 || desc->heads > 64 || desc->dim % desc->heads != 0) return ITB_ERR_SIZE;
    const int dh = desc->dim / desc->heads;
    const int ve = bf16 ? 8 : 4;
    if (dh % ve != 0) return ITB_ERR_UNSUPPORTED;  // a lane's 16-byte vector must lie inside one head
    const bool hubs = split && split->n_hubs > 0;
    Carver cv(workspace);
    uint32_t *long_count = cv.take<uint32_t>(64);
    int64_t *own_bounds = cv.take<int64_t>(32);
    int32_t *long_list = cv.take<int32_t>((size_t)n_nodes);
    float *part_acc = cv.take<float>(hubs ? (size_t)split->n_shadows * desc->dim : 0);
    float *part_m = cv.take<float>(hubs ? (size_t)split->n_shadows * desc->heads : 0);
    float *part_l = cv.take<float>(hubs ? (size_t)split->n_shadows * desc->heads : 0);
    if (!workspace) {
        *workspace_bytes = cv.off;
        return ITB_OK;
    }
    if (*workspace_bytes < cv.off || (cv.off > 0 && (reinterpret_cast<uintptr_t>(workspace) & 255u))) return ITB_ERR_WORKSPACE;
    if (!rowptr || (n_nodes > 0 && (!out || !z || !s_src || !s_dst))) return ITB_ERR_NULL;
    if (!aligned16(z) || !aligned16(out)) return ITB_ERR_UNSUPPORTED;
    if (hubs && (!split->hub_ids || !split->hub_shadow_off || !split->shadow_begin || !split->shadow_end || !split->shadow_owner))
        return ITB_ERR_NULL;
    if (n_nodes == 0) return ITB_OK;

    GatArgs a{};
    a.n_nodes = n_nodes;
    a.rowptr = rowptr;
    a.col = col;
    a.z = static_cast<const uint4 *>(z);
    a.stream_rows = stream_rows_for(n_nodes * (int64_t)desc->dim * (bf16 ? 2 : 4));
    a.s_src = s_src;
    a.s_dst = s_dst;
    a.bias = desc->bias;
    a.out = out;
    a.threshold = split ? split->threshold : INT64_MAX;
    a.edge_lo = edge_lo;
    a.edge_hi = edge_hi;
    if (!bounds && (edge_lo > 0 || edge_hi < INT64_MAX)) {   // a partial range: find its rows, segments and hubs once
        const int32_t brc = enqueue_range_bounds(1, 0, edge_lo, edge_hi, n_nodes, rowptr, split, own_bounds, st);
        if (brc != ITB_OK) return brc;
        bounds = own_bounds;
    }
    a.bounds = bounds;
    a.row_vecs = desc->dim * (bf16 ? 2 : 4) / 16;
    a.heads = desc->heads;
    a.dh = dh;
    a.act = desc->act;
    a.slope = desc->leaky_slope;
    int G = 1;
    while (G < a.row_vecs && G < kWave) G <<= 1;
    const int tuned_small = g_tuning.small_limit.load(), tuned_long = g_tuning.long_row.load();
    a.small_limit = tuned_small >= 0 ? tuned_small : 2 * (kWave / G);
    a.long_limit = tuned_long > a.small_limit ? tuned_long : a.small_limit;
    a.long_list = long_list;
    a.long_count = long_count;
    if (hubs) {
        a.n_shadows = split->n_shadows;
        a.shadow_begin = split->shadow_begin;
        a.shadow_end = split->shadow_end;
        a.shadow_owner = split->shadow_owner;
        a.part_acc = part_acc;
        a.part_m = part_m;
        a.part_l = part_l;
    }
    return bf16 ? dispatch<true>(G, a, hubs, hubs ? split->n_hubs : 0, hubs ? split->hub_ids : nullptr,
                                 hubs ? split->hub_shadow_off : nullptr, opt, st)
                : dispatch<false>(G, a, hubs, hubs ? split->n_hubs : 0, hubs ? split->hub_ids : nullptr,
                                  hubs ? split->hub_shadow_off : nullptr, opt, st);
}
}  // namespace itb
