// gather_layer: degree-segmented sum / mean / degree-normalised sum / max / min over in-edges (pull over CSR rows).
//
// Data movement is the whole cost (one 16-byte vector per lane per edge, one fp32 FMA per element), so the
// kernels are organised around keeping many independent row loads in flight per wavefront:
//   * a row of `dim` elements is covered by G = next_pow2(dim*elem/16) lanes, each owning one 16-byte
//     vector; a 64-lane wavefront therefore carries 64/G edges per load instruction;
//   * each wavefront owns 64 consecutive destination rows (their row pointers are one coalesced load);
//     rows with few in-edges are processed 64/G at a time, one lane group per row; longer rows are
//     processed by the whole wavefront, the lane groups taking interleaved edges and a fixed xor-butterfly
//     combining the group partials;
//   * column indices (and per-source scales) are fetched 64 (or G) at a time with one coalesced load and
//     handed to the lane groups by cross-lane shuffles, so the dependent row loads are issued back to back;
//   * rows longer than kLongRow edges would leave one wavefront working alone for a long time, so the row
//     kernel only appends their ids to a work list (integer atomics; the list order does not enter any
//     result) and a second kernel gives each such row a whole 8-wave block;
//   * hub rows (in-degree > threshold) are skipped here; each shadow segment is summed by one 8-wave block
//     into one fp32 partial (wave w takes the 64-edge chunks congruent to w, the wave results are added in
//     wave order through LDS) and a block per hub adds the partials in ascending segment order.
// No floating-point atomics anywhere: every summation order is a function of the sizes only.
#include "common.h"

namespace itb {
namespace {
constexpr int kMaxDevices = 64;
SideStream g_side[kMaxDevices];
bool g_side_made[kMaxDevices];
std::mutex g_side_mu;
}  // namespace
SideStream *side_stream() {
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDevices) return nullptr;
    std::lock_guard<std::mutex> lock(g_side_mu);
    if (!g_side_made[dev]) {
        SideStream &s = g_side[dev];
        if (hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking) != hipSuccess) return nullptr;
        if (hipEventCreateWithFlags(&s.fork, hipEventDisableTiming) != hipSuccess) {
            (void)hipStreamDestroy(s.stream);
            return nullptr;
        }
        if (hipEventCreateWithFlags(&s.join, hipEventDisableTiming) != hipSuccess) {
            (void)hipEventDestroy(s.fork);
            (void)hipStreamDestroy(s.stream);
            return nullptr;
        }
        g_side_made[dev] = true;
    }
    return &g_side[dev];
}
// Destroys the helper stream and events of every device that has them (the next call that wants one makes it again).
void destroy_side_streams() {
    std::lock_guard<std::mutex> lock(g_side_mu);
    int cur = -1;
    (void)hipGetDevice(&cur);
    for (int dev = 0; dev < kMaxDevices; ++dev) {
        if (!g_side_made[dev]) continue;
        if (hipSetDevice(dev) == hipSuccess) {
            std::lock_guard<std::mutex> in_use(g_side[dev].mu);
            (void)hipStreamSynchronize(g_side[dev].stream);
            (void)hipEventDestroy(g_side[dev].fork);
            (void)hipEventDestroy(g_side[dev].join);
            (void)hipStreamDestroy(g_side[dev].stream);
        }
        g_side_made[dev] = false;
    }
    if (cur >= 0) (void)hipSetDevice(cur);
}
// Dynamic LDS that limits a 256-thread (4-wave) block to `waves` wavefronts per SIMD: a CU has 4 SIMDs and
// 160 KB of LDS, so `waves` blocks fit when each asks for 160 KB / waves.
size_t lds_for_occupancy(int waves, int lanes_per_row, bool beside_hub_passes) {
    // Measured on MI355X: with rows of 512 bytes and more (32+ lanes per row) the random row gather runs ~10 %
    // faster with 4 resident wavefronts per SIMD than with 8 (fewer requests queued per memory channel); 256-byte
    // rows gain 2-3 % from a cap of 5 when the kernel has the chip to itself and lose 5 % when the hub passes run
    // beside it (the LDS request then keeps segment blocks off the CU); shorter rows want every wavefront.
    if (waves < 0) waves = lanes_per_row >= 32 ? 4 : (lanes_per_row == 16 && !beside_hub_passes ? 5 : 0);
    if (waves <= 0 || waves >= 8) return 0;
    return (size_t)(160 * 1024 / waves) - 512;
}
}  // namespace itb

namespace {
using namespace itb;

enum { kModeSum = 0, kModeMean = 1, kModeScaleDst = 2, kModeMax = 3, kModeMin = 4 };

// The extremum aggregators (EXT kernels) run as a maximum of sign * x with sign = +1 (max) or -1 (min); the
// multiplication by +-1 is exact, so the result is bit-for-bit the extremum of the stored values.
__device__ __forceinline__ float ext_sign(int mode) { return mode == kModeMin ? -1.f : 1.f; }

struct GatherArgs {
    int64_t n_nodes;
    const int64_t *rowptr;
    const int32_t *col;      // nullptr: the source row of in-edge e is row e of `h` (a per-edge table in CSR order)
    const uint4 *h;          // [n_nodes x row_vecs] 16-byte vectors
    const float *src_scale;  // nullable: per-source coefficient, looked up per edge
    const float *edge_coef;  // nullable: per-edge coefficient in CSR order (read beside the column index); wins over src_scale
    const float *dst_scale;  // kModeScaleDst only
    void *out;               // agg rows, or fp32 partial rows in the segment kernel
    // update epilogue (all nullable / 0): out = act(agg + addend + bias), applied when a row is finished
    const void *addend;      // [n_nodes x dim] of the output dtype
    const float *bias;       // [dim]
    int32_t act;
    int64_t threshold;       // rows with in-degree > threshold are hubs (skipped by the row kernel)
    int64_t edge_lo, edge_hi;
    // nullable: {row_lo, row_hi, seg_lo, seg_hi, hub_lo, hub_hi} = the rows, shadow segments and hubs whose first edge
    // offset can lie in [edge_lo, edge_hi); wavefronts and blocks outside leave after one scalar load
    const int64_t *bounds;
    int32_t row_vecs;        // 16-byte vectors per input row
    int32_t stream_rows;     // source rows are read with non-temporal loads (tables far beyond the caches)
    int32_t mode;
    int32_t small_limit;
    int32_t long_limit;      // rows with more in-edges than this go to the work list
    int32_t *long_list;      // [n_nodes] work list of long rows
    uint32_t *long_count;    // its length
    // segment kernel only
    int64_t n_shadows;
    const int64_t *shadow_begin, *shadow_end;
    const int32_t *shadow_owner;
};

template <bool BF16>
struct Elems {
    static constexpr int kPerVec = BF16 ? 8 : 4;
};

template <bool BF16, bool EXT = false>
__device__ __forceinline__ void accumulate(float (&acc)[Elems<BF16>::kPerVec], const uint4 &raw, float s) {
    if constexpr (EXT) {
        if constexpr (BF16) {
            acc[0] = fmaxf(acc[0], s * bf16_lo(raw.x));
            acc[1] = fmaxf(acc[1], s * bf16_hi(raw.x));
            acc[2] = fmaxf(acc[2], s * bf16_lo(raw.y));
            acc[3] = fmaxf(acc[3], s * bf16_hi(raw.y));
            acc[4] = fmaxf(acc[4], s * bf16_lo(raw.z));
            acc[5] = fmaxf(acc[5], s * bf16_hi(raw.z));
            acc[6] = fmaxf(acc[6], s * bf16_lo(raw.w));
            acc[7] = fmaxf(acc[7], s * bf16_hi(raw.w));
        } else {
            acc[0] = fmaxf(acc[0], s * __uint_as_float(raw.x));
            acc[1] = fmaxf(acc[1], s * __uint_as_float(raw.y));
            acc[2] = fmaxf(acc[2], s * __uint_as_float(raw.z));
            acc[3] = fmaxf(acc[3], s * __uint_as_float(raw.w));
        }
    } else if constexpr (BF16) {
        acc[0] = fmaf(s, bf16_lo(raw.x), acc[0]);
        acc[1] = fmaf(s, bf16_hi(raw.x), acc[1]);
        acc[2] = fmaf(s, bf16_lo(raw.y), acc[2]);
        acc[3] = fmaf(s, bf16_hi(raw.y), acc[3]);
        acc[4] = fmaf(s, bf16_lo(raw.z), acc[4]);
        acc[5] = fmaf(s, bf16_hi(raw.z), acc[5]);
        acc[6] = fmaf(s, bf16_lo(raw.w), acc[6]);
        acc[7] = fmaf(s, bf16_hi(raw.w), acc[7]);
    } else {
        acc[0] = fmaf(s, __uint_as_float(raw.x), acc[0]);
        acc[1] = fmaf(s, __uint_as_float(raw.y), acc[1]);
        acc[2] = fmaf(s, __uint_as_float(raw.z), acc[2]);
        acc[3] = fmaf(s, __uint_as_float(raw.w), acc[3]);
    }
}

// What a masked-off lane feeds to accumulate(): (raw, scale) that leave the accumulator unchanged.  Sums: 0 * 0.
// Extrema: sign * (-sign * inf) = -inf, the identity of the running maximum.
// (One 32-bit word of the vector; the callers build the vector as a temporary so that the select stays a select
// of values and never becomes a select of addresses.)
template <bool BF16, bool EXT>
__device__ __forceinline__ uint32_t idle_word(float sign) {
    if constexpr (!EXT) return 0u;
    const uint32_t inf = BF16 ? 0x7f807f80u : 0x7f800000u, ninf = BF16 ? 0xff80ff80u : 0xff800000u;
    return sign > 0.f ? ninf : inf;
}

// Store one lane's slice of an output row.  `vec` is the lane's 16-byte vector index in the INPUT row.
template <bool BF16_IN, bool BF16_OUT>
__device__ __forceinline__ void store_row_slice(void *out, int64_t row, int32_t row_vecs, int vec,
                                                const float (&acc)[Elems<BF16_IN>::kPerVec], bool stream = false) {
    constexpr int VE = Elems<BF16_IN>::kPerVec;
    const int64_t elem0 = (row * row_vecs + vec) * VE;
    if constexpr (BF16_OUT) {
        static_assert(BF16_IN, "bf16 output needs bf16 input");
        uint4 p;
        p.x = pack_bf16x2(acc[0], acc[1]);
        p.y = pack_bf16x2(acc[2], acc[3]);
        p.z = pack_bf16x2(acc[4], acc[5]);
        p.w = pack_bf16x2(acc[6], acc[7]);
        store_piece(static_cast<uint16_t *>(out) + elem0, p, stream);
    } else {
        float *o = static_cast<float *>(out) + elem0;
        store_piece(o, make_uint4(__float_as_uint(acc[0]), __float_as_uint(acc[1]), __float_as_uint(acc[2]), __float_as_uint(acc[3])), stream);
        if constexpr (VE == 8)
            store_piece(o + 4, make_uint4(__float_as_uint(acc[4]), __float_as_uint(acc[5]), __float_as_uint(acc[6]), __float_as_uint(acc[7])), stream);
    }
}

template <int VE, bool EXT = false>
__device__ __forceinline__ void finish_row(float (&acc)[VE], int mode, int64_t deg, const float *dst_scale, int64_t row) {
    if constexpr (EXT) {
        // back from sign * x to x; a vertex without in-edges aggregates to 0
        const float s = deg > 0 ? ext_sign(mode) : 0.f;
#pragma unroll
        for (int i = 0; i < VE; ++i) acc[i] = deg > 0 ? acc[i] * s : 0.f;
    } else if (mode == kModeMean) {
        if (deg > 0) {
            const float inv = 1.0f / (float)deg;  // one division per lane and row; the elements are scaled by it
#pragma unroll
            for (int i = 0; i < VE; ++i) acc[i] *= inv;
        }
    } else if (mode == kModeScaleDst) {
        const float s = dst_scale[row];
#pragma unroll
        for (int i = 0; i < VE; ++i) acc[i] *= s;
    }
}

// The update fused into the gather (a layer whose neighbour matrix was applied before the gather): the finished
// aggregate of a lane's VE columns gets the lane's slice of the addend row and of the bias, then the activation.
template <bool BF16_OUT, int VE>
__device__ __forceinline__ void update_epilogue(float (&acc)[VE], const void *addend, const float *bias, int act, int64_t row,
                                                int32_t row_vecs, int vec) {
    if (!addend && !bias && act == ITB_ACT_NONE) return;
    if (addend) {
        const int64_t elem0 = (row * row_vecs + vec) * VE;
        if constexpr (BF16_OUT) {
            static_assert(VE == 8, "bf16 output rows come from bf16 input rows");
            const uint4 ad = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(addend) + elem0);
            acc[0] += bf16_lo(ad.x); acc[1] += bf16_hi(ad.x); acc[2] += bf16_lo(ad.y); acc[3] += bf16_hi(ad.y);
            acc[4] += bf16_lo(ad.z); acc[5] += bf16_hi(ad.z); acc[6] += bf16_lo(ad.w); acc[7] += bf16_hi(ad.w);
        } else {
            const float4 *ad = reinterpret_cast<const float4 *>(static_cast<const float *>(addend) + elem0);
#pragma unroll
            for (int k = 0; k < VE / 4; ++k) {
                const float4 x = ad[k];
                acc[4 * k + 0] += x.x; acc[4 * k + 1] += x.y; acc[4 * k + 2] += x.z; acc[4 * k + 3] += x.w;
            }
        }
    }
    if (bias) {
        const float4 *b4 = reinterpret_cast<const float4 *>(bias + (int64_t)vec * VE);
#pragma unroll
        for (int k = 0; k < VE / 4; ++k) {
            const float4 b = b4[k];
            acc[4 * k + 0] += b.x; acc[4 * k + 1] += b.y; acc[4 * k + 2] += b.z; acc[4 * k + 3] += b.w;
        }
    }
    if (act == ITB_ACT_RELU) {
#pragma unroll
        for (int i = 0; i < VE; ++i) acc[i] = fmaxf(acc[i], 0.f);
    }
}

__device__ __forceinline__ int64_t shfl_i64(int64_t v, int src) {
    int lo = __shfl((int)(v & 0xffffffff), src, kWave);
    int hi = __shfl((int)(v >> 32), src, kWave);
    return ((int64_t)hi << 32) | (uint32_t)lo;
}

// Whole-wavefront sum of h[col[e]] * scale over the 64-edge chunks first_chunk, first_chunk + chunk_stride, ...
// of the edge range [start, start+deg).  Group g takes the edges congruent to g modulo 64/G inside every
// chunk; on return every lane group holds the sum over all the wavefront's chunks.
template <bool BF16, int G, bool EXT = false, int U = 8>
__device__ __forceinline__ void wave_segment_sum(float (&acc)[Elems<BF16>::kPerVec], const GatherArgs &a, int64_t start,
                                                 int64_t deg, int vec, bool lane_on, int first_chunk = 0,
                                                 int chunk_stride = 1) {
    constexpr int NG = kWave / G;
    constexpr int VE = Elems<BF16>::kPerVec;
    // U = row loads in flight per lane (8 instead of 4: 3-4 % on 256-byte rows in the segment and long-row kernels; the
    // row kernel takes 4, whose registers buy it three more resident wavefronts per SIMD)
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / G;
    const bool has_scale = !EXT && (a.src_scale != nullptr || a.edge_coef != nullptr);
    const float unit = EXT ? ext_sign(a.mode) : 1.f;  // scale of an edge without a source coefficient
    const float idle_s = EXT ? unit : 0.f;
    const uint32_t idle = idle_word<BF16, EXT>(unit);
#pragma unroll
    for (int i = 0; i < VE; ++i) acc[i] = EXT ? -INFINITY : 0.f;
    for (int64_t c = (int64_t)first_chunk * kWave; c < deg; c += (int64_t)chunk_stride * kWave) {
        int myc = 0;
        float mys = unit;
        if (c + lane < deg) {
            myc = a.col ? a.col[start + c + lane] : (int)(start + c + lane);
            if (has_scale) mys = a.edge_coef ? a.edge_coef[start + c + lane] : a.src_scale[myc];
        }
        const int cnt = (deg - c < kWave) ? (int)(deg - c) : kWave;  // wave-uniform
        const int steps = (cnt + NG - 1) / NG;
        for (int t = 0; t < steps; t += U) {
            uint4 raw[U];
            float sc[U];
            auto issue = [&](auto stream_tag) {
#pragma unroll
                for (int q = 0; q < U; ++q) {
                    const int ei = (t + q) * NG + g;
                    const int u = __shfl(myc, ei & (kWave - 1), kWave);
                    const float s = __shfl(mys, ei & (kWave - 1), kWave);
                    const bool on = lane_on && ei < cnt;
                    raw[q] = on ? load_row_piece<decltype(stream_tag)::value>(a.h + ((int64_t)u * a.row_vecs + vec))
                                : make_uint4(idle, idle, idle, idle);
                    sc[q] = on ? s : idle_s;
                }
            };
            if (a.stream_rows) issue(std::true_type{}); else issue(std::false_type{});  // kernel argument: wave-uniform
#pragma unroll
            for (int q = 0; q < U; ++q) accumulate<BF16, EXT>(acc, raw[q], sc[q]);
        }
    }
#pragma unroll
    for (int off = G; off < kWave; off <<= 1) {
#pragma unroll
        for (int i = 0; i < VE; ++i) {
            const float o = __shfl_xor(acc[i], off, kWave);
            acc[i] = EXT ? fmaxf(acc[i], o) : acc[i] + o;
        }
    }
}

template <bool BF16_IN, bool BF16_OUT, int G, bool EXT>
__global__ __launch_bounds__(256) void gather_rows_kernel(GatherArgs a) {
    constexpr int NG = kWave / G;
    constexpr int VE = Elems<BF16_IN>::kPerVec;
    constexpr int U = (G < 4) ? G : 4;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / G;
    const int li = lane % G;
    const int64_t r0 = ((int64_t)blockIdx.x * (blockDim.x / kWave) + (threadIdx.x / kWave)) * kWave;
    if (r0 >= a.n_nodes) return;
    if (a.bounds && (r0 + kWave <= a.bounds[0] || r0 >= a.bounds[1])) return;  // no row of this wavefront starts in the range
    const int vec = blockIdx.y * G + li;
    const bool lane_on = vec < a.row_vecs;
    const bool has_scale = !EXT && (a.src_scale != nullptr || a.edge_coef != nullptr);
    const float unit = EXT ? ext_sign(a.mode) : 1.f;
    const float idle_s = EXT ? unit : 0.f;
    const uint32_t idle = idle_word<BF16_IN, EXT>(unit);

    const int64_t my_row = r0 + lane;
    int64_t rs = 0, re = 0;
    if (my_row < a.n_nodes) {
        rs = a.rowptr[my_row];
        re = a.rowptr[my_row + 1];
    }
    const int64_t deg64 = re - rs;
    const bool mine = my_row < a.n_nodes && rs >= a.edge_lo && rs < a.edge_hi && deg64 <= a.threshold;
    const int deg = (int)deg64;
    const uint64_t small_mask = __ballot(mine && deg <= a.small_limit);
    uint64_t large_mask = __ballot(mine && deg > a.small_limit && deg <= a.long_limit);
    const uint64_t long_mask = __ballot(mine && deg > a.long_limit);
    // hand the long rows to the block-per-row kernel; one entry per row: of the blocks that share these rows
    // (blockIdx.y walks the row's width) only the first appends, every column block of the long-rows kernel
    // reads the same list
    if (long_mask && blockIdx.y == 0) {
        uint32_t base = 0;
        if (lane == 0) base = atomicAdd(a.long_count, (uint32_t)__popcll(long_mask));
        base = __shfl(base, 0, kWave);
        if ((long_mask >> lane) & 1ull) {
            const uint64_t below = (lane == 0) ? 0ull : (long_mask & (~0ull >> (kWave - lane)));
            a.long_list[base + (uint32_t)__popcll(below)] = (int32_t)my_row;
        }
    }

    // ---- rows with few in-edges: one lane group per row --------------------------------------------------
    // The 64/G lane groups walk the wavefront's short rows independently: a group that finishes its row takes
    // the next one not yet started (ascending, decided by wave-uniform bit arithmetic), so a 30-edge row next to
    // seven 2-edge rows holds up one group, not eight.  A row is still summed by one group, G edges per step in U
    // at a time, so its result does not depend on which group took it or on what else the wavefront had to do.
    if (small_mask) {
        uint64_t remaining = small_mask;  // wave-uniform: short rows nobody has started
        int rl = -1;                      // the group's current row (same in its G lanes), -1 = none
        int d = 0, j = 0;
        int64_t st = 0;
        float acc[VE];
#pragma unroll
        for (int i = 0; i < VE; ++i) acc[i] = EXT ? -INFINITY : 0.f;
        for (;;) {
            uint64_t idle_groups = __ballot(li == 0 && rl < 0);  // one bit per idle group, at its first lane
            int take = -1;
            while (idle_groups && remaining) {                   // wave-uniform, at most 64/G rounds
                const int first_lane = __ffsll((unsigned long long)idle_groups) - 1;
                idle_groups &= idle_groups - 1;
                const int row = __ffsll((unsigned long long)remaining) - 1;
                remaining &= remaining - 1;
                if (first_lane == g * G) take = row;
            }
            {   // every lane takes part in the shuffles; a group without a new row keeps what it has
                const int src = take >= 0 ? take : 0;
                const int nd = __shfl(deg, src, kWave);
                const int64_t nst = shfl_i64(rs, src);
                if (take >= 0) {
                    rl = take;
                    d = nd;
                    st = nst;
                    j = 0;
#pragma unroll
                    for (int i = 0; i < VE; ++i) acc[i] = EXT ? -INFINITY : 0.f;
                }
            }
            const bool busy = rl >= 0;
            if (__ballot(busy) == 0ull) break;
            int myc = 0;
            float mys = unit;
            if (busy && j + li < d) {
                myc = a.col ? a.col[st + j + li] : (int)(st + j + li);
                if (has_scale) mys = a.edge_coef ? a.edge_coef[st + j + li] : a.src_scale[myc];
            }
            const int cnt = busy ? d - j : 0;  // edges left for this group
            for (int t = 0; t < G; t += U) {
                if (__ballot(t < cnt) == 0ull) break;
                uint4 raw[U];
                float sc[U];
                int src_row[U];
#pragma unroll
                for (int q = 0; q < U; ++q) {  // all shuffles first: the loads then go out back to back
                    const int sl = g * G + t + q;
                    src_row[q] = __shfl(myc, sl, kWave);
                    const float s = __shfl(mys, sl, kWave);
                    sc[q] = (lane_on && (t + q) < cnt) ? s : idle_s;
                }
                auto issue = [&](auto stream_tag) {
#pragma unroll
                    for (int q = 0; q < U; ++q) {
                        const bool on = lane_on && (t + q) < cnt;
                        raw[q] = on ? load_row_piece<decltype(stream_tag)::value>(a.h + ((int64_t)src_row[q] * a.row_vecs + vec))
                                    : make_uint4(idle, idle, idle, idle);
                    }
                };
                if (a.stream_rows) issue(std::true_type{}); else issue(std::false_type{});
#pragma unroll
                for (int q = 0; q < U; ++q) accumulate<BF16_IN, EXT>(acc, raw[q], sc[q]);
            }
            j += G;
            if (busy && j >= d) {  // row finished (a row without in-edges finishes at once)
                if (lane_on) {
                    finish_row<VE, EXT>(acc, a.mode, d, a.dst_scale, r0 + rl);
                    update_epilogue<BF16_OUT, VE>(acc, a.addend, a.bias, a.act, r0 + rl, a.row_vecs, vec);
                    store_row_slice<BF16_IN, BF16_OUT>(a.out, r0 + rl, a.row_vecs, vec, acc, a.stream_rows);
                }
                rl = -1;
            }
        }
    }

    // ---- longer rows: the whole wavefront per row ---------------------------------------------------------
    while (large_mask) {
        const int rl = __ffsll((unsigned long long)large_mask) - 1;
        large_mask &= large_mask - 1;
        const int d = __shfl(deg, rl, kWave);
        const int64_t st = shfl_i64(rs, rl);
        float acc[VE];
        wave_segment_sum<BF16_IN, G, EXT, 4>(acc, a, st, d, vec, lane_on);
        if (g == 0 && lane_on) {
            finish_row<VE, EXT>(acc, a.mode, d, a.dst_scale, r0 + rl);
            update_epilogue<BF16_OUT, VE>(acc, a.addend, a.bias, a.act, r0 + rl, a.row_vecs, vec);
            store_row_slice<BF16_IN, BF16_OUT>(a.out, r0 + rl, a.row_vecs, vec, acc, a.stream_rows);
        }
    }
}

constexpr int kRangeWaves = 8;  // wavefronts that share one edge range (a shadow segment or a long row)

// Block-cooperative sum over one edge range: wave w takes the 64-edge chunks congruent to w modulo kRangeWaves,
// the wave results are added in wave order.  On return lane group 0 of wave 0 holds the sum.
template <bool BF16, int G, bool EXT>
__device__ __forceinline__ void block_range_sum(float (&acc)[Elems<BF16>::kPerVec], const GatherArgs &a, int64_t start,
                                                int64_t deg, int vec, bool lane_on, float *sm) {
    constexpr int VE = Elems<BF16>::kPerVec;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    wave_segment_sum<BF16, G, EXT>(acc, a, start, deg, vec, lane_on, w, kRangeWaves);
    __syncthreads();  // the buffer may still be read from the previous range
    if (lane < G) {
#pragma unroll
        for (int i = 0; i < VE; ++i) sm[(w * G + lane) * VE + i] = acc[i];
    }
    __syncthreads();
    if (w == 0 && lane < G) {
#pragma unroll
        for (int i = 0; i < VE; ++i) acc[i] = EXT ? -INFINITY : 0.f;
        for (int ww = 0; ww < kRangeWaves; ++ww) {
#pragma unroll
            for (int i = 0; i < VE; ++i) {
                const float o = sm[(ww * G + lane) * VE + i];
                acc[i] = EXT ? fmaxf(acc[i], o) : acc[i] + o;
            }
        }
    }
}

// One block per shadow segment: one fp32 partial row (source scales applied, destination finish deferred; for the
// extrema the partial is the maximum of sign * x).
template <bool BF16_IN, int G, bool EXT>
__global__ __launch_bounds__(kRangeWaves * kWave) void gather_segments_kernel(GatherArgs a) {
    constexpr int VE = Elems<BF16_IN>::kPerVec;
    __shared__ float sm[kRangeWaves * G * VE];
    const int lane = threadIdx.x & (kWave - 1);
    const int li = lane % G;
    const int64_t s = blockIdx.x;
    if (a.bounds && (s < a.bounds[2] || s >= a.bounds[3])) return;
    const int64_t owner_start = a.rowptr[a.shadow_owner[s]];
    if (owner_start < a.edge_lo || owner_start >= a.edge_hi) return;
    const int vec = blockIdx.y * G + li;
    const bool lane_on = vec < a.row_vecs;
    const int64_t b = a.shadow_begin[s];
    float acc[VE];
    block_range_sum<BF16_IN, G, EXT>(acc, a, b, a.shadow_end[s] - b, vec, lane_on, sm);
    if (threadIdx.x < G && lane_on) store_row_slice<BF16_IN, false>(a.out, s, a.row_vecs, vec, acc);
}

// Long rows from the work list, one block per row at a time.
template <bool BF16_IN, bool BF16_OUT, int G, bool EXT>
__global__ __launch_bounds__(kRangeWaves * kWave) void gather_long_rows_kernel(GatherArgs a) {
    constexpr int VE = Elems<BF16_IN>::kPerVec;
    __shared__ float sm[kRangeWaves * G * VE];
    const int lane = threadIdx.x & (kWave - 1);
    const int li = lane % G;
    const int vec = blockIdx.y * G + li;
    const bool lane_on = vec < a.row_vecs;
    const uint32_t count = *a.long_count;
    for (uint32_t i = blockIdx.x; i < count; i += gridDim.x) {
        const int64_t row = a.long_list[i];
        const int64_t b = a.rowptr[row];
        const int64_t d = a.rowptr[row + 1] - b;
        float acc[VE];
        block_range_sum<BF16_IN, G, EXT>(acc, a, b, d, vec, lane_on, sm);
        if (threadIdx.x < G && lane_on) {
            finish_row<VE, EXT>(acc, a.mode, d, a.dst_scale, row);
            update_epilogue<BF16_OUT, VE>(acc, a.addend, a.bias, a.act, row, a.row_vecs, vec);
            store_row_slice<BF16_IN, BF16_OUT>(a.out, row, a.row_vecs, vec, acc, a.stream_rows);
        }
    }
}

__global__ void zero_u32_kernel(uint32_t *p) { *p = 0u; }

// One block per hub: partial rows are added in ascending segment order within each of `slices` interleaved
// chains, then the chains are added in ascending slice order (extrema: merged by maximum in the same order).
template <bool BF16_OUT, bool EXT>
__global__ __launch_bounds__(1024) void combine_hubs_kernel(const float *part, int32_t dim, int64_t n_hubs,
                                                            const int32_t *hub_ids, const int64_t *hub_shadow_off,
                                                            const int64_t *rowptr, const float *dst_scale, int32_t mode,
                                                            int64_t edge_lo, int64_t edge_hi, void *out, const void *addend,
                                                            const float *bias, int32_t act, const int64_t *bounds) {
    __shared__ float4 sm[1024];
    const int64_t hub = blockIdx.x;
    if (bounds && (hub < bounds[4] || hub >= bounds[5])) return;
    const int32_t v = hub_ids[hub];
    const int64_t rs = rowptr[v];
    if (rs < edge_lo || rs >= edge_hi) return;
    const int64_t deg = rowptr[v + 1] - rs;
    const int64_t s0 = hub_shadow_off[hub], s1 = hub_shadow_off[hub + 1];
    const int lanes_per_row = dim / 4;
    for (int q0 = 0; q0 < lanes_per_row; q0 += 1024) {  // column tiles of 4096 elements
        const int cols_here = (lanes_per_row - q0 < 1024) ? (lanes_per_row - q0) : 1024;
        const int slices = 1024 / cols_here;
        const int slice = threadIdx.x / cols_here;
        const int lv = threadIdx.x % cols_here;
        const float zero = EXT ? -INFINITY : 0.f;
        auto join = [](float x, float y) { return EXT ? fmaxf(x, y) : x + y; };
        float4 acc = make_float4(zero, zero, zero, zero);
        if (slice < slices) {
            const float4 *p = reinterpret_cast<const float4 *>(part) + q0 + lv;
            int64_t s = s0 + slice;
            for (; s + 3 * (int64_t)slices < s1; s += 4 * (int64_t)slices) {
                const float4 x0 = p[s * lanes_per_row];
                const float4 x1 = p[(s + slices) * lanes_per_row];
                const float4 x2 = p[(s + 2 * (int64_t)slices) * lanes_per_row];
                const float4 x3 = p[(s + 3 * (int64_t)slices) * lanes_per_row];
                acc.x = join(acc.x, x0.x); acc.y = join(acc.y, x0.y); acc.z = join(acc.z, x0.z); acc.w = join(acc.w, x0.w);
                acc.x = join(acc.x, x1.x); acc.y = join(acc.y, x1.y); acc.z = join(acc.z, x1.z); acc.w = join(acc.w, x1.w);
                acc.x = join(acc.x, x2.x); acc.y = join(acc.y, x2.y); acc.z = join(acc.z, x2.z); acc.w = join(acc.w, x2.w);
                acc.x = join(acc.x, x3.x); acc.y = join(acc.y, x3.y); acc.z = join(acc.z, x3.z); acc.w = join(acc.w, x3.w);
            }
            for (; s < s1; s += slices) {
                const float4 x0 = p[s * lanes_per_row];
                acc.x = join(acc.x, x0.x); acc.y = join(acc.y, x0.y); acc.z = join(acc.z, x0.z); acc.w = join(acc.w, x0.w);
            }
        }
        __syncthreads();
        sm[threadIdx.x] = acc;
        __syncthreads();
        if (slice == 0) {
            float r[4] = {zero, zero, zero, zero};
            for (int k = 0; k < slices; ++k) {
                const float4 x = sm[k * cols_here + lv];
                r[0] = join(r[0], x.x); r[1] = join(r[1], x.y); r[2] = join(r[2], x.z); r[3] = join(r[3], x.w);
            }
            finish_row<4, EXT>(r, mode, deg, dst_scale, v);
            const int64_t elem0 = (int64_t)v * dim + (int64_t)(q0 + lv) * 4;
            if (addend) {   // the fused update, as in the row kernels
                if constexpr (BF16_OUT) {
                    const uint2 ad = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(addend) + elem0);
                    r[0] += bf16_lo(ad.x); r[1] += bf16_hi(ad.x); r[2] += bf16_lo(ad.y); r[3] += bf16_hi(ad.y);
                } else {
                    const float4 ad = *reinterpret_cast<const float4 *>(static_cast<const float *>(addend) + elem0);
                    r[0] += ad.x; r[1] += ad.y; r[2] += ad.z; r[3] += ad.w;
                }
            }
            if (bias) {
                const float4 b = *reinterpret_cast<const float4 *>(bias + (int64_t)(q0 + lv) * 4);
                r[0] += b.x; r[1] += b.y; r[2] += b.z; r[3] += b.w;
            }
            if (act == ITB_ACT_RELU) {
#pragma unroll
                for (int i = 0; i < 4; ++i) r[i] = fmaxf(r[i], 0.f);
            }
            if constexpr (BF16_OUT) {
                uint2 pk;
                pk.x = pack_bf16x2(r[0], r[1]);
                pk.y = pack_bf16x2(r[2], r[3]);
                *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(out) + elem0) = pk;
            } else {
                *reinterpret_cast<float4 *>(static_cast<float *>(out) + elem0) = make_float4(r[0], r[1], r[2], r[3]);
            }
        }
    }
}

// first index i in [0, n) with key[i] >= x (n if none); key non-decreasing
template <typename T>
__device__ __forceinline__ int64_t lower_bound_dev(const T *key, int64_t n, int64_t x) {
    int64_t lo = 0, hi = n;
    while (lo < hi) {
        const int64_t mid = lo + (hi - lo) / 2;
        if ((int64_t)key[mid] < x) lo = mid + 1;
        else hi = mid;
    }
    return lo;
}

}  // namespace

namespace itb {
// Range r (r < n_ranges) covers the edge offsets [r * edge_step, (r + 1) * edge_step), the last one to the end; a
// single range [edge_lo, edge_hi) is given with n_ranges = 1 and edge_step = 0.  Row pointers are non-decreasing, so
// the rows whose first edge offset lies in a range are a contiguous run of vertex ids: out[6 r ..] =
// {row_lo, row_hi, seg_lo, seg_hi, hub_lo, hub_hi}.
__global__ void range_bounds_kernel(int64_t n_ranges, int64_t edge_step, int64_t edge_lo, int64_t edge_hi, int64_t n_nodes,
                                    const int64_t *rowptr, int64_t n_hubs, const int32_t *hub_ids, const int64_t *hub_shadow_off,
                                    int64_t *out) {
    const int64_t r = blockIdx.x * (int64_t)blockDim.x + threadIdx.x;
    if (r >= n_ranges) return;
    const int64_t lo = edge_step > 0 ? r * edge_step : edge_lo;
    const int64_t hi = edge_step > 0 ? (r == n_ranges - 1 ? INT64_MAX : (r + 1) * edge_step) : edge_hi;
    const int64_t row_lo = lower_bound_dev(rowptr, n_nodes, lo);
    const int64_t row_hi = lower_bound_dev(rowptr, n_nodes, hi);
    int64_t hub_lo = 0, hub_hi = 0;
    if (n_hubs > 0) {
        hub_lo = lower_bound_dev(hub_ids, n_hubs, row_lo);
        hub_hi = lower_bound_dev(hub_ids, n_hubs, row_hi);
    }
    int64_t *o = out + 6 * r;
    o[0] = row_lo;
    o[1] = row_hi;
    o[2] = n_hubs > 0 ? hub_shadow_off[hub_lo] : 0;
    o[3] = n_hubs > 0 ? hub_shadow_off[hub_hi] : 0;
    o[4] = hub_lo;
    o[5] = hub_hi;
}

int32_t enqueue_range_bounds(int64_t n_ranges, int64_t edge_step, int64_t edge_lo, int64_t edge_hi, int64_t n_nodes,
                             const int64_t *rowptr, const itb_split *split, int64_t *out, hipStream_t st) {
    const bool hubs = split && split->n_hubs > 0;
    range_bounds_kernel<<<(unsigned)((n_ranges + 63) / 64), 64, 0, st>>>(n_ranges, edge_step, edge_lo, edge_hi, n_nodes, rowptr,
                                                                          hubs ? split->n_hubs : 0, hubs ? split->hub_ids : nullptr,
                                                                          hubs ? split->hub_shadow_off : nullptr, out);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}
}  // namespace itb

namespace {
template <bool BF16_IN, bool BF16_OUT, int G, bool EXT>
int32_t launch_rows(const GatherArgs &a, hipStream_t st) {
    const int64_t waves = (a.n_nodes + kWave - 1) / kWave;
    dim3 grid((unsigned)((waves + 3) / 4), (unsigned)((a.row_vecs + G - 1) / G));
    if (a.n_nodes > 0) {
        zero_u32_kernel<<<1, 1, 0, st>>>(a.long_count);
        ITB_LAUNCH_CHECK();
        gather_rows_kernel<BF16_IN, BF16_OUT, G, EXT><<<grid, 256, lds_for_occupancy(g_tuning.rows_waves_per_simd.load(), G, a.n_shadows > 0), st>>>(a);
        ITB_LAUNCH_CHECK();
        // the list length is only known on the device: a fixed grid walks it (blocks beyond the length exit)
        int64_t lg = (a.n_nodes + 63) / 64;
        if (lg > 2048) lg = 2048;
        gather_long_rows_kernel<BF16_IN, BF16_OUT, G, EXT><<<dim3((unsigned)lg, grid.y), kRangeWaves * kWave, 0, st>>>(a);
        ITB_LAUNCH_CHECK();
    }
    return ITB_OK;
}

template <bool BF16_IN, int G, bool EXT>
int32_t launch_segments(const GatherArgs &a, hipStream_t st) {
    dim3 grid((unsigned)a.n_shadows, (unsigned)((a.row_vecs + G - 1) / G));
    gather_segments_kernel<BF16_IN, G, EXT><<<grid, kRangeWaves * kWave, 0, st>>>(a);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

template <bool BF16_IN, bool BF16_OUT, bool EXT>
int32_t dispatch_rows(int G, const GatherArgs &a, hipStream_t st) {
    switch (G) {
        case 1: return launch_rows<BF16_IN, BF16_OUT, 1, EXT>(a, st);
        case 2: return launch_rows<BF16_IN, BF16_OUT, 2, EXT>(a, st);
        case 4: return launch_rows<BF16_IN, BF16_OUT, 4, EXT>(a, st);
        case 8: return launch_rows<BF16_IN, BF16_OUT, 8, EXT>(a, st);
        case 16: return launch_rows<BF16_IN, BF16_OUT, 16, EXT>(a, st);
        case 32: return launch_rows<BF16_IN, BF16_OUT, 32, EXT>(a, st);
        default: return launch_rows<BF16_IN, BF16_OUT, 64, EXT>(a, st);
    }
}

template <bool BF16_IN, bool EXT>
int32_t dispatch_segments(int G, const GatherArgs &a, hipStream_t st) {
    switch (G) {
        case 1: return launch_segments<BF16_IN, 1, EXT>(a, st);
        case 2: return launch_segments<BF16_IN, 2, EXT>(a, st);
        case 4: return launch_segments<BF16_IN, 4, EXT>(a, st);
        case 8: return launch_segments<BF16_IN, 8, EXT>(a, st);
        case 16: return launch_segments<BF16_IN, 16, EXT>(a, st);
        case 32: return launch_segments<BF16_IN, 32, EXT>(a, st);
        default: return launch_segments<BF16_IN, 64, EXT>(a, st);
    }
}

}  // namespace

namespace itb {
int32_t gat_gather_impl(const itb_gather_desc *desc, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                        const itb_split *split, const void *z, const float *s_src, const float *s_dst, void *out,
                        int64_t edge_lo, int64_t edge_hi, void *workspace, size_t *workspace_bytes, const GatherOptions &opt,
                        hipStream_t st);

// gather_layer with its internal knobs (see GatherOptions).
int32_t gather_layer_impl(const itb_gather_desc *desc, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                          const itb_split *split, const void *h_src, const float *src_scale, const float *dst_scale,
                          void *agg_out, int64_t edge_lo, int64_t edge_hi, void *workspace, size_t *workspace_bytes,
                          const GatherOptions &opt, void *stream) {
    const int64_t *bounds = opt.bounds;
    const bool per_edge_rows = opt.per_edge_rows;
    if (!desc || !workspace_bytes) return ITB_ERR_NULL;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31)) return ITB_ERR_SIZE;
    if (desc->agg < ITB_AGG_SUM || desc->agg > ITB_AGG_MIN) return ITB_ERR_DTYPE;
    if ((desc->dtype_in != ITB_F32 && desc->dtype_in != ITB_BF16) || (desc->dtype_out != ITB_F32 && desc->dtype_out != ITB_BF16))
        return ITB_ERR_DTYPE;
    if (desc->dtype_in == ITB_F32 && desc->dtype_out == ITB_BF16) return ITB_ERR_UNSUPPORTED;
    if (desc->dim <= 0) return ITB_ERR_SIZE;
    const int elem = desc->dtype_in == ITB_BF16 ? 2 : 4;
    if ((desc->dim * elem) % 16 != 0) return ITB_ERR_UNSUPPORTED;
    if (split && (split->threshold <= 0 || split->n_hubs < 0 || split->n_shadows < 0)) return ITB_ERR_SIZE;
    if (desc->agg == ITB_AGG_GAT)
        return gat_gather_impl(desc, n_nodes, rowptr, col, split, h_src, src_scale, dst_scale, agg_out, edge_lo, edge_hi,
                               workspace, workspace_bytes, opt, static_cast<hipStream_t>(stream));

    if (desc->act != ITB_ACT_NONE && desc->act != ITB_ACT_RELU) return ITB_ERR_DTYPE;
    // bias and addend are read as 16-byte vectors
    if ((reinterpret_cast<uintptr_t>(desc->bias) & 15u) || !aligned16(desc->addend)) return ITB_ERR_UNSUPPORTED;
    const bool hubs = split && split->n_hubs > 0;
    Carver cv(workspace);
    uint32_t *long_count = cv.take<uint32_t>(64);
    int64_t *own_bounds = cv.take<int64_t>(32);
    int32_t *long_list = cv.take<int32_t>((size_t)n_nodes);
    float *part = cv.take<float>(hubs ? (size_t)split->n_shadows * desc->dim : 0);
    if (!workspace) {
        *workspace_bytes = cv.off;
        return ITB_OK;
    }
    if (*workspace_bytes < cv.off || (cv.off > 0 && (reinterpret_cast<uintptr_t>(workspace) & 255u))) return ITB_ERR_WORKSPACE;
    if (!rowptr || (n_nodes > 0 && (!h_src || !agg_out))) return ITB_ERR_NULL;
    if (!aligned16(h_src) || !aligned16(agg_out)) return ITB_ERR_UNSUPPORTED;
    if (desc->agg == ITB_AGG_GCN && n_nodes > 0 && !dst_scale) return ITB_ERR_NULL;  // src_scale NULL: rows already carry it
    if (hubs && (!split->hub_ids || !split->hub_shadow_off || !split->shadow_begin || !split->shadow_end || !split->shadow_owner))
        return ITB_ERR_NULL;
    if (n_nodes == 0) return ITB_OK;

    hipStream_t st = static_cast<hipStream_t>(stream);
    GatherArgs a{};
    a.n_nodes = n_nodes;
    a.rowptr = rowptr;
    a.col = per_edge_rows ? nullptr : col;
    a.h = static_cast<const uint4 *>(h_src);
    {
        // non-temporal row loads and stores once the table is far beyond what the caches hold
        const int64_t table_bytes = n_nodes * (int64_t)desc->dim * (desc->dtype_in == ITB_BF16 ? 2 : 4);
        a.stream_rows = per_edge_rows ? 0 : stream_rows_for(table_bytes);
    }
    a.src_scale = (desc->agg == ITB_AGG_GCN && !per_edge_rows) ? src_scale : nullptr;
    // per-edge scalar: the source coefficient of a GCN edge, or the weight of an edge-weighted sum / mean
    a.edge_coef = (desc->agg == ITB_AGG_GCN || desc->agg == ITB_AGG_SUM || desc->agg == ITB_AGG_MEAN) ? desc->edge_coef : nullptr;
    a.dst_scale = (desc->agg == ITB_AGG_GCN) ? dst_scale : nullptr;
    a.out = agg_out;
    a.addend = desc->addend;
    a.bias = desc->bias;
    a.act = desc->act;
    a.threshold = split ? split->threshold : INT64_MAX;
    a.edge_lo = edge_lo;
    a.edge_hi = edge_hi;
    if (!bounds && (edge_lo > 0 || edge_hi < INT64_MAX)) {   // a partial range: find its rows, segments and hubs once
        const int32_t brc = enqueue_range_bounds(1, 0, edge_lo, edge_hi, n_nodes, rowptr, split, own_bounds, st);
        if (brc != ITB_OK) return brc;
        bounds = own_bounds;
    }
    a.bounds = bounds;
    a.row_vecs = desc->dim * elem / 16;
    const bool ext = desc->agg == ITB_AGG_MAX || desc->agg == ITB_AGG_MIN;
    a.mode = desc->agg == ITB_AGG_MEAN ? kModeMean
             : desc->agg == ITB_AGG_GCN ? kModeScaleDst
             : desc->agg == ITB_AGG_MAX ? kModeMax
             : desc->agg == ITB_AGG_MIN ? kModeMin
                                        : kModeSum;
    int G = 1;
    while (G < a.row_vecs && G < kWave) G <<= 1;
    const int ng = kWave / G;
    // one lane group per row up to 32 in-edges (measured on 256-byte rows: 4 % faster than handing rows of 9-32
    // edges to the whole wavefront, whose last load batch is mostly masked), never below two batches of groups
    const int tuned_small = g_tuning.small_limit.load(), tuned_long = g_tuning.long_row.load();
    a.small_limit = tuned_small >= 0 ? tuned_small : (2 * ng > 32 ? 2 * ng : 32);
    a.long_limit = tuned_long > a.small_limit ? tuned_long : a.small_limit;
    a.long_list = long_list;
    a.long_count = long_count;
    a.n_shadows = hubs ? split->n_shadows : 0;  // > 0: hub passes run beside the row passes

    const bool bin = desc->dtype_in == ITB_BF16, bout = desc->dtype_out == ITB_BF16;
    int32_t rc;
    // The hub passes touch other rows and other workspace than the row passes: they go first and, when the helper
    // stream exists, run beside the row passes, whose many small blocks fill the gaps the large segment blocks leave.
    SideFork own_fork;
    SideFork &fork = opt.outer_fork ? *opt.outer_fork : own_fork;
    if (!opt.outer_fork) {
        rc = own_fork.begin((hubs && opt.allow_side && g_tuning.overlap_hubs.load()) ? side_stream() : nullptr, st);
        if (rc != ITB_OK) return rc;
    }
    if (hubs) {
        hipStream_t hst = fork.stream();
        GatherArgs s = a;
        s.out = part;
        s.n_shadows = split->n_shadows;
        s.shadow_begin = split->shadow_begin;
        s.shadow_end = split->shadow_end;
        s.shadow_owner = split->shadow_owner;
        if (ext) rc = bin ? dispatch_segments<true, true>(G, s, hst) : dispatch_segments<false, true>(G, s, hst);
        else rc = bin ? dispatch_segments<true, false>(G, s, hst) : dispatch_segments<false, false>(G, s, hst);
        if (rc != ITB_OK) return rc;
        auto combine = bout ? (ext ? combine_hubs_kernel<true, true> : combine_hubs_kernel<true, false>)
                            : (ext ? combine_hubs_kernel<false, true> : combine_hubs_kernel<false, false>);
        combine<<<(unsigned)split->n_hubs, 1024, 0, hst>>>(part, desc->dim, split->n_hubs, split->hub_ids, split->hub_shadow_off,
                                                           rowptr, a.dst_scale, a.mode, edge_lo, edge_hi, agg_out, a.addend, a.bias,
                                                           a.act, a.bounds);
        ITB_LAUNCH_CHECK();
        if (!opt.outer_fork) {
            rc = own_fork.mark_done();
            if (rc != ITB_OK) return rc;
        }
    }
    if (ext) {
        if (!bin) rc = dispatch_rows<false, false, true>(G, a, st);
        else if (bout) rc = dispatch_rows<true, true, true>(G, a, st);
        else rc = dispatch_rows<true, false, true>(G, a, st);
    } else {
        if (!bin) rc = dispatch_rows<false, false, false>(G, a, st);
        else if (bout) rc = dispatch_rows<true, true, false>(G, a, st);
        else rc = dispatch_rows<true, false, false>(G, a, st);
    }
    if (rc != ITB_OK) return rc;
    return opt.outer_fork ? ITB_OK : own_fork.finish();
}
}  // namespace itb

namespace {
// Scratch of gather_layer_noalloc: device memory that belongs to the library image, one copy per GPU, held until the
// process ends.  In host code the array's name is only a handle for hipGetSymbolAddress; kernels and memory
// operations get the per-device address looked up below.
constexpr size_t kStaticScratchBytes = (size_t)ITB_NOALLOC_SCRATCH_BYTES;
static __device__ __align__(256) unsigned char scratch[kStaticScratchBytes];

void *static_scratch_of_current_device() {
    constexpr int kMaxDev = 64;
    static void *table[kMaxDev];
    static std::mutex mu;
    int dev = -1;
    if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= kMaxDev) return nullptr;
    std::lock_guard<std::mutex> lock(mu);
    if (!table[dev]) {
        void *ptr = nullptr;
        if (hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch)) != hipSuccess || !ptr) return nullptr;
        table[dev] = ptr;
    }
    return table[dev];
}
}  // namespace

extern "C" int32_t gather_layer(const itb_gather_desc *desc, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                                const itb_split *split, const void *h_src, const float *src_scale, const float *dst_scale,
                                void *agg_out, int64_t edge_lo, int64_t edge_hi, void *workspace, size_t *workspace_bytes,
                                void *stream) {
    return itb::gather_layer_impl(desc, n_nodes, rowptr, col, split, h_src, src_scale, dst_scale, agg_out, edge_lo, edge_hi,
                                  workspace, workspace_bytes, GatherOptions{}, stream);
}

extern "C" int32_t aggregate_edge_features(int32_t agg, int32_t dtype, int64_t n_nodes, const int64_t *rowptr,
                                           const itb_split *split, int32_t edge_dim, const void *edge_feat,
                                           const float *edge_coef, const float *dst_scale, void *out, void *workspace,
                                           size_t *workspace_bytes, void *stream) {
    if (agg != ITB_AGG_SUM && agg != ITB_AGG_MEAN && agg != ITB_AGG_GCN) return ITB_ERR_UNSUPPORTED;
    if (agg == ITB_AGG_GCN && workspace && n_nodes > 0 && (!edge_coef || !dst_scale)) return ITB_ERR_NULL;
    itb_gather_desc d{agg, dtype, dtype, edge_dim, 1, 0.f, ITB_ACT_NONE, nullptr, agg == ITB_AGG_GCN ? edge_coef : nullptr, nullptr};
    itb::GatherOptions opt;
    opt.per_edge_rows = true;
    return itb::gather_layer_impl(&d, n_nodes, rowptr, nullptr, split, edge_feat, nullptr, dst_scale, out, 0, INT64_MAX, workspace,
                                  workspace_bytes, opt, stream);
}

extern "C" int32_t gather_layer_noalloc(const itb_gather_desc *desc, int64_t n_nodes, const int64_t *rowptr, const int32_t *col,
                                        const itb_split *split, const void *h_src, const float *src_scale,
                                        const float *dst_scale, void *agg_out, int64_t edge_lo, int64_t edge_hi, void *stream) {
    size_t need = 0;
    itb::GatherOptions opt;
    opt.allow_side = false;
    int32_t rc = itb::gather_layer_impl(desc, n_nodes, nullptr, nullptr, split, nullptr, nullptr, nullptr, nullptr, edge_lo, edge_hi,
                                        nullptr, &need, opt, nullptr);
    if (rc != ITB_OK) return rc;
    if (need > kStaticScratchBytes) return ITB_ERR_WORKSPACE;  // sizes beyond the built-in scratch: use gather_layer
    void *ptr = static_scratch_of_current_device();
    if (!ptr) return ITB_ERR_DEVICE;
    size_t have = kStaticScratchBytes;
    return itb::gather_layer_impl(desc, n_nodes, rowptr, col, split, h_src, src_scale, dst_scale, agg_out, edge_lo, edge_hi, ptr,
                                  &have, opt, stream);
}

extern "C" int32_t itb_shutdown(void) {
    itb::destroy_side_streams();
    return ITB_OK;
}
