// build_csr_by_dst: stable grouping of the edge table by destination.
//
// Method: least-significant-digit radix sort of (dst, src) pairs over the ceil(log2 N) key bits
// (each pass: per-tile digit histogram -> exclusive scan -> stable scatter), then the row pointers are
// read off the run boundaries of the sorted keys.  Every step is insensitive to degree skew: a hub with
// millions of in-edges costs the same per edge as a uniform graph, and nothing depends on atomics
// ordering, so the result is the unique stable grouping.
#include "common.h"

namespace itb {
int g_csr_xcd_remap = 1;  // tuning hook (key 2): 0 = tiles in launch order
}

namespace {
using namespace itb;

constexpr int kThreads = 256;
constexpr int kWaves = kThreads / kWave;
constexpr int kItems = 16;
constexpr int kTile = kThreads * kItems;  // keys per block
constexpr int kMaxRadix = 256;

constexpr int kScanThreads = 256;
constexpr int kScanItems = 8;
constexpr int kScanTile = kScanThreads * kScanItems;

// Workgroups are handed to the 8 XCDs round-robin by linear id, and every XCD has its own L2.  Giving XCD x a
// CONTIGUOUS range of tiles makes neighbouring tiles -- which append to neighbouring positions of every digit
// bucket -- meet in one L2, where their partial-line stores merge before they are written back.
__device__ __forceinline__ int64_t xcd_contiguous_tile(int64_t block, int64_t nblocks, int remap) {
    if (!remap) return block;
    constexpr int64_t kXcds = 8;
    const int64_t per = nblocks / kXcds, rem = nblocks % kXcds;
    const int64_t x = block % kXcds, j = block / kXcds;
    return x * per + (x < rem ? x : rem) + j;
}

__global__ void fill_i64_kernel(int64_t *p, int64_t n, int64_t v) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
__global__ void fill_u32_kernel(uint32_t *p, int64_t n, uint32_t v) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

// First read of the raw edge table: range check of both endpoints and, in the same pass, the first-digit tile
// histograms of both sorts (the destinations' for the CSR, the sources' for the out-degrees when WITH_SRC).
// Layout of each histogram as in radix_hist_kernel.
template <bool WITH_SRC>
__global__ __launch_bounds__(kThreads) void first_pass_kernel(int64_t n_edges, uint32_t n_nodes, const int32_t *src,
                                                              const int32_t *dst, int bits, uint32_t *hist_dst,
                                                              uint32_t *hist_src, int64_t nblocks, int remap,
                                                              uint32_t *bad_flag) {
    __shared__ uint32_t hd[kMaxRadix];
    __shared__ uint32_t hs[WITH_SRC ? kMaxRadix : 1];
    const int64_t tile = xcd_contiguous_tile(blockIdx.x, nblocks, remap);
    const int radix = 1 << bits;
    const uint32_t mask = radix - 1;
    for (int d = threadIdx.x; d < radix; d += kThreads) {
        hd[d] = 0;
        if constexpr (WITH_SRC) hs[d] = 0;
    }
    __syncthreads();
    const int64_t base = tile * kTile;
    bool bad = false;
    uint32_t kd[kItems], ks[kItems];
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int64_t idx = base + i * kThreads + threadIdx.x;
        kd[i] = idx < n_edges ? (uint32_t)dst[idx] : 0u;
        ks[i] = idx < n_edges ? (uint32_t)src[idx] : 0u;
    }
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int64_t idx = base + i * kThreads + threadIdx.x;
        if (idx < n_edges) {
            bad = bad || kd[i] >= n_nodes || ks[i] >= n_nodes;
            atomicAdd(&hd[kd[i] & mask], 1u);
            if constexpr (WITH_SRC) atomicAdd(&hs[ks[i] & mask], 1u);
        }
    }
    if (bad) atomicOr(bad_flag, 1u);
    __syncthreads();
    for (int d = threadIdx.x; d < radix; d += kThreads) {
        hist_dst[(int64_t)d * nblocks + tile] = hd[d];
        if constexpr (WITH_SRC) hist_src[(int64_t)d * nblocks + tile] = hs[d];
    }
}

// hist[digit * nblocks + block] = number of keys of this block's tile with that digit.
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(const uint32_t *keys, int64_t n, int shift, int bits,
                                                              uint32_t *hist, int64_t nblocks, int remap) {
    __shared__ uint32_t h[kMaxRadix];
    const int64_t tile = xcd_contiguous_tile(blockIdx.x, nblocks, remap);
    const int radix = 1 << bits;
    const uint32_t mask = radix - 1;
    for (int d = threadIdx.x; d < radix; d += kThreads) h[d] = 0;
    __syncthreads();
    const int64_t base = tile * kTile;
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        int64_t idx = base + i * kThreads + threadIdx.x;
        if (idx < n) atomicAdd(&h[(keys[idx] >> shift) & mask], 1u);
    }
    __syncthreads();
    for (int d = threadIdx.x; d < radix; d += kThreads) hist[(int64_t)d * nblocks + tile] = h[d];
}

// Stable scatter of one digit.  Tile order is (wave, slot, lane) = ascending input index, and the rank of a
// key among equal digits is: keys of earlier blocks (scanned histogram) + earlier waves of the tile + earlier
// slots of the wave + lower lanes of the slot.  The tile is first put in digit order in LDS and then written
// out by consecutive threads, so that each digit's run leaves the block as contiguous, coalesced stores
// (scattering straight from registers costs one memory transaction per 4-byte element).
template <bool HAS_VALS>
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(const uint32_t *keys_in, const int32_t *vals_in,
                                                                 uint32_t *keys_out, int32_t *vals_out, int64_t n,
                                                                 int shift, int bits, const uint32_t *hist_scanned,
                                                                 int64_t nblocks, int remap) {
    __shared__ uint32_t cnt[kWaves][kMaxRadix];   // per wave and digit: count, then start inside the sorted tile
    __shared__ uint32_t gbase[kMaxRadix];         // global position of the tile's first key of the digit
    __shared__ uint32_t lstart[kMaxRadix];        // position of the digit's first key inside the sorted tile
    __shared__ uint32_t skey[kTile];
    __shared__ int32_t sval[HAS_VALS ? kTile : 1];
    __shared__ uint32_t scan_sm[17];
    const int radix = 1 << bits;
    const uint32_t mask = radix - 1;
    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    for (int d = threadIdx.x; d < kWaves * kMaxRadix; d += kThreads) (&cnt[0][0])[d] = 0;
    const int64_t tile = xcd_contiguous_tile(blockIdx.x, nblocks, remap);
    for (int d = threadIdx.x; d < radix; d += kThreads) gbase[d] = hist_scanned[(int64_t)d * nblocks + tile];
    __syncthreads();

    const int64_t tile_base = tile * kTile;
    const int64_t wave_base = tile_base + (int64_t)w * (kWave * kItems);
    const uint64_t lower = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    uint32_t key[kItems];
    int32_t val[kItems];
    uint32_t rank[kItems];
#pragma unroll
    for (int s = 0; s < kItems; ++s) {
        const int64_t idx = wave_base + s * kWave + lane;
        key[s] = (idx < n) ? keys_in[idx] : 0u;
        if constexpr (HAS_VALS) val[s] = (idx < n) ? vals_in[idx] : 0;
    }
#pragma unroll
    for (int s = 0; s < kItems; ++s) {
        const int64_t idx = wave_base + s * kWave + lane;
        const bool valid = idx < n;
        const uint32_t d = (key[s] >> shift) & mask;
        uint64_t peers = __ballot(valid);
        for (int b = 0; b < bits; ++b) {
            const bool bit = (d >> b) & 1u;
            const uint64_t vote = __ballot(valid && bit);
            peers &= bit ? vote : ~vote;
        }
        const uint32_t prev = valid ? cnt[w][d] : 0u;
        rank[s] = prev + (uint32_t)__popcll(peers & lower);
        __builtin_amdgcn_wave_barrier();
        if (valid && (peers & lower) == 0) cnt[w][d] = prev + (uint32_t)__popcll(peers);
        __builtin_amdgcn_wave_barrier();
    }
    __syncthreads();
    // per digit: exclusive prefix over the waves, tile total; then exclusive prefix over the digits
    uint32_t total_d = 0;
    if (threadIdx.x < radix) {
        const int d = threadIdx.x;
        for (int ww = 0; ww < kWaves; ++ww) {
            const uint32_t t = cnt[ww][d];
            cnt[ww][d] = total_d;
            total_d += t;
        }
    }
    uint32_t tile_total;
    const uint32_t ls = block_exclusive_scan<uint32_t>(total_d, scan_sm, &tile_total);
    if (threadIdx.x < radix) lstart[threadIdx.x] = ls;
    __syncthreads();
#pragma unroll
    for (int s = 0; s < kItems; ++s) {
        const int64_t idx = wave_base + s * kWave + lane;
        if (idx < n) {
            const uint32_t d = (key[s] >> shift) & mask;
            const uint32_t lp = lstart[d] + cnt[w][d] + rank[s];
            skey[lp] = key[s];
            if constexpr (HAS_VALS) sval[lp] = val[s];
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < tile_total; i += kThreads) {
        const uint32_t k = skey[i];
        const uint32_t d = (k >> shift) & mask;
        const uint32_t pos = gbase[d] + (i - lstart[d]);
        keys_out[pos] = k;
        if constexpr (HAS_VALS) vals_out[pos] = sval[i];
    }
}

// ---- exclusive scan of a uint32 array, in place -------------------------------------------------------
__global__ __launch_bounds__(kScanThreads) void scan_reduce_kernel(const uint32_t *in, int64_t n, uint32_t *partial) {
    __shared__ uint32_t sm[17];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i)
        if (base + i < n) s += in[base + i];
    uint32_t total;
    block_exclusive_scan<uint32_t>(s, sm, &total);
    if (threadIdx.x == 0) partial[blockIdx.x] = total;
}

__global__ __launch_bounds__(kScanThreads) void scan_apply_kernel(uint32_t *data, int64_t n, const uint32_t *offsets) {
    __shared__ uint32_t sm[17];
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    uint32_t v[kScanItems];
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        v[i] = (base + i < n) ? data[base + i] : 0u;
        s += v[i];
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan<uint32_t>(s, sm, &total) + (offsets ? offsets[blockIdx.x] : 0u);
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        if (base + i < n) data[base + i] = run;
        run += v[i];
    }
}

size_t scan_workspace_elems(int64_t n) {
    size_t total = 0;
    while (n > kScanTile) {
        n = (n + kScanTile - 1) / kScanTile;
        total += align_up((size_t)n * sizeof(uint32_t)) / sizeof(uint32_t);
    }
    return total;
}

int32_t exclusive_scan_u32(uint32_t *data, int64_t n, uint32_t *ws, hipStream_t st) {
    if (n <= 0) return ITB_OK;
    const int64_t nb = (n + kScanTile - 1) / kScanTile;
    if (nb == 1) {
        scan_apply_kernel<<<1, kScanThreads, 0, st>>>(data, n, nullptr);
        ITB_LAUNCH_CHECK();
        return ITB_OK;
    }
    scan_reduce_kernel<<<(unsigned)nb, kScanThreads, 0, st>>>(data, n, ws);
    ITB_LAUNCH_CHECK();
    int32_t rc = exclusive_scan_u32(ws, nb, ws + align_up((size_t)nb * sizeof(uint32_t)) / sizeof(uint32_t), st);
    if (rc != ITB_OK) return rc;
    scan_apply_kernel<<<(unsigned)nb, kScanThreads, 0, st>>>(data, n, ws);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

// rowptr[v] = index of the first sorted key >= v.  The thread at the start of each run of equal keys fills
// the row pointers of its own key and of the empty rows just before it; the last thread fills the tail.
// A thread looks at four consecutive keys (one 16-byte load; `keys` is 16-byte aligned) and the key before them.
template <typename OutT>
__global__ void rowptr_from_sorted_kernel(const uint32_t *keys, int64_t n_edges, int64_t n_nodes, OutT *rowptr) {
    const int64_t n_quads = (n_edges + 3) / 4;
    for (int64_t q = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; q < n_quads; q += (int64_t)gridDim.x * blockDim.x) {
        const int64_t i0 = 4 * q;
        uint32_t kk[4];
        if (i0 + 3 < n_edges) {
            const uint4 v = *reinterpret_cast<const uint4 *>(keys + i0);
            kk[0] = v.x; kk[1] = v.y; kk[2] = v.z; kk[3] = v.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) kk[j] = (i0 + j < n_edges) ? keys[i0 + j] : 0u;
        }
        int64_t kp = (i0 == 0) ? -1 : (int64_t)keys[i0 - 1];
#pragma unroll
        for (int j = 0; j < 4; ++j) {
            const int64_t i = i0 + j;
            if (i < n_edges) {
                const int64_t k = kk[j];
                if (k != kp) {
                    const int64_t hi = k < n_nodes ? k : n_nodes;
                    for (int64_t v = kp + 1; v <= hi; ++v) rowptr[v] = (OutT)i;
                }
                if (i == n_edges - 1)
                    for (int64_t v = k + 1; v <= n_nodes; ++v) rowptr[v] = (OutT)n_edges;
                kp = k;
            }
        }
    }
}

__global__ void adjacent_difference_kernel(const uint32_t *bounds, int64_t n, int32_t *out) {
    for (int64_t v = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; v < n; v += (int64_t)gridDim.x * blockDim.x)
        out[v] = (int32_t)(bounds[v + 1] - bounds[v]);
}

int ceil_log2(int64_t n) {
    int b = 0;
    while (((int64_t)1 << b) < n) ++b;
    return b;
}

unsigned grid_for(int64_t n, int threads, int64_t cap = 65536) {
    int64_t g = (n + threads - 1) / threads;
    if (g < 1) g = 1;
    if (g > cap) g = cap;
    return (unsigned)g;
}

}  // namespace

extern "C" int32_t build_csr_by_dst(int64_t n_nodes, int64_t n_edges, const int32_t *src, const int32_t *dst,
                                    int64_t *rowptr, int32_t *col, int32_t *deg_out, void *workspace,
                                    size_t *workspace_bytes, void *stream) {
    if (!workspace_bytes) return ITB_ERR_NULL;
    if (n_nodes < 0 || n_edges < 0 || n_nodes >= ((int64_t)1 << 31) || n_edges >= ((int64_t)1 << 31)) return ITB_ERR_SIZE;

    const int64_t nblocks = (n_edges + kTile - 1) / kTile;
    const int64_t hist_elems = (int64_t)kMaxRadix * (nblocks > 0 ? nblocks : 1);
    Carver cv(workspace);
    uint32_t *flag = cv.take<uint32_t>(64);
    uint32_t *kbuf0 = cv.take<uint32_t>((size_t)n_edges);
    uint32_t *kbuf1 = cv.take<uint32_t>((size_t)n_edges);
    int32_t *vtmp = cv.take<int32_t>((size_t)n_edges);
    uint32_t *hist = cv.take<uint32_t>((size_t)hist_elems);
    uint32_t *hist_src = cv.take<uint32_t>((size_t)hist_elems);  // histograms of the source sort (reserved whether or not
                                                                  // deg_out is asked for: the size query passes no pointers)
    uint32_t *scan_ws = cv.take<uint32_t>(scan_workspace_elems(hist_elems) + 64);
    uint32_t *bounds = cv.take<uint32_t>((size_t)n_nodes + 1);
    if (!workspace) {
        *workspace_bytes = cv.off;
        return ITB_OK;
    }
    if (*workspace_bytes < cv.off || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return ITB_ERR_WORKSPACE;
    if (!rowptr || (n_edges > 0 && (!src || !dst || !col))) return ITB_ERR_NULL;

    hipStream_t st = static_cast<hipStream_t>(stream);
    if (n_edges == 0 || n_nodes == 0) {
        fill_i64_kernel<<<grid_for(n_nodes + 1, 256), 256, 0, st>>>(rowptr, n_nodes + 1, 0);
        ITB_LAUNCH_CHECK();
        if (deg_out && n_nodes > 0) {
            fill_u32_kernel<<<grid_for(n_nodes, 256), 256, 0, st>>>(reinterpret_cast<uint32_t *>(deg_out), n_nodes, 0u);
            ITB_LAUNCH_CHECK();
        }
        ITB_HIP(hipStreamSynchronize(st));
        return (n_edges > 0) ? ITB_ERR_RANGE : ITB_OK;
    }

    int bits_total = ceil_log2(n_nodes);
    if (bits_total < 1) bits_total = 1;
    const int passes = (bits_total + 7) / 8;
    const int base_bits = bits_total / passes, extra = bits_total % passes;
    uint32_t *kbuf[2] = {kbuf0, kbuf1};

    fill_u32_kernel<<<1, 64, 0, st>>>(flag, 64, 0u);
    ITB_LAUNCH_CHECK();
    {
        const int bits0 = base_bits + (0 < extra ? 1 : 0);
        if (deg_out)
            first_pass_kernel<true><<<(unsigned)nblocks, kThreads, 0, st>>>(n_edges, (uint32_t)n_nodes, src, dst, bits0, hist, hist_src,
                                                                            nblocks, itb::g_csr_xcd_remap, flag);
        else
            first_pass_kernel<false><<<(unsigned)nblocks, kThreads, 0, st>>>(n_edges, (uint32_t)n_nodes, src, dst, bits0, hist, nullptr,
                                                                             nblocks, itb::g_csr_xcd_remap, flag);
        ITB_LAUNCH_CHECK();
    }

    // One radix sort, run once or twice: keys only over the sources (their run lengths are the out-degrees;
    // a histogram by atomics would cost one memory-side atomic per edge), then (dst, src) pairs for the CSR.
    const uint32_t *kin = nullptr;
    for (int which = deg_out ? 0 : 1; which < 2; ++which) {
        const bool pairs = which == 1;
        kin = reinterpret_cast<const uint32_t *>(pairs ? dst : src);
        const int32_t *vin = src;
        int shift = 0;
        for (int p = 0; p < passes; ++p) {
            const int bits = base_bits + (p < extra ? 1 : 0);
            uint32_t *kout = kbuf[p & 1];
            int32_t *vout = ((passes - 1 - p) % 2 == 0) ? col : vtmp;
            const int64_t hist_n = ((int64_t)1 << bits) * nblocks;
            // the first digit of both sorts was counted while the raw table was range-checked
            uint32_t *h = pairs ? hist : hist_src;  // separate buffers: the pairs' first histogram must survive the source sort
            if (p > 0) {
                radix_hist_kernel<<<(unsigned)nblocks, kThreads, 0, st>>>(kin, n_edges, shift, bits, h, nblocks, itb::g_csr_xcd_remap);
                ITB_LAUNCH_CHECK();
            }
            int32_t rc = exclusive_scan_u32(h, hist_n, scan_ws, st);
            if (rc != ITB_OK) return rc;
            if (pairs)
                radix_scatter_kernel<true><<<(unsigned)nblocks, kThreads, 0, st>>>(kin, vin, kout, vout, n_edges, shift, bits, h,
                                                                                   nblocks, itb::g_csr_xcd_remap);
            else
                radix_scatter_kernel<false><<<(unsigned)nblocks, kThreads, 0, st>>>(kin, nullptr, kout, nullptr, n_edges, shift, bits,
                                                                                    h, nblocks, itb::g_csr_xcd_remap);
            ITB_LAUNCH_CHECK();
            kin = kout;
            vin = vout;
            shift += bits;
        }
        if (!pairs) {
            rowptr_from_sorted_kernel<uint32_t><<<grid_for(n_edges, 256), 256, 0, st>>>(kin, n_edges, n_nodes, bounds);
            ITB_LAUNCH_CHECK();
            adjacent_difference_kernel<<<grid_for(n_nodes, 256), 256, 0, st>>>(bounds, n_nodes, deg_out);
            ITB_LAUNCH_CHECK();
        }
    }
    rowptr_from_sorted_kernel<int64_t><<<grid_for(n_edges, 256), 256, 0, st>>>(kin, n_edges, n_nodes, rowptr);
    ITB_LAUNCH_CHECK();

    uint32_t host_flag = 0;
    ITB_HIP(hipMemcpyAsync(&host_flag, flag, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    ITB_HIP(hipStreamSynchronize(st));
    return host_flag ? ITB_ERR_RANGE : ITB_OK;
}
