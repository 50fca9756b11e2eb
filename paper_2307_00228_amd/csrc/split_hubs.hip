// split_hubs: even split of every high-in-degree row into contiguous segments ("shadow" mirrors).
//
// Small kernels over the row pointers: per-block (hub, segment) counts, a single-block exclusive scan of those
// counts, an emit pass that recomputes the in-block prefix and writes the hub arrays in ascending vertex
// order, and one thread per segment that finds its hub by binary search and writes its bounds (a hub with
// millions of in-edges has thousands of segments, so they must not be written by one thread).
// Integer only; the output is unique.
#include "common.h"

#include <cmath>

namespace {
using namespace itb;

constexpr int kThreads = 1024;  // 4096 rows per block: the single-block scan over the per-block counts stays short (24 k entries for 1e8 rows)
constexpr int kRowsPerThread = 4;
constexpr int kRowsPerBlock = kThreads * kRowsPerThread;

__device__ __forceinline__ void row_counts(const int64_t *rowptr, int64_t n_nodes, int64_t threshold, int64_t row0,
                                           int64_t &hubs, int64_t &segs) {
    hubs = 0;
    segs = 0;
#pragma unroll
    for (int i = 0; i < kRowsPerThread; ++i) {
        const int64_t v = row0 + i;
        if (v < n_nodes) {
            const int64_t d = rowptr[v + 1] - rowptr[v];
            if (d > threshold) {
                hubs += 1;
                segs += (d + threshold - 1) / threshold;
            }
        }
    }
}

__global__ __launch_bounds__(kThreads) void hub_count_kernel(const int64_t *rowptr, int64_t n_nodes, int64_t threshold,
                                                             int64_t *blk_hubs, int64_t *blk_segs) {
    __shared__ int64_t sm[17];
    int64_t h, s, th, ts;
    row_counts(rowptr, n_nodes, threshold, (int64_t)blockIdx.x * kRowsPerBlock + (int64_t)threadIdx.x * kRowsPerThread, h, s);
    block_exclusive_scan<int64_t>(h, sm, &th);
    block_exclusive_scan<int64_t>(s, sm, &ts);
    if (threadIdx.x == 0) {
        blk_hubs[blockIdx.x] = th;
        blk_segs[blockIdx.x] = ts;
    }
}

// One block: exclusive scan of both per-block arrays in place; totals[0] = H, totals[1] = S.
__global__ __launch_bounds__(1024) void hub_scan_kernel(int64_t *blk_hubs, int64_t *blk_segs, int64_t nblocks, int64_t *totals) {
    __shared__ int64_t sm[17];
    int64_t carry_h = 0, carry_s = 0;
    for (int64_t base = 0; base < nblocks; base += blockDim.x) {
        const int64_t i = base + threadIdx.x;
        const int64_t h = (i < nblocks) ? blk_hubs[i] : 0;
        const int64_t s = (i < nblocks) ? blk_segs[i] : 0;
        int64_t th, ts;
        const int64_t eh = block_exclusive_scan<int64_t>(h, sm, &th);
        const int64_t es = block_exclusive_scan<int64_t>(s, sm, &ts);
        if (i < nblocks) {
            blk_hubs[i] = carry_h + eh;
            blk_segs[i] = carry_s + es;
        }
        carry_h += th;
        carry_s += ts;
    }
    if (threadIdx.x == 0) {
        totals[0] = carry_h;
        totals[1] = carry_s;
    }
}

__global__ __launch_bounds__(kThreads) void hub_emit_kernel(const int64_t *rowptr, int64_t n_nodes, int64_t threshold,
                                                            const int64_t *blk_hubs, const int64_t *blk_segs,
                                                            const int64_t *totals, int32_t *hub_ids, int64_t *hub_shadow_off) {
    __shared__ int64_t sm[17];
    const int64_t row0 = (int64_t)blockIdx.x * kRowsPerBlock + (int64_t)threadIdx.x * kRowsPerThread;
    int64_t h, s, th, ts;
    row_counts(rowptr, n_nodes, threshold, row0, h, s);
    int64_t hi = block_exclusive_scan<int64_t>(h, sm, &th) + blk_hubs[blockIdx.x];
    int64_t si = block_exclusive_scan<int64_t>(s, sm, &ts) + blk_segs[blockIdx.x];
    if (blockIdx.x == 0 && threadIdx.x == 0) hub_shadow_off[totals[0]] = totals[1];
    if (h == 0) return;
    for (int i = 0; i < kRowsPerThread; ++i) {
        const int64_t v = row0 + i;
        if (v >= n_nodes) break;
        const int64_t d = rowptr[v + 1] - rowptr[v];
        if (d > threshold) {
            hub_ids[hi] = (int32_t)v;
            hub_shadow_off[hi] = si;
            hi += 1;
            si += (d + threshold - 1) / threshold;
        }
    }
}

// Segment s belongs to the hub h with hub_shadow_off[h] <= s < hub_shadow_off[h+1]; it is group g = s - off[h]
// of n = off[h+1] - off[h] and covers [floor(g*d/n), floor((g+1)*d/n)) of the hub's row.
__global__ void segment_emit_kernel(const int64_t *rowptr, int64_t n_hubs, int64_t n_shadows, const int32_t *hub_ids,
                                    const int64_t *hub_shadow_off, int64_t *shadow_begin, int64_t *shadow_end,
                                    int32_t *shadow_owner) {
    for (int64_t s = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; s < n_shadows; s += (int64_t)gridDim.x * blockDim.x) {
        int64_t lo = 0, hi = n_hubs - 1;  // last h with off[h] <= s
        while (lo < hi) {
            const int64_t mid = (lo + hi + 1) >> 1;
            if (hub_shadow_off[mid] <= s) lo = mid; else hi = mid - 1;
        }
        const int64_t v = hub_ids[lo];
        const int64_t b = rowptr[v];
        const int64_t d = rowptr[v + 1] - b;
        const int64_t n = hub_shadow_off[lo + 1] - hub_shadow_off[lo];
        const int64_t g = s - hub_shadow_off[lo];
        shadow_begin[s] = b + (g * d) / n;   // g*d < 2^62: d < 2^31 and n <= d
        shadow_end[s] = b + ((g + 1) * d) / n;
        shadow_owner[s] = (int32_t)v;
    }
}

}  // namespace

extern "C" int32_t hub_threshold_heuristic(int64_t total_edges, int64_t total_workers, double lambda, int64_t *threshold) {
    if (!threshold) return ITB_ERR_NULL;
    if (total_edges < 0 || total_workers <= 0 || !(lambda > 0.0) || lambda > 1.0e6) return ITB_ERR_SIZE;
    // floor of the real quotient, formed in long double and nudged up by one part in 2^52: a lambda like 0.1, which a
    // double holds up to 2^-53 off, still lands on the integer it means (0.1 * 1e9 / 1000 = 100000, not 99999)
    const long double t = (long double)lambda * (long double)total_edges / (long double)total_workers;
    long double f = floorl(t * (1.0L + 0x1p-52L));
    if (f < 1.0L) f = 1.0L;
    if (f > 9.0e18L) f = 9.0e18L;
    *threshold = (int64_t)f;
    return ITB_OK;
}

extern "C" int32_t split_hubs(int64_t n_nodes, const int64_t *rowptr, int64_t threshold, int64_t *n_hubs,
                              int64_t *n_shadows, int32_t *hub_ids, int64_t *hub_shadow_off, int64_t *shadow_begin,
                              int64_t *shadow_end, int32_t *shadow_owner, void *workspace, size_t *workspace_bytes,
                              void *stream) {
    if (!workspace_bytes) return ITB_ERR_NULL;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31) || threshold <= 0) return ITB_ERR_SIZE;
    const int64_t nblocks = (n_nodes + kRowsPerBlock - 1) / kRowsPerBlock;
    Carver cv(workspace);
    int64_t *totals = cv.take<int64_t>(32);
    int64_t *blk_hubs = cv.take<int64_t>((size_t)(nblocks > 0 ? nblocks : 1));
    int64_t *blk_segs = cv.take<int64_t>((size_t)(nblocks > 0 ? nblocks : 1));
    if (!workspace) {
        *workspace_bytes = cv.off;
        return ITB_OK;
    }
    if (*workspace_bytes < cv.off || (reinterpret_cast<uintptr_t>(workspace) & 255u)) return ITB_ERR_WORKSPACE;
    if (!rowptr || !n_hubs || !n_shadows) return ITB_ERR_NULL;
    const bool fill = hub_ids || hub_shadow_off || shadow_begin || shadow_end || shadow_owner;
    if (fill && !hub_shadow_off) return ITB_ERR_NULL;

    hipStream_t st = static_cast<hipStream_t>(stream);
    int64_t host_totals[2] = {0, 0};
    // An in-degree is at most the edge count, which is below 2^31: a threshold from there on selects no vertex, and
    // the answer needs neither a kernel nor a round trip to the host.
    const bool nothing_can_exceed = threshold >= ((int64_t)1 << 31);
    if (nothing_can_exceed) {
        *n_hubs = 0;
        *n_shadows = 0;
        if (fill) ITB_HIP(hipMemsetAsync(hub_shadow_off, 0, sizeof(int64_t), st));
        return ITB_OK;
    }
    if (nblocks > 0) {
        hub_count_kernel<<<(unsigned)nblocks, kThreads, 0, st>>>(rowptr, n_nodes, threshold, blk_hubs, blk_segs);
        ITB_LAUNCH_CHECK();
        hub_scan_kernel<<<1, 1024, 0, st>>>(blk_hubs, blk_segs, nblocks, totals);
        ITB_LAUNCH_CHECK();
        ITB_HIP(hipMemcpyAsync(host_totals, totals, 2 * sizeof(int64_t), hipMemcpyDeviceToHost, st));
        ITB_HIP(hipStreamSynchronize(st));
    }
    *n_hubs = host_totals[0];
    *n_shadows = host_totals[1];
    if (!fill) return ITB_OK;
    if (host_totals[0] > 0 && (!hub_ids || !shadow_begin || !shadow_end || !shadow_owner)) return ITB_ERR_NULL;
    if (nblocks > 0) {
        hub_emit_kernel<<<(unsigned)nblocks, kThreads, 0, st>>>(rowptr, n_nodes, threshold, blk_hubs, blk_segs, totals,
                                                              hub_ids, hub_shadow_off);
        ITB_LAUNCH_CHECK();
        if (host_totals[1] > 0) {
            int64_t g = (host_totals[1] + 255) / 256;
            if (g > 65536) g = 65536;
            segment_emit_kernel<<<(unsigned)g, 256, 0, st>>>(rowptr, host_totals[0], host_totals[1], hub_ids, hub_shadow_off,
                                                            shadow_begin, shadow_end, shadow_owner);
            ITB_LAUNCH_CHECK();
        }
    } else {
        ITB_HIP(hipMemsetAsync(hub_shadow_off, 0, sizeof(int64_t), st));
    }
    return ITB_OK;  // the arrays are ordered on the stream like any other output; only the two counts needed the host
}
