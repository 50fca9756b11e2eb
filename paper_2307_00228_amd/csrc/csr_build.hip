// build_csr_by_dst: stable grouping of the edge table by destination.
//
// Method: least-significant-digit radix sort of (dst, src) pairs over the ceil(log2 N) key bits
// (each pass: per-tile digit histogram -> exclusive scan -> stable scatter), then the row pointers are
// read off the run boundaries of the sorted keys.  Every step is insensitive to degree skew: a hub with
// millions of in-edges costs the same per edge as a uniform graph, and nothing depends on atomics
// ordering, so the result is the unique stable grouping.
#include "common.h"

namespace {
using namespace itb;

constexpr int kThreads = 512;
constexpr int kWaves = kThreads / kWave;
constexpr int kItems = 16;
constexpr int kTile = kThreads * kItems;  // keys per block: 8192 (with 8-bit digits a tile's run of one digit averages a whole
                                          // 128-byte line; measured 2.5 % faster than 4096 on 2e9 edges, neutral on small graphs)
constexpr int kMaxRadix = 256;
constexpr int kMaxPartRadix = 512;  // buckets of the out-degree partition (top bits of the source id)
constexpr int kMaxLowBits = 13;     // vertex ids per bucket: 2^13 counters of 4 bytes in LDS
constexpr int kDegThreads = 1024;
constexpr int kDegSlice = 1 << 18;  // keys one block counts per visit
constexpr int kDegSlicesY = 16;

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

// Digit of the out-degree partition: the bits above `shift`, clamped so that an out-of-range id (reported as an
// error by the range check) still lands in a valid bucket.
__device__ __forceinline__ uint32_t partition_digit(uint32_t key, int shift, int radix) {
    const uint32_t d = key >> shift;
    return d < (uint32_t)radix ? d : (uint32_t)radix - 1u;
}

// LDS counter update of one wavefront: h[d] += 1 for every valid lane; returns the lane's slot (the counter value
// it would have seen), which only the unstable partition uses.  Popular digits -- the ids of hubs -- would make
// dozens of lanes hit one counter and serialise, so up to two rounds first fold all lanes that share the digit of
// the first pending lane into one atomic (worth it from four lanes on); what is left goes lane by lane.
// `fold` (wave-uniform, in/out): folding is tried only while it is set; a wavefront whose probe finds nothing to fold
// clears it and pays one atomic per lane from then on -- on uniform ids the votes would be pure overhead.
__device__ __forceinline__ uint32_t wave_count(uint32_t *h, uint32_t d, bool valid, bool &fold) {
    if (!fold) return valid ? atomicAdd(&h[d], 1u) : 0u;
    bool folded = false;
    const int lane = threadIdx.x & (kWave - 1);
    const uint64_t lower = (lane == 0) ? 0ull : (~0ull >> (kWave - lane));
    uint64_t pending = __ballot(valid);
    uint32_t slot = 0;
#pragma unroll
    for (int r = 0; r < 2; ++r) {
        if (pending == 0) break;  // wave-uniform
        const int leader = __ffsll((unsigned long long)pending) - 1;
        const uint32_t dl = (uint32_t)__shfl((int)d, leader, kWave);
        const uint64_t same = __ballot(valid && d == dl) & pending;
        if (__popcll(same) < 4) break;
        folded = true;
        uint32_t base = 0;
        if (lane == leader) base = atomicAdd(&h[dl], (uint32_t)__popcll(same));
        base = (uint32_t)__shfl((int)base, leader, kWave);
        if ((same >> lane) & 1ull) slot = base + (uint32_t)__popcll(same & lower);
        pending &= ~same;
    }
    if ((pending >> lane) & 1ull) slot = atomicAdd(&h[d], 1u);
    fold = folded;
    return slot;
}

__global__ void fill_i64_kernel(int64_t *p, int64_t n, int64_t v) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}
__global__ void fill_u32_kernel(uint32_t *p, int64_t n, uint32_t v) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n; i += (int64_t)gridDim.x * blockDim.x) p[i] = v;
}

// First read of the raw edge table: range check of the endpoints and, in the same pass, the first-digit tile
// histograms of both sorts (the destinations' for the CSR, the sources' for the out-degrees when WITH_SRC).  Without
// out-degrees the source column is not read here: the first scatter pass, which moves it anyway, checks its range.
// Layout of each histogram as in radix_hist_kernel.
// SRC_MODE 0: destinations only; 1: source digit = key & (src_radix - 1) (first pass of the keys-only sort);
// 2: source digit = partition_digit(key, src_shift, src_radix).
template <int SRC_MODE>
__global__ __launch_bounds__(kThreads) void first_pass_kernel(int64_t n_edges, uint32_t n_nodes, const int32_t *src,
                                                              const int32_t *dst, int bits, uint32_t *hist_dst,
                                                              int src_shift, int src_radix, uint32_t *hist_src,
                                                              int64_t nblocks, int remap, uint32_t *bad_flag) {
    __shared__ uint32_t hd[kMaxRadix];
    constexpr bool WITH_SRC = SRC_MODE != 0;
    __shared__ uint32_t hs[WITH_SRC ? kMaxPartRadix : 1];
    const int64_t tile = xcd_contiguous_tile(blockIdx.x, nblocks, remap);
    const int radix = 1 << bits;
    const uint32_t mask = radix - 1;
    for (int d = threadIdx.x; d < radix; d += kThreads) hd[d] = 0;
    if constexpr (WITH_SRC)
        for (int d = threadIdx.x; d < src_radix; d += kThreads) hs[d] = 0;
    __syncthreads();
    const int64_t base = tile * kTile;
    bool bad = false;
    bool fold_d = true, fold_s = true;
    // 16-byte loads where the caller's arrays allow them (counting does not care about the order inside the tile)
    const bool vec = (((WITH_SRC ? reinterpret_cast<uintptr_t>(src) : 0) | reinterpret_cast<uintptr_t>(dst)) & 15u) == 0;
    uint32_t kd[kItems], ks[WITH_SRC ? kItems : 1];
#pragma unroll
    for (int i = 0; i < kItems / 4; ++i) {
        const int64_t idx = base + ((int64_t)i * kThreads + threadIdx.x) * 4;
        if (vec && idx + 3 < n_edges) {
            const uint4 a = *reinterpret_cast<const uint4 *>(dst + idx);
            kd[4 * i] = a.x; kd[4 * i + 1] = a.y; kd[4 * i + 2] = a.z; kd[4 * i + 3] = a.w;
            if constexpr (WITH_SRC) {
                const uint4 b = *reinterpret_cast<const uint4 *>(src + idx);
                ks[4 * i] = b.x; ks[4 * i + 1] = b.y; ks[4 * i + 2] = b.z; ks[4 * i + 3] = b.w;
            }
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) {
                kd[4 * i + j] = idx + j < n_edges ? (uint32_t)dst[idx + j] : 0u;
                if constexpr (WITH_SRC) ks[4 * i + j] = idx + j < n_edges ? (uint32_t)src[idx + j] : 0u;
            }
        }
    }
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        const int64_t idx = base + ((int64_t)(i / 4) * kThreads + threadIdx.x) * 4 + (i & 3);
        const bool valid = idx < n_edges;
        if (valid) bad = bad || kd[i] >= n_nodes;
        if constexpr (WITH_SRC)
            if (valid) bad = bad || ks[i] >= n_nodes;
        wave_count(hd, kd[i] & mask, valid, fold_d);
        if constexpr (SRC_MODE == 1) wave_count(hs, ks[i] & (uint32_t)(src_radix - 1), valid, fold_s);
        if constexpr (SRC_MODE == 2) wave_count(hs, partition_digit(ks[i], src_shift, src_radix), valid, fold_s);
    }
    if (bad) atomicOr(bad_flag, 1u);
    __syncthreads();
    for (int d = threadIdx.x; d < radix; d += kThreads) hist_dst[(int64_t)d * nblocks + tile] = hd[d];
    if constexpr (WITH_SRC)
        for (int d = threadIdx.x; d < src_radix; d += kThreads) hist_src[(int64_t)d * nblocks + tile] = hs[d];
}

// ---- out-degrees: one partition pass + one histogram per bucket -----------------------------------------
// deg_out is the histogram of the source column.  Only counts are wanted, so nothing has to be stable: the
// sources are partitioned once by their top bits (order inside a bucket arbitrary, only the low bits are kept,
// as 16-bit values), and each bucket -- a contiguous range of at most 2^13 vertex ids -- is counted in LDS and
// stored.  All counters are integers, so the result does not depend on any ordering.
//
// Unstable partition of one tile: local slot by LDS atomics, tile put in digit order in LDS, runs written out
// by consecutive threads.  Same tile numbering and histogram layout as the stable scatter.
__global__ __launch_bounds__(kThreads) void partition_scatter_kernel(const uint32_t *keys_in, uint16_t *low_out, int64_t n,
                                                                     int shift, int radix, const uint32_t *hist_scanned,
                                                                     int64_t nblocks, int remap) {
    __shared__ uint32_t cnt[kMaxPartRadix];
    __shared__ uint32_t lstart[kMaxPartRadix];
    __shared__ uint32_t gbase[kMaxPartRadix];
    __shared__ uint32_t skey[kTile];  // (digit << 16) | low bits
    __shared__ uint32_t scan_sm[17];
    const int64_t tile = xcd_contiguous_tile(blockIdx.x, nblocks, remap);
    for (int d = threadIdx.x; d < radix; d += kThreads) {
        cnt[d] = 0;
        gbase[d] = hist_scanned[(int64_t)d * nblocks + tile];
    }
    __syncthreads();
    const int64_t base = tile * kTile;
    const uint32_t low_mask = (1u << shift) - 1u;
    uint32_t key[kItems], slot[kItems];
    bool fold = true;
    // any order inside the tile will do: 16-byte loads where the caller's array allows them
    const bool vec = (reinterpret_cast<uintptr_t>(keys_in) & 15u) == 0;
    auto item_index = [&](int i) { return base + ((int64_t)(i / 4) * kThreads + threadIdx.x) * 4 + (i & 3); };
#pragma unroll
    for (int i = 0; i < kItems / 4; ++i) {
        const int64_t idx = item_index(4 * i);
        if (vec && idx + 3 < n) {
            const uint4 v = *reinterpret_cast<const uint4 *>(keys_in + idx);
            key[4 * i] = v.x; key[4 * i + 1] = v.y; key[4 * i + 2] = v.z; key[4 * i + 3] = v.w;
        } else {
#pragma unroll
            for (int j = 0; j < 4; ++j) key[4 * i + j] = idx + j < n ? keys_in[idx + j] : 0u;
        }
    }
#pragma unroll
    for (int i = 0; i < kItems; ++i)
        slot[i] = wave_count(cnt, partition_digit(key[i], shift, radix), item_index(i) < n, fold);
    __syncthreads();
    // exclusive prefix over the digits, two digits per thread (radix <= 2 * kThreads)
    const int d0 = 2 * threadIdx.x, d1 = d0 + 1;
    const uint32_t c0 = d0 < radix ? cnt[d0] : 0u, c1 = d1 < radix ? cnt[d1] : 0u;
    uint32_t tile_total;
    const uint32_t ex = block_exclusive_scan<uint32_t>(c0 + c1, scan_sm, &tile_total);
    if (d0 < radix) lstart[d0] = ex;
    if (d1 < radix) lstart[d1] = ex + c0;
    __syncthreads();
#pragma unroll
    for (int i = 0; i < kItems; ++i) {
        if (item_index(i) < n) {
            const uint32_t d = partition_digit(key[i], shift, radix);
            skey[lstart[d] + slot[i]] = (d << 16) | (key[i] & low_mask);
        }
    }
    __syncthreads();
    for (uint32_t i = threadIdx.x; i < tile_total; i += kThreads) {
        const uint32_t k = skey[i];
        const uint32_t d = k >> 16;
        low_out[gbase[d] + (i - lstart[d])] = (uint16_t)(k & 0xffffu);
    }
}

// Block (b, y): bucket b = vertex ids [b << low, (b+1) << low), its keys are low_keys[start_b, start_{b+1}).
// The bucket is cut into slices of kDegSlice keys; block y counts slices y, y + gridDim.y, ...  A bucket with one
// slice (the normal case) is stored directly; a larger one adds its non-zero counters with integer atomics to
// deg_out, which the caller has zeroed.
__global__ __launch_bounds__(kDegThreads) void bucket_degree_kernel(const uint16_t *low_keys, int64_t n_edges,
                                                                    const uint32_t *hist_scanned, int64_t nblocks, int radix,
                                                                    int low, int64_t n_nodes, int32_t *deg_out) {
    __shared__ uint32_t h[1 << kMaxLowBits];
    const int b = blockIdx.x;
    const int64_t start = hist_scanned[(int64_t)b * nblocks];
    const int64_t end = (b + 1 < radix) ? (int64_t)hist_scanned[(int64_t)(b + 1) * nblocks] : n_edges;
    const int64_t len = end - start;
    const int64_t n_slices = (len + kDegSlice - 1) / kDegSlice;
    if ((int64_t)blockIdx.y >= (n_slices > 1 ? n_slices : 1)) return;
    const int bins = 1 << low;
    for (int i = threadIdx.x; i < bins; i += kDegThreads) h[i] = 0;
    __syncthreads();
    for (int64_t sl = blockIdx.y; sl < n_slices; sl += gridDim.y) {
        const int64_t s0 = start + sl * kDegSlice;
        const int64_t s1 = (s0 + kDegSlice < end) ? s0 + kDegSlice : end;
        // head and tail by single elements, the 16-byte aligned body eight keys at a time
        int64_t a0 = (s0 + 7) & ~(int64_t)7, a1 = s1 & ~(int64_t)7;
        if (a0 > a1) { a0 = s1; a1 = s1; }
        for (int64_t i = s0 + threadIdx.x; i < a0; i += kDegThreads) atomicAdd(&h[low_keys[i]], 1u);
        for (int64_t i = a1 + threadIdx.x; i < s1; i += kDegThreads) atomicAdd(&h[low_keys[i]], 1u);
        const uint4 *body = reinterpret_cast<const uint4 *>(low_keys + a0);
        const int64_t n_vec = (a1 - a0) / 8;
        for (int64_t i0 = 0; i0 < n_vec; i0 += kDegThreads) {  // block-uniform trip count: wave_count votes
            const int64_t i = i0 + threadIdx.x;
            const bool valid = i < n_vec;
            const uint4 v = valid ? body[i] : make_uint4(0, 0, 0, 0);
            bool fold = true;  // probed again for every 16-byte vector
            wave_count(h, v.x & 0xffffu, valid, fold); wave_count(h, v.x >> 16, valid, fold);
            wave_count(h, v.y & 0xffffu, valid, fold); wave_count(h, v.y >> 16, valid, fold);
            wave_count(h, v.z & 0xffffu, valid, fold); wave_count(h, v.z >> 16, valid, fold);
            wave_count(h, v.w & 0xffffu, valid, fold); wave_count(h, v.w >> 16, valid, fold);
        }
    }
    __syncthreads();
    const int64_t v0 = (int64_t)b << low;
    for (int i = threadIdx.x; i < bins; i += kDegThreads) {
        const int64_t v = v0 + i;
        if (v < n_nodes) {
            if (n_slices <= 1) deg_out[v] = (int32_t)h[i];
            else if (h[i]) atomicAdd(&deg_out[v], (int32_t)h[i]);
        }
    }
}

// hist[digit * nblocks + block] = number of keys of this block's tile with that digit.
// The counters are kept four times over, lane l adding to copy l & 3 (copy c of digit d sits at word 4 d + c, so the
// copies of a digit lie in different LDS banks): lanes that hold the same digit -- frequent once the lower digits are
// sorted and the edges of a heavy row sit together -- then spread over four addresses instead of serialising on one.
__global__ __launch_bounds__(kThreads) void radix_hist_kernel(const uint32_t *keys, int64_t n, int shift, int bits,
                                                              uint32_t *hist, int64_t nblocks, int remap) {
    constexpr int kCopies = 4;
    __shared__ uint32_t h[kMaxRadix * kCopies];
    const int64_t tile = xcd_contiguous_tile(blockIdx.x, nblocks, remap);
    const int radix = 1 << bits;
    const uint32_t mask = radix - 1;
    for (int d = threadIdx.x; d < radix * kCopies; d += kThreads) h[d] = 0;
    __syncthreads();
    const int64_t base = tile * kTile;
    const uint32_t copy = threadIdx.x & (kCopies - 1);
    // counting does not care about the order inside the tile: 16-byte loads (the key buffers are 16-byte aligned and a
    // tile starts at a multiple of 4096 keys); only the last tile can be ragged
    uint32_t k[kItems];
#pragma unroll
    for (int i = 0; i < kItems / 4; ++i) {
        const int64_t idx = base + ((int64_t)i * kThreads + threadIdx.x) * 4;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (idx + 3 < n) v = *reinterpret_cast<const uint4 *>(keys + idx);
        else {
            if (idx < n) v.x = keys[idx];
            if (idx + 1 < n) v.y = keys[idx + 1];
            if (idx + 2 < n) v.z = keys[idx + 2];
        }
        k[4 * i] = v.x; k[4 * i + 1] = v.y; k[4 * i + 2] = v.z; k[4 * i + 3] = v.w;
    }
    // A thread holds four runs of four consecutive keys; a run that holds one digit four times is counted by one
    // atomic of 4.
#pragma unroll
    for (int i = 0; i < kItems; i += 4) {
        const int64_t idx = base + ((int64_t)(i / 4) * kThreads + threadIdx.x) * 4;
        const uint32_t d0 = (k[i] >> shift) & mask, d1 = (k[i + 1] >> shift) & mask, d2 = (k[i + 2] >> shift) & mask,
                       d3 = (k[i + 3] >> shift) & mask;
        if (idx + 3 < n && d0 == d1 && d0 == d2 && d0 == d3) {
            atomicAdd(&h[d0 * kCopies + copy], 4u);
        } else {
            if (idx < n) atomicAdd(&h[d0 * kCopies + copy], 1u);
            if (idx + 1 < n) atomicAdd(&h[d1 * kCopies + copy], 1u);
            if (idx + 2 < n) atomicAdd(&h[d2 * kCopies + copy], 1u);
            if (idx + 3 < n) atomicAdd(&h[d3 * kCopies + copy], 1u);
        }
    }
    __syncthreads();
    for (int d = threadIdx.x; d < radix; d += kThreads)
        hist[(int64_t)d * nblocks + tile] = h[d * kCopies] + h[d * kCopies + 1] + h[d * kCopies + 2] + h[d * kCopies + 3];
}

// Stable scatter of one digit.  Tile order is (wave, slot, lane) = ascending input index, and the rank of a
// key among equal digits is: keys of earlier blocks (scanned histogram) + earlier waves of the tile + earlier
// slots of the wave + lower lanes of the slot.  The tile is first put in digit order in LDS and then written
// out by consecutive threads, so that each digit's run leaves the block as contiguous, coalesced stores
// (scattering straight from registers costs one memory transaction per 4-byte element).
//
// LAST (the pass over the top digit of the pair sort): the sorted keys themselves are wanted only for the row
// pointers, so they are not written.  A digit's run of a tile is a contiguous piece of the final order: every key of
// the run that differs from the key before it in the run starts a row (and the empty rows just before it) at its
// global position, stored here; what the run cannot see -- whether its FIRST key continues the row that ends the
// previous non-empty run -- is left to rowptr_run_starts_kernel, for which the first and last key of every run are
// kept in `run_keys` (two arrays in the histogram's layout).
// BITS > 0: the digit width as a compile-time constant (the vote loop unrolls into straight-line code, 6 vector
// instructions per bit); BITS == 0: any width, taken from the `bits` argument.
template <bool HAS_VALS, bool LAST, int BITS>
__global__ __launch_bounds__(kThreads) void radix_scatter_kernel(const uint32_t *keys_in, const int32_t *vals_in,
                                                                 uint32_t *keys_out, int32_t *vals_out, int64_t n,
                                                                 int shift, int bits, const uint32_t *hist_scanned,
                                                                 int64_t nblocks, int remap, int64_t n_nodes,
                                                                 int64_t *rowptr, uint32_t *run_keys, uint32_t val_limit,
                                                                 uint32_t *bad_flag) {
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
    if constexpr (HAS_VALS) {
        if (val_limit) {  // first pass over a source column that nothing has range-checked yet (padding lanes hold 0)
            bool bad = false;
#pragma unroll
            for (int s = 0; s < kItems; ++s) bad = bad || (uint32_t)val[s] >= val_limit;
            if (bad) atomicOr(bad_flag, 1u);
        }
    }
#pragma unroll
    for (int s = 0; s < kItems; ++s) {
        const int64_t idx = wave_base + s * kWave + lane;
        const bool valid = idx < n;
        const uint32_t d = (key[s] >> shift) & mask;
        // lanes of this slot with the same digit: one vote per bit; a lane keeps the voters when its own bit is set
        // and the others when it is not (an invalid lane holds key 0, so it never votes and is masked out by `all`)
        const uint64_t all = __ballot(valid);
        uint32_t peers_lo = (uint32_t)all, peers_hi = (uint32_t)(all >> 32);
        auto vote_on = [&](int b) {
            const uint32_t own = 0u - ((d >> b) & 1u);  // all ones when the lane's bit is set
            const uint64_t vote = __ballot(own != 0u);
            peers_lo &= ~((uint32_t)vote ^ own);
            peers_hi &= ~((uint32_t)(vote >> 32) ^ own);
        };
        if constexpr (BITS > 0) {
#pragma unroll
            for (int b = 0; b < BITS; ++b) vote_on(b);
        } else {
            for (int b = 0; b < bits; ++b) vote_on(b);
        }
        const uint64_t peers = ((uint64_t)peers_hi << 32) | peers_lo;
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
    if constexpr (LAST) {
        if (threadIdx.x < radix && total_d > 0) {
            const int64_t e = (int64_t)threadIdx.x * nblocks + tile;
            run_keys[e] = skey[ls];
            run_keys[(int64_t)radix * nblocks + e] = skey[ls + total_d - 1];
        }
    }
    for (uint32_t i = threadIdx.x; i < tile_total; i += kThreads) {
        const uint32_t k = skey[i];
        const uint32_t d = (k >> shift) & mask;
        const uint32_t pos = gbase[d] + (i - lstart[d]);
        if constexpr (LAST) {
            // rows (kp, k] start here when the key before this one in the run, kp, differs; the first key of a run
            // takes kp = k, which leaves the loop empty (ids are clamped so that invalid input cannot run it long)
            const uint32_t ls_d = lstart[d];
            const uint32_t kp = i > ls_d ? skey[i - 1] : k;
            const uint32_t hi = k < (uint32_t)n_nodes ? k : (uint32_t)n_nodes;
            for (uint32_t v = (kp < 0x7fffffffu ? kp : 0x7fffffffu) + 1u; v <= hi; ++v) rowptr[v] = (int64_t)pos;
        } else {
            keys_out[pos] = k;
        }
        if constexpr (HAS_VALS) vals_out[pos] = sval[i];
    }
}

// Row pointers at the run starts of the last pass.  Entry e = digit * nblocks + tile of the scanned histogram is a
// run of the final order starting at position gb[e]; entries in ascending e are consecutive pieces of that order.  For
// a non-empty run the key before its first key is the last key of the closest non-empty run before it (normally
// e - 1; otherwise found by bisection of the non-decreasing gb, so that long stretches of empty runs cost
// nothing).  The first run of all also starts the rows from 0, the last one ends the rows up to n_nodes.
__global__ void rowptr_run_starts_kernel(const uint32_t *gb, const uint32_t *run_keys, int64_t n_entries, int64_t n_edges,
                                         int64_t n_nodes, int64_t *rowptr) {
    const uint32_t *first_key = run_keys, *last_key = run_keys + n_entries;
    for (int64_t e = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; e < n_entries; e += (int64_t)gridDim.x * blockDim.x) {
        const int64_t start = gb[e];
        const int64_t end = e + 1 < n_entries ? (int64_t)gb[e + 1] : n_edges;
        if (end == start) continue;
        int64_t kp = -1;
        if (start > 0) {
            int64_t prev = e - 1;
            if ((int64_t)gb[prev] == start) {
                // first entry whose start equals this one's, minus one: that run is non-empty and ends at `start`
                int64_t lo = 0, hi = prev;  // invariant: gb[hi] == start, gb[lo] < start or lo == 0
                while (lo < hi) {
                    const int64_t mid = (lo + hi) >> 1;
                    if ((int64_t)gb[mid] < start) lo = mid + 1; else hi = mid;
                }
                prev = lo - 1;
            }
            kp = last_key[prev];
        }
        const int64_t k = first_key[e];
        if (k != kp) {
            const int64_t hi = k < n_nodes ? k : n_nodes;
            for (int64_t v = kp + 1; v <= hi; ++v) rowptr[v] = start;
        }
        if (end == n_edges) {
            const int64_t kl = last_key[e];
            for (int64_t v = kl + 1; v <= n_nodes; ++v) rowptr[v] = n_edges;
        }
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

// Second level folded into the first: with at most kScanTile partial sums every block adds up the partials of the
// blocks before it by itself (one 8-item read per thread), which saves the launch of a one-block scan in between.
__global__ __launch_bounds__(kScanThreads) void scan_apply_self_offset_kernel(uint32_t *data, int64_t n, const uint32_t *partial) {
    __shared__ uint32_t sm[17];
    uint32_t before = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        const int j = threadIdx.x * kScanItems + i;
        if (j < (int)blockIdx.x) before += partial[j];
    }
    uint32_t offset;
    block_exclusive_scan<uint32_t>(before, sm, &offset);   // offset = sum over the whole block = sum of partial[0 .. blockIdx)
    const int64_t base = (int64_t)blockIdx.x * kScanTile + (int64_t)threadIdx.x * kScanItems;
    uint32_t v[kScanItems];
    uint32_t s = 0;
#pragma unroll
    for (int i = 0; i < kScanItems; ++i) {
        v[i] = (base + i < n) ? data[base + i] : 0u;
        s += v[i];
    }
    uint32_t total;
    uint32_t run = block_exclusive_scan<uint32_t>(s, sm, &total) + offset;
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
    if (nb <= kScanTile) {
        scan_apply_self_offset_kernel<<<(unsigned)nb, kScanThreads, 0, st>>>(data, n, ws);
        ITB_LAUNCH_CHECK();
        return ITB_OK;
    }
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

template <bool HAS_VALS, bool LAST>
void launch_scatter_bits(int bits, unsigned grid, hipStream_t st, const uint32_t *kin, const int32_t *vin, uint32_t *kout, int32_t *vout,
                         int64_t n, int shift, const uint32_t *h, int64_t nblocks, int remap, int64_t n_nodes, int64_t *rowptr,
                         uint32_t *run_keys, uint32_t val_limit, uint32_t *bad_flag) {
#define ITB_SCATTER(B)                                                                                                          \
    radix_scatter_kernel<HAS_VALS, LAST, B><<<grid, kThreads, 0, st>>>(kin, vin, kout, vout, n, shift, bits, h, nblocks, remap, \
                                                                       n_nodes, rowptr, run_keys, val_limit, bad_flag)
    switch (bits) {  // the widths that graphs beyond a few thousand vertices use get straight-line vote code
        case 5: ITB_SCATTER(5); break;
        case 6: ITB_SCATTER(6); break;
        case 7: ITB_SCATTER(7); break;
        case 8: ITB_SCATTER(8); break;
        default: ITB_SCATTER(0); break;
    }
#undef ITB_SCATTER
}

void launch_scatter(bool pairs, bool last, int bits, unsigned grid, hipStream_t st, const uint32_t *kin, const int32_t *vin,
                    uint32_t *kout, int32_t *vout, int64_t n, int shift, const uint32_t *h, int64_t nblocks, int remap,
                    int64_t n_nodes, int64_t *rowptr, uint32_t *run_keys, uint32_t val_limit, uint32_t *bad_flag) {
    if (last)
        launch_scatter_bits<true, true>(bits, grid, st, kin, vin, kout, vout, n, shift, h, nblocks, remap, n_nodes, rowptr, run_keys,
                                        val_limit, bad_flag);
    else if (pairs)
        launch_scatter_bits<true, false>(bits, grid, st, kin, vin, kout, vout, n, shift, h, nblocks, remap, n_nodes, rowptr, run_keys,
                                         val_limit, bad_flag);
    else
        launch_scatter_bits<false, false>(bits, grid, st, kin, vin, kout, vout, n, shift, h, nblocks, remap, n_nodes, rowptr, run_keys,
                                          0u, nullptr);
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
    const int64_t part_hist_elems = (int64_t)kMaxPartRadix * (nblocks > 0 ? nblocks : 1);
    Carver cv(workspace);
    uint32_t *flag = cv.take<uint32_t>(64);
    uint32_t *kbuf0 = cv.take<uint32_t>((size_t)n_edges);
    uint32_t *kbuf1 = cv.take<uint32_t>((size_t)n_edges);
    int32_t *vtmp = cv.take<int32_t>((size_t)n_edges);
    uint32_t *hist = cv.take<uint32_t>((size_t)hist_elems);
    uint32_t *hist_src = cv.take<uint32_t>((size_t)part_hist_elems);  // histograms of the source sort (reserved whether or not
                                                                  // deg_out is asked for: the size query passes no pointers)
    uint32_t *scan_ws = cv.take<uint32_t>(scan_workspace_elems(part_hist_elems) + 64);
    // buffers of the out-degree branch, separate so that it can run beside the pair sort
    uint32_t *scan_ws_deg = cv.take<uint32_t>(scan_workspace_elems(part_hist_elems) + 64);
    uint16_t *low_keys = cv.take<uint16_t>((size_t)n_edges);
    uint32_t *bounds = cv.take<uint32_t>((size_t)n_nodes + 1);
    uint32_t *run_keys = cv.take<uint32_t>(2 * (size_t)hist_elems);  // first and last key of every run of the last pass
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

    // Out-degrees by partition + bucket histogram when a bucket's id range fits the LDS counters (N <= 2^22);
    // otherwise by a keys-only run of the stable sort (run lengths of the sorted sources).
    int part_high = bits_total - 6;
    if (part_high < 1) part_high = 1;
    if (part_high > 9) part_high = 9;
    if (part_high > bits_total) part_high = bits_total;
    const int part_low = bits_total - part_high;
    const bool deg_by_partition = deg_out && part_low <= kMaxLowBits && itb::g_tuning.csr_deg_by_sort.load() == 0;

    const int xcd_remap = itb::g_tuning.csr_xcd_remap.load();
    fill_u32_kernel<<<1, 64, 0, st>>>(flag, 64, 0u);
    ITB_LAUNCH_CHECK();
    {
        const int bits0 = base_bits + (0 < extra ? 1 : 0);
        if (deg_by_partition)
            first_pass_kernel<2><<<(unsigned)nblocks, kThreads, 0, st>>>(n_edges, (uint32_t)n_nodes, src, dst, bits0, hist, part_low,
                                                                         1 << part_high, hist_src, nblocks, xcd_remap, flag);
        else if (deg_out)
            first_pass_kernel<1><<<(unsigned)nblocks, kThreads, 0, st>>>(n_edges, (uint32_t)n_nodes, src, dst, bits0, hist, 0, 1 << bits0,
                                                                         hist_src, nblocks, xcd_remap, flag);
        else
            first_pass_kernel<0><<<(unsigned)nblocks, kThreads, 0, st>>>(n_edges, (uint32_t)n_nodes, src, dst, bits0, hist, 0, 1,
                                                                             nullptr, nblocks, xcd_remap, flag);
        ITB_LAUNCH_CHECK();
    }
    // The out-degree branch shares nothing with the pair sort but the raw table and the first-pass histograms: it is
    // enqueued on the helper stream (when there is one) and joins before the final synchronisation.
    itb::SideFork fork;
    {
        const int32_t rc = fork.begin((deg_by_partition && itb::g_tuning.overlap_hubs.load()) ? itb::side_stream() : nullptr, st);
        if (rc != ITB_OK) return rc;
    }
    if (deg_by_partition) {
        hipStream_t dst_stream = fork.stream();
        const int radix = 1 << part_high;
        int32_t rc = exclusive_scan_u32(hist_src, (int64_t)radix * nblocks, scan_ws_deg, dst_stream);
        if (rc != ITB_OK) return rc;
        partition_scatter_kernel<<<(unsigned)nblocks, kThreads, 0, dst_stream>>>(reinterpret_cast<const uint32_t *>(src), low_keys,
                                                                                 n_edges, part_low, radix, hist_src, nblocks,
                                                                                 xcd_remap);
        ITB_LAUNCH_CHECK();
        fill_u32_kernel<<<grid_for(n_nodes, 256), 256, 0, dst_stream>>>(reinterpret_cast<uint32_t *>(deg_out), n_nodes, 0u);
        ITB_LAUNCH_CHECK();
        bucket_degree_kernel<<<dim3((unsigned)radix, kDegSlicesY), kDegThreads, 0, dst_stream>>>(low_keys, n_edges, hist_src, nblocks,
                                                                                                 radix, part_low, n_nodes, deg_out);
        ITB_LAUNCH_CHECK();
        rc = fork.mark_done();
        if (rc != ITB_OK) return rc;
    }

    // One radix sort, run once or twice: keys only over the sources (their run lengths are the out-degrees;
    // a histogram by atomics would cost one memory-side atomic per edge), then (dst, src) pairs for the CSR.
    const uint32_t *kin = nullptr;
    for (int which = (deg_out && !deg_by_partition) ? 0 : 1; which < 2; ++which) {
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
                radix_hist_kernel<<<(unsigned)nblocks, kThreads, 0, st>>>(kin, n_edges, shift, bits, h, nblocks, xcd_remap);
                ITB_LAUNCH_CHECK();
            }
            int32_t rc = exclusive_scan_u32(h, hist_n, scan_ws, st);
            if (rc != ITB_OK) return rc;
            const bool last = pairs && p == passes - 1;
            // last pass of the pair sort: no sorted keys are written, the row pointers come from the runs themselves
            launch_scatter(pairs, last, bits, (unsigned)nblocks, st, kin, pairs ? vin : nullptr, last ? nullptr : kout,
                           pairs ? vout : nullptr, n_edges, shift, h, nblocks, xcd_remap, n_nodes, last ? rowptr : nullptr,
                           last ? run_keys : nullptr, (pairs && p == 0 && !deg_out) ? (uint32_t)n_nodes : 0u, flag);
            ITB_LAUNCH_CHECK();
            if (last) rowptr_run_starts_kernel<<<grid_for(hist_n, 256), 256, 0, st>>>(h, run_keys, hist_n, n_edges, n_nodes, rowptr);
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
    {
        const int32_t rc = fork.finish();
        if (rc != ITB_OK) return rc;
    }
    uint32_t host_flag = 0;
    ITB_HIP(hipMemcpyAsync(&host_flag, flag, sizeof(uint32_t), hipMemcpyDeviceToHost, st));
    ITB_HIP(hipStreamSynchronize(st));
    return host_flag ? ITB_ERR_RANGE : ITB_OK;
}
