// Measurement aids (not part of the method): the A/B switches, the plain copy kernel that hardware byte counters
// are scaled against, and a random-row read probe that measures what this machine's memory system delivers for the
// access pattern of a gather (sequential index stream, one random row of a given size per index) with no
// arithmetic at all.
#include "common.h"

#include "inferturbo_aids.h"

namespace itb {
Tuning g_tuning;
}

namespace {
using namespace itb;

// Plain 16-byte-per-lane copy: the known-size reference against which hardware byte counters are scaled.
__global__ void copy_kernel(const uint4 *src, uint4 *dst, int64_t n_vec) {
    for (int64_t i = blockIdx.x * (int64_t)blockDim.x + threadIdx.x; i < n_vec; i += (int64_t)gridDim.x * blockDim.x) dst[i] = src[i];
}

// A lane group of G lanes reads the row idx[i] (16 bytes per lane), U independent rows in flight per lane group;
// the words are folded by xor and one word per thread reaches `sink`, so that no load can be dropped.
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));

// NT: non-temporal loads, as the gather uses them for tables far beyond the caches.
template <int G, int U, bool NT>
__global__ __launch_bounds__(256) void random_rows_kernel(const uint4 *table, const int32_t *idx, int64_t n_idx, uint32_t *sink) {
    constexpr int NG = kWave / G;
    const int lane = threadIdx.x & (kWave - 1);
    const int g = lane / G, li = lane % G;
    const int64_t wave = (blockIdx.x * (int64_t)blockDim.x + threadIdx.x) / kWave;
    const int64_t n_waves = (int64_t)gridDim.x * blockDim.x / kWave;
    uint32_t fold = 0;
    // a wavefront takes 64 consecutive indices at a time (one coalesced load), lane group g the ones congruent to g
    for (int64_t base = wave * kWave; base < n_idx; base += n_waves * kWave) {
        const int myi = (base + lane < n_idx) ? idx[base + lane] : -1;
        for (int t = 0; t < G; t += U) {
            uint4 raw[U];
#pragma unroll
            for (int q = 0; q < U; ++q) {
                const int u = __shfl(myi, (t + q) * NG + g, kWave);
                if (u < 0) raw[q] = make_uint4(0, 0, 0, 0);
                else if constexpr (NT) {
                    const u32x4 v = __builtin_nontemporal_load(reinterpret_cast<const u32x4 *>(table) + ((int64_t)u * G + li));
                    raw[q] = make_uint4(v.x, v.y, v.z, v.w);
                } else raw[q] = table[(int64_t)u * G + li];
            }
#pragma unroll
            for (int q = 0; q < U; ++q) fold ^= raw[q].x ^ raw[q].y ^ raw[q].z ^ raw[q].w;
        }
    }
    sink[blockIdx.x * (int64_t)blockDim.x + threadIdx.x] = fold;
}

template <int G>
int32_t launch_probe(const void *table, int64_t table_bytes, const int32_t *idx, int64_t n_idx, void *sink, int blocks, hipStream_t st) {
    constexpr int U = G < 4 ? G : 4;
    constexpr int U8 = G < 8 ? G : 8;
    const int want = itb::g_tuning.gather_unroll.load();  // A/B switch 7: row loads in flight per lane
    // A/B switch 8: 1 = non-temporal loads, 0 = plain, -1 = as the gather would choose for a table of this size
    const int policy = itb::g_tuning.row_load_policy.load();
    const bool nt = policy >= 0 ? policy == 1 : table_bytes >= itb::kStreamRowsFromBytes;
    const uint4 *t = static_cast<const uint4 *>(table);
    uint32_t *s = static_cast<uint32_t *>(sink);
    if (nt) {
        if (want == 8) random_rows_kernel<G, U8, true><<<blocks, 256, 0, st>>>(t, idx, n_idx, s);
        else random_rows_kernel<G, U, true><<<blocks, 256, 0, st>>>(t, idx, n_idx, s);
    } else if (want == 8)
        random_rows_kernel<G, U8, false><<<blocks, 256, 0, st>>>(t, idx, n_idx, s);
    else if (want == 1)
        random_rows_kernel<G, 1, false><<<blocks, 256, 0, st>>>(t, idx, n_idx, s);
    else
        random_rows_kernel<G, U, false><<<blocks, 256, 0, st>>>(t, idx, n_idx, s);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

}  // namespace

extern "C" int32_t itb_copy_bytes(const void *src, void *dst, int64_t n_bytes, void *stream) {
    if (n_bytes < 0 || (n_bytes & 15)) return ITB_ERR_SIZE;
    if (n_bytes > 0 && (!src || !dst)) return ITB_ERR_NULL;
    if (n_bytes == 0) return ITB_OK;
    copy_kernel<<<8192, 256, 0, static_cast<hipStream_t>(stream)>>>(static_cast<const uint4 *>(src), static_cast<uint4 *>(dst), n_bytes / 16);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

extern "C" int32_t itb_random_row_read(const void *table, int64_t n_rows, int32_t row_bytes, const int32_t *idx, int64_t n_idx,
                                       void *sink, int64_t sink_bytes, void *stream) {
    if (n_rows <= 0 || n_rows >= ((int64_t)1 << 31) || n_idx < 0) return ITB_ERR_SIZE;
    if (row_bytes != 16 && row_bytes != 32 && row_bytes != 64 && row_bytes != 128 && row_bytes != 256 && row_bytes != 512 &&
        row_bytes != 1024)
        return ITB_ERR_UNSUPPORTED;
    if (!table || !sink || (n_idx > 0 && !idx)) return ITB_ERR_NULL;
    if (!aligned16(table)) return ITB_ERR_UNSUPPORTED;
    const int blocks = 256 * 8;  // 8 blocks of 4 wavefronts per compute unit: every SIMD full
    if (sink_bytes < (int64_t)blocks * 256 * 4) return ITB_ERR_WORKSPACE;
    hipStream_t st = static_cast<hipStream_t>(stream);
    switch (row_bytes / 16) {
        case 1: return launch_probe<1>(table, n_rows * (int64_t)row_bytes, idx, n_idx, sink, blocks, st);
        case 2: return launch_probe<2>(table, n_rows * (int64_t)row_bytes, idx, n_idx, sink, blocks, st);
        case 4: return launch_probe<4>(table, n_rows * (int64_t)row_bytes, idx, n_idx, sink, blocks, st);
        case 8: return launch_probe<8>(table, n_rows * (int64_t)row_bytes, idx, n_idx, sink, blocks, st);
        case 16: return launch_probe<16>(table, n_rows * (int64_t)row_bytes, idx, n_idx, sink, blocks, st);
        case 32: return launch_probe<32>(table, n_rows * (int64_t)row_bytes, idx, n_idx, sink, blocks, st);
        default: return launch_probe<64>(table, n_rows * (int64_t)row_bytes, idx, n_idx, sink, blocks, st);
    }
}

extern "C" int32_t itb_set_tuning(int32_t key, int32_t value) {
    Tuning &t = itb::g_tuning;
    if (key == 0) { t.small_limit = value; return ITB_OK; }
    if (key == 2) { t.csr_xcd_remap = value; return ITB_OK; }
    if (key == 3 && value > 0) { t.long_row = value; return ITB_OK; }
    if (key == 4) { t.rows_waves_per_simd = value; return ITB_OK; }
    if (key == 5) { t.csr_deg_by_sort = value; return ITB_OK; }
    if (key == 6) { t.overlap_hubs = value; return ITB_OK; }
    if (key == 7) { t.gather_unroll = value; return ITB_OK; }
    if (key == 8 && value >= -1 && value <= 1) { t.row_load_policy = value; return ITB_OK; }
    if (key == 9) { t.chain_updates = value; return ITB_OK; }
    if (key == 10) { t.epilogue_scores = value; return ITB_OK; }
    return ITB_ERR_UNSUPPORTED;
}
