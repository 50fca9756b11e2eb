// Internal helpers shared by the HIP translation units of libinferturbo_hip.
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>

#include "inferturbo.h"

#define ITB_HIP(call)                                   \
    do {                                                \
        if ((call) != hipSuccess) return ITB_ERR_DEVICE; \
    } while (0)

#define ITB_LAUNCH_CHECK()                                       \
    do {                                                         \
        if (hipGetLastError() != hipSuccess) return ITB_ERR_DEVICE; \
    } while (0)

#include <atomic>
#include <type_traits>
#include <mutex>

namespace itb {

// Feature tensors are read and written as 16-byte vectors.
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

// Library-owned state, one per device, created at the first call that uses it and destroyed by itb_shutdown():
// a helper stream on which gather_layer runs the hub passes (segment partials + combine) and build_csr_by_dst the
// out-degree branch, next to the work on the caller's stream.  fork = event recorded on the caller's stream that
// the helper waits for, join = event recorded on the helper that the caller's stream waits for.  Default
// priority, non-blocking.
struct SideStream {
    hipStream_t stream;
    hipEvent_t fork, join;
    std::mutex mu;  // held from the fork record to the join wait: host threads sharing the device must not interleave them
};
SideStream *side_stream();  // nullptr if it cannot be created (callers then stay on the one stream)
void destroy_side_streams();

// Process-wide A/B switches of the measurement aids (itb_set_tuning, keys in brackets); atomics because a caller may
// flip one while another host thread is inside a call.
struct Tuning {
    std::atomic<int> small_limit{-1};         // [0] rows with in-degree <= limit use one lane group per row (-1 = built-in)
    std::atomic<int> csr_xcd_remap{1};        // [2] XCD-contiguous tile order in the radix passes
    std::atomic<int> long_row{512};           // [3] rows with more in-edges get a whole block
    std::atomic<int> rows_waves_per_simd{-1}; // [4] resident wavefronts per SIMD of the row gather (0 = no cap, -1 = built-in)
    std::atomic<int> csr_deg_by_sort{0};      // [5] out-degrees always from a keys-only run of the stable sort
    std::atomic<int> overlap_hubs{1};         // [6] 0 = everything on the caller's stream
    std::atomic<int> gather_unroll{-1};       // [7] row loads in flight per lane of the gather loops (-1 = built-in)
    std::atomic<int> row_load_policy{-1};     // [8] random row loads: 0 = plain, 1 = non-temporal, -1 = by table size
    std::atomic<int> chain_updates{1};        // [9] an update feeds the next (narrowing) layer's projection in the same launch
    std::atomic<int> epilogue_scores{1};      // [10] attention scores of a projection from its epilogue (0 = always by the score tile)
};
extern Tuning g_tuning;

// One 16-byte piece of a randomly addressed source row.  STREAM: non-temporal load.  Measured on MI355X with random
// rows of 16..256 bytes: a table of 12.8 GB is read at 52 G rows/s (6.9 TB/s of 128-byte lines) non-temporally against
// 47 G rows/s (6.2 TB/s) with plain loads, a 3 GB table 4 % faster; tables of 1 GB and less, which partly live in the
// caches, are 5-10 % faster with plain loads.  The host picks per launch (stream_rows_for).
typedef uint32_t u32x4_t __attribute__((ext_vector_type(4)));
constexpr int64_t kStreamRowsFromBytes = (int64_t)3 << 30;  // the smallest table size measured to gain
template <bool STREAM>
__device__ __forceinline__ uint4 load_row_piece(const uint4 *p) {
    if constexpr (STREAM) {
        const u32x4_t v = __builtin_nontemporal_load(reinterpret_cast<const u32x4_t *>(p));
        return make_uint4(v.x, v.y, v.z, v.w);
    } else {
        return *p;
    }
}
template <bool STREAM>
__device__ __forceinline__ float load_row_scalar(const float *p) {
    if constexpr (STREAM) return __builtin_nontemporal_load(p);
    else return *p;
}
// 16-byte store; `stream`: non-temporal (rows of a table far beyond the caches, written once and read by a later launch)
__device__ __forceinline__ void store_piece(void *p, uint4 v, bool stream) {
    if (stream) {
        u32x4_t w;
        w.x = v.x; w.y = v.y; w.z = v.z; w.w = v.w;
        __builtin_nontemporal_store(w, static_cast<u32x4_t *>(p));
    } else {
        *static_cast<uint4 *>(p) = v;
    }
}
// A/B switch 8: 0 never, 1 always, -1 by the size of the table the rows come from.
inline int32_t stream_rows_for(int64_t table_bytes) {
    const int policy = g_tuning.row_load_policy.load();
    return policy >= 0 ? policy : (table_bytes >= kStreamRowsFromBytes);
}

// One fork/join of the helper stream.  Whatever path a call takes after begin() -- an error return included --
// the destructor records the join on the helper stream and makes the caller's stream wait for it, so that no
// call leaves the caller's stream (or a stream capture) with an open fork.
class SideFork {
   public:
    SideFork() = default;
    SideFork(const SideFork &) = delete;
    SideFork &operator=(const SideFork &) = delete;
    ~SideFork() { finish(); }
    // `side` may be nullptr: everything then stays on `main`.
    int32_t begin(SideStream *side, hipStream_t main) {
        main_ = main;
        if (!side) return ITB_OK;
        lock_ = std::unique_lock<std::mutex>(side->mu);
        if (hipEventRecord(side->fork, main) != hipSuccess) { lock_.unlock(); return ITB_ERR_DEVICE; }
        side_ = side;  // from here on the helper stream depends on `main`: it must be joined back
        if (hipStreamWaitEvent(side->stream, side->fork, 0) != hipSuccess) return ITB_ERR_DEVICE;
        return ITB_OK;
    }
    hipStream_t stream() const { return side_ ? side_->stream : main_; }
    // The helper's work is enqueued: record the join point (the caller's stream waits for it in finish()).
    int32_t mark_done() {
        if (!side_ || recorded_) return ITB_OK;
        recorded_ = true;
        return hipEventRecord(side_->join, side_->stream) == hipSuccess ? ITB_OK : ITB_ERR_DEVICE;
    }
    int32_t finish() {
        if (!side_) return ITB_OK;
        int32_t rc = mark_done();
        if (hipStreamWaitEvent(main_, side_->join, 0) != hipSuccess) rc = ITB_ERR_DEVICE;
        side_ = nullptr;
        lock_.unlock();
        return rc;
    }

   private:
    SideStream *side_ = nullptr;
    hipStream_t main_ = nullptr;
    bool recorded_ = false;
    std::unique_lock<std::mutex> lock_;
};

// Internal knobs of a gather_layer call.
struct GatherOptions {
    // device array {row_lo, row_hi, seg_lo, seg_hi, hub_lo, hub_hi} of the edge range, or nullptr: computed by the
    // call itself when the range is not the whole graph
    const int64_t *bounds = nullptr;
    // the hub passes may run on the library's helper stream (false: everything on the caller's stream, no
    // library-owned object is created or touched)
    bool allow_side = true;
    // h_src is a table with one row per in-edge in CSR order and `col` is not used
    bool per_edge_rows = false;
    // a fork the CALLER has begun and will finish: the hub passes of this call are enqueued on its stream and the
    // call does not join.  The layer loop uses one fork for all edge ranges of a layer, so that the hub passes of one
    // range overlap the row passes of the next instead of every range ending in a join.
    SideFork *outer_fork = nullptr;
};

constexpr int kWave = 64;

static inline size_t align_up(size_t x, size_t a = 256) { return (x + a - 1) / a * a; }

// Carves 256-byte aligned pieces out of the caller's workspace; with base == nullptr it only sizes.
struct Carver {
    char *base;
    size_t off = 0;
    explicit Carver(void *b) : base(static_cast<char *>(b)) {}
    template <typename T>
    T *take(size_t count) {
        size_t o = off;
        off += align_up(count * sizeof(T));
        return base ? reinterpret_cast<T *>(base + o) : nullptr;
    }
};

// ---- bf16 storage format -----------------------------------------------------------------
__device__ __forceinline__ float bf16_lo(uint32_t packed) { return __uint_as_float(packed << 16); }
__device__ __forceinline__ float bf16_hi(uint32_t packed) { return __uint_as_float(packed & 0xffff0000u); }

// fp32 -> bf16, round to nearest even: the conversion of a float pair is one gfx950 instruction
// (v_cvt_pk_bf16_f32); written as a vector conversion so that the compiler selects it.
typedef __bf16 itb_bf16x2 __attribute__((ext_vector_type(2)));
typedef float itb_f32x2 __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
    const itb_f32x2 v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, itb_bf16x2));
}
__device__ __forceinline__ uint32_t f32_to_bf16(float f) { return pack_bf16x2(f, 0.f) & 0xffffu; }

// ---- wave / block scans ------------------------------------------------------------------
template <typename T>
__device__ __forceinline__ T wave_inclusive_scan(T v) {
    const int lane = threadIdx.x & (kWave - 1);
#pragma unroll
    for (int d = 1; d < kWave; d <<= 1) {
        T o = __shfl_up(v, d, kWave);
        if (lane >= d) v += o;
    }
    return v;
}

// Exclusive scan across a block of up to 1024 threads; every thread must call it.
// `smem` must hold 17 elements of T.  Returns the exclusive prefix; *total gets the block sum.
template <typename T>
__device__ __forceinline__ T block_exclusive_scan(T v, T *smem, T *total) {
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int nwaves = (blockDim.x + kWave - 1) / kWave;
    T inc = wave_inclusive_scan(v);
    __syncthreads();  // protects smem reuse between consecutive calls
    if (lane == kWave - 1) smem[wave] = inc;
    __syncthreads();
    if (threadIdx.x == 0) {
        T run = 0;
        for (int w = 0; w < nwaves; ++w) {
            T t = smem[w];
            smem[w] = run;
            run += t;
        }
        smem[16] = run;
    }
    __syncthreads();
    *total = smem[16];
    return inc - v + smem[wave];
}

}  // namespace itb
