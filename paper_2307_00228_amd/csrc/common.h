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

#include <mutex>

namespace itb {

// A helper stream per device on which gather_layer runs the hub passes (segment partials + combine) next to the
// row passes of the caller's stream: fork = event recorded on the caller's stream that the helper waits for,
// join = event recorded on the helper that the caller's stream waits for.  Default priority, non-blocking.
// Feature tensors are read and written as 16-byte vectors.
inline bool aligned16(const void *p) { return (reinterpret_cast<uintptr_t>(p) & 15u) == 0; }

struct SideStream {
    hipStream_t stream;
    hipEvent_t fork, join;
    std::mutex mu;  // held from the fork record to the join wait: host threads sharing the device must not interleave them
};
SideStream *side_stream();  // nullptr if it cannot be created (callers then stay on the one stream)
extern int g_overlap_hubs;  // tuning hook (key 6): 0 = everything on the caller's stream

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
