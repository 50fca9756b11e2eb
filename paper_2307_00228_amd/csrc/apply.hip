// apply_layer: h_out = act([h_self | agg] . [W_self ; W_nbr] + bias) on the matrix cores.
//
// The weights are tiny (<= 256 KB) and the activations are a tall-skinny stream, so:
//   * each block is persistent: it loads the whole [K_total x BN] weight panel into LDS once, in the exact
//     fragment order of the MFMA B operand (one conflict-free 16-byte LDS read per lane per k-chunk), and
//     then walks over 32*waves-row tiles;
//   * every wavefront owns 32 rows and all BN = 32*NT output columns (NT independent 32x32 accumulators,
//     so consecutive MFMAs never wait on each other);
//   * the A operand goes straight from global memory to registers: lane (row i, half kh) loads 16 bytes of
//     its row per k-chunk.  The k index inside a chunk is permuted identically for A and B (a dot product
//     does not care), which lets one 16-byte load feed 4 fp32 MFMAs (32x32x2) or 1 bf16 MFMA (32x32x16);
//   * bias, activation and the store (the scatter of the new state) are fused into the epilogue.
#include "common.h"

namespace {
using namespace itb;

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kApplyThreads = 512;
constexpr int kApplyWaves = kApplyThreads / kWave;
constexpr int kRowsPerBlockTile = 32 * kApplyWaves;
constexpr size_t kMaxWeightLds = 128 * 1024;  // weight panel of the plain update
constexpr size_t kMaxLds = 160 * 1024;        // whole LDS of a CU (weight panel + score panel)

struct ApplyArgs {
    int64_t n;
    const uint4 *h_self;  // nullable
    const uint4 *agg;
    const void *w_self;   // nullable
    const void *w_nbr;
    const float *bias;    // nullable
    void *out;
    int32_t d_in, d_out;
    int32_t act;
    int64_t n_row_tiles;
    // attention-score epilogue (GAT projection): s[v,k] = sum_d att[k,d] * y[v,k,d] from the fp32 accumulators
    int32_t heads;         // 0 = none
    const float *att_src;  // [heads x d_out/heads]
    const float *att_dst;
    float *s_src;          // [n x heads]
    float *s_dst;
    // message output (the scatter-side apply_edge): msg_out[v] = h_out[v] * msg_scale[v], both nullable together
    const float *msg_scale;
    void *msg_out;
    // optional addend [n x d_out] of the storage dtype, added before the activation (the gathered projection when
    // the neighbour product was taken before the gather)
    const void *addend;
};

// LDS weight panel: chunk kc (8 fp32 / 16 bf16 values of k), half kh, column j -> one uint4 holding the
// 4 (fp32) or 8 (bf16) consecutive-k weights W[kc*KC + kh*KC/2 + t][col0 + j].
template <bool BF16, int NT>
__device__ __forceinline__ void load_weight_panel(uint4 *wlds, const ApplyArgs &a, int col0) {
    constexpr int BN = 32 * NT;
    constexpr int KC = BF16 ? 16 : 8;
    constexpr int KH = KC / 2;
    const int phases = a.h_self ? 2 : 1;
    const int chunks_per_phase = a.d_in / KC;
    const int total = phases * chunks_per_phase * 2 * BN;
#pragma unroll 4
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int j = idx % BN;
        const int kh = (idx / BN) & 1;
        const int kcg = idx / (2 * BN);
        const int phase = kcg / chunks_per_phase;
        const int kc = kcg % chunks_per_phase;
        const void *wbase = (phases == 2 && phase == 0) ? a.w_self : a.w_nbr;
        const int col = col0 + j;
        const int k0 = kc * KC + kh * KH;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (col < a.d_out) {
            if constexpr (BF16) {
                const uint16_t *w = static_cast<const uint16_t *>(wbase);
                uint32_t e[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) e[t] = w[(int64_t)(k0 + t) * a.d_out + col];
                v.x = e[0] | (e[1] << 16);
                v.y = e[2] | (e[3] << 16);
                v.z = e[4] | (e[5] << 16);
                v.w = e[6] | (e[7] << 16);
            } else {
                const uint32_t *w = static_cast<const uint32_t *>(wbase);
                v.x = w[(int64_t)(k0 + 0) * a.d_out + col];
                v.y = w[(int64_t)(k0 + 1) * a.d_out + col];
                v.z = w[(int64_t)(k0 + 2) * a.d_out + col];
                v.w = w[(int64_t)(k0 + 3) * a.d_out + col];
            }
        }
        wlds[idx] = v;
    }
}

template <bool BF16, int NT>
__device__ __forceinline__ void mfma_chunk(v16f (&acc)[NT], const uint4 &av, const uint4 (&bv)[NT]) {
    if constexpr (BF16) {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
            acc[nt] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(__builtin_bit_cast(v8bf, av), __builtin_bit_cast(v8bf, bv[nt]), acc[nt], 0, 0, 0);
    } else {
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.x), __uint_as_float(bv[nt].x), acc[nt], 0, 0, 0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.y), __uint_as_float(bv[nt].y), acc[nt], 0, 0, 0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.z), __uint_as_float(bv[nt].z), acc[nt], 0, 0, 0);
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) acc[nt] = __builtin_amdgcn_mfma_f32_32x32x2f32(__uint_as_float(av.w), __uint_as_float(bv[nt].w), acc[nt], 0, 0, 0);
    }
}

// Attention-score panel for the GAT projection.  s[v,j] = sum_d att[j][d] * (h[v] . W[:, head(j)*dh + d]) is
// linear in h[v], so it equals h[v] . U[:, j] with U[k][j] = sum_d W[k][head*dh + d] * att[j][d]: 2*heads extra
// output columns.  Every block folds U once (fp32) and keeps it in LDS in B-fragment order as a fifth 32-column
// tile; the scores then come out of the matrix cores with the projection, with no cross-lane reduction.
// Column j < heads is the source score of head j, heads <= j < 2*heads the destination score of head j - heads.
// bf16: U is split into hi + lo bf16 parts (two B fragments per chunk, same accumulator), which keeps it
// accurate to ~2^-17 relative.
template <bool BF16>
__device__ __forceinline__ void load_score_panel(uint4 *slds, const ApplyArgs &a) {
    constexpr int KC = BF16 ? 16 : 8;
    constexpr int KH = KC / 2;
    constexpr int PARTS = BF16 ? 2 : 1;
    const int chunks = a.d_in / KC;
    const int dh = a.d_out / a.heads;
    const int total = chunks * 2 * 32;
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int j = idx & 31;
        const int kh = (idx >> 5) & 1;
        const int kc = idx >> 6;
        const int k0 = kc * KC + kh * KH;
        float u[KH];
#pragma unroll
        for (int t = 0; t < KH; ++t) u[t] = 0.f;
        if (j < 2 * a.heads) {
            const int hd = j < a.heads ? j : j - a.heads;
            const float *att = (j < a.heads ? a.att_src : a.att_dst) + hd * dh;
            for (int d = 0; d < dh; ++d) {
                const float av = att[d];
#pragma unroll
                for (int t = 0; t < KH; ++t) {
                    const int64_t wi = (int64_t)(k0 + t) * a.d_out + hd * dh + d;
                    float wv;
                    if constexpr (BF16) wv = __uint_as_float((uint32_t)static_cast<const uint16_t *>(a.w_nbr)[wi] << 16);
                    else wv = static_cast<const float *>(a.w_nbr)[wi];
                    u[t] = fmaf(wv, av, u[t]);
                }
            }
        }
        if constexpr (BF16) {
            uint32_t hi[8], lo[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) {
                hi[t] = f32_to_bf16(u[t]);
                lo[t] = f32_to_bf16(u[t] - __uint_as_float(hi[t] << 16));
            }
            slds[idx] = make_uint4(hi[0] | (hi[1] << 16), hi[2] | (hi[3] << 16), hi[4] | (hi[5] << 16), hi[6] | (hi[7] << 16));
            slds[total + idx] = make_uint4(lo[0] | (lo[1] << 16), lo[2] | (lo[3] << 16), lo[4] | (lo[5] << 16), lo[6] | (lo[7] << 16));
        } else {
            slds[idx] = make_uint4(__float_as_uint(u[0]), __float_as_uint(u[1]), __float_as_uint(u[2]), __float_as_uint(u[3]));
        }
    }
    (void)PARTS;
}

// PF = k-chunks per group; it divides the number of k-chunks, so the unrolled group body has no branches.
// A fragments are double-buffered by group and the request stream runs on across row tiles (the first
// fragments of the next tile are requested while the current tile finishes and stores).
template <bool BF16, int NT, int PF, bool SCORES, bool MSG, bool ADD>
__global__ __launch_bounds__(kApplyThreads) void apply_kernel(ApplyArgs a) {
    constexpr int SPARTS = BF16 ? 2 : 1;  // B fragments of the score tile per chunk (bf16: hi and lo part)
    extern __shared__ uint4 wlds[];
    constexpr int BN = 32 * NT;
    constexpr int KC = BF16 ? 16 : 8;
    const int col0 = blockIdx.y * BN;
    load_weight_panel<BF16, NT>(wlds, a, col0);
    uint4 *slds = wlds + (int64_t)(a.d_in / KC) * (a.h_self ? 2 : 1) * 2 * BN;  // score panel behind the weight panel
    if constexpr (SCORES) load_score_panel<BF16>(slds, a);
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const int i = lane & 31;
    const int kh = lane >> 5;
    const int chunks = a.d_in / KC;
    const int chunks_self = a.h_self ? chunks : 0;
    const int total = chunks_self + chunks;
    const int64_t row_vecs = 2 * chunks;
    const uint4 *wbase = wlds + kh * BN + i;
    const uint4 *sbase = slds + kh * 32 + i;   // score panel: [part][chunk][kh][32]

    auto tile_rowoff = [&](int64_t tile) -> int64_t {
        int64_t r = tile * kRowsPerBlockTile + (int64_t)w * 32 + i;
        r = r < a.n ? r : a.n - 1;  // clamped rows are computed but never stored
        return r * row_vecs + kh;
    };
    // 16-byte fragment c of the concatenated [h_self | agg] row at vector offset `rowoff`
    auto frag_ptr = [&](int64_t rowoff, int c) -> const uint4 * {
        const bool in_self = c < chunks_self;
        const uint4 *base = in_self ? a.h_self : a.agg;
        const int ci = in_self ? c : c - chunks_self;
        return base + rowoff + 2 * ci;
    };

    float bias_v[NT];  // this lane's bias per column tile, fetched once
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int col = col0 + nt * 32 + i;
        bias_v[nt] = (a.bias && col < a.d_out) ? a.bias[col] : 0.f;
    }

    int64_t tile = blockIdx.x;
    if (tile >= a.n_row_tiles) return;
    int64_t rowoff = tile_rowoff(tile);
    uint4 cur[PF];
#pragma unroll
    for (int p = 0; p < PF; ++p) cur[p] = *frag_ptr(rowoff, p);
    uint4 bcur[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) bcur[nt] = wbase[nt * 32];
    uint4 scur[SCORES ? SPARTS : 1];
    if constexpr (SCORES) {
#pragma unroll
        for (int q = 0; q < SPARTS; ++q) scur[q] = sbase[(int64_t)q * total * 64];
    }

    for (; tile < a.n_row_tiles; tile += gridDim.x) {
        const int64_t next_tile = tile + gridDim.x;
        const int64_t rowoff_next = next_tile < a.n_row_tiles ? tile_rowoff(next_tile) : rowoff;
        v16f acc[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt)
#pragma unroll
            for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;
        v16f sacc;
#pragma unroll
        for (int r = 0; r < 16; ++r) sacc[r] = 0.f;

        for (int c0 = 0; c0 < total; c0 += PF) {
            // Double-buffered A: the PF fragments of the NEXT k-group (running on into the next row tile) are
            // requested first and are only touched a whole group of MFMAs later.
            uint4 nxt[PF];
            {
                const int s0 = c0 + PF;
                const bool wrap = s0 >= total;  // PF divides total: a group never straddles two tiles
                const int64_t ro = wrap ? rowoff_next : rowoff;
                const int sb = wrap ? s0 - total : s0;
#pragma unroll
                for (int p = 0; p < PF; ++p) nxt[p] = *frag_ptr(ro, sb + p);
            }
            __builtin_amdgcn_sched_barrier(0);
#pragma unroll
            for (int p = 0; p < PF; ++p) {
                const int c = c0 + p;
                const int cn = (c + 1 == total) ? 0 : c + 1;
                uint4 bnext[NT];  // B fragments of the next chunk, read from LDS under the current MFMAs
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bnext[nt] = wbase[(int64_t)cn * 2 * BN + nt * 32];
                uint4 snext[SCORES ? SPARTS : 1];
                if constexpr (SCORES) {
#pragma unroll
                    for (int q = 0; q < SPARTS; ++q) snext[q] = sbase[(int64_t)q * total * 64 + (int64_t)cn * 64];
                }
                __builtin_amdgcn_sched_barrier(0);
                mfma_chunk<BF16, NT>(acc, cur[p], bcur);
                if constexpr (SCORES) {
#pragma unroll
                    for (int q = 0; q < SPARTS; ++q) {
                        v16f one[1] = {sacc};
                        const uint4 bq[1] = {scur[q]};
                        mfma_chunk<BF16, 1>(one, cur[p], bq);
                        sacc = one[0];
                    }
                }
                __builtin_amdgcn_sched_barrier(0);
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bcur[nt] = bnext[nt];
                if constexpr (SCORES) {
#pragma unroll
                    for (int q = 0; q < SPARTS; ++q) scur[q] = snext[q];
                }
            }
#pragma unroll
            for (int p = 0; p < PF; ++p) cur[p] = nxt[p];
        }

        // Epilogue.  Accumulator register r of a lane holds row 8*(r/4) + 4*kh + (r%4), column i of the tile.
        const int64_t m0 = tile * kRowsPerBlockTile + (int64_t)w * 32;
        const bool full = (m0 + 32 <= a.n) && (col0 + BN <= a.d_out) && (a.d_out % 4 == 0);
        if (full) {
            // 4x4 transposes inside lane quads (two butterfly steps, lanes ^1 then ^2) turn "4 rows of one column"
            // into "4 consecutive columns of one row", so a lane stores 16 bytes (fp32) / 8 bytes (bf16) at once:
            // lane i ends up with row 8*b + 4*kh + (i&3) and columns 4*(i>>2) .. +3 of the tile.
            const bool odd = (i & 1) != 0, hi = (i & 2) != 0;
            const int64_t row_q = m0 + 4 * kh + (i & 3);
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const float b = bias_v[nt];
                const float b1 = __shfl_xor(b, 1, kWave);   // bias of the neighbouring column
                const float blo = odd ? b1 : b, bhi = odd ? b : b1;   // biases of columns (pair start, pair start + 1)
                const int colq = col0 + nt * 32 + 4 * (i >> 2);
#pragma unroll
                for (int bq = 0; bq < 4; ++bq) {
                    float p0[2], p1[2];  // after step 1: pair jj holds two adjacent columns of one row
#pragma unroll
                    for (int jj = 0; jj < 2; ++jj) {
                        const float va = acc[nt][4 * bq + 2 * jj], vb = acc[nt][4 * bq + 2 * jj + 1];
                        const float got = __shfl_xor(odd ? va : vb, 1, kWave);
                        p0[jj] = odd ? got : va;   // even lane: row 2jj, cols (c, c+1); odd lane: row 2jj+1, cols (c-1, c)
                        p1[jj] = odd ? vb : got;
                        p0[jj] += blo;
                        p1[jj] += bhi;
                        if (!ADD && a.act == ITB_ACT_RELU) {
                            p0[jj] = fmaxf(p0[jj], 0.f);
                            p1[jj] = fmaxf(p1[jj], 0.f);
                        }
                    }
                    const int64_t off = (row_q + 8 * bq) * a.d_out + colq;
                    if constexpr (ADD) {
                        // finish the transpose in fp32, add the addend's four columns of this lane's row, then the
                        // activation, rounding and stores
                        const float g0 = __shfl_xor(hi ? p0[0] : p0[1], 2, kWave);
                        const float g1 = __shfl_xor(hi ? p1[0] : p1[1], 2, kWave);
                        float o[4] = {hi ? g0 : p0[0], hi ? g1 : p1[0], hi ? p0[1] : g0, hi ? p1[1] : g1};
                        if constexpr (BF16) {
                            const uint2 ad = *reinterpret_cast<const uint2 *>(static_cast<const uint16_t *>(a.addend) + off);
                            o[0] += bf16_lo(ad.x); o[1] += bf16_hi(ad.x); o[2] += bf16_lo(ad.y); o[3] += bf16_hi(ad.y);
                        } else {
                            const float4 ad = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.addend) + off);
                            o[0] += ad.x; o[1] += ad.y; o[2] += ad.z; o[3] += ad.w;
                        }
                        if (a.act == ITB_ACT_RELU) {
#pragma unroll
                            for (int t = 0; t < 4; ++t) o[t] = fmaxf(o[t], 0.f);
                        }
                        float ms = 0.f;
                        if constexpr (MSG) ms = a.msg_scale[row_q + 8 * bq];
                        if constexpr (BF16) {
                            *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.out) + off) =
                                make_uint2(pack_bf16x2(o[0], o[1]), pack_bf16x2(o[2], o[3]));
                            if constexpr (MSG)
                                *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.msg_out) + off) =
                                    make_uint2(pack_bf16x2(o[0] * ms, o[1] * ms), pack_bf16x2(o[2] * ms, o[3] * ms));
                        } else {
                            *reinterpret_cast<float4 *>(static_cast<float *>(a.out) + off) = make_float4(o[0], o[1], o[2], o[3]);
                            if constexpr (MSG)
                                *reinterpret_cast<float4 *>(static_cast<float *>(a.msg_out) + off) =
                                    make_float4(o[0] * ms, o[1] * ms, o[2] * ms, o[3] * ms);
                        }
                        continue;
                    }
                    // after step 1 pair jj of a lane belongs to row 8*bq + 4*kh + 2*jj + (i&1) of the tile
                    float ms0 = 0.f, ms1 = 0.f;
                    if constexpr (MSG) {
                        ms0 = a.msg_scale[m0 + 8 * bq + 4 * kh + (i & 1)];
                        ms1 = a.msg_scale[m0 + 8 * bq + 4 * kh + 2 + (i & 1)];
                    }
                    if constexpr (BF16) {
                        const uint32_t k0 = pack_bf16x2(p0[0], p1[0]), k1 = pack_bf16x2(p0[1], p1[1]);
                        const uint32_t got = (uint32_t)__shfl_xor((int)(hi ? k0 : k1), 2, kWave);
                        uint2 o;
                        o.x = hi ? got : k0;   // lanes with bit1 clear keep pair 0 (their row), receive columns +2,+3
                        o.y = hi ? k1 : got;
                        *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.out) + off) = o;
                        if constexpr (MSG) {
                            const uint32_t q0 = pack_bf16x2(p0[0] * ms0, p1[0] * ms0), q1 = pack_bf16x2(p0[1] * ms1, p1[1] * ms1);
                            const uint32_t gq = (uint32_t)__shfl_xor((int)(hi ? q0 : q1), 2, kWave);
                            uint2 m;
                            m.x = hi ? gq : q0;
                            m.y = hi ? q1 : gq;
                            *reinterpret_cast<uint2 *>(static_cast<uint16_t *>(a.msg_out) + off) = m;
                        }
                    } else {
                        const float g0 = __shfl_xor(hi ? p0[0] : p0[1], 2, kWave);
                        const float g1 = __shfl_xor(hi ? p1[0] : p1[1], 2, kWave);
                        float4 o;
                        o.x = hi ? g0 : p0[0];
                        o.y = hi ? g1 : p1[0];
                        o.z = hi ? p0[1] : g0;
                        o.w = hi ? p1[1] : g1;
                        *reinterpret_cast<float4 *>(static_cast<float *>(a.out) + off) = o;
                        if constexpr (MSG) {
                            const float ms = hi ? ms1 : ms0;  // this lane's final row is 8*bq + 4*kh + (i&3)
                            *reinterpret_cast<float4 *>(static_cast<float *>(a.msg_out) + off) =
                                make_float4(o.x * ms, o.y * ms, o.z * ms, o.w * ms);
                        }
                    }
                }
            }
        } else {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt) {
                const int col = col0 + nt * 32 + i;
                const bool col_ok = col < a.d_out;
                const float b = bias_v[nt];
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t orow = m0 + 8 * (r / 4) + 4 * kh + (r % 4);
                    float y = acc[nt][r] + b;
                    if constexpr (ADD) {
                        if (col_ok && orow < a.n) {
                            if constexpr (BF16) y += __uint_as_float((uint32_t)static_cast<const uint16_t *>(a.addend)[orow * a.d_out + col] << 16);
                            else y += static_cast<const float *>(a.addend)[orow * a.d_out + col];
                        }
                    }
                    if (a.act == ITB_ACT_RELU) y = fmaxf(y, 0.f);
                    if (col_ok && orow < a.n) {
                        if constexpr (BF16) {
                            static_cast<uint16_t *>(a.out)[orow * a.d_out + col] = (uint16_t)f32_to_bf16(y);
                            if constexpr (MSG)
                                static_cast<uint16_t *>(a.msg_out)[orow * a.d_out + col] = (uint16_t)f32_to_bf16(y * a.msg_scale[orow]);
                        } else {
                            static_cast<float *>(a.out)[orow * a.d_out + col] = y;
                            if constexpr (MSG) static_cast<float *>(a.msg_out)[orow * a.d_out + col] = y * a.msg_scale[orow];
                        }
                    }
                }
            }
        }
        if constexpr (SCORES) {
            // column i of the score tile: source score of head i, or destination score of head i - heads
            if (blockIdx.y == 0 && i < 2 * a.heads) {
                float *dst = i < a.heads ? a.s_src : a.s_dst;
                const int hd = i < a.heads ? i : i - a.heads;
#pragma unroll
                for (int r = 0; r < 16; ++r) {
                    const int64_t orow = m0 + 8 * (r / 4) + 4 * kh + (r % 4);
                    if (orow < a.n) dst[orow * a.heads + hd] = sacc[r];
                }
            }
        }
        rowoff = rowoff_next;
    }
}

template <bool BF16, int NT, int PF, bool SCORES, bool MSG, bool ADD>
int32_t launch_apply_cfg(const ApplyArgs &a, int n_cus, hipStream_t st) {
    constexpr int BN = 32 * NT;
    const int k_total = a.d_in * (a.h_self ? 2 : 1);
    const size_t lds = (size_t)k_total * (BN + (SCORES ? 32 * (BF16 ? 2 : 1) : 0)) * (BF16 ? 2 : 4);
    if (lds > kMaxLds) return ITB_ERR_UNSUPPORTED;
    static bool attr_set = false;
    if (!attr_set) {
        ITB_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&apply_kernel<BF16, NT, PF, SCORES, MSG, ADD>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLds));
        attr_set = true;
    }
    const int col_tiles = (a.d_out + BN - 1) / BN;
    int blocks_per_cu = (int)((160 * 1024) / (lds + 1024));
    if (blocks_per_cu < 1) blocks_per_cu = 1;
    if (blocks_per_cu > 2) blocks_per_cu = 2;
    int64_t gx = (int64_t)n_cus * blocks_per_cu / col_tiles;
    if (gx < 1) gx = 1;
    if (gx > a.n_row_tiles) gx = a.n_row_tiles;
    dim3 grid((unsigned)gx, (unsigned)col_tiles);
    apply_kernel<BF16, NT, PF, SCORES, MSG, ADD><<<grid, kApplyThreads, lds, st>>>(a);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

template <bool BF16, int NT, int PF, bool SCORES>
int32_t launch_apply_pf(const ApplyArgs &a, int n_cus, hipStream_t st) {
    if constexpr (!SCORES) {
        if (a.msg_out && a.addend) return launch_apply_cfg<BF16, NT, PF, false, true, true>(a, n_cus, st);
        if (a.msg_out) return launch_apply_cfg<BF16, NT, PF, false, true, false>(a, n_cus, st);
        if (a.addend) return launch_apply_cfg<BF16, NT, PF, false, false, true>(a, n_cus, st);
    }
    return launch_apply_cfg<BF16, NT, PF, SCORES, false, false>(a, n_cus, st);
}

template <bool BF16, int NT>
int32_t launch_apply(const ApplyArgs &a, int n_cus, hipStream_t st) {
    const int total = (a.d_in / (BF16 ? 16 : 8)) * (a.h_self ? 2 : 1);
    if (a.heads > 0) {
        if (total % 4 == 0) return launch_apply_pf<BF16, NT, 4, true>(a, n_cus, st);
        if (total % 2 == 0) return launch_apply_pf<BF16, NT, 2, true>(a, n_cus, st);
        return launch_apply_pf<BF16, NT, 1, true>(a, n_cus, st);
    }
    if (total % 8 == 0) return launch_apply_pf<BF16, NT, 8, false>(a, n_cus, st);
    if (total % 4 == 0) return launch_apply_pf<BF16, NT, 4, false>(a, n_cus, st);
    if (total % 2 == 0) return launch_apply_pf<BF16, NT, 2, false>(a, n_cus, st);
    return launch_apply_pf<BF16, NT, 1, false>(a, n_cus, st);
}

template <bool BF16>
int32_t dispatch_apply(const ApplyArgs &a, int n_cus, hipStream_t st) {
    const int k_total = a.d_in * (a.h_self ? 2 : 1);
    const size_t per_tile = (size_t)k_total * 32 * (BF16 ? 2 : 4);
    int nt = 4;  // 8 accumulator tiles per wave would not leave registers for the prefetch buffers
    while (nt > 1 && (per_tile * nt > kMaxWeightLds || 32 * (nt / 2) >= a.d_out)) nt /= 2;
    if (per_tile * nt > kMaxWeightLds) return ITB_ERR_UNSUPPORTED;
    if (a.heads > 0) {  // leave room for the score panel
        const size_t score = (size_t)k_total * 32 * (BF16 ? 4 : 4);
        while (nt > 1 && per_tile * nt + score > kMaxLds) nt /= 2;
        if (per_tile * nt + score > kMaxLds) return ITB_ERR_UNSUPPORTED;
    }
    switch (nt) {
        case 4: return launch_apply<BF16, 4>(a, n_cus, st);
        case 2: return launch_apply<BF16, 2>(a, n_cus, st);
        default: return launch_apply<BF16, 1>(a, n_cus, st);
    }
}

int cached_cu_count() {
    static int cus = 0;
    if (cus == 0) {
        int dev = 0;
        hipDeviceProp_t prop;
        if (hipGetDevice(&dev) == hipSuccess && hipGetDeviceProperties(&prop, dev) == hipSuccess) cus = prop.multiProcessorCount;
        if (cus <= 0) cus = 256;
    }
    return cus;
}

}  // namespace

extern "C" int32_t apply_layer(const itb_apply_desc *desc, int64_t n_nodes, const void *h_self, const void *agg,
                               const void *w_self, const void *w_nbr, const float *bias, void *h_out, const float *att_src,
                               const float *att_dst, float *s_src, float *s_dst, const float *msg_scale, void *msg_out,
                               const void *addend, void *stream) {
    if (!desc) return ITB_ERR_NULL;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31)) return ITB_ERR_SIZE;
    if (desc->dtype != ITB_F32 && desc->dtype != ITB_BF16) return ITB_ERR_DTYPE;
    if (desc->act != ITB_ACT_NONE && desc->act != ITB_ACT_RELU) return ITB_ERR_DTYPE;
    if (desc->d_in <= 0 || desc->d_out <= 0) return ITB_ERR_SIZE;
    const int kc = desc->dtype == ITB_BF16 ? 16 : 8;
    if (desc->d_in % kc != 0 || desc->d_in > 512 || desc->d_out > 256) return ITB_ERR_UNSUPPORTED;
    if (desc->heads < 0) return ITB_ERR_SIZE;
    if (desc->heads == 0 && (att_src || att_dst || s_src || s_dst)) return ITB_ERR_SIZE;
    if (desc->heads > 0) {
        if (!att_src || !att_dst || !s_src || !s_dst) return ITB_ERR_NULL;
        if (desc->d_out % desc->heads != 0) return ITB_ERR_SIZE;
        if (desc->heads > 16 || h_self) return ITB_ERR_UNSUPPORTED;  // 2*heads score columns share one 32-column tile
    }
    if ((h_self == nullptr) != (w_self == nullptr)) return ITB_ERR_NULL;
    if ((msg_scale == nullptr) != (msg_out == nullptr)) return ITB_ERR_NULL;
    if ((msg_out || addend) && desc->heads > 0) return ITB_ERR_UNSUPPORTED;
    if (!w_nbr || (n_nodes > 0 && (!agg || !h_out))) return ITB_ERR_NULL;
    if (n_nodes == 0) return ITB_OK;

    ApplyArgs a{};
    a.n = n_nodes;
    a.h_self = static_cast<const uint4 *>(h_self);
    a.agg = static_cast<const uint4 *>(agg);
    a.w_self = w_self;
    a.w_nbr = w_nbr;
    a.bias = bias;
    a.out = h_out;
    a.d_in = desc->d_in;
    a.d_out = desc->d_out;
    a.act = desc->act;
    a.n_row_tiles = (n_nodes + kRowsPerBlockTile - 1) / kRowsPerBlockTile;
    a.heads = desc->heads;
    a.att_src = att_src;
    a.att_dst = att_dst;
    a.s_src = s_src;
    a.s_dst = s_dst;
    a.msg_scale = msg_scale;
    a.msg_out = msg_out;
    a.addend = addend;
    hipStream_t st = static_cast<hipStream_t>(stream);
    return desc->dtype == ITB_BF16 ? dispatch_apply<true>(a, cached_cu_count(), st)
                                   : dispatch_apply<false>(a, cached_cu_count(), st);
}
