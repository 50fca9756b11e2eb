// apply_layer: h_out = act([h_self | agg] . [W_self ; W_nbr] + bias (+ addend)) on the matrix cores.
//
// The weights are tiny (<= 256 KB) and the activations are a tall-skinny stream, so:
//   * each block is persistent: it loads the whole [K_total x BN] weight panel into LDS once, in the exact
//     fragment order of the MFMA B operand (one conflict-free 16-byte LDS read per lane per k-chunk), and
//     then walks over 32*waves-row tiles;
//   * every wavefront owns 32 rows and all BN = 32*NT output columns (NT independent 32x32 accumulators,
//     so consecutive MFMAs never wait on each other);
//   * rows travel global -> registers -> a per-wavefront LDS staging area -> A fragments, and the finished tile
//     goes back through the same area, so that every global access is a full 64-byte piece of one row;
//   * the k index inside a chunk is permuted identically for A and B (a dot product does not care), which lets
//     one 16-byte fragment feed 4 fp32 MFMAs (32x32x2) or 1 bf16 MFMA (32x32x16);
//   * bias, addend, activation, rounding, the store (the scatter of the new state) and the optional message rows
//     are fused into the epilogue.
#include "common.h"

namespace {
using namespace itb;

typedef float v16f __attribute__((ext_vector_type(16)));
typedef __bf16 v8bf __attribute__((ext_vector_type(8)));

constexpr int kApplyThreads = 512;
constexpr int kApplyWaves = kApplyThreads / kWave;
constexpr int kRowsPerBlockTile = 32 * kApplyWaves;
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
    // optional second product of the same rows: out2 = agg . w2 ([d_in x d_out], no bias, no activation).  The kernel
    // then runs over n_cols = 2 * d_out logical columns: column c < d_out belongs to (w_nbr, out), column c >= d_out
    // to (w2, out2) at c - d_out.
    const void *w2;
    void *out2;
    int32_t n_cols;
    // optional chained projection (bf16, d_out == 16 * PF so that a finished row tile is exactly one staging area): the
    // finished rows y = act(...), rounded to the storage type, are multiplied by [wc_first | wc_second] (each
    // [d_out x dc]) on the spot and stored to outc_first / outc_second ([n x dc]); `out` may then be NULL (y is never
    // written).  It is the next layer's projection h.[W_nbr | W_self] taken while h is still in the staging area.
    const void *wc_first, *wc_second;
    void *outc_first, *outc_second;
    int32_t dc;
};

// LDS weight panel: chunk kc (8 fp32 / 16 bf16 values of k), half kh, column j -> one uint4 holding the
// 4 (fp32) or 8 (bf16) consecutive-k weights W[kc*KC + kh*KC/2 + t][col0 + j].
// `chunks_per_phase` may exceed d_in / KC (the k range is padded to whole k-groups): weights of k >= d_in are zero.
template <bool BF16, int NT, bool DUAL>
__device__ __forceinline__ void load_weight_panel(uint4 *wlds, const ApplyArgs &a, int col0, int chunks_per_phase) {
    constexpr int BN = 32 * NT;
    constexpr int KC = BF16 ? 16 : 8;
    constexpr int KH = KC / 2;
    const int phases = a.h_self ? 2 : 1;
    const int total = phases * chunks_per_phase * 2 * BN;
#pragma unroll 4
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int j = idx % BN;
        const int kh = (idx / BN) & 1;
        const int kcg = idx / (2 * BN);
        const int phase = kcg / chunks_per_phase;
        const int kc = kcg % chunks_per_phase;
        const int lcol = col0 + j;                       // logical column
        const bool second = DUAL && lcol >= a.d_out;     // (only with a second product)
        const void *wbase = second ? a.w2 : ((phases == 2 && phase == 0) ? a.w_self : a.w_nbr);
        const int col = second ? lcol - a.d_out : lcol;
        const int k0 = kc * KC + kh * KH;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (lcol < a.n_cols) {
            if constexpr (BF16) {
                const uint16_t *w = static_cast<const uint16_t *>(wbase);
                uint32_t e[8];
#pragma unroll
                for (int t = 0; t < 8; ++t) e[t] = (k0 + t < a.d_in) ? w[(int64_t)(k0 + t) * a.d_out + col] : 0u;
                v.x = e[0] | (e[1] << 16);
                v.y = e[2] | (e[3] << 16);
                v.z = e[4] | (e[5] << 16);
                v.w = e[6] | (e[7] << 16);
            } else {
                const uint32_t *w = static_cast<const uint32_t *>(wbase);
                if (k0 < a.d_in) {  // d_in is a multiple of 4: a 4-value piece is whole or absent
                    v.x = w[(int64_t)(k0 + 0) * a.d_out + col];
                    v.y = w[(int64_t)(k0 + 1) * a.d_out + col];
                    v.z = w[(int64_t)(k0 + 2) * a.d_out + col];
                    v.w = w[(int64_t)(k0 + 3) * a.d_out + col];
                }
            }
        }
        wlds[idx] = v;
    }
}

// LDS panel of the chained projection (bf16): K = d_out of the first product, logical columns [0, dc) from wc_first,
// [dc, 2 dc) from wc_second, zero beyond; same fragment order as the main panel.
template <int NT>
__device__ __forceinline__ void load_chain_panel(uint4 *clds, const ApplyArgs &a) {
    constexpr int BN = 32 * NT;
    const int chunks = a.d_out / 16;
    const int total = chunks * 2 * BN;
    for (int idx = threadIdx.x; idx < total; idx += blockDim.x) {
        const int j = idx % BN;
        const int kh = (idx / BN) & 1;
        const int kc = idx / (2 * BN);
        const int k0 = kc * 16 + kh * 8;
        uint4 v = make_uint4(0, 0, 0, 0);
        if (j < 2 * a.dc) {
            const uint16_t *w = static_cast<const uint16_t *>(j < a.dc ? a.wc_first : a.wc_second);
            const int col = j < a.dc ? j : j - a.dc;
            uint32_t e[8];
#pragma unroll
            for (int t = 0; t < 8; ++t) e[t] = w[(int64_t)(k0 + t) * a.dc + col];
            v.x = e[0] | (e[1] << 16);
            v.y = e[2] | (e[3] << 16);
            v.z = e[4] | (e[5] << 16);
            v.w = e[6] | (e[7] << 16);
        }
        clds[idx] = v;
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
__device__ __forceinline__ void load_score_panel(uint4 *slds, const ApplyArgs &a, int chunks) {
    constexpr int KC = BF16 ? 16 : 8;
    constexpr int KH = KC / 2;
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
                    if (k0 + t < a.d_in) {  // padded k range: nothing beyond d_in
                        const int64_t wi = (int64_t)(k0 + t) * a.d_out + hd * dh + d;
                        float wv;
                        if constexpr (BF16) wv = __uint_as_float((uint32_t)static_cast<const uint16_t *>(a.w_nbr)[wi] << 16);
                        else wv = static_cast<const float *>(a.w_nbr)[wi];
                        u[t] = fmaf(wv, av, u[t]);
                    }
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
}

// ---------------------------------------------------------------------------------------------------------
// The fragment layout of the matrix cores puts 32 different rows into adjacent lanes, so loading
// A fragments (and storing C fragments) straight from/to global memory gives the vector cache one 16-byte (or
// 8-byte) access per lane: measured, this costs four times the cache accesses of row-contiguous traffic.  Here every
// wavefront owns a staging area in LDS: it loads its 32 rows x 32*PF bytes with 2*PF adjacent lanes on one
// row (full 64-byte accesses), writes them to LDS, and reads the fragments from there; the finished 32 x 32*NT
// tile goes back through the same area so that it leaves as row-contiguous 16-byte stores.  Staging is private
// to a wavefront (LDS operations of one wavefront execute in program order), so the row-tile loop needs no
// block-level synchronisation.  Loads run two k-groups ahead in registers.
// Staging layout for A: 16-byte unit (row r, piece c) at r*LPR + (c ^ swz(r)), LPR = 2*PF pieces per row,
// swz(r) = (r / (16/LPR)) % LPR: both the row-major writes and the column-wise fragment reads touch 64 distinct
// banks per 16 lanes.
template <int LPR>
__device__ __forceinline__ int stage_swz(int r) { return (r / (16 / LPR)) % LPR; }

// RAGGED: d_out is not a multiple of the 16-byte store width; the epilogue then stores element by element (a small
// loop, kept out of the vector variant because memory operations inside a loop of unknown length make the
// compiler's wait counts for the prefetched rows conservative).
// GTS > 0: the number of k-groups per row tile is this compile-time constant (even); the tile body is then one
// straight line of code and the wait counts for the rows in flight are exact.  GTS == 0: any number of groups.
// DUAL: a second product of the same rows (logical columns d_out .. 2 d_out - 1 belong to w2 / out2).
// CHAIN: the finished row tile is multiplied by a second weight panel before it leaves (ApplyArgs::wc_first).
// ESC: attention scores taken in the epilogue instead of by a score tile: the finished fp32 rows pass through the lanes
// row by row anyway, so a lane multiplies its piece of the row by the matching piece of att_src / att_dst, the lanes
// of one head add up by xor-shuffles, and heads wider than one epilogue pass carry their partial sum to the next pass.
// No score panel in LDS and no extra matrix instructions, which also leaves the registers for the straight-line tile
// body.  Needs a power-of-two head width that divides the block's column range.
template <bool BF16, int NT, int PF, bool SCORES, bool RAGGED, int GTS, bool DUAL, bool CHAIN = false, bool ESC = false>
__global__ __launch_bounds__(kApplyThreads) void apply_staged_kernel(ApplyArgs a) {
    static_assert(!CHAIN || (BF16 && !SCORES && !RAGGED && !DUAL), "the chained projection is built for plain bf16 updates");
    static_assert(!ESC || (!SCORES && !RAGGED && !DUAL && !CHAIN), "epilogue scores replace the score tile of a plain projection");
    constexpr int SPARTS = BF16 ? 2 : 1;
    constexpr int BN = 32 * NT;
    constexpr int KC = BF16 ? 16 : 8;
    constexpr int LPR = 2 * PF;              // lanes (16-byte pieces) per row and group
    constexpr int RPL = 64 / LPR;            // rows per load instruction
    constexpr int STG_VECS = (32 * LPR > 256) ? 32 * LPR : 256;  // per wavefront: the A group, at least 4 KB for the epilogue
    constexpr int ENT = STG_VECS / 256;      // 32-column tiles the epilogue stages at a time (fp32): 2 or 1
    constexpr int W = ENT * 32;              // dwords per staged output row
    constexpr int VE = BF16 ? 8 : 4;         // output elements per 16-byte store
    constexpr int UPL = VE / 4;              // 16-byte fp32 units a lane reads back
    constexpr int LPRO = (W / 4) / UPL;      // lanes per output row
    constexpr int RPI = 64 / LPRO;           // output rows per store instruction
    extern __shared__ uint4 wlds[];
    const int col0 = blockIdx.y * BN;
    // k range of a phase: d_in values = row_vecs 16-byte pieces per row, padded up to whole groups of PF chunks (the
    // padding reads as zeros on both operands)
    const int gpp = ((a.d_in + KC - 1) / KC + PF - 1) / PF;   // groups per phase
    const int chunks = gpp * PF;                                // padded chunks per phase
    const int phases = a.h_self ? 2 : 1;
    const int total = phases * chunks;
    load_weight_panel<BF16, NT, DUAL>(wlds, a, col0, chunks);
    uint4 *slds = wlds + (int64_t)total * 2 * BN;
    if constexpr (SCORES) load_score_panel<BF16>(slds, a, chunks);
    uint4 *clds = slds + (SCORES ? (int64_t)total * 64 * SPARTS : 0) + (int64_t)kApplyWaves * STG_VECS;  // behind the staging areas
    if constexpr (CHAIN) load_chain_panel<NT>(clds, a);
    float *attl = reinterpret_cast<float *>(clds);   // ESC: att_src then att_dst of this block's columns
    if constexpr (ESC) {
        for (int c = threadIdx.x; c < 2 * BN; c += blockDim.x) {
            const int col = col0 + (c % BN);
            const float *att = c < BN ? a.att_src : a.att_dst;
            attl[c] = col < a.d_out ? att[col] : 0.f;     // att is [heads x dh] = d_out consecutive values
        }
    }
    __syncthreads();

    const int lane = threadIdx.x & (kWave - 1);
    const int w = threadIdx.x / kWave;
    const int i = lane & 31;
    const int kh = lane >> 5;
    uint4 *stage = slds + (SCORES ? (int64_t)total * 64 * SPARTS : 0) + (int64_t)w * STG_VECS;
    uint32_t *stage32 = reinterpret_cast<uint32_t *>(stage);
    const int GT = GTS > 0 ? GTS : phases * gpp;  // groups per row tile
    const int64_t row_vecs = a.d_in / (KC / 2);    // 16-byte pieces of a stored row (2 * chunks unless the k range is padded)
    // (the variants with a compile-time group count are dispatched for unpadded k ranges only)
    const bool padded_k = GTS == 0 && (int64_t)2 * chunks != row_vecs;
    const uint4 *wbase = wlds + kh * BN + i;
    const uint4 *sbase = slds + kh * 32 + i;
    const int lr = lane / LPR, lc = lane % LPR;
    const int frag_swz = stage_swz<LPR>(i);

    float bias_v[NT];
#pragma unroll
    for (int nt = 0; nt < NT; ++nt) {
        const int col = col0 + nt * 32 + i;
        bias_v[nt] = (a.bias && col < a.d_out) ? a.bias[col] : 0.f;   // (the second product carries no bias)
    }

    // fetch cursor: the next group to request (runs two groups ahead of the compute cursor)
    int64_t f_tile = blockIdx.x;
    int f_g = 0;
    // Always issues its PF loads, so that the number of requests in flight at every point of the loop is the same
    // on every path and the compiler's wait counts stay exact (a conditional request made it wait for everything
    // outstanding).  Past the block's last tile the requests go to the first rows of `agg` (cache hits, never used).
    auto issue = [&](uint4(&R)[PF]) __attribute__((always_inline)) {
        const bool live = f_tile < a.n_row_tiles;
        const int phase = (f_g >= gpp) ? 1 : 0;
        const uint4 *base = (live && phases == 2 && phase == 0) ? a.h_self : a.agg;
        const int gi = live ? f_g - phase * gpp : 0;
        const int64_t row0 = live ? f_tile * kRowsPerBlockTile + (int64_t)w * 32 + lr : 0;
        // A piece of the padded k range past the row's end re-reads the row's last piece, so that the load needs no
        // predicate; stage_write replaces it by zeros (the zero weights it meets would cancel finite values only).
        int piece = gi * LPR + lc;
        piece = piece < (int)row_vecs ? piece : (int)row_vecs - 1;
#pragma unroll
        for (int q = 0; q < PF; ++q) {
            int64_t row = row0 + q * RPL;
            row = row < a.n ? row : a.n - 1;  // clamped rows are computed but never stored
            R[q] = base[row * row_vecs + piece];
        }
        if (++f_g == GT) {
            f_g = 0;
            f_tile += gridDim.x;
        }
    };
    v16f acc[NT];
    v16f sacc;
    int64_t tile = blockIdx.x;
    int g = 0;   // compute cursor: the group whose rows are written to the staging area and multiplied next

    auto stage_write = [&](const uint4(&R)[PF]) __attribute__((always_inline)) {
        if (padded_k) {  // uniform over the launch: pieces of group g beyond the row's width enter as zeros
            const int gi = (g >= gpp) ? g - gpp : g;
            const bool pad = gi * LPR + lc >= (int)row_vecs;
#pragma unroll
            for (int q = 0; q < PF; ++q) {
                const int r = q * RPL + lr;
                stage[r * LPR + (lc ^ stage_swz<LPR>(r))] = pad ? make_uint4(0, 0, 0, 0) : R[q];
            }
        } else {
#pragma unroll
            for (int q = 0; q < PF; ++q) {
                const int r = q * RPL + lr;
                stage[r * LPR + (lc ^ stage_swz<LPR>(r))] = R[q];
            }
        }
    };

    auto compute = [&]() __attribute__((always_inline)) {
        const int cb = g * PF;
        uint4 av = stage[i * LPR + (kh ^ frag_swz)];
        uint4 bv[NT];
#pragma unroll
        for (int nt = 0; nt < NT; ++nt) bv[nt] = wbase[(int64_t)cb * 2 * BN + nt * 32];
        uint4 sv[SCORES ? SPARTS : 1];
        if constexpr (SCORES) {
#pragma unroll
            for (int q = 0; q < SPARTS; ++q) sv[q] = sbase[(int64_t)q * total * 64 + (int64_t)cb * 64];
        }
#pragma unroll
        for (int p = 0; p < PF; ++p) {
            uint4 an = av;
            uint4 bn[NT];
            uint4 sn[SCORES ? SPARTS : 1];
            if (p + 1 < PF) {  // fragments of the next chunk, read under the current MFMAs
                an = stage[i * LPR + ((2 * (p + 1) + kh) ^ frag_swz)];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bn[nt] = wbase[(int64_t)(cb + p + 1) * 2 * BN + nt * 32];
                if constexpr (SCORES) {
#pragma unroll
                    for (int q = 0; q < SPARTS; ++q) sn[q] = sbase[(int64_t)q * total * 64 + (int64_t)(cb + p + 1) * 64];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            mfma_chunk<BF16, NT>(acc, av, bv);
            if constexpr (SCORES) {
#pragma unroll
                for (int q = 0; q < SPARTS; ++q) {
                    v16f one[1] = {sacc};
                    const uint4 bq[1] = {sv[q]};
                    mfma_chunk<BF16, 1>(one, av, bq);
                    sacc = one[0];
                }
            }
            __builtin_amdgcn_sched_barrier(0);
            if (p + 1 < PF) {
                av = an;
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bv[nt] = bn[nt];
                if constexpr (SCORES) {
#pragma unroll
                    for (int q = 0; q < SPARTS; ++q) sv[q] = sn[q];
                }
            }
        }
    };

    // Accumulator register r of a lane holds row 8*(r/4) + 4*kh + (r%4), column i of its 32-column tile.
    auto epilogue = [&]() __attribute__((always_inline)) {
        const int64_t m0 = tile * kRowsPerBlockTile + (int64_t)w * 32;
        // CHAIN: the finished rows of this wavefront's tile, as the lanes hold them after the row-wise read-back
        // (one 16-byte piece = 8 bf16 columns of one row each)
        constexpr int YK = CHAIN ? ((NT + ENT - 1) / ENT) * (32 / RPI) : 1;
        uint4 yk[YK];
        // ESC: running score sums of the rows this lane reads back (one per read-back step), carried across passes
        float esc_s[ESC ? 32 / RPI : 1], esc_d[ESC ? 32 / RPI : 1];
        if constexpr (ESC) {
#pragma unroll
            for (int t = 0; t < 32 / RPI; ++t) esc_s[t] = esc_d[t] = 0.f;
        }
#pragma unroll
        for (int nt0 = 0; nt0 < NT; nt0 += ENT) {
            const int npass = (NT - nt0 < ENT) ? NT - nt0 : ENT;
            // fp32 tile (+bias) into the staging area; rows 4 apart (kh = 0 / 1) are kept in different bank halves:
            // with two tiles per row by flipping the tile half, with one tile per row by swapping the row pair
#pragma unroll
            for (int e = 0; e < ENT; ++e) {
                if (e < npass) {
                    const int nt = nt0 + e;
#pragma unroll
                    for (int r = 0; r < 16; ++r) {
                        const int rho = 8 * (r / 4) + 4 * kh + (r % 4);
                        const int col = e * 32 + i;
                        const int unit = (ENT == 2) ? ((col >> 2) ^ (kh * 8)) : (col >> 2);
                        const int slot = (ENT == 2) ? rho : (rho ^ kh);
                        stage32[slot * W + unit * 4 + (col & 3)] = __float_as_uint(acc[nt][r] + bias_v[nt]);
                    }
                }
            }
            // back as rows: a lane takes VE consecutive columns of one row
#pragma unroll
            for (int t = 0; t < 32 / RPI; ++t) {
                const int rho = t * RPI + lane / LPRO;
                const int u0 = (lane % LPRO) * UPL;
                const int khr = (rho >> 2) & 1;
                const int slot = (ENT == 2) ? rho : (rho ^ khr);
                const int uswz = (ENT == 2) ? khr * 8 : 0;
                float v[VE];
#pragma unroll
                for (int j = 0; j < UPL; ++j) {
                    const uint4 x = stage[(slot * W) / 4 + ((u0 + j) ^ uswz)];
                    v[4 * j + 0] = __uint_as_float(x.x);
                    v[4 * j + 1] = __uint_as_float(x.y);
                    v[4 * j + 2] = __uint_as_float(x.z);
                    v[4 * j + 3] = __uint_as_float(x.w);
                }
                const int64_t row = m0 + rho;
                const int col = col0 + nt0 * 32 + u0 * 4;
                if constexpr (CHAIN) yk[(nt0 / ENT) * (32 / RPI) + t] = make_uint4(0, 0, 0, 0);
                if constexpr (ESC) {
                    const int dh = a.d_out / a.heads;
                    const int cl = nt0 * 32 + u0 * 4;                 // column inside the block
                    float ps = 0.f, pd = 0.f;
                    if (u0 * 4 < npass * 32) {                         // (att is zero beyond d_out)
#pragma unroll
                        for (int e = 0; e < VE; ++e) {
                            ps = fmaf(v[e], attl[cl + e], ps);
                            pd = fmaf(v[e], attl[BN + cl + e], pd);
                        }
                    }
                    const int lanes_per_head = dh / VE < LPRO ? dh / VE : LPRO;   // of this pass; a power of two
                    for (int off = 1; off < lanes_per_head; off <<= 1) {
                        ps += __shfl_xor(ps, off, kWave);
                        pd += __shfl_xor(pd, off, kWave);
                    }
                    esc_s[t] += ps;
                    esc_d[t] += pd;
                    const int pass_end = col0 + nt0 * 32 + npass * 32;   // first column after this pass
                    const bool head_done = dh <= npass * 32 || pass_end % dh == 0;
                    if (head_done) {
                        if ((lane % LPRO) % lanes_per_head == 0 && row < a.n && col < a.d_out && u0 * 4 < npass * 32) {
                            const int k = col / dh;
                            a.s_src[row * a.heads + k] = esc_s[t];
                            a.s_dst[row * a.heads + k] = esc_d[t];
                        }
                        esc_s[t] = esc_d[t] = 0.f;
                    }
                }
                if (DUAL && row < a.n && u0 * 4 < npass * 32 && col >= a.d_out && col < a.n_cols) {
                    // the second product: plain rows of out2 (d_out is a multiple of the vector width here)
                    const int64_t off = row * a.d_out + (col - a.d_out);
                    if constexpr (BF16)
                        *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.out2) + off) =
                            make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                    else
                        *reinterpret_cast<float4 *>(static_cast<float *>(a.out2) + off) = make_float4(v[0], v[1], v[2], v[3]);
                } else if (row < a.n && u0 * 4 < npass * 32 && col < a.d_out) {
                    const int64_t off = row * a.d_out + col;
                    const float ms = a.msg_out ? a.msg_scale[row] : 0.f;
                    if constexpr (!RAGGED) {  // d_out % VE == 0: every vector is whole and 16-byte aligned
                        if (a.addend) {
                            if constexpr (BF16) {
                                const uint4 ad = *reinterpret_cast<const uint4 *>(static_cast<const uint16_t *>(a.addend) + off);
                                v[0] += bf16_lo(ad.x); v[1] += bf16_hi(ad.x); v[2] += bf16_lo(ad.y); v[3] += bf16_hi(ad.y);
                                v[4] += bf16_lo(ad.z); v[5] += bf16_hi(ad.z); v[6] += bf16_lo(ad.w); v[7] += bf16_hi(ad.w);
                            } else {
                                const float4 ad = *reinterpret_cast<const float4 *>(static_cast<const float *>(a.addend) + off);
                                v[0] += ad.x; v[1] += ad.y; v[2] += ad.z; v[3] += ad.w;
                            }
                        }
                        if (a.act == ITB_ACT_RELU) {
#pragma unroll
                            for (int e = 0; e < VE; ++e) v[e] = fmaxf(v[e], 0.f);
                        }
                        if constexpr (BF16) {
                            const uint4 pk =
                                make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                            if constexpr (CHAIN) {
                                yk[(nt0 / ENT) * (32 / RPI) + t] = pk;
                                if (a.out) *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.out) + off) = pk;
                            } else {
                                *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.out) + off) = pk;
                            }
                            if (a.msg_out)
                                *reinterpret_cast<uint4 *>(static_cast<uint16_t *>(a.msg_out) + off) =
                                    make_uint4(pack_bf16x2(v[0] * ms, v[1] * ms), pack_bf16x2(v[2] * ms, v[3] * ms),
                                               pack_bf16x2(v[4] * ms, v[5] * ms), pack_bf16x2(v[6] * ms, v[7] * ms));
                        } else {
                            *reinterpret_cast<float4 *>(static_cast<float *>(a.out) + off) = make_float4(v[0], v[1], v[2], v[3]);
                            if (a.msg_out)
                                *reinterpret_cast<float4 *>(static_cast<float *>(a.msg_out) + off) =
                                    make_float4(v[0] * ms, v[1] * ms, v[2] * ms, v[3] * ms);
                        }
                    } else {
                        // element by element, read again from the staging area so that the path stays a small loop
#pragma unroll 1
                        for (int e = 0; e < VE; ++e) {
                            if (col + e < a.d_out) {
                                float y = __uint_as_float(stage32[slot * W + ((u0 + e / 4) ^ uswz) * 4 + (e & 3)]);
                                if (a.addend) {
                                    if constexpr (BF16) y += __uint_as_float((uint32_t)static_cast<const uint16_t *>(a.addend)[off + e] << 16);
                                    else y += static_cast<const float *>(a.addend)[off + e];
                                }
                                if (a.act == ITB_ACT_RELU) y = fmaxf(y, 0.f);
                                if constexpr (BF16) {
                                    static_cast<uint16_t *>(a.out)[off + e] = (uint16_t)f32_to_bf16(y);
                                    if (a.msg_out) static_cast<uint16_t *>(a.msg_out)[off + e] = (uint16_t)f32_to_bf16(y * ms);
                                } else {
                                    static_cast<float *>(a.out)[off + e] = y;
                                    if (a.msg_out) static_cast<float *>(a.msg_out)[off + e] = y * ms;
                                }
                            }
                        }
                    }
                }
            }
        }
        if constexpr (CHAIN) {
            // The row tile y [32 x d_out] (d_out == 8 * LPR columns: LPR pieces per row) goes back into the staging area
            // in the layout the A fragments are read from, is multiplied by the chained panel (PF chunks of 16 k) and
            // leaves through the staging area once more, as rows of outc_first / outc_second.
            static_assert(UPL == 2, "a lane holds one 8-column piece per read-back");
#pragma unroll
            for (int p = 0; p < (NT + ENT - 1) / ENT; ++p) {
#pragma unroll
                for (int t = 0; t < 32 / RPI; ++t) {
                    const int rho = t * RPI + lane / LPRO;
                    const int piece = p * ENT * 4 + lane % LPRO;      // 8 columns per piece, 4 pieces per 32-column tile
                    if (piece < LPR) stage[rho * LPR + (piece ^ stage_swz<LPR>(rho))] = yk[p * (32 / RPI) + t];
                }
            }
            v16f acc2[NT];
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc2[nt][r] = 0.f;
            const uint4 *cbase = clds + kh * BN + i;
#pragma unroll
            for (int c2 = 0; c2 < PF; ++c2) {
                const uint4 av = stage[i * LPR + ((2 * c2 + kh) ^ frag_swz)];
                uint4 bv[NT];
#pragma unroll
                for (int nt = 0; nt < NT; ++nt) bv[nt] = cbase[(int64_t)c2 * 2 * BN + nt * 32];
                mfma_chunk<true, NT>(acc2, av, bv);
            }
#pragma unroll
            for (int nt0 = 0; nt0 < NT; nt0 += ENT) {
                const int npass = (NT - nt0 < ENT) ? NT - nt0 : ENT;
#pragma unroll
                for (int e = 0; e < ENT; ++e) {
                    if (e < npass) {
                        const int nt = nt0 + e;
#pragma unroll
                        for (int r = 0; r < 16; ++r) {
                            const int rho = 8 * (r / 4) + 4 * kh + (r % 4);
                            const int col = e * 32 + i;
                            const int unit = (ENT == 2) ? ((col >> 2) ^ (kh * 8)) : (col >> 2);
                            const int slot = (ENT == 2) ? rho : (rho ^ kh);
                            stage32[slot * W + unit * 4 + (col & 3)] = __float_as_uint(acc2[nt][r]);
                        }
                    }
                }
#pragma unroll
                for (int t = 0; t < 32 / RPI; ++t) {
                    const int rho = t * RPI + lane / LPRO;
                    const int u0 = (lane % LPRO) * UPL;
                    const int khr = (rho >> 2) & 1;
                    const int slot = (ENT == 2) ? rho : (rho ^ khr);
                    const int uswz = (ENT == 2) ? khr * 8 : 0;
                    float v[8];
#pragma unroll
                    for (int j = 0; j < UPL; ++j) {
                        const uint4 x = stage[(slot * W) / 4 + ((u0 + j) ^ uswz)];
                        v[4 * j + 0] = __uint_as_float(x.x);
                        v[4 * j + 1] = __uint_as_float(x.y);
                        v[4 * j + 2] = __uint_as_float(x.z);
                        v[4 * j + 3] = __uint_as_float(x.w);
                    }
                    const int64_t row = m0 + rho;
                    const int col = nt0 * 32 + u0 * 4;   // logical column of the chained product (dc is a multiple of 8)
                    if (row < a.n && u0 * 4 < npass * 32 && col < 2 * a.dc) {
                        uint16_t *dst = static_cast<uint16_t *>(col < a.dc ? a.outc_first : a.outc_second);
                        const int64_t off = row * a.dc + (col < a.dc ? col : col - a.dc);
                        *reinterpret_cast<uint4 *>(dst + off) =
                            make_uint4(pack_bf16x2(v[0], v[1]), pack_bf16x2(v[2], v[3]), pack_bf16x2(v[4], v[5]), pack_bf16x2(v[6], v[7]));
                    }
                }
            }
        }
        if constexpr (SCORES) {
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
    };

    auto item = [&](uint4(&R)[PF]) __attribute__((always_inline)) {
        stage_write(R);   // this group's rows (requested two groups ago) into the staging area
        __builtin_amdgcn_sched_barrier(0);
        issue(R);         // and its registers carry the request two groups ahead
        __builtin_amdgcn_sched_barrier(0);
        if (g == 0) {
#pragma unroll
            for (int nt = 0; nt < NT; ++nt)
#pragma unroll
                for (int r = 0; r < 16; ++r) acc[nt][r] = 0.f;
#pragma unroll
            for (int r = 0; r < 16; ++r) sacc[r] = 0.f;
        }
        compute();
        if (++g == GT) {
            epilogue();
            g = 0;
            tile += gridDim.x;
        }
    };

    if (tile >= a.n_row_tiles) return;
    uint4 R0[PF], R1[PF];
#pragma unroll
    for (int q = 0; q < PF; ++q) R0[q] = R1[q] = make_uint4(0, 0, 0, 0);
    // (the barriers keep the two request batches in program order: the wait counts assume R0's rows were asked
    // for before R1's)
    issue(R0);
    __builtin_amdgcn_sched_barrier(0);
    issue(R1);
    __builtin_amdgcn_sched_barrier(0);
    if constexpr (GTS > 0) {
        static_assert(GTS % 2 == 0, "static group count must be even");
        while (tile < a.n_row_tiles) {
#pragma unroll
            for (int gg = 0; gg < GTS; gg += 2) {
                g = gg;
                item(R0);
                g = gg + 1;
                item(R1);
            }
        }
    } else {
        while (tile < a.n_row_tiles) {
            item(R0);
            if (tile >= a.n_row_tiles) break;
            item(R1);
        }
    }
}

// chunks of KC values per phase, rounded up to whole groups of pf chunks
int padded_chunks(int d_in, int kc, int pf) { return ((d_in + kc - 1) / kc + pf - 1) / pf * pf; }

template <bool BF16, int NT, int PF, bool SCORES, bool RAGGED, int GTS, bool DUAL, bool CHAIN = false, bool ESC = false>
int32_t launch_staged_one(const ApplyArgs &a, int n_cus, hipStream_t st) {
    constexpr int BN = 32 * NT;
    constexpr size_t stage_bytes = (size_t)kApplyWaves * ((32 * 2 * PF > 256) ? 32 * 2 * PF : 256) * 16;
    constexpr int KC = BF16 ? 16 : 8;
    const int k_total = padded_chunks(a.d_in, KC, PF) * KC * (a.h_self ? 2 : 1);
    const size_t chain_bytes = CHAIN ? (size_t)a.d_out * BN * 2 : (ESC ? (size_t)2 * BN * 4 : 0);   // [d_out x BN] bf16 / att pieces
    const size_t lds = (size_t)k_total * (BN + (SCORES ? 32 * (BF16 ? 2 : 1) : 0)) * (BF16 ? 2 : 4) + stage_bytes + chain_bytes;
    if (lds > kMaxLds) return ITB_ERR_UNSUPPORTED;
    // once per kernel variant (setting it again is harmless, so a race between two first callers is too)
    static std::atomic<bool> attr_set{false};
    if (!attr_set.load(std::memory_order_acquire)) {
        ITB_HIP(hipFuncSetAttribute(reinterpret_cast<const void *>(&apply_staged_kernel<BF16, NT, PF, SCORES, RAGGED, GTS, DUAL, CHAIN, ESC>),
                                    hipFuncAttributeMaxDynamicSharedMemorySize, (int)kMaxLds));
        attr_set.store(true, std::memory_order_release);
    }
    const int col_tiles = (a.n_cols + BN - 1) / BN;
    int blocks_per_cu = (int)((160 * 1024) / (lds + 1024));
    if (blocks_per_cu < 1) blocks_per_cu = 1;
    if (blocks_per_cu > 2) blocks_per_cu = 2;
    int64_t gx = (int64_t)n_cus * blocks_per_cu / col_tiles;
    if (gx < 1) gx = 1;
    if (gx > a.n_row_tiles) gx = a.n_row_tiles;
    dim3 grid((unsigned)gx, (unsigned)col_tiles);
    apply_staged_kernel<BF16, NT, PF, SCORES, RAGGED, GTS, DUAL, CHAIN, ESC><<<grid, kApplyThreads, lds, st>>>(a);
    ITB_LAUNCH_CHECK();
    return ITB_OK;
}

// (the second product exists for whole-vector output rows without score columns only)
template <bool BF16, int NT, int PF, bool SCORES, bool RAGGED, int GTS = 0>
int32_t launch_staged_cfg(const ApplyArgs &a, int n_cus, hipStream_t st) {
    if constexpr (!SCORES && !RAGGED) {
        if (a.w2) return launch_staged_one<BF16, NT, PF, SCORES, RAGGED, GTS, true>(a, n_cus, st);
    }
    return launch_staged_one<BF16, NT, PF, SCORES, RAGGED, GTS, false>(a, n_cus, st);
}

// Widest column tile first (fewer re-reads of A), then the largest k-group whose staging still fits the LDS.
template <bool BF16, bool SCORES>
int32_t dispatch_staged(const ApplyArgs &a, int n_cus, hipStream_t st) {
    constexpr int KC = BF16 ? 16 : 8;
    const int phases = a.h_self ? 2 : 1;
    const size_t esz = BF16 ? 2 : 4;
    const int real_chunks = (a.d_in + KC - 1) / KC;
    const bool ragged = a.d_out % (BF16 ? 8 : 4) != 0;
    for (int nt = 4; nt >= 1; nt /= 2) {
        if (nt > 1 && 32 * (nt / 2) >= a.n_cols) continue;  // narrower tile already covers every column
        // LDS of a configuration: weight panel (+ score panel) over the padded k range, plus the staging areas
        auto fits = [&](int pf) {
            const int chunks = padded_chunks(a.d_in, KC, pf);
            if (pf > 1 && 4 * (chunks - real_chunks) > real_chunks) return false;  // more than 25 % padding: smaller groups
            const size_t k_total = (size_t)chunks * KC * phases;
            const size_t panel = k_total * 32 * nt * esz + (SCORES ? k_total * 32 * (BF16 ? 2 : 1) * esz : 0);
            const size_t stage = (size_t)kApplyWaves * ((64 * pf > 256) ? 64 * pf : 256) * 16;
            return panel + stage <= kMaxLds;
        };
        if (ragged) {  // rare widths: one instantiation per tile width, smallest k-group
            if (!fits(1)) continue;
            if (nt == 4) return launch_staged_cfg<BF16, 4, 1, SCORES, true>(a, n_cus, st);
            if (nt == 2) return launch_staged_cfg<BF16, 2, 1, SCORES, true>(a, n_cus, st);
            return launch_staged_cfg<BF16, 1, 1, SCORES, true>(a, n_cus, st);
        }
        // First choice: a k-group size (8 or 4 chunks) that cuts the row tile into 2, 4, 8 or 16 groups -- those have
        // variants with a compile-time group count (straight-line tile body, exact wait counts; measured 1.5-2x on
        // shapes whose run-time variant waits for every outstanding request at the loop head).
        if constexpr (!SCORES) {  // (with the score tile the straight-line body runs out of registers; so does the widest
                                  // bf16 tile with a second product)
            if (nt >= 2 && !(BF16 && nt == 4 && a.w2)) {
                for (int pf = 8; pf >= 4; pf /= 2) {
                    if (!fits(pf)) continue;
                    if (padded_chunks(a.d_in, KC, pf) != real_chunks || a.d_in % KC != 0) continue;  // padded k range: run-time variant
                    const int gt = (padded_chunks(a.d_in, KC, pf) / pf) * phases;
#define ITB_STATIC_CASE(NT_, PF_, GT_) \
    if (nt == NT_ && pf == PF_ && gt == GT_) return launch_staged_cfg<BF16, NT_, PF_, false, false, GT_>(a, n_cus, st);
                    ITB_STATIC_CASE(4, 8, 2) ITB_STATIC_CASE(4, 8, 4) ITB_STATIC_CASE(4, 8, 8) ITB_STATIC_CASE(4, 8, 16)
                    ITB_STATIC_CASE(4, 4, 2) ITB_STATIC_CASE(4, 4, 4) ITB_STATIC_CASE(4, 4, 8) ITB_STATIC_CASE(4, 4, 16)
                    ITB_STATIC_CASE(2, 8, 2) ITB_STATIC_CASE(2, 8, 4) ITB_STATIC_CASE(2, 8, 8) ITB_STATIC_CASE(2, 8, 16)
                    ITB_STATIC_CASE(2, 4, 2) ITB_STATIC_CASE(2, 4, 4) ITB_STATIC_CASE(2, 4, 8) ITB_STATIC_CASE(2, 4, 16)
#undef ITB_STATIC_CASE
                }
            }
        }
        for (int pf = 8; pf >= 1; pf /= 2) {
            if (!fits(pf)) continue;
#define ITB_STAGED_CASE(NT_, PF_) \
    if (nt == NT_ && pf == PF_) return launch_staged_cfg<BF16, NT_, PF_, SCORES, false>(a, n_cus, st);
            ITB_STAGED_CASE(4, 8) ITB_STAGED_CASE(4, 4) ITB_STAGED_CASE(4, 2) ITB_STAGED_CASE(4, 1)
            ITB_STAGED_CASE(2, 8) ITB_STAGED_CASE(2, 4) ITB_STAGED_CASE(2, 2) ITB_STAGED_CASE(2, 1)
            ITB_STAGED_CASE(1, 8) ITB_STAGED_CASE(1, 4) ITB_STAGED_CASE(1, 2) ITB_STAGED_CASE(1, 1)
#undef ITB_STAGED_CASE
        }
    }
    return ITB_ERR_UNSUPPORTED;
}

// Projection with attention scores taken in the epilogue: no score panel, so the shapes that have a straight-line
// variant keep it.  Column tile of 128 (or the narrowest that covers d_out); returns ITB_ERR_UNSUPPORTED when the
// caller should fall back to the score-tile variant.
template <bool BF16>
int32_t dispatch_epilogue_scores(const ApplyArgs &a, int n_cus, hipStream_t st) {
    constexpr int KC = BF16 ? 16 : 8;
    constexpr int VE = BF16 ? 8 : 4;
    const int want = g_tuning.epilogue_scores.load();   // A/B switch 10: 0 never, 1 by shape, 2 whenever possible
    if (a.bias || a.h_self || a.heads <= 0 || a.d_out % a.heads != 0 || a.d_out % VE != 0 || want == 0) return ITB_ERR_UNSUPPORTED;
    // The epilogue work is fixed per row tile, the score tile costs two matrix instructions per 16 values of k: measured
    // (bf16, 4 heads, 2e6 rows) 256 -> 256: 0.61 ms against 0.77 ms with the score tile; 128 -> 128: 0.33 against 0.30.
    if (want == 1 && a.d_in < 256) return ITB_ERR_UNSUPPORTED;
    const int dh = a.d_out / a.heads;
    if (dh < VE || (dh & (dh - 1)) != 0) return ITB_ERR_UNSUPPORTED;      // power-of-two head width, whole pieces
    const int nt = a.d_out > 64 ? 4 : (a.d_out > 32 ? 2 : 1);
    if ((32 * nt) % dh != 0) return ITB_ERR_UNSUPPORTED;                    // a head must not straddle column blocks
    const int real_chunks = (a.d_in + KC - 1) / KC;
    const size_t esz = BF16 ? 2 : 4;
    auto fits = [&](int pf) {
        const int chunks = padded_chunks(a.d_in, KC, pf);
        if (pf > 1 && 4 * (chunks - real_chunks) > real_chunks) return false;
        const size_t panel = (size_t)chunks * KC * 32 * nt * esz;
        const size_t stage = (size_t)kApplyWaves * ((64 * pf > 256) ? 64 * pf : 256) * 16;
        return panel + stage + (size_t)2 * 32 * nt * 4 <= kMaxLds;
    };
    if (nt == 4) {
        for (int pf = 8; pf >= 4; pf /= 2) {
            if (!fits(pf) || padded_chunks(a.d_in, KC, pf) != real_chunks || a.d_in % KC != 0) continue;
            const int gt = real_chunks / pf;
#define ITB_ESC_STATIC(PF_, GT_) \
    if (pf == PF_ && gt == GT_) return launch_staged_one<BF16, 4, PF_, false, false, GT_, false, false, true>(a, n_cus, st);
            ITB_ESC_STATIC(8, 2) ITB_ESC_STATIC(8, 4) ITB_ESC_STATIC(8, 8) ITB_ESC_STATIC(4, 2) ITB_ESC_STATIC(4, 4) ITB_ESC_STATIC(4, 8)
#undef ITB_ESC_STATIC
        }
    }
    for (int pf = 8; pf >= 1; pf /= 2) {
        if (pf == 2 || !fits(pf)) continue;
#define ITB_ESC_CASE(NT_, PF_) \
    if (nt == NT_ && pf == PF_) return launch_staged_one<BF16, NT_, PF_, false, false, 0, false, false, true>(a, n_cus, st);
        ITB_ESC_CASE(4, 8) ITB_ESC_CASE(4, 4) ITB_ESC_CASE(4, 1) ITB_ESC_CASE(2, 8) ITB_ESC_CASE(2, 4) ITB_ESC_CASE(2, 1)
        ITB_ESC_CASE(1, 8) ITB_ESC_CASE(1, 4) ITB_ESC_CASE(1, 1)
#undef ITB_ESC_CASE
    }
    return ITB_ERR_UNSUPPORTED;
}

// The chained projection: bf16, a finished row tile of exactly one staging area.  Built for 64 output columns (two
// 32-column tiles, k-groups of 4 chunks); the k range of the first product must be whole groups.
constexpr int kChainWidth = 64;
size_t chain_lds_bytes(int d_in, bool has_self) {
    return (size_t)d_in * (has_self ? 2 : 1) * kChainWidth * 2 + (size_t)kApplyWaves * 256 * 16 + (size_t)kChainWidth * kChainWidth * 2;
}
int32_t dispatch_chain(const ApplyArgs &a, int n_cus, hipStream_t st) {
    if (a.d_out != kChainWidth || a.d_in % 64 != 0 || chain_lds_bytes(a.d_in, a.h_self != nullptr) > kMaxLds) return ITB_ERR_UNSUPPORTED;
    const int gt = (a.d_in / 64) * (a.h_self ? 2 : 1);
    if (gt == 2) return launch_staged_one<true, 2, 4, false, false, 2, false, true>(a, n_cus, st);
    if (gt == 4) return launch_staged_one<true, 2, 4, false, false, 4, false, true>(a, n_cus, st);
    if (gt == 8) return launch_staged_one<true, 2, 4, false, false, 8, false, true>(a, n_cus, st);
    return launch_staged_one<true, 2, 4, false, false, 0, false, true>(a, n_cus, st);
}

}  // namespace

namespace itb {
// Whether apply_layer takes a chained projection for this shape (the same conditions as its argument checks).
bool apply_chain_supported(int32_t dtype, int32_t d_in, int32_t d_out, bool has_self, int32_t dc) {
    return dtype == ITB_BF16 && d_out == kChainWidth && d_in > 0 && d_in % 64 == 0 && dc > 0 && dc % 8 == 0 && 2 * dc <= kChainWidth &&
           chain_lds_bytes(d_in, has_self) <= kMaxLds;
}

// Whether some configuration of the update kernel holds this shape in LDS (the same walk as dispatch_staged): lets
// the layer loop refuse a model before it has enqueued anything.
bool apply_shape_supported(int32_t dtype, int32_t d_in, int32_t d_out, bool has_self, int32_t heads) {
    const bool bf16 = dtype == ITB_BF16;
    const int kc = bf16 ? 16 : 8;
    if (d_in <= 0 || d_out <= 0 || d_in % (kc / 2) != 0) return false;
    if (heads > 0 && (has_self || heads > 16 || d_out % heads != 0)) return false;
    const size_t esz = bf16 ? 2 : 4;
    const int phases = has_self ? 2 : 1;
    const int real_chunks = (d_in + kc - 1) / kc;
    const bool ragged = d_out % (bf16 ? 8 : 4) != 0;
    for (int nt = 4; nt >= 1; nt /= 2) {
        if (nt > 1 && 32 * (nt / 2) >= d_out) continue;
        for (int pf = ragged ? 1 : 8; pf >= 1; pf /= 2) {
            const int chunks = padded_chunks(d_in, kc, pf);
            if (pf > 1 && 4 * (chunks - real_chunks) > real_chunks) continue;
            const size_t k_total = (size_t)chunks * kc * phases;
            const size_t panel = k_total * 32 * nt * esz + (heads > 0 ? k_total * 32 * (bf16 ? 2 : 1) * esz : 0);
            const size_t stage = (size_t)kApplyWaves * ((64 * pf > 256) ? 64 * pf : 256) * 16;
            if (panel + stage <= kMaxLds) return true;
        }
    }
    return false;
}
}  // namespace itb

namespace {
using namespace itb;

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
                               const void *addend, const void *w_second, void *out_second, const itb_apply_chain *chain,
                               void *stream) {
    if (!desc) return ITB_ERR_NULL;
    if (n_nodes < 0 || n_nodes >= ((int64_t)1 << 31)) return ITB_ERR_SIZE;
    if (desc->dtype != ITB_F32 && desc->dtype != ITB_BF16) return ITB_ERR_DTYPE;
    if (desc->act != ITB_ACT_NONE && desc->act != ITB_ACT_RELU) return ITB_ERR_DTYPE;
    if (desc->d_in <= 0 || desc->d_out <= 0) return ITB_ERR_SIZE;
    const int piece = desc->dtype == ITB_BF16 ? 8 : 4;  // elements of one 16-byte piece of a row
    if (desc->d_in % piece != 0) return ITB_ERR_UNSUPPORTED;  // rows are read as 16-byte pieces
    if (desc->heads < 0) return ITB_ERR_SIZE;
    if (n_nodes == 0) return ITB_OK;  // nothing to read or write: the per-vertex pointers may all be NULL
    if (desc->heads == 0 && (att_src || att_dst || s_src || s_dst)) return ITB_ERR_SIZE;
    if (desc->heads > 0) {
        if (!att_src || !att_dst || !s_src || !s_dst) return ITB_ERR_NULL;
        if (desc->d_out % desc->heads != 0) return ITB_ERR_SIZE;
        if (desc->heads > 16 || h_self) return ITB_ERR_UNSUPPORTED;  // 2*heads score columns share one 32-column tile
    }
    if ((h_self == nullptr) != (w_self == nullptr)) return ITB_ERR_NULL;
    if ((msg_scale == nullptr) != (msg_out == nullptr)) return ITB_ERR_NULL;
    if ((msg_out || addend) && desc->heads > 0) return ITB_ERR_UNSUPPORTED;
    if ((w_second == nullptr) != (out_second == nullptr)) return ITB_ERR_NULL;
    // the second product shares the rows of `agg`: no self term, no score columns, whole 16-byte vectors per row
    if (w_second && (h_self || desc->heads > 0 || desc->d_out % piece != 0)) return ITB_ERR_UNSUPPORTED;
    if (chain) {
        if (!chain->w_first || !chain->w_second || !chain->out_first || !chain->out_second) return ITB_ERR_NULL;
        if (desc->heads > 0 || w_second || msg_out || desc->d_out % piece != 0 ||
            !itb::apply_chain_supported(desc->dtype, desc->d_in, desc->d_out, h_self != nullptr, chain->dc))
            return ITB_ERR_UNSUPPORTED;
        if (!aligned16(chain->out_first) || !aligned16(chain->out_second)) return ITB_ERR_UNSUPPORTED;
    }
    if (!w_nbr || !agg || (!h_out && !chain)) return ITB_ERR_NULL;
    if (!aligned16(h_self) || !aligned16(agg) || !aligned16(h_out) || !aligned16(addend) || !aligned16(msg_out) ||
        !aligned16(out_second))
        return ITB_ERR_UNSUPPORTED;  // rows are moved as 16-byte vectors (a ragged d_out is stored element by element,
                                     // its base must still be aligned)

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
    a.w2 = w_second;
    a.out2 = out_second;
    a.n_cols = w_second ? 2 * desc->d_out : desc->d_out;
    hipStream_t st = static_cast<hipStream_t>(stream);
    const int cus = cached_cu_count();
    if (chain) {
        a.wc_first = chain->w_first;
        a.wc_second = chain->w_second;
        a.outc_first = chain->out_first;
        a.outc_second = chain->out_second;
        a.dc = chain->dc;
        return dispatch_chain(a, cus, st);
    }
    if (a.heads > 0 && aligned16(att_src) && aligned16(att_dst)) {
        // scores in the epilogue where the head width allows it, else by the score tile
        const int32_t rc = desc->dtype == ITB_BF16 ? dispatch_epilogue_scores<true>(a, cus, st) : dispatch_epilogue_scores<false>(a, cus, st);
        if (rc != ITB_ERR_UNSUPPORTED) return rc;
    }
    if (desc->dtype == ITB_BF16) return a.heads > 0 ? dispatch_staged<true, true>(a, cus, st) : dispatch_staged<true, false>(a, cus, st);
    return a.heads > 0 ? dispatch_staged<false, true>(a, cus, st) : dispatch_staged<false, false>(a, cus, st);
}
