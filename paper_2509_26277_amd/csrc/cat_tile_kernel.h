// MFMA tile kernel of the CAT hot path for gfx950: device code, kernel template and its launcher.
// Included by cat_tile.hip (host logic) and by the per-KT instantiation units cat_tile_kN.hip.
//
// One wavefront owns a tile of 16 rows.  The rows stream in with fully coalesced
// dword loads (lane = channel), are split into bf16 (hi, lo) pairs and staged through
// a small wave-private LDS buffer into the operand layout of
// v_mfma_f32_16x16x32_bf16, and are contracted against the centroids, which sit in
// LDS for the whole kernel, already split and packed in operand order.  The scores
// -2 x.c + |c|^2 rank the centroids; a row whose two best scores are closer than the
// error bound of the split arithmetic is re-ranked with direct-form double-precision
// distances over the candidates inside that bound, so the result is the exact
// nearest centroid (lowest index on ties).
//
//   assign      writes assignments (+ counts, objective, first row of each cluster)
//   lloyd       assign + the rows that changed cluster since the previous pass are
//               added to / subtracted from the running per-cluster sums
//   apply       assign + corrected = gamma[a] * x + beta[a] in the same pass
#pragma once
#include "cat_tile.h"

namespace cat {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kRows = 16;          // rows per wave tile (the N of the 16x16x32 MFMA)
constexpr int kChunk = 128;        // channels staged at a time (4 MFMA steps)
constexpr int kStageStride = 68;   // dwords per staged row: 64 + 4 pad, keeps ds_read_b128 conflict-free
constexpr int kStagePlane = kRows * kStageStride;  // dwords
constexpr int kMaxWaves = 8;
constexpr int kListCap = 1024;     // changed rows a workgroup can defer per launch
constexpr int kDirectRows = 8;     // up to this many deferred rows skip the LDS panel
constexpr size_t kLdsLimit = 160 * 1024;
constexpr float kPadNorm = 3.0e38f;

enum { MODE_ASSIGN = 0, MODE_APPLY_RETAIN = 1, MODE_APPLY_REREAD = 2 };
constexpr int kRetainCols = 8;     // retained inference: D <= 64 * kRetainCols

struct TileParams {
    const void* lq;
    int64_t N, D;
    int32_t K, K16, nchunks, waves;
    int64_t ntiles;
    const uint16_t* packA;   // [chunk][step][ktile][part][lane][8] bf16
    const float* cnorm;      // K16
    const float* cent;       // K x D fp32 (exact re-rank)
    int32_t* assign;         // nullable (apply)
    int32_t* counts;         // nullable
    double* inertia;         // nullable
    unsigned long long* rep; // nullable
    double* delta;           // K x D, lloyd delta mode only
    int32_t delta_mode;      // 0: off, 1: rows carry a previous assignment
    int32_t reverse;         // walk the tiles from the last to the first (see tile_lloyd)
    const float* gamma;      // apply
    const float* beta;
    void* out;
    float tau, tau2;         // re-rank threshold T = tau |x| cmax + tau2 cmax^2
    uint32_t ldsA_bytes, off_stage, off_cnorm, off_hist, off_rep, off_list, off_misc, stage_planes;
};

// ---- small device helpers ---------------------------------------------------------
__device__ __forceinline__ uint32_t pack_bf16(float a, float b) {  // a -> low half, b -> high half, RNE
    f32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2));
}
__device__ __forceinline__ float lo_half(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float hi_half(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }
__device__ __forceinline__ float readlane_f(float v, int l) {
    return __int_as_float(__builtin_amdgcn_readlane(__float_as_int(v), l));
}

// Row totals of 16 per-lane partials: lane l returns the sum over all 64 lanes of p[l & 15].
__device__ __forceinline__ float rowsum16(const float (&p)[16], int lane) {
    float a8[8], a4[4], a2[2];
    {
        const bool up = lane & 8;
#pragma unroll
        for (int j = 0; j < 8; j++) {
            float keep = up ? p[j + 8] : p[j], send = up ? p[j] : p[j + 8];
            a8[j] = keep + __shfl_xor(send, 8, kWave);
        }
    }
    {
        const bool up = lane & 4;
#pragma unroll
        for (int j = 0; j < 4; j++) {
            float keep = up ? a8[j + 4] : a8[j], send = up ? a8[j] : a8[j + 4];
            a4[j] = keep + __shfl_xor(send, 4, kWave);
        }
    }
    {
        const bool up = lane & 2;
#pragma unroll
        for (int j = 0; j < 2; j++) {
            float keep = up ? a4[j + 2] : a4[j], send = up ? a4[j] : a4[j + 2];
            a2[j] = keep + __shfl_xor(send, 2, kWave);
        }
    }
    const bool up = lane & 1;
    float keep = up ? a2[1] : a2[0], send = up ? a2[0] : a2[1];
    float v = keep + __shfl_xor(send, 1, kWave);
    v += __shfl_xor(v, 16, kWave);
    v += __shfl_xor(v, 32, kWave);
    return v;
}

template <bool BF16>
__device__ __forceinline__ double exact_dist(const void* lq, int64_t row, int64_t D, const float* c, int lane) {
    double s = 0.0;
    if (BF16) {
        const bf16_t* x = (const bf16_t*)lq + row * D;
        for (int64_t j = lane; j < D; j += kWave) {
            double d = (double)bf16_to_f32(x[j]) - (double)c[j];
            s = fma(d, d, s);
        }
    } else {
        const float* x = (const float*)lq + row * D;
        for (int64_t j = lane; j < D; j += kWave) {
            double d = (double)x[j] - (double)c[j];
            s = fma(d, d, s);
        }
    }
    return wave_sum(s);
}

// One chunk of 128 channels of the 16 rows, as loaded: lane l holds channels 2 l and 2 l + 1 of the
// chunk (f32 input: one 8-byte load per row, bf16 input: one 4-byte load per row).
template <bool BF16>
struct ChunkRegs {
    uint32_t w[kRows][BF16 ? 1 : 2];
};

// Rows beyond N repeat the last valid row and channels beyond D read channel 0 (both valid
// addresses), so every load is unconditional; the consumer masks the padding channels to zero
// (masking here would make the loads wait where they are issued).  `tile` is wave-uniform:
// the 16 row pointers live in scalar registers and each load is pointer + 32-bit lane offset.
template <bool BF16>
__device__ __forceinline__ void load_chunk(ChunkRegs<BF16>& r, const TileParams& p, int tile, int chunk, int lane) {
    const int64_t row0 = (int64_t)(p.reverse ? (int)p.ntiles - 1 - tile : tile) * kRows;
    const int nv = (p.N - row0) < kRows ? (int)(p.N - row0) : kRows;
    if (BF16) {
        const bf16_t* x = (const bf16_t*)p.lq + row0 * p.D;
        const int ch = chunk * kChunk + 2 * lane;
        const int o = ch < p.D ? ch : 0;
#pragma unroll
        for (int i = 0; i < kRows; i++) {
            r.w[i][0] = *(const uint32_t*)(x + o);
            if (i + 1 < nv) x += p.D;
        }
    } else {
        const float* x = (const float*)p.lq + row0 * p.D;
        const int ch = chunk * kChunk + 2 * lane;
        const int o = ch < p.D ? ch : 0;  // D is even: a pair is valid or padding as a whole
#pragma unroll
        for (int i = 0; i < kRows; i++) {
            const f32x2 v = *(const f32x2*)(x + o);
            r.w[i][0] = __float_as_uint(v.x);
            r.w[i][1] = __float_as_uint(v.y);
            if (i + 1 < nv) x += p.D;
        }
    }
}

// Stage one chunk and run its 4 MFMA steps against the resident centroids.
template <int KT, int PASSES, bool BF16>
__device__ __forceinline__ void contract_chunk(const ChunkRegs<BF16>& r, f32x4 (&acc)[KT], float (&nrm)[kRows],
                                               const unsigned char* ldsA_chunk, uint32_t* stage, int lane,
                                               int chunk, int64_t D) {
    constexpr int P = PASSES == 1 ? 1 : 2;
    uint32_t* stage_lo = stage + kStagePlane;
    // padding channels (>= D) were loaded from channel 0: mask them to zero
    const uint32_t m0 = chunk * kChunk + 2 * lane < D ? 0xFFFFFFFFu : 0u;
#pragma unroll
    for (int i = 0; i < kRows; i++) {
        if (BF16) {
            uint32_t w = r.w[i][0] & m0;
            float x0 = lo_half(w), x1 = hi_half(w);
            nrm[i] = fmaf(x0, x0, fmaf(x1, x1, nrm[i]));
            stage[i * kStageStride + lane] = w;
        } else {
            float x0 = __uint_as_float(r.w[i][0] & m0), x1 = __uint_as_float(r.w[i][BF16 ? 0 : 1] & m0);
            nrm[i] = fmaf(x0, x0, fmaf(x1, x1, nrm[i]));
            uint32_t h = pack_bf16(x0, x1);
            stage[i * kStageStride + lane] = h;
            if (PASSES == 3) stage_lo[i * kStageStride + lane] = pack_bf16(x0 - lo_half(h), x1 - hi_half(h));
        }
    }
    __builtin_amdgcn_wave_barrier();
    const int n = lane & 15, g = lane >> 4;
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const uint32_t* bp = stage + n * kStageStride + 16 * s + 4 * g;
        bf16x8 bh = __builtin_bit_cast(bf16x8, *(const u32x4*)bp);
        bf16x8 bl;
        if (PASSES == 3 && !BF16) bl = __builtin_bit_cast(bf16x8, *(const u32x4*)(bp + kStagePlane));
#pragma unroll
        for (int t = 0; t < KT; t++) {
            const unsigned char* ap = ldsA_chunk + (size_t)((s * KT + t) * P) * 1024 + lane * 16;
            bf16x8 ah = __builtin_bit_cast(bf16x8, *(const u32x4*)ap);
            acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bh, acc[t], 0, 0, 0);
            if (PASSES == 3) {
                bf16x8 al = __builtin_bit_cast(bf16x8, *(const u32x4*)(ap + 1024));
                acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(al, bh, acc[t], 0, 0, 0);
                if (!BF16) acc[t] = __builtin_amdgcn_mfma_f32_16x16x32_bf16(ah, bl, acc[t], 0, 0, 0);
            }
        }
    }
    __builtin_amdgcn_wave_barrier();
}

// Rank the centroids of the 16 rows from the accumulated dot products; exact re-rank of
// the rows inside the error bound.  On return every lane (n, *) holds row n's result.
template <int KT, bool BF16>
__device__ __forceinline__ void rank_rows(const TileParams& p, const f32x4 (&acc)[KT], const float* s_cnorm,
                                          float xn2, float cmax, int64_t row0, int lane, int& idx, float& dmin) {
    const int n = lane & 15, q = lane >> 4;
    float b1 = __builtin_inff(), b2 = __builtin_inff();
    int i1 = 0;
#pragma unroll
    for (int t = 0; t < KT; t++)
#pragma unroll
        for (int i = 0; i < 4; i++) {
            int k = 16 * t + 4 * q + i;
            float s = fmaf(-2.f, acc[t][i], s_cnorm[k]);
            if (s < b1) {
                b2 = b1;
                b1 = s;
                i1 = k;
            } else if (s < b2) {
                b2 = s;
            }
        }
#pragma unroll
    for (int o = 16; o <= 32; o <<= 1) {
        float ob1 = __shfl_xor(b1, o, kWave), ob2 = __shfl_xor(b2, o, kWave);
        int oi1 = __shfl_xor(i1, o, kWave);
        bool take = (ob1 < b1) || (ob1 == b1 && oi1 < i1);
        float loser = take ? b1 : ob1;
        b1 = take ? ob1 : b1;
        i1 = take ? oi1 : i1;
        b2 = fminf(fminf(b2, ob2), loser);
    }
    const float T = p.tau * sqrtf(xn2) * cmax + p.tau2 * cmax * cmax;
    const bool valid = row0 + n < p.N;
    const bool flag = valid && !(b2 - b1 > T);
    dmin = fmaxf(xn2 + b1, 0.f);
    unsigned long long mask = __ballot(flag && q == 0);
    while (mask) {
        const int r = __builtin_amdgcn_readfirstlane(__builtin_ctzll(mask));
        mask &= mask - 1;
        const float thr = readlane_f(b1, r) + readlane_f(T, r);
        const int64_t row = row0 + r;
        double dbest = __builtin_inf();
        int kbest = 0x7fffffff;
#pragma unroll
        for (int t = 0; t < KT; t++)
#pragma unroll
            for (int i = 0; i < 4; i++) {
                float s = fmaf(-2.f, acc[t][i], s_cnorm[16 * t + 4 * q + i]);
                unsigned long long m = __ballot(n == r && s <= thr);
                while (m) {
                    const int l = __builtin_amdgcn_readfirstlane(__builtin_ctzll(m));
                    m &= m - 1;
                    const int k = 16 * t + 4 * (l >> 4) + i;
                    if (k < p.K) {
                        double d = exact_dist<BF16>(p.lq, row, p.D, p.cent + (int64_t)k * p.D, lane);
                        if (d < dbest || (d == dbest && k < kbest)) {
                            dbest = d;
                            kbest = k;
                        }
                    }
                }
            }
        if (n == r && kbest != 0x7fffffff) {
            i1 = kbest;
            dmin = (float)dbest;
        }
    }
    idx = i1;
}

// Per-tile finishing work of the streaming modes: rank, write, book-keep; resets acc / nrm.
template <int KT, bool BF16, int MODE>
__device__ __forceinline__ void finish_tile(const TileParams& p, unsigned char* smem, f32x4 (&acc)[KT],
                                            float (&nrm)[kRows], int tile, int lane, float cmax, double& in_acc) {
    const int n = lane & 15, q = lane >> 4;
    const int64_t row0 = (int64_t)(p.reverse ? (int)p.ntiles - 1 - tile : tile) * kRows;
    const float* s_cnorm = (const float*)(smem + p.off_cnorm);
    const float xn2 = rowsum16(nrm, lane);
    int idx;
    float dmin;
    rank_rows<KT, BF16>(p, acc, s_cnorm, xn2, cmax, row0, lane, idx, dmin);
#pragma unroll
    for (int t = 0; t < KT; t++) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < kRows; i++) nrm[i] = 0.f;
    const bool owner = q == 0 && row0 + n < p.N;

    if (MODE == MODE_APPLY_REREAD) {
        if (p.assign && owner) p.assign[row0 + n] = idx;
        const int nv = (p.N - row0) < kRows ? (int)(p.N - row0) : kRows;
        // 8 rows at a time: 24 independent loads per lane in flight
#pragma unroll 1
        for (int i0 = 0; i0 < kRows; i0 += 8) {
            int a[8];
#pragma unroll
            for (int u = 0; u < 8; u++) a[u] = __builtin_amdgcn_readfirstlane(__shfl(idx, i0 + u, kWave));
            if (BF16) {
                for (int c2 = lane; 2 * c2 < p.D; c2 += kWave) {
                    uint32_t w[8];
                    f32x2 g[8], b[8];
#pragma unroll
                    for (int u = 0; u < 8; u++)
                        if (i0 + u < nv) {
                            w[u] = *((const uint32_t*)((const bf16_t*)p.lq + (row0 + i0 + u) * p.D) + c2);
                            g[u] = *((const f32x2*)(p.gamma + (int64_t)a[u] * p.D) + c2);
                            b[u] = *((const f32x2*)(p.beta + (int64_t)a[u] * p.D) + c2);
                        }
#pragma unroll
                    for (int u = 0; u < 8; u++)
                        if (i0 + u < nv)
                            *((uint32_t*)((bf16_t*)p.out + (row0 + i0 + u) * p.D) + c2) =
                                pack_bf16(fmaf(g[u].x, lo_half(w[u]), b[u].x), fmaf(g[u].y, hi_half(w[u]), b[u].y));
                }
            } else {
                for (int ch = lane; ch < p.D; ch += kWave) {
                    float x[8], g[8], b[8];
#pragma unroll
                    for (int u = 0; u < 8; u++)
                        if (i0 + u < nv) {
                            x[u] = ((const float*)p.lq + (row0 + i0 + u) * p.D)[ch];
                            g[u] = (p.gamma + (int64_t)a[u] * p.D)[ch];
                            b[u] = (p.beta + (int64_t)a[u] * p.D)[ch];
                        }
#pragma unroll
                    for (int u = 0; u < 8; u++)
                        if (i0 + u < nv)
                            __builtin_nontemporal_store(fmaf(g[u], x[u], b[u]), (float*)p.out + (row0 + i0 + u) * p.D + ch);
                }
            }
        }
        return;
    }

    // assign / lloyd bookkeeping (lanes 0..15 own one row each)
    int* s_hist = (int*)(smem + p.off_hist);
    unsigned long long* s_rep = (unsigned long long*)(smem + p.off_rep);
    int* s_misc = (int*)(smem + p.off_misc);
    int prev = -1;
    if (owner) {
        if (p.delta_mode) prev = p.assign[row0 + n];
        p.assign[row0 + n] = idx;
        if (p.counts) atomicAdd(&s_hist[idx], 1);
        if (p.rep) atomicMin(&s_rep[idx], (unsigned long long)(row0 + n));
        in_acc += (double)dmin;
    }
    if (p.delta) {
        const bool changed = owner && prev != idx;
        bool ovf = false;
        if (changed) {
            int pos = atomicAdd(&s_misc[0], 1);
            if (pos < kListCap) {
                ((int64_t*)(smem + p.off_list))[pos] = row0 + n;
                ((uint32_t*)(smem + p.off_list + (size_t)kListCap * 8))[pos] = ((uint32_t)(prev + 1) << 16) | (uint32_t)idx;
            } else {
                ovf = true;
            }
        }
        unsigned long long om = __ballot(ovf);
        while (om) {  // list full: this row goes straight to the global sums
            const int r = __builtin_amdgcn_readfirstlane(__builtin_ctzll(om));
            om &= om - 1;
            const int nw = __builtin_amdgcn_readlane(idx, r), od = __builtin_amdgcn_readlane(prev, r);
            const int64_t row = row0 + r;
            for (int64_t ch = lane; ch < p.D; ch += kWave) {
                double x = BF16 ? (double)bf16_to_f32(((const bf16_t*)p.lq)[row * p.D + ch])
                                : (double)((const float*)p.lq)[row * p.D + ch];
                atomicAdd(p.delta + (int64_t)nw * p.D + ch, x);
                if (od >= 0) atomicAdd(p.delta + (int64_t)od * p.D + ch, -x);
            }
        }
    }
}

// ---- the kernel ----------------------------------------------------------------------
template <int KT, int PASSES, bool BF16, int MODE, bool CA>
__global__ __launch_bounds__(kMaxWaves * kWave) void k_tile(const TileParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // wave-uniform: keeps tile/row math scalar
    const int n = lane & 15, q = lane >> 4;
    constexpr int P = PASSES == 1 ? 1 : 2;
    float* s_cnorm = (float*)(smem + p.off_cnorm);
    int* s_hist = (int*)(smem + p.off_hist);
    unsigned long long* s_rep = (unsigned long long*)(smem + p.off_rep);
    int* s_misc = (int*)(smem + p.off_misc);  // [0] list count, [2..] doubles for the objective
    uint32_t* stage = (uint32_t*)(smem + p.off_stage) + (size_t)wave * p.stage_planes * kStagePlane;

    const int ntiles = (int)p.ntiles;
    const int tstride = (int)gridDim.x * p.waves;
    const int tile0 = __builtin_amdgcn_readfirstlane((int)blockIdx.x * p.waves + wave);
    // streaming modes: the first two chunks are requested before the prologue touches LDS
    int tl = tile0, cl = 0;  // load cursor
    ChunkRegs<BF16> b0, b1, b2;
#define CAT_ISSUE(buf)                            \
    if (tl < ntiles) {                            \
        load_chunk<BF16>(buf, p, tl, cl, lane);   \
        if (++cl == p.nchunks) {                  \
            cl = 0;                               \
            tl += tstride;                        \
        }                                         \
    }
    if (MODE != MODE_APPLY_RETAIN) {
        CAT_ISSUE(b0)
        CAT_ISSUE(b1)
    }

    // prologue: centroids (operand order) and their norms into LDS
    {
        // resident operand: all of it; chunked operand (CA): the first chunk into the first of two buffers
        const u32x4* src = (const u32x4*)p.packA;
        u32x4* dst = (u32x4*)smem;
        const uint32_t nvec = CA ? (uint32_t)(4 * KT * P * 1024 / 16) : p.ldsA_bytes / 16;
        for (uint32_t i = threadIdx.x; i < nvec; i += blockDim.x) dst[i] = src[i];
        for (int k = threadIdx.x; k < p.K16; k += blockDim.x) s_cnorm[k] = p.cnorm[k];
        for (int k = threadIdx.x; k < p.K; k += blockDim.x) {
            s_hist[k] = 0;
            s_rep[k] = ~0ull;
        }
        if (threadIdx.x == 0) s_misc[0] = 0;
    }
    __syncthreads();
    float cmax2 = 0.f;
    for (int k = 0; k < p.K; k++) cmax2 = fmaxf(cmax2, s_cnorm[k]);
    const float cmax = sqrtf(cmax2);

    double in_acc = 0.0;

    if (MODE == MODE_APPLY_RETAIN) {
        // the 16 rows stay in registers between ranking and the affine map
        for (int tile = tile0; tile < ntiles; tile += tstride) {
            const int64_t row0 = (int64_t)(p.reverse ? ntiles - 1 - tile : tile) * kRows;
            ChunkRegs<false> xr[kRetainCols / 2];
#pragma unroll
            for (int c = 0; c < kRetainCols / 2; c++)
                if (c < p.nchunks) load_chunk<false>(xr[c], p, tile, c, lane);
            f32x4 acc[KT];
            float nrm[kRows];
#pragma unroll
            for (int t = 0; t < KT; t++) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
            for (int i = 0; i < kRows; i++) nrm[i] = 0.f;
#pragma unroll
            for (int c = 0; c < kRetainCols / 2; c++)
                if (c < p.nchunks)
                    contract_chunk<KT, PASSES, false>(xr[c], acc, nrm, smem + (size_t)c * 4 * KT * P * 1024, stage, lane, c,
                                                      p.D);
            const float xn2 = rowsum16(nrm, lane);
            int idx;
            float dmin;
            rank_rows<KT, false>(p, acc, s_cnorm, xn2, cmax, row0, lane, idx, dmin);
            if (p.assign && q == 0 && row0 + n < p.N) p.assign[row0 + n] = idx;
            float* out = (float*)p.out + row0 * p.D;
#pragma unroll
            for (int i = 0; i < kRows; i++) {
                const int a = __builtin_amdgcn_readlane(idx, i);
                if (row0 + i < p.N) {
                    const float* g = p.gamma + (int64_t)a * p.D;
                    const float* b = p.beta + (int64_t)a * p.D;
                    float* o = out + (int64_t)i * p.D;
#pragma unroll
                    for (int c = 0; c < kRetainCols / 2; c++) {
                        const int ch = c * kChunk + 2 * lane;
                        if (c < p.nchunks && ch < p.D) {
                            const f32x2 gv = *(const f32x2*)(g + ch), bv = *(const f32x2*)(b + ch);
                            f32x2 ov;
                            ov.x = fmaf(gv.x, __uint_as_float(xr[c].w[i][0]), bv.x);
                            ov.y = fmaf(gv.y, __uint_as_float(xr[c].w[i][1]), bv.y);
                            __builtin_nontemporal_store(ov, (f32x2*)(o + ch));
                        }
                    }
                }
            }
        }
        return;
    }

    // streaming modes: a three-buffer register pipeline keeps two chunks of loads in flight
    // while a third is contracted; the (tile, chunk) cursors run across tile boundaries
    f32x4 acc[KT];
    float nrm[kRows];
#pragma unroll
    for (int t = 0; t < KT; t++) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
#pragma unroll
    for (int i = 0; i < kRows; i++) nrm[i] = 0.f;
    int tc = tile0, cc = 0;  // compute cursor
#define CAT_STEP(buf)                                                                                              \
    contract_chunk<KT, PASSES, BF16>(buf, acc, nrm, smem + (size_t)cc * 4 * KT * P * 1024, stage, lane, cc, p.D); \
    if (++cc == p.nchunks) {                                                                                       \
        finish_tile<KT, BF16, MODE>(p, smem, acc, nrm, tc, lane, cmax, in_acc);                                    \
        cc = 0;                                                                                                    \
        tc += tstride;                                                                                             \
    }
    if (CA) {
        // The centroid operand does not fit in LDS: it streams through two LDS buffers one
        // 128-channel chunk at a time.  All waves of the workgroup walk the chunks in lockstep (a wave
        // that has run out of tiles still takes part in the copies and barriers), the next chunk of
        // the operand travels global -> registers -> LDS while the current one is contracted.
        constexpr int chunkA = 4 * KT * P * 1024;
        constexpr int AREG = (chunkA / 16 + kMaxWaves * kWave - 1) / (kMaxWaves * kWave);
        const int wg_tile0 = (int)blockIdx.x * p.waves;
        const int wg_tiles = wg_tile0 < ntiles ? (ntiles - 1 - wg_tile0) / tstride + 1 : 0;
        const int nsteps = wg_tiles * p.nchunks;
        int s = 0, ca = 0;
        u32x4 areg[AREG];
#define CAT_CA_STEP(bufcur, bufnext)                                                                          \
    {                                                                                                         \
        const int cn_ = ca + 1 == p.nchunks ? 0 : ca + 1;                                                     \
        const bool more_ = s + 1 < nsteps;                                                                    \
        if (more_) {                                                                                          \
            const u32x4* src_ = (const u32x4*)((const unsigned char*)p.packA + (size_t)cn_ * chunkA);         \
            _Pragma("unroll") for (int i_ = 0; i_ < AREG; i_++) {                                             \
                const int v_ = i_ * (int)blockDim.x + (int)threadIdx.x;                                       \
                if (v_ < chunkA / 16) areg[i_] = src_[v_];                                                    \
            }                                                                                                 \
        }                                                                                                     \
        CAT_ISSUE(bufnext)                                                                                    \
        if (tc < ntiles) {                                                                                    \
            contract_chunk<KT, PASSES, BF16>(bufcur, acc, nrm, smem + (size_t)(s & 1) * chunkA, stage, lane, cc, p.D); \
            if (++cc == p.nchunks) {                                                                          \
                finish_tile<KT, BF16, MODE>(p, smem, acc, nrm, tc, lane, cmax, in_acc);                       \
                cc = 0;                                                                                       \
                tc += tstride;                                                                                \
            }                                                                                                 \
        }                                                                                                     \
        if (more_) {                                                                                          \
            u32x4* dst_ = (u32x4*)(smem + (size_t)((s + 1) & 1) * chunkA);                                    \
            _Pragma("unroll") for (int i_ = 0; i_ < AREG; i_++) {                                             \
                const int v_ = i_ * (int)blockDim.x + (int)threadIdx.x;                                       \
                if (v_ < chunkA / 16) dst_[v_] = areg[i_];                                                    \
            }                                                                                                 \
        }                                                                                                     \
        __syncthreads();                                                                                      \
        ca = cn_;                                                                                             \
        s++;                                                                                                  \
    }
        while (s < nsteps) {
            CAT_CA_STEP(b0, b2)
            if (s >= nsteps) break;
            CAT_CA_STEP(b1, b0)
            if (s >= nsteps) break;
            CAT_CA_STEP(b2, b1)
        }
#undef CAT_CA_STEP
    } else {
        while (tc < ntiles) {
            CAT_ISSUE(b2)
            CAT_STEP(b0)
            if (tc >= ntiles) break;
            CAT_ISSUE(b0)
            CAT_STEP(b1)
            if (tc >= ntiles) break;
            CAT_ISSUE(b1)
            CAT_STEP(b2)
        }
    }
#undef CAT_ISSUE
#undef CAT_STEP

    if (MODE != MODE_ASSIGN) return;

    // workgroup epilogue: counts, first rows, objective
    double* s_in = (double*)(s_misc + 2);
    if (lane == 0) s_in[wave] = 0.0;
    in_acc = wave_sum(in_acc);
    if (lane == 0) s_in[wave] = in_acc;
    __syncthreads();
    for (int k = threadIdx.x; k < p.K; k += blockDim.x) {
        if (p.counts && s_hist[k]) atomicAdd(&p.counts[k], s_hist[k]);
        if (p.rep && s_rep[k] != ~0ull) atomicMin(&p.rep[k], s_rep[k]);
    }
    if (p.inertia && threadIdx.x == 0) {
        double tot = 0.0;
        for (int w = 0; w < p.waves; w++) tot += s_in[w];
        atomicAdd(p.inertia, tot);
    }
    if (!p.delta) return;

    // deferred sums of the rows that changed cluster: the centroid operand is dead now,
    // its LDS becomes a K x CW panel of doubles, filled panel by panel over the channels
    const int cnt = s_misc[0] < kListCap ? s_misc[0] : kListCap;
    if (cnt == 0) return;  // uniform: s_misc[0] is final after the barrier above
    const int64_t* l_row = (const int64_t*)(smem + p.off_list);
    const uint32_t* l_on = (const uint32_t*)(smem + p.off_list + (size_t)kListCap * 8);
    double* S = (double*)smem;
    // panel width: everything below the norm table (operand + staging) is free now
    int CW = (int)((p.off_cnorm / 8 / p.K) & ~63u);
    if (CW > 1024) CW = 1024;
    if (cnt <= kDirectRows || CW == 0) {
        // a handful of rows (the usual case once Lloyd has nearly converged), or no room for a
        // panel: one wave per row, all loads first, then straight to the global sums
        for (int e = wave; e < cnt; e += p.waves) {
            const int64_t row = l_row[e];
            const int nw = (int)(l_on[e] & 0xFFFFu), od = (int)(l_on[e] >> 16) - 1;
            for (int64_t c0 = 0; c0 < p.D; c0 += 16 * kWave) {
                float x[16];
#pragma unroll
                for (int u = 0; u < 16; u++) {
                    const int64_t ch = c0 + u * kWave + lane;
                    x[u] = ch < p.D ? (BF16 ? bf16_to_f32(((const bf16_t*)p.lq)[row * p.D + ch])
                                            : ((const float*)p.lq)[row * p.D + ch])
                                    : 0.f;
                }
#pragma unroll
                for (int u = 0; u < 16; u++) {
                    const int64_t ch = c0 + u * kWave + lane;
                    if (ch < p.D) {
                        atomicAdd(p.delta + (int64_t)nw * p.D + ch, (double)x[u]);
                        if (od >= 0) atomicAdd(p.delta + (int64_t)od * p.D + ch, -(double)x[u]);
                    }
                }
            }
        }
        return;
    }
    for (int64_t base = 0; base < p.D; base += CW) {
        const int cw = (p.D - base) < CW ? (int)(p.D - base) : CW;
        __syncthreads();
        for (int i = threadIdx.x; i < p.K * CW; i += blockDim.x) S[i] = 0.0;
        __syncthreads();
        for (int e = wave; e < cnt; e += p.waves) {
            const int64_t row = l_row[e];
            const int nw = (int)(l_on[e] & 0xFFFFu), od = (int)(l_on[e] >> 16) - 1;
            for (int c = lane; c < cw; c += kWave) {
                double x = BF16 ? (double)bf16_to_f32(((const bf16_t*)p.lq)[row * p.D + base + c])
                                : (double)((const float*)p.lq)[row * p.D + base + c];
                atomicAdd(S + (size_t)nw * CW + c, x);
                if (od >= 0) atomicAdd(S + (size_t)od * CW + c, -x);
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < p.K * CW; i += blockDim.x) {
            const int k = i / CW, c = i - k * CW;
            const double v = S[i];
            if (c < cw && v != 0.0) atomicAdd(p.delta + (int64_t)k * p.D + base + c, v);
        }
    }
}

struct TileCfg {
    bool ok = false;
    int KT = 0, P = 0, waves = 0, nchunks = 0, planes = 0, mode = MODE_ASSIGN;
    bool chunked = false;  // the centroid operand streams through LDS instead of living there
    uint32_t ldsA = 0, off_stage = 0, off_cnorm = 0, off_hist = 0, off_rep = 0, off_list = 0, off_misc = 0;
    size_t lds_total = 0;
};

template <int KT, int PASSES, bool BF16, int MODE, bool CA>
static inline cat_status launch_one(const TileParams& p, const TileCfg& c, hipStream_t st) {
    auto kern = k_tile<KT, PASSES, BF16, MODE, CA>;
    CAT_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c.lds_total));
    int64_t want = (p.ntiles + c.waves - 1) / c.waves;
    int per_cu = (int)(kLdsLimit / c.lds_total);
    if (per_cu > 2) per_cu = 2;
    if (per_cu < 1) per_cu = 1;
    int64_t cap = 256 * (int64_t)per_cu;
    unsigned blocks = (unsigned)(want < cap ? want : cap);
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(c.waves * kWave), c.lds_total, st, p);
    CAT_LAUNCH_CHECK("k_tile");
    return CAT_OK;
}

template <int KT, int PASSES, bool BF16>
static inline cat_status launch_mode(const TileParams& p, const TileCfg& c, hipStream_t st) {
    if (c.chunked) {
        if (c.mode == MODE_ASSIGN) return launch_one<KT, PASSES, BF16, MODE_ASSIGN, true>(p, c, st);
        if (c.mode == MODE_APPLY_REREAD) return launch_one<KT, PASSES, BF16, MODE_APPLY_REREAD, true>(p, c, st);
    } else {
        if (c.mode == MODE_ASSIGN) return launch_one<KT, PASSES, BF16, MODE_ASSIGN, false>(p, c, st);
        if (c.mode == MODE_APPLY_REREAD) return launch_one<KT, PASSES, BF16, MODE_APPLY_REREAD, false>(p, c, st);
        if (!BF16 && c.mode == MODE_APPLY_RETAIN) return launch_one<KT, PASSES, false, MODE_APPLY_RETAIN, false>(p, c, st);
    }
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernel: no instance for this mode");
}

template <int KT, bool BF16>
static inline cat_status launch_kt(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return c.P == 2 ? launch_mode<KT, 3, BF16>(p, c, st) : launch_mode<KT, 1, BF16>(p, c, st);
}


// one translation unit per (KT, dtype), for compile time: cat_tile_k<KT>_<dtype>.hip
cat_status launch_kt1_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt1_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt2_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt2_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt4_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt4_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt8_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt8_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt16_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_kt16_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);

}  // namespace cat
