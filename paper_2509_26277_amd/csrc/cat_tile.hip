// MFMA tile kernels of the CAT hot path for gfx950.
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
template <int KT, int PASSES, bool BF16, int MODE>
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
        const u32x4* src = (const u32x4*)p.packA;
        u32x4* dst = (u32x4*)smem;
        for (uint32_t i = threadIdx.x; i < p.ldsA_bytes / 16; i += blockDim.x) dst[i] = src[i];
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

// ---- centroid preparation: (sums -> centroids), split to bf16 (hi, lo), operand order ----
// One workgroup per cluster slot k in [0, K16).  With `base` given: S = base + delta is
// folded back into base, delta is cleared, centroid = S / count (kept if the cluster is
// empty).  Then the row is split and scattered into packA, and its squared norm stored.  Last,
// the outputs of the following pass are reset: counts (after its value was used), the objective
// slot and the first-row table.
__global__ __launch_bounds__(256) void k_tile_prep(float* cent, double* base, double* delta, int32_t* counts,
                                                   int64_t D, int32_t K, int32_t KT, int32_t P, int32_t nchunks,
                                                   uint16_t* packA, float* cnorm, double* inertia_slot,
                                                   unsigned long long* rep) {
    __shared__ double s_red[256];
    const int k = blockIdx.x;
    const int t = k >> 4, m = k & 15;
    double nn = 0.0;
    const int64_t Dpad = (int64_t)nchunks * kChunk;
    const int cntk = (base && k < K) ? counts[k] : 0;
    for (int64_t ch = threadIdx.x; ch < Dpad; ch += blockDim.x) {
        float c = 0.f;
        if (k < K && ch < D) {
            const int64_t i = (int64_t)k * D + ch;
            if (base) {
                double S = base[i] + delta[i];
                base[i] = S;
                delta[i] = 0.0;
                if (cntk > 0) cent[i] = (float)(S / (double)cntk);
            }
            c = cent[i];
        }
        nn += (double)c * (double)c;
        // position of channel ch in the operand: chunk, MFMA step s, lane group g, then the 8
        // consecutive channels a lane feeds to one MFMA
        const int cc = (int)(ch / kChunk), r = (int)(ch % kChunk);
        const int h = r & 1, d = r >> 1;
        const int s = d >> 4, g = (d >> 2) & 3, ii = d & 3;
        const int lane = g * 16 + m;
        const uint32_t hw = pack_bf16(c, 0.f) & 0xFFFFu;
        const size_t blk = ((size_t)(cc * 4 + s) * KT + t) * P;
        packA[(blk * 64 + lane) * 8 + 2 * ii + h] = (uint16_t)hw;
        if (P == 2) {
            const uint32_t lw = pack_bf16(c - lo_half(hw), 0.f) & 0xFFFFu;
            packA[((blk + 1) * 64 + lane) * 8 + 2 * ii + h] = (uint16_t)lw;
        }
    }
    s_red[threadIdx.x] = nn;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) s_red[threadIdx.x] += s_red[threadIdx.x + o];
        __syncthreads();
    }
    if (threadIdx.x == 0) {
        cnorm[k] = k < K ? (float)s_red[0] : kPadNorm;
        // outputs the following pass accumulates into (the count was read above, before the barriers)
        if (k < K) {
            if (counts) counts[k] = 0;
            if (rep) rep[k] = ~0ull;
        }
        if (k == 0 && inertia_slot) *inertia_slot = 0.0;
    }
}

// ---- host side ----------------------------------------------------------------------------
struct TileCfg {
    bool ok = false;
    int KT = 0, P = 0, waves = 0, nchunks = 0, planes = 0, mode = MODE_ASSIGN;
    uint32_t ldsA = 0, off_stage = 0, off_cnorm = 0, off_hist = 0, off_rep = 0, off_list = 0, off_misc = 0;
    size_t lds_total = 0;
};

static inline uint32_t up16(size_t x) { return (uint32_t)((x + 15) & ~(size_t)15); }

static TileCfg tile_config(TileMode mode, int64_t D, int32_t K, cat_dtype dt) {
    TileCfg c;
    const int K16 = (K + 15) & ~15;
    int KT = 1;
    while (KT * 16 < K16) KT *= 2;
    if (KT > 16) return c;
    if (D & 1) return c;      // rows must keep the 8-byte alignment of the paired loads
    if (D > 65536) return c;  // also bounds the fp32 accumulation term of the re-rank threshold
    const int nchunks = (int)((D + kChunk - 1) / kChunk);
    const bool bf16 = dt == CAT_BF16;
    const bool lists = mode == TILE_LLOYD;
    for (int P = 2; P >= 1; P--) {
        const int planes = (P == 2 && !bf16) ? 2 : 1;
        const size_t ldsA = (size_t)nchunks * 4 * KT * P * 1024;
        for (int waves = kMaxWaves; waves >= 4; waves -= 2) {
            size_t off = ldsA;
            TileCfg t;
            t.off_stage = up16(off);
            off = t.off_stage + (size_t)waves * planes * kStagePlane * 4;
            t.off_cnorm = up16(off);
            off = t.off_cnorm + (size_t)KT * 16 * 4;
            t.off_hist = up16(off);
            off = t.off_hist + (size_t)K * 4;
            t.off_rep = up16(off);
            off = t.off_rep + (size_t)K * 8;
            t.off_list = up16(off);
            off = t.off_list + (lists ? (size_t)kListCap * 12 : 0);
            t.off_misc = up16(off);
            off = t.off_misc + 16 + 8 * kMaxWaves;
            if (off > kLdsLimit) continue;
            t.ok = true;
            t.KT = KT;
            t.P = P;
            t.waves = waves;
            t.nchunks = nchunks;
            t.planes = planes;
            t.ldsA = (uint32_t)ldsA;
            t.lds_total = off;
            if (mode == TILE_APPLY) t.mode = (!bf16 && D <= 64 * kRetainCols && KT <= 8) ? MODE_APPLY_RETAIN : MODE_APPLY_REREAD;
            return t;
        }
    }
    return c;
}

bool tile_supports(TileMode mode, int64_t D, int32_t K, cat_dtype dt) { return tile_config(mode, D, K, dt).ok; }

static size_t packA_bytes(int64_t D, int32_t K) {
    const int K16 = (K + 15) & ~15;
    int KT = 1;
    while (KT * 16 < K16) KT *= 2;
    const size_t nchunks = (size_t)((D + kChunk - 1) / kChunk);
    return nchunks * 4 * KT * 2 * 1024;
}
static inline size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t tile_workspace_bytes(int64_t D, int32_t K, cat_dtype dt) {
    if (!tile_config(TILE_ASSIGN, D, K, dt).ok) return 0;
    return a256(packA_bytes(D, K)) + a256(16 * 16 * 4 * sizeof(float)) + a256((size_t)K * D * sizeof(float));
}
TileWs tile_carve(void* base, int64_t D, int32_t K, cat_dtype dt) {
    TileWs w;
    w.bytes = tile_workspace_bytes(D, K, dt);
    if (!base || w.bytes == 0) return w;
    char* b = (char*)base;
    w.packA = (uint16_t*)b;
    b += a256(packA_bytes(D, K));
    w.cnorm = (float*)b;
    b += a256(16 * 16 * 4 * sizeof(float));
    w.cent = (float*)b;
    return w;
}

static cat_status launch_prep(cat_dtype dt, float* cent, double* base, double* delta, int32_t* counts, int64_t D,
                              int32_t K, const TileCfg& c, const TileWs& ws, double* inertia_slot,
                              unsigned long long* rep, hipStream_t st) {
    dim3 grid(c.KT * 16), block(256);
    (void)dt;
    hipLaunchKernelGGL(k_tile_prep, grid, block, 0, st, cent, base, delta, counts, D, K, c.KT, c.P, c.nchunks, ws.packA,
                       ws.cnorm, inertia_slot, rep);
    CAT_LAUNCH_CHECK("k_tile_prep");
    return CAT_OK;
}

template <int KT, int PASSES, bool BF16, int MODE>
static cat_status launch_one(const TileParams& p, const TileCfg& c, hipStream_t st) {
    auto kern = k_tile<KT, PASSES, BF16, MODE>;
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

template <int KT, bool BF16>
static cat_status launch_kt(const TileParams& p, const TileCfg& c, hipStream_t st) {
    if (c.P == 2) {
        if (c.mode == MODE_ASSIGN) return launch_one<KT, 3, BF16, MODE_ASSIGN>(p, c, st);
        if (c.mode == MODE_APPLY_REREAD) return launch_one<KT, 3, BF16, MODE_APPLY_REREAD>(p, c, st);
        if (!BF16) return launch_one<KT, 3, false, MODE_APPLY_RETAIN>(p, c, st);
    } else {
        if (c.mode == MODE_ASSIGN) return launch_one<KT, 1, BF16, MODE_ASSIGN>(p, c, st);
        if (c.mode == MODE_APPLY_REREAD) return launch_one<KT, 1, BF16, MODE_APPLY_REREAD>(p, c, st);
        if (!BF16) return launch_one<KT, 1, false, MODE_APPLY_RETAIN>(p, c, st);
    }
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernel: no instance for this mode");
}

static cat_status launch_tile(const TileParams& p, const TileCfg& c, cat_dtype dt, hipStream_t st) {
#define CAT_KT(KT_)                                                   \
    case KT_:                                                         \
        return dt == CAT_BF16 ? launch_kt<KT_, true>(p, c, st) : launch_kt<KT_, false>(p, c, st);
    switch (c.KT) {
        CAT_KT(1)
        CAT_KT(2)
        CAT_KT(4)
        CAT_KT(8)
        CAT_KT(16)
    }
#undef CAT_KT
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernel: K tile count %d", c.KT);
}

static TileParams base_params(const void* lq, int64_t N, int64_t D, int32_t K, const TileCfg& c, const TileWs& ws,
                              cat_dtype dt) {
    TileParams p = {};
    p.lq = lq;
    p.N = N;
    p.D = D;
    p.K = K;
    p.K16 = c.KT * 16;
    p.nchunks = c.nchunks;
    p.waves = c.waves;
    p.ntiles = (N + kRows - 1) / kRows;
    p.packA = ws.packA;
    p.cnorm = ws.cnorm;
    // error bound of the split arithmetic, as a fraction of |x| |c|: two bf16 parts per operand
    // leave 2^-16 relative per product (one part: 2^-8), four such terms enter a score difference,
    // and the fp32 accumulation of n_acc MFMA partial sums; tau2 covers the rounding of |c|^2
    const bool exact_x = dt == CAT_BF16;
    const int passes = c.P == 2 ? (exact_x ? 2 : 3) : 1;
    const float n_acc = (float)(passes * c.nchunks * 4 + 8);
    const float split = c.P == 2 ? (exact_x ? 3.1e-5f : 9.4e-5f) : (exact_x ? 8.0e-3f : 1.6e-2f);
    p.tau = split + 4.f * n_acc * 5.96e-8f;
    p.tau2 = 4.0e-7f;
    p.ldsA_bytes = c.ldsA;
    p.off_stage = c.off_stage;
    p.off_cnorm = c.off_cnorm;
    p.off_hist = c.off_hist;
    p.off_rep = c.off_rep;
    p.off_list = c.off_list;
    p.off_misc = c.off_misc;
    p.stage_planes = c.planes;
    return p;
}

cat_status tile_assign(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                       int32_t* assign, int32_t* counts, double* inertia, unsigned long long* rep,
                       const float* gamma, const float* beta, void* corrected, const TileWs& ws, hipStream_t st) {
    const TileMode mode = gamma ? TILE_APPLY : TILE_ASSIGN;
    TileCfg c = tile_config(mode, D, K, dt);
    if (!c.ok) return set_error(CAT_ERR_UNSUPPORTED, "tile kernels do not fit D=%lld K=%d", (long long)D, (int)K);
    cat_status s = launch_copy_words(cent, ws.cent, (int64_t)K * D, st);
    if (s != CAT_OK) return s;
    s = launch_prep(dt, ws.cent, nullptr, nullptr, nullptr, D, K, c, ws, nullptr, nullptr, st);
    if (s != CAT_OK) return s;
    TileParams p = base_params(lq, N, D, K, c, ws, dt);
    p.cent = ws.cent;
    p.assign = assign;
    p.counts = counts;
    p.inertia = inertia;
    p.rep = rep;
    p.gamma = gamma;
    p.beta = beta;
    p.out = corrected;
    return launch_tile(p, c, dt, st);
}

cat_status tile_lloyd(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, int32_t iters,
                      float* cent_io, double* sums, int32_t* assign, int32_t* counts, double* inertia,
                      unsigned long long* rep, const TileWs& ws, hipStream_t st) {
    TileCfg c = tile_config(TILE_LLOYD, D, K, dt);
    if (!c.ok) return set_error(CAT_ERR_UNSUPPORTED, "tile kernels do not fit D=%lld K=%d", (long long)D, (int)K);
    const size_t KD = (size_t)K * (size_t)D;
    double* base = sums;
    double* delta = sums + KD;
    cat_status s;
#define CAT_T(expr)            \
    do {                       \
        s = (expr);            \
        if (s != CAT_OK) return s; \
    } while (0)
    TileParams p = base_params(lq, N, D, K, c, ws, dt);
    p.cent = cent_io;
    p.assign = assign;
    p.counts = counts;
    for (int32_t t = 0; t <= iters; t++) {
        const bool last = t == iters;
        // centroids of this pass: the initial ones, or the running sums over the counts of the last pass;
        // the same launch resets what this pass accumulates into
        CAT_T(launch_prep(dt, cent_io, t ? base : nullptr, t ? delta : nullptr, counts, D, K, c, ws,
                          inertia ? inertia + t : nullptr, last ? rep : nullptr, st));
        p.inertia = inertia ? inertia + t : nullptr;
        p.rep = last ? rep : nullptr;  // the final pass describes the partition that is returned
        p.delta = (t > 0 && !last) ? delta : nullptr;
        p.delta_mode = p.delta ? 1 : 0;
        // alternate the scan direction: the rows a pass reads last are the ones most likely still in
        // the memory-side cache when the next pass starts
        p.reverse = t & 1;
        CAT_T(launch_tile(p, c, dt, st));
        if (t == 0 && iters > 0) {  // first full sums: one segmented pass; later passes only move the changed rows
            CAT_T(launch_fill_zero(sums, 2 * KD * sizeof(double), st));
            CAT_T(launch_segsum(1, lq, nullptr, dt, assign, N, D, K, nullptr, nullptr, base, st));
        }
    }
#undef CAT_T
    return CAT_OK;
}

}  // namespace cat
