// MFMA tile kernels of the CAT hot path: host side (variant selection, workspace, the Lloyd
// driver) and the centroid preparation kernel.  The tile kernel itself is in cat_tile_kernel.h.
#include "cat_tile_kernel.h"

namespace cat {

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
        // position of channel ch in the operand: chunk, MFMA step s (32 channels), lane group g, then
        // the 8 consecutive channels j that lane (m, g) feeds to one MFMA
        const int cc = (int)(ch / kChunk), r = (int)(ch % kChunk);
        const int s = r >> 5, g = (r >> 3) & 3, j = r & 7;
        const int lane = g * 16 + m;
        const uint32_t hw = pack_bf16(c, 0.f) & 0xFFFFu;
        const size_t blk = ((size_t)(cc * 4 + s) * KT + t) * P;
        packA[(blk * 64 + lane) * 8 + j] = (uint16_t)hw;
        if (P == 2) {
            const uint32_t lw = pack_bf16(c - lo_half(hw), 0.f) & 0xFFFFu;
            packA[((blk + 1) * 64 + lane) * 8 + j] = (uint16_t)lw;
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

static inline uint32_t up16(size_t x) { return (uint32_t)((x + 15) & ~(size_t)15); }

static TileCfg tile_config(TileMode mode, int64_t D, int32_t K, cat_dtype dt) {
    TileCfg c;
    const int K16 = (K + 15) & ~15;
    int KT = 1;
    while (KT * 16 < K16) KT *= 2;
    if (KT > 16) return c;
    if (D % (dt == CAT_BF16 ? 8 : 4)) return c;  // rows must keep the 16-byte alignment of the operand loads
    if (D > 65536) return c;  // also bounds the fp32 accumulation term of the re-rank threshold
    const int nchunks = (int)((D + kChunk - 1) / kChunk);
    const bool lists = mode == TILE_LLOYD;
    // first choice: the whole operand resident in LDS (hi + lo parts, else hi only); otherwise
    // the chunked operand (two chunk buffers, 8 waves)
    for (int pass = 0; pass < 4; pass++) {
        const bool chunked = pass >= 2;
        const int P = (pass & 1) ? 1 : 2;
        const size_t ldsA = chunked ? (size_t)2 * 4 * KT * P * 1024 : (size_t)nchunks * 4 * KT * P * 1024;
        for (int waves = kMaxWaves; waves >= kMaxWaves; waves -= 2) {
            size_t off = ldsA;
            TileCfg t;
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
            t.chunked = chunked;
            t.ldsA = (uint32_t)ldsA;
            t.lds_total = off;
            if (mode == TILE_APPLY)
                t.mode = MODE_APPLY;
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

static cat_status launch_tile(const TileParams& p, const TileCfg& c, cat_dtype dt, hipStream_t st) {
    const bool bf = dt == CAT_BF16;
    switch (c.KT) {
        case 1: return bf ? launch_kt1_bf16(p, c, st) : launch_kt1_f32(p, c, st);
        case 2: return bf ? launch_kt2_bf16(p, c, st) : launch_kt2_f32(p, c, st);
        case 4: return bf ? launch_kt4_bf16(p, c, st) : launch_kt4_f32(p, c, st);
        case 8: return bf ? launch_kt8_bf16(p, c, st) : launch_kt8_f32(p, c, st);
        case 16: return bf ? launch_kt16_bf16(p, c, st) : launch_kt16_f32(p, c, st);
    }
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
    p.off_cnorm = c.off_cnorm;
    p.off_hist = c.off_hist;
    p.off_rep = c.off_rep;
    p.off_list = c.off_list;
    p.off_misc = c.off_misc;
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
