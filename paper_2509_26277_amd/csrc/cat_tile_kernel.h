// MFMA tile kernel of the CAT hot path for gfx950: device code, kernel template and its launcher.
// Included by cat_tile.hip (host logic) and by the instantiation units cat_tile_k<KT>_<dtype>.hip.
//
// One wavefront owns a tile of 16 rows.  Lane (n, g) = (lane & 15, lane >> 4) loads, with
// 16-byte loads, 8 consecutive channels of row n per MFMA step -- which is exactly the
// B-operand layout of v_mfma_f32_16x16x32_bf16, so nothing is staged or transposed: fp32
// data is split in registers into bf16 (hi, lo) pairs, bf16 data is used as loaded.  The
// A operand is the centroids, split and packed in operand order by k_tile_prep and held
// in LDS (whole, or streamed through two buffers when it does not fit).  Clusters are
// the M dimension and rows the N dimension, so a lane ends up with 4 KT cluster scores
// of ONE row: the argmin is in-register plus two cross-lane steps.  The scores
// -2 x.c + |c|^2 rank the centroids; a row whose two best scores are closer than the
// error bound of the split arithmetic is re-ranked with direct-form double-precision
// distances over the candidates inside that bound, so the result is the exact nearest
// centroid (lowest index on ties).
//
//   assign      writes assignments (+ counts, objective, first row of each cluster)
//   lloyd       assign + the rows that changed cluster since the previous pass are
//               listed (row, old, new) for the sums update that follows (k_delta_prep)
//   apply       assign + corrected = gamma[a] * x + beta[a] in the same pass
#pragma once
#include <type_traits>

#include "cat_tile.h"

namespace cat {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 bf16x2;
typedef __attribute__((ext_vector_type(2))) float f32x2;
typedef __attribute__((ext_vector_type(4))) float f32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t u32x4;

constexpr int kRows = 16;          // rows per wave tile (the N of the 16x16x32 MFMA)
constexpr int kChunk = 128;        // channels per pipeline stage (4 MFMA steps of 32)
constexpr int kMaxWaves = 8;
constexpr int kQueueCap = 256;     // rows a workgroup queues in LDS for the exact re-rank at the end of its tiles
constexpr int kListCap = 1024;     // changed rows a workgroup collects in LDS before they go to the global list
constexpr size_t kLdsLimit = 160 * 1024;
constexpr float kPadNorm = 3.0e38f;

enum { MODE_ASSIGN = 0, MODE_APPLY = 2 };

struct TileParams {
    const void* lq;
    int64_t N, D;
    int32_t K, K16, nchunks, waves;
    int64_t ntiles;
    const uint16_t* packA;   // [chunk][step][ktile][part][lane][8] bf16
    const float* cnorm;      // K16 squared centroid norms, or (norm_slices > 0) their per-slice shares:
    const double* norm_part; //   norm_slices x K doubles, added up here in slice order
    int32_t norm_slices;
    const float* cent;       // K x D fp32 (exact re-rank)
    int32_t* assign;         // nullable (apply)
    int32_t* counts;         // nullable
    double* inertia;         // nullable
    unsigned long long* rep; // nullable
    unsigned long long* list;  // lloyd: rows that changed cluster, (row << 24) | ((old + 1) << 12) | new
    uint32_t* list_count;      // entries in list (appended to with atomics)
    int32_t delta_mode;      // 0: off, 1: rows carry a previous assignment
    int32_t list_cap;        // entries of the workgroup's LDS list in use (<= kListCap)
    int32_t reverse;         // walk the tiles from the last to the first (see tile_lloyd)
    const uint32_t* skip_when_zero;  // nullable: the launch does nothing if this word is zero (tile_lloyd: the
                                     // list length of the pass before, when the loop may stop early)
    const float* gamma;      // apply
    const float* beta;
    void* out;
    float tau, tau2;         // re-rank threshold T = tau |x| cmax + tau2 cmax^2
    uint32_t ldsA_bytes, off_cnorm, off_hist, off_rep, off_list, off_misc;
    // Plain assignment passes: rows inside the error bound are not measured where they are found (the wave would
    // leave the pipeline of row loads it has in flight, and in the chunked-operand loop hold up the other seven) but
    // queued in LDS, queue_cap entries of DeferredRow after a 16-byte header at off_queue, and measured by all waves
    // when the workgroup has run out of tiles.  A row that finds the queue full, or has more than kQueueCand
    // candidates, is measured on the spot; queue_cap = 0: every row is.
    uint32_t off_queue;
    int32_t queue_cap;
    // Several independent centroid sets side by side (fits for a grid of cluster counts that share every read of
    // the rows; MULTI instantiations only).  Set s owns the cluster tiles set_t0[s] .. set_t0[s + 1] - 1, of whose
    // 16-cluster slots the first set_k[s] hold centroids.  Cluster numbers everywhere (assignments, counts, list
    // entries, first rows) are slot numbers of the concatenation.  `assign` then holds 16 int32 per row (set s at
    // [row * 16 + s]) and `inertia` one double per set.
    int32_t nsets;
    int16_t set_k[16];
    uint8_t set_t0[17];
    // Distance bounds (BOUNDS instantiations only; Hamerly, SDM 2010).  A pass that evaluates a row leaves in
    // expire[row] the value the accumulated centroid drift *gnow must reach before the row's nearest centroid can
    // change: the drift at the evaluation plus a lower bound of (distance to the second nearest) - (distance to the
    // nearest).  With `rows` given the pass walks only the *n_rows listed rows (16 to a tile, in list order) instead
    // of all N; row numbers everywhere (assignments, list entries, expire) are the real ones.
    double* expire;            // N doubles, nullable
    const double* gnow;        // accumulated drift up to this pass
    const int32_t* rows;       // nullable: listed rows
    const uint32_t* n_rows;    // their number
    int32_t* evaluated_slot;   // nullable: receives the number of rows this pass evaluates
    // More clusters than one launch ranks with the two-part operand (SPLIT instantiations only): the clusters are
    // split over two launches.  This launch ranks the K clusters k_base .. k_base + K - 1 (packA, cnorm point at its
    // share).  The first launch (carry_out given) only leaves, per row, the best score of its share and the exact
    // nearest centroid of its share; the second (carry_in given) ranks that pair as one more cluster beside its own
    // and does the bookkeeping of the pass.  Tables per cluster (counts, first rows) span k_hist clusters.
    int32_t k_base, k_hist, norm_stride;
    const float2* carry_in;
    float2* carry_out;
    float* cmax_io;  // the first launch leaves the largest centroid norm of its share, the second takes the larger of the two
};

// A row whose exact re-rank waits for the end of the workgroup's tiles: its number, the assignment it had before the
// pass (-1: none), and the clusters whose scores are within the error bound of the best one.
constexpr int kQueueCand = 8;
struct DeferredRow {
    long long row;
    int prev, ncand;
    short cand[kQueueCand];
};
static_assert(sizeof(DeferredRow) == 32, "queue entries are 32 bytes");

// Which lane group g (0..3) and which of its 8 operand elements j hold channel r (0..31) of a
// 32-channel MFMA step.  The contraction does not care how channels map to the k index as long as
// rows and centroids agree, so the map is chosen for the row loads: bf16 rows give a lane 8
// consecutive channels (one 16-byte load); fp32 rows give it channels 4g..4g+3 and 16+4g..16+4g+3,
// so that each of its two 16-byte loads forms, with the other three lanes of the row, 64
// contiguous bytes (whole 32-byte sectors) instead of 16-byte pieces with gaps.
__host__ __device__ __forceinline__ void operand_slot(int r, bool f32_rows, int& g, int& j) {
    if (f32_rows) {
        g = (r & 15) >> 2;
        j = (r & 3) + ((r >> 4) << 2);
    } else {
        g = r >> 3;
        j = r & 7;
    }
}

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

// Exact squared distances (fp64, direct form) of one row to NC centroids at once, the whole wave
// on the row: 16-byte loads, every lane's loads of a round issued before any is used.  D is a
// multiple of the 16-byte group (4 fp32 / 8 bf16 channels), as everywhere in the tile path.
template <bool BF16, int NC>
__device__ __forceinline__ void exact_dists(const void* lq, int64_t row, int64_t D, const float* cent,
                                            const int (&k)[NC], int lane, double (&out)[NC]) {
    constexpr int EPL = BF16 ? 8 : 4;
    double s[NC];
#pragma unroll
    for (int c = 0; c < NC; c++) s[c] = 0.0;
    const unsigned char* xrow = (const unsigned char*)lq + row * D * (BF16 ? 2 : 4);
    for (int64_t j0 = (int64_t)lane * EPL; j0 < D; j0 += 2 * kWave * EPL) {
        const int64_t j1 = j0 + kWave * EPL;
        const bool two = j1 < D;
        const int64_t j[2] = {j0, two ? j1 : j0};
        u32x4 xv[2];
        f32x4 cv[2][NC][BF16 ? 2 : 1];
#pragma unroll
        for (int u = 0; u < 2; u++) {
            xv[u] = *(const u32x4*)(xrow + j[u] * (BF16 ? 2 : 4));
#pragma unroll
            for (int c = 0; c < NC; c++) {
                const float* cr = cent + (int64_t)k[c] * D + j[u];
                cv[u][c][0] = *(const f32x4*)cr;
                if (BF16) cv[u][c][BF16 ? 1 : 0] = *(const f32x4*)(cr + 4);
            }
        }
#pragma unroll
        for (int u = 0; u < 2; u++) {
            if (u == 1 && !two) break;
            float x[EPL];
#pragma unroll
            for (int e = 0; e < 4; e++) {
                if (BF16) {
                    x[2 * e] = lo_half(xv[u][e]);
                    x[2 * e + 1] = hi_half(xv[u][e]);
                } else {
                    x[e] = __uint_as_float(xv[u][e]);
                }
            }
#pragma unroll
            for (int c = 0; c < NC; c++)
#pragma unroll
                for (int e = 0; e < EPL; e++) {
                    const double d = (double)x[e] - (double)cv[u][c][e >> 2][e & 3];
                    s[c] = fma(d, d, s[c]);
                }
        }
    }
#pragma unroll
    for (int c = 0; c < NC; c++) out[c] = wave_sum(s[c]);
}

// One chunk (128 channels) of the tile as loaded: per MFMA step s, lane (n, g) holds 8 channels of
// row n out of 128 c + 32 s .. + 31: 8 g .. 8 g + 7 in one 16-byte load (bf16), or 4 g .. 4 g + 3 and
// 16 + 4 g .. 16 + 4 g + 3 in two (fp32); see operand_slot.
template <bool BF16>
struct ChunkRegs {
    u32x4 v[BF16 ? 4 : 8];
    int prev;     // previous assignment of row n (assignment passes only)
    u32x4 prevv;  // several sets: previous assignments of row n in the sets 4 g .. 4 g + 3
    int row;      // listed rows: the number of row n
    float2 carry; // split clusters: (best score, its cluster as int bits) of row n in the clusters ranked before
};

// Rows past N repeat the last row and channel groups past D read the start of the row (valid
// addresses either way), so no load is conditional; the consumer masks the padding channels
// (masking here would make the loads wait where they are issued).  D is a multiple of 4 (fp32)
// or 8 (bf16): rows are 16-byte aligned and a 16-byte group is valid or padding as a whole.
// With PREV the row's previous assignment rides along with every chunk: fetched inside the
// tile's finishing code it would have to be waited for there, and since loads return in order
// that wait would also drain the chunks requested ahead.
// LISTED: the tile's rows are not consecutive; lrow is the number of the row this lane loads (already clamped).
template <bool BF16, int PREV, bool LISTED = false>  // PREV: 0 none, 1 the row's previous assignment, 2 its previous assignments in all sets, 3 as 1 plus the carried pair of a split ranking
__device__ __forceinline__ void load_chunk(ChunkRegs<BF16>& r, const TileParams& p, int tile, int chunk, int lane, int lrow = 0) {
    const int n = lane & 15, g = lane >> 4;
    int64_t row;
    if (LISTED) {
        row = lrow;
        r.row = lrow;
    } else {
        const int64_t row0 = (int64_t)(p.reverse ? (int)p.ntiles - 1 - tile : tile) * kRows;
        const int nv = (p.N - row0) < kRows ? (int)(p.N - row0) : kRows;
        row = row0 + (n < nv ? n : nv - 1);
    }
    const int ch = chunk * kChunk + 8 * g;
    if (PREV == 1 || PREV == 3) r.prev = p.assign[row];
    if (PREV == 3 && p.carry_in) r.carry = p.carry_in[row];
    if (PREV == 2) r.prevv = *(const u32x4*)(p.assign + row * 16 + 4 * g);
    if (BF16) {
        const bf16_t* x = (const bf16_t*)p.lq + row * p.D;
#pragma unroll
        for (int s = 0; s < 4; s++) {
            const int c = ch + 32 * s;
            r.v[s] = *(const u32x4*)(x + (c < p.D ? c : 0));
        }
    } else {
        const float* x = (const float*)p.lq + row * p.D;
        const int chf = chunk * kChunk + 4 * g;  // see operand_slot
#pragma unroll
        for (int s = 0; s < 4; s++) {
            const int c = chf + 32 * s;
            r.v[2 * s] = *(const u32x4*)(x + (c < p.D ? c : 0));
            r.v[2 * s + 1] = *(const u32x4*)(x + (c + 16 < p.D ? c + 16 : 0));
        }
    }
}

// The 4 MFMA steps of one chunk against the centroid operand in LDS.  nrm accumulates the
// lane's share of |x|^2 of row n.
template <int KT, int PASSES, bool BF16>
__device__ __forceinline__ void contract_chunk(const ChunkRegs<BF16>& r, f32x4 (&acc)[KT], float& nrm,
                                               const unsigned char* ldsA_chunk, int lane, int chunk, int64_t D) {
    constexpr int P = PASSES == 1 ? 1 : 2;
    const int ch = chunk * kChunk + 8 * (lane >> 4);
#pragma unroll
    for (int s = 0; s < 4; s++) {
        const int c = ch + 32 * s;
        bf16x8 bh, bl;
        if (BF16) {
            u32x4 w = r.v[s];
            const uint32_t m = c < D ? 0xFFFFFFFFu : 0u;
            w.x &= m; w.y &= m; w.z &= m; w.w &= m;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                const float x0 = lo_half(w[j]), x1 = hi_half(w[j]);
                nrm = fmaf(x0, x0, fmaf(x1, x1, nrm));
            }
            bh = __builtin_bit_cast(bf16x8, w);
        } else {
            const int cf = chunk * kChunk + 4 * (lane >> 4) + 32 * s;  // see operand_slot
            const uint32_t m0 = cf < D ? 0xFFFFFFFFu : 0u, m1 = cf + 16 < D ? 0xFFFFFFFFu : 0u;
            float x[8];
#pragma unroll
            for (int j = 0; j < 4; j++) {
                x[j] = __uint_as_float(r.v[2 * s][j] & m0);
                x[4 + j] = __uint_as_float(r.v[2 * s + 1][j] & m1);
            }
            u32x4 h, l;
#pragma unroll
            for (int j = 0; j < 4; j++) {
                nrm = fmaf(x[2 * j], x[2 * j], fmaf(x[2 * j + 1], x[2 * j + 1], nrm));
                h[j] = pack_bf16(x[2 * j], x[2 * j + 1]);
                if (PASSES == 3) l[j] = pack_bf16(x[2 * j] - lo_half(h[j]), x[2 * j + 1] - hi_half(h[j]));
            }
            bh = __builtin_bit_cast(bf16x8, h);
            if (PASSES == 3) bl = __builtin_bit_cast(bf16x8, l);
        }
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
            // keep at most four cluster tiles of operand reads in registers at a time
            if (KT > 4 && (t & 3) == 3) __builtin_amdgcn_sched_barrier(0);
        }
    }
}

// Rank the centroids of the 16 rows from the accumulated dot products; exact re-rank of
// the rows inside the error bound.  On return every lane (n, *) holds row n's result.
// (t0, t1: the cluster tiles that take part, wave-uniform; all of them unless several sets share the kernel)
// myrow: the number of row n (lanes of q = 0 at least), valid: whether it exists.  first / second / reranked / bound
// (optional outputs): the best score, the best among the other centroids, whether the row goes through the exact
// re-rank, and the threshold of that decision.
// DEFER (with queue, the LDS queue, and prev, lane n's previous assignment of row n): such a row is queued instead,
// if the queue has room and the row at most kQueueCand candidates, and *deferred says so for row n.
template <int KT, bool BF16, bool DEFER = false>
__device__ __forceinline__ void rank_rows(const TileParams& p, const f32x4 (&acc)[KT], const float* s_cnorm,
                                          float xn2, float cmax, int64_t myrow, bool valid, int lane, int& idx, float& dmin,
                                          int t0 = 0, int t1 = KT, float* first = nullptr, float* second = nullptr,
                                          bool* reranked = nullptr, float* bound = nullptr, int k_base = 0,
                                          bool has_carry = false, float carry_s = 0.f, int carry_i = 0,
                                          unsigned char* queue = nullptr, int prev = -1, bool* deferred = nullptr,
                                          int k_last = -1) {
    const int n = lane & 15, q = lane >> 4;
    float b1 = __builtin_inff(), b2 = __builtin_inff();
    int i1 = 16 * t0;
#pragma unroll
    for (int t = 0; t < KT; t++) {
        if (t < t0 || t >= t1) continue;
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
    {
        // A slot past the last cluster (k_last; p.K - 1 unless given) holds no centroid and a huge norm: it can only
        // win when every real score is non-finite.  The label stays a cluster number whatever the input.
        const int kl = k_last >= 0 ? k_last : p.K - 1;
        i1 = i1 < kl ? i1 : kl;
    }
    i1 += k_base;
    if (has_carry) {
        // the clusters ranked by the launch before count as one more cluster: its score is the best score there, its
        // index the exact nearest centroid there (lower than every index here, so it wins an equal score)
        if (carry_s <= b1) {
            b2 = b1;
            b1 = carry_s;
            i1 = carry_i;
        } else if (carry_s < b2) {
            b2 = carry_s;
        }
    }
    const float T = p.tau * sqrtf(xn2) * cmax + p.tau2 * cmax * cmax;
    const bool flag = valid && !(b2 - b1 > T);
    if (first) *first = b1;
    if (second) *second = b2;
    if (reranked) *reranked = flag;
    if (bound) *bound = T;
    dmin = fmaxf(xn2 + b1, 0.f);
    unsigned long long mask = __ballot(flag && q == 0);
    while (mask) {
        const int r = __builtin_amdgcn_readfirstlane(__builtin_ctzll(mask));
        mask &= mask - 1;
        const float thr = readlane_f(b1, r) + readlane_f(T, r);
        const int64_t row = ((int64_t)__builtin_amdgcn_readlane((int)(myrow >> 32), r) << 32) |
                            (int64_t)(uint32_t)__builtin_amdgcn_readlane((int)myrow, r);
        double dbest = __builtin_inf();
        int kbest = 0x7fffffff;
        // the candidates (scores within the bound of the best) are listed first, one per lane (entry c in lane
        // c mod 64 of register c / 64: every cluster of the pass may be one), then measured two at a time: the
        // usual case is exactly two
        constexpr int NCR = (KT * 16 + kWave) / kWave;
        int cand[NCR];
#pragma unroll
        for (int j = 0; j < NCR; j++) cand[j] = 0;
        int cnt = 0;
        auto add = [&](int k) {
#pragma unroll
            for (int j = 0; j < NCR; j++)
                if ((cnt >> 6) == j && lane == (cnt & (kWave - 1))) cand[j] = k;
            ++cnt;
        };
        auto get = [&](int c) -> int {  // c is wave-uniform
            int v = cand[0];
#pragma unroll
            for (int j = 1; j < NCR; j++) v = (c >> 6) == j ? cand[j] : v;
            return __builtin_amdgcn_readlane(v, c & (kWave - 1));
        };
        auto measure = [&]() {
            for (int c0 = 0; c0 < cnt; c0 += 2) {
                const int k0 = get(c0);
                if (c0 + 1 < cnt) {
                    const int kk[2] = {k0, get(c0 + 1)};
                    double d[2];
                    exact_dists<BF16, 2>(p.lq, row, p.D, p.cent, kk, lane, d);
#pragma unroll
                    for (int c = 0; c < 2; c++)
                        if (d[c] < dbest || (d[c] == dbest && kk[c] < kbest)) {
                            dbest = d[c];
                            kbest = kk[c];
                        }
                } else {
                    const int kk[1] = {k0};
                    double d[1];
                    exact_dists<BF16, 1>(p.lq, row, p.D, p.cent, kk, lane, d);
                    if (d[0] < dbest || (d[0] == dbest && k0 < kbest)) {
                        dbest = d[0];
                        kbest = k0;
                    }
                }
            }
        };
        if (has_carry && readlane_f(carry_s, r) <= thr) {
            add(__builtin_amdgcn_readlane(carry_i, r));
        }
#pragma unroll
        for (int t = 0; t < KT; t++) {
            if (t < t0 || t >= t1) continue;
#pragma unroll
            for (int i = 0; i < 4; i++) {
                float s = fmaf(-2.f, acc[t][i], s_cnorm[16 * t + 4 * q + i]);
                unsigned long long m = __ballot(n == r && s <= thr);
                while (m) {
                    const int l = __builtin_amdgcn_readfirstlane(__builtin_ctzll(m));
                    m &= m - 1;
                    const int k = 16 * t + 4 * (l >> 4) + i;
                    if (k < p.K) add(k + k_base);
                }
            }
        }
        if (DEFER && p.queue_cap > 0 && cnt >= 1 && cnt <= kQueueCand) {
            int pos = 0;
            if (lane == 0) pos = atomicAdd((int*)queue, 1);
            pos = __builtin_amdgcn_readfirstlane(pos);
            if (pos < p.queue_cap) {
                DeferredRow* e = (DeferredRow*)(queue + 16) + pos;
                if (lane < cnt) e->cand[lane] = (short)cand[0];
                const int pv = __builtin_amdgcn_readlane(prev, r);
                if (lane == 0) {
                    e->row = row;
                    e->prev = pv;
                    e->ncand = cnt;
                }
                if (n == r) *deferred = true;
                continue;
            }
        }
        measure();
        if (n == r && kbest != 0x7fffffff) {
            i1 = kbest;
            dmin = (float)dbest;
        }
    }
    idx = i1;
}

// A queued row, measured by one wave: the exact nearest centroid among its candidates and the bookkeeping of the pass
// for that row (what finish_tile does for the rows ranked on the spot), by lane 0.
template <bool BF16>
__device__ __forceinline__ void finish_deferred(const TileParams& p, unsigned char* smem, const DeferredRow& e, int lane,
                                                double& in_acc) {
    double dbest = __builtin_inf();
    int kbest = 0x7fffffff;
    const int nc = __builtin_amdgcn_readfirstlane(e.ncand);
    const int64_t row = ((int64_t)__builtin_amdgcn_readfirstlane((int)(e.row >> 32)) << 32) |
                        (int64_t)(uint32_t)__builtin_amdgcn_readfirstlane((int)e.row);
    for (int c0 = 0; c0 < nc; c0 += 2) {
        const int k0 = __builtin_amdgcn_readfirstlane((int)e.cand[c0]);
        if (c0 + 1 < nc) {
            const int kk[2] = {k0, __builtin_amdgcn_readfirstlane((int)e.cand[c0 + 1])};
            double d[2];
            exact_dists<BF16, 2>(p.lq, row, p.D, p.cent, kk, lane, d);
#pragma unroll
            for (int c = 0; c < 2; c++)
                if (d[c] < dbest || (d[c] == dbest && kk[c] < kbest)) {
                    dbest = d[c];
                    kbest = kk[c];
                }
        } else {
            const int kk[1] = {k0};
            double d[1];
            exact_dists<BF16, 1>(p.lq, row, p.D, p.cent, kk, lane, d);
            if (d[0] < dbest || (d[0] == dbest && k0 < kbest)) {
                dbest = d[0];
                kbest = k0;
            }
        }
    }
    if (lane != 0) return;
    if (kbest == 0x7fffffff) kbest = (int)e.cand[0];  // no distance compares (non-finite input): any listed cluster
    int* s_hist = (int*)(smem + p.off_hist);
    unsigned long long* s_rep = (unsigned long long*)(smem + p.off_rep);
    int* s_misc = (int*)(smem + p.off_misc);
    p.assign[row] = kbest;
    if (p.counts) atomicAdd(&s_hist[kbest], 1);
    if (p.rep) atomicMin(&s_rep[kbest], (unsigned long long)row);
    in_acc += (double)(float)dbest;
    if (p.list && e.prev != kbest) {
        const unsigned long long entry =
            ((unsigned long long)row << 24) | ((unsigned long long)(e.prev + 1) << 12) | (unsigned long long)kbest;
        const int pos = atomicAdd(&s_misc[0], 1);
        if (pos < p.list_cap)
            ((unsigned long long*)(smem + p.off_list))[pos] = entry;
        else
            p.list[atomicAdd(p.list_count, 1u)] = entry;
    }
}

// Per-tile finishing work of the streaming modes: rank, write, book-keep; resets acc / nrm.
// BOUNDS: the pass also leaves the row's distance bound (TileParams::expire); with listed rows (row_in >= 0 is the
// number of row n, n_listed their count) the tile is 16 entries of the list instead of 16 consecutive rows.
// SPLIT: the clusters of the pass are ranked by two launches (TileParams::carry_in / carry_out).
template <int KT, bool BF16, int MODE, bool BOUNDS = false, bool SPLIT = false>
__device__ __forceinline__ void finish_tile(const TileParams& p, unsigned char* smem, f32x4 (&acc)[KT], float& nrm,
                                            int tile, int lane, float cmax, double& in_acc, int prev_in, int row_in = -1,
                                            uint32_t n_listed = 0, double gnow = 0.0, float2 carry = float2{0.f, 0.f}) {
    const int n = lane & 15, q = lane >> 4;
    const bool listed = BOUNDS && p.rows != nullptr;
    const int64_t row0 = BOUNDS ? 0 : (int64_t)(p.reverse ? (int)p.ntiles - 1 - tile : tile) * kRows;
    const int64_t myrow = BOUNDS ? (int64_t)row_in : row0 + n;  // (BOUNDS: the clamped row the lane loaded)
    const bool valid = listed ? (uint32_t)(tile * kRows + n) < n_listed
                              : (BOUNDS ? (int64_t)(p.reverse ? (int)p.ntiles - 1 - tile : tile) * kRows + n < p.N : myrow < p.N);
    const float* s_cnorm = (const float*)(smem + p.off_cnorm);
    float xn2 = nrm;
    xn2 += __shfl_xor(xn2, 16, kWave);
    xn2 += __shfl_xor(xn2, 32, kWave);
    int idx;
    float dmin, first = 0.f, second = 0.f, bound = 0.f;
    bool reranked = false, deferred = false;
    constexpr bool DEFER = !BOUNDS && !SPLIT && MODE == MODE_ASSIGN;
    const int prev = p.delta_mode ? prev_in : -1;
    if (DEFER)
        rank_rows<KT, BF16, true>(p, acc, s_cnorm, xn2, cmax, myrow, valid, lane, idx, dmin, 0, KT, nullptr, nullptr, nullptr,
                                  nullptr, 0, false, 0.f, 0, smem + p.off_queue, prev, &deferred);
    else if (SPLIT)
        rank_rows<KT, BF16>(p, acc, s_cnorm, xn2, cmax, myrow, valid, lane, idx, dmin, 0, KT, &first, nullptr, nullptr, nullptr,
                            p.k_base, p.carry_in != nullptr, carry.x, __float_as_int(carry.y));
    else
        rank_rows<KT, BF16>(p, acc, s_cnorm, xn2, cmax, myrow, valid, lane, idx, dmin, 0, KT, BOUNDS ? &first : nullptr,
                            BOUNDS ? &second : nullptr, BOUNDS ? &reranked : nullptr, BOUNDS ? &bound : nullptr);
#pragma unroll
    for (int t = 0; t < KT; t++) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    nrm = 0.f;
    const bool owner = q == 0 && valid && !deferred;
    if (SPLIT && p.carry_out) {  // the first of the two launches: hand the pair on, nothing else
        if (owner) p.carry_out[myrow] = float2{first, __int_as_float(idx)};
        return;
    }

    if (MODE == MODE_APPLY) {
        // The affine map walks the 16 rows again, this time one row per instruction with the
        // lanes side by side over the channels (16 bytes each): the row was fetched a moment ago and
        // comes from L2, its cluster id is wave-uniform, so the gamma / beta rows are scalar-addressed
        // and everything is coalesced.  Four rows (fp32; two for bf16) are in flight at a time: 24
        // independent 16-byte loads per lane.
        if (p.assign && owner) p.assign[row0 + n] = idx;
        const int nv = (p.N - row0) < kRows ? (int)(p.N - row0) : kRows;
        constexpr int EPL = BF16 ? 8 : 4;  // elements per lane per load
        constexpr int RB = BF16 ? 2 : 4;   // rows in flight (bf16 rows need two gamma and two beta loads per x load)
        typedef typename std::conditional<BF16, bf16_t, float>::type T;
#pragma unroll 1
        for (int i0 = 0; i0 < kRows; i0 += RB) {
            // row pointers are wave-uniform (scalar registers).  Rows past the end repeat the last row and
            // channels past D repeat channel 0: those lanes recompute and store again exactly what the
            // owning lanes store, so neither the loads nor the stores are conditional
            const T* xr[RB];
            const float* gr[RB];
            const float* br[RB];
            T* orow[RB];
#pragma unroll
            for (int u = 0; u < RB; u++) {
                const int iu = i0 + u < nv ? i0 + u : nv - 1;
                const int a = __builtin_amdgcn_readfirstlane(__shfl(idx, iu, kWave));
                xr[u] = (const T*)p.lq + (row0 + iu) * p.D;
                orow[u] = (T*)p.out + (row0 + iu) * p.D;
                gr[u] = p.gamma + (int64_t)a * p.D;
                br[u] = p.beta + (int64_t)a * p.D;
            }
#pragma unroll 1
            for (int cb = 0; cb < p.D; cb += 2 * EPL * kWave) {
                int o[2];
#pragma unroll
                for (int j = 0; j < 2; j++) {
                    const int ch = cb + (j * kWave + lane) * EPL;
                    o[j] = ch < p.D ? ch : 0;
                }
                u32x4 xv[RB][2];
                f32x4 gv[RB][2][BF16 ? 2 : 1], bv[RB][2][BF16 ? 2 : 1];
#pragma unroll
                for (int u = 0; u < RB; u++)
#pragma unroll
                    for (int j = 0; j < 2; j++) {
                        xv[u][j] = *(const u32x4*)(xr[u] + o[j]);
                        gv[u][j][0] = *(const f32x4*)(gr[u] + o[j]);
                        bv[u][j][0] = *(const f32x4*)(br[u] + o[j]);
                        if (BF16) {
                            gv[u][j][1] = *(const f32x4*)(gr[u] + o[j] + 4);
                            bv[u][j][1] = *(const f32x4*)(br[u] + o[j] + 4);
                        }
                    }
#pragma unroll
                for (int u = 0; u < RB; u++)
#pragma unroll
                    for (int j = 0; j < 2; j++) {
                        u32x4 r;
                        if (BF16) {
                            const f32x4 g0 = gv[u][j][0], g1 = gv[u][j][BF16 ? 1 : 0], b0 = bv[u][j][0], b1 = bv[u][j][BF16 ? 1 : 0];
                            const u32x4 w = xv[u][j];
                            r.x = pack_bf16(fmaf(g0.x, lo_half(w.x), b0.x), fmaf(g0.y, hi_half(w.x), b0.y));
                            r.y = pack_bf16(fmaf(g0.z, lo_half(w.y), b0.z), fmaf(g0.w, hi_half(w.y), b0.w));
                            r.z = pack_bf16(fmaf(g1.x, lo_half(w.z), b1.x), fmaf(g1.y, hi_half(w.z), b1.y));
                            r.w = pack_bf16(fmaf(g1.z, lo_half(w.w), b1.z), fmaf(g1.w, hi_half(w.w), b1.w));
                        } else {
                            const f32x4 g = gv[u][j][0], b = bv[u][j][0];
                            r.x = __float_as_uint(fmaf(g.x, __uint_as_float(xv[u][j].x), b.x));
                            r.y = __float_as_uint(fmaf(g.y, __uint_as_float(xv[u][j].y), b.y));
                            r.z = __float_as_uint(fmaf(g.z, __uint_as_float(xv[u][j].z), b.z));
                            r.w = __float_as_uint(fmaf(g.w, __uint_as_float(xv[u][j].w), b.w));
                        }
                        __builtin_nontemporal_store(r, (u32x4*)(orow[u] + o[j]));
                    }
            }
        }
        return;
    }

    // assign / lloyd bookkeeping (lanes 0..15 own one row each)
    int* s_hist = (int*)(smem + p.off_hist);
    unsigned long long* s_rep = (unsigned long long*)(smem + p.off_rep);
    int* s_misc = (int*)(smem + p.off_misc);
    if (owner) {
        p.assign[myrow] = idx;
        if (p.counts) atomicAdd(&s_hist[idx], 1);
        if (p.rep) atomicMin(&s_rep[idx], (unsigned long long)myrow);
        in_acc += (double)dmin;
    }
    if (BOUNDS && p.expire && owner) {
        // How far the centroids may drift before this row's nearest centroid can change: with e the error bound of
        // a score (the re-rank threshold, which bounds a difference of two scores, plus the rounding of |x|^2), the
        // nearest centroid is at most sqrt(|x|^2 + s1 + e) away and every other at least sqrt(|x|^2 + s2 - e).  A row
        // that was re-ranked has two centroids within the bound of each other: no margin.  No second centroid
        // (s2 = inf): never again.
        double m = 0.0;
        if (!reranked) {
            const double e = (double)bound + (double)xn2 * (double)p.D * 1.5e-8;
            const double hi1 = (double)xn2 + (double)first + e;
            const double lo2 = (double)xn2 + (double)second - e;
            if (lo2 > hi1) m = (sqrt(lo2) - sqrt(hi1 > 0.0 ? hi1 : 0.0)) * (1.0 - 1e-9);
        }
        p.expire[myrow] = gnow + m;
    }
    if (p.list) {
        // rows that changed cluster: into the workgroup's LDS list; when that is full, straight to
        // the global list (one reservation per tile)
        const bool changed = owner && prev != idx;
        const unsigned long long entry =
            ((unsigned long long)myrow << 24) | ((unsigned long long)(prev + 1) << 12) | (unsigned long long)idx;
        bool ovf = false;
        if (changed) {
            int pos = atomicAdd(&s_misc[0], 1);
            if (pos < p.list_cap)
                ((unsigned long long*)(smem + p.off_list))[pos] = entry;
            else
                ovf = true;
        }
        const unsigned long long om = __ballot(ovf);
        if (om) {
            uint32_t base = 0;
            if (lane == 0) base = atomicAdd(p.list_count, (uint32_t)__builtin_popcountll(om));
            base = __builtin_amdgcn_readfirstlane(base);
            if (ovf) p.list[base + __builtin_popcountll(om & ((1ull << lane) - 1ull))] = entry;
        }
    }
}

// Several centroid sets side by side (assignment passes of a fit for a grid of cluster counts): the same finishing
// work once per set, over that set's cluster tiles.  The previous assignments of the row in the sets 4 g .. 4 g + 3
// came with the chunk loads (prevv); lane (n, s / 4) owns row n in set s: it counts, lists the row if its cluster
// changed, and keeps the new assignment, and the 16 int32 of the row are written back with one 16-byte store per
// lane.  The objective of each set is accumulated in LDS doubles.
template <int KT, bool BF16>
__device__ __forceinline__ void finish_tile_multi(const TileParams& p, unsigned char* smem, f32x4 (&acc)[KT], float& nrm,
                                                  int tile, int lane, float cmax, u32x4 prevv) {
    const int n = lane & 15, q = lane >> 4;
    const int64_t row0 = (int64_t)(p.reverse ? (int)p.ntiles - 1 - tile : tile) * kRows;
    const float* s_cnorm = (const float*)(smem + p.off_cnorm);
    int* s_hist = (int*)(smem + p.off_hist);
    unsigned long long* s_rep = (unsigned long long*)(smem + p.off_rep);
    int* s_misc = (int*)(smem + p.off_misc);
    double* s_inset = (double*)(s_misc + 2) + kMaxWaves;
    float xn2 = nrm;
    xn2 += __shfl_xor(xn2, 16, kWave);
    xn2 += __shfl_xor(xn2, 32, kWave);
    const bool valid = row0 + n < p.N;
    u32x4 newa = prevv;
#pragma unroll 1
    for (int s = 0; s < p.nsets; s++) {
        int idx;
        float dmin;
        rank_rows<KT, BF16>(p, acc, s_cnorm, xn2, cmax, row0 + n, valid, lane, idx, dmin, (int)p.set_t0[s], (int)p.set_t0[s + 1],
                            nullptr, nullptr, nullptr, nullptr, 0, false, 0.f, 0, nullptr, -1, nullptr,
                            16 * (int)p.set_t0[s] + (int)p.set_k[s] - 1);
        const bool owner = valid && q == (s >> 2);
        const int e = s & 3;
        const int prev = p.delta_mode ? (int)(e == 0 ? prevv.x : e == 1 ? prevv.y : e == 2 ? prevv.z : prevv.w) : -1;
        if (owner) {
            if (e == 0) newa.x = (uint32_t)idx;
            if (e == 1) newa.y = (uint32_t)idx;
            if (e == 2) newa.z = (uint32_t)idx;
            if (e == 3) newa.w = (uint32_t)idx;
            if (p.counts) atomicAdd(&s_hist[idx], 1);
            if (p.rep) atomicMin(&s_rep[idx], (unsigned long long)(row0 + n));
            atomicAdd(&s_inset[s], (double)dmin);
        }
        if (p.list) {
            const bool changed = owner && prev != idx;
            const unsigned long long entry =
                ((unsigned long long)(row0 + n) << 24) | ((unsigned long long)(prev + 1) << 12) | (unsigned long long)idx;
            bool ovf = false;
            if (changed) {
                int pos = atomicAdd(&s_misc[0], 1);
                if (pos < p.list_cap)
                    ((unsigned long long*)(smem + p.off_list))[pos] = entry;
                else
                    ovf = true;
            }
            const unsigned long long om = __ballot(ovf);
            if (om) {
                uint32_t base = 0;
                if (lane == 0) base = atomicAdd(p.list_count, (uint32_t)__builtin_popcountll(om));
                base = __builtin_amdgcn_readfirstlane(base);
                if (ovf) p.list[base + __builtin_popcountll(om & ((1ull << lane) - 1ull))] = entry;
            }
        }
    }
#pragma unroll
    for (int t = 0; t < KT; t++) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    nrm = 0.f;
    if (valid) *(u32x4*)(p.assign + (row0 + n) * 16 + 4 * q) = newa;
}

// ---- the kernel ----------------------------------------------------------------------
// VAR: 0 the plain pass, 1 several centroid sets side by side (finish_tile_multi), 2 a pass that keeps distance
// bounds and may walk a list of rows instead of all of them (TileParams::expire, rows), 3 one of the two launches
// that rank the halves of a large cluster set (TileParams::carry_in, carry_out).
enum { VAR_PLAIN = 0, VAR_MULTI = 1, VAR_BOUNDS = 2, VAR_SPLIT = 3 };
template <int KT, int PASSES, bool BF16, int MODE, bool CA, int VAR = VAR_PLAIN>
__global__ __launch_bounds__(kMaxWaves * kWave) void k_tile(const TileParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr bool MULTI = VAR == VAR_MULTI, BOUNDS = VAR == VAR_BOUNDS, SPLIT = VAR == VAR_SPLIT;
    if (p.skip_when_zero && *p.skip_when_zero == 0u) return;  // uniform over the grid, before any barrier
    const bool listed = BOUNDS && p.rows != nullptr;
    const uint32_t n_listed = listed ? *p.n_rows : 0u;
    const double gnow = (BOUNDS && p.gnow) ? *p.gnow : 0.0;
    if (BOUNDS && p.evaluated_slot && blockIdx.x == 0 && threadIdx.x == 0)
        *p.evaluated_slot = listed ? (int32_t)n_listed : (int32_t)p.N;
    // listed rows: a workgroup none of whose waves has a tile leaves before any barrier
    if (listed && (uint32_t)blockIdx.x * (uint32_t)p.waves * kRows >= n_listed) return;
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);  // wave-uniform: keeps tile math scalar
    constexpr int P = PASSES == 1 ? 1 : 2;
    float* s_cnorm = (float*)(smem + p.off_cnorm);
    int* s_hist = (int*)(smem + p.off_hist);
    unsigned long long* s_rep = (unsigned long long*)(smem + p.off_rep);
    int* s_misc = (int*)(smem + p.off_misc);  // [0] list count, [2..] doubles for the objective

    const int ntiles = listed ? (int)((n_listed + kRows - 1) / kRows) : (int)p.ntiles;
    const int tstride = (int)gridDim.x * p.waves;
    const int tile0 = __builtin_amdgcn_readfirstlane((int)blockIdx.x * p.waves + wave);
    int tl = tile0, cl = 0;  // load cursor
    float cmax_out;
    ChunkRegs<BF16> b0, b1, b2;
    // BOUNDS: the number of the row this lane loads in the tile at the load cursor, and in the tile after it: an
    // entry of the list (requested a whole tile ahead: waiting for it where it is needed would drain the chunks in
    // flight) or, without a list, the tile's own rows.  Either way the chunk loads themselves sit in no branch.
    int lrow = 0, lrow_nx = 0;
    auto tile_row = [&](int tile) -> int {
        if (listed) {
            uint32_t e = (uint32_t)tile * kRows + (uint32_t)(lane & 15);
            e = e < n_listed ? e : n_listed - 1u;  // n_listed > 0 here (the workgroup has a tile)
            return p.rows[e];
        }
        const int64_t row0 = (int64_t)(p.reverse ? ntiles - 1 - tile : tile) * kRows;
        const int nv = (p.N - row0) < kRows ? (int)(p.N - row0) : kRows;
        return (int)row0 + ((lane & 15) < nv ? (lane & 15) : nv - 1);  // (N is below 2^31 in these passes)
    };
    if (BOUNDS) {
        lrow = tile_row(tile0 < ntiles ? tile0 : 0);
        lrow_nx = tile_row(tile0 + tstride < ntiles ? tile0 + tstride : 0);
    }
    // A wave stops requesting rows once its cursor has passed its last tile.  (Requesting them
    // unconditionally, the last tile again, lets the compiler count on two chunks in flight at
    // every wait instead of draining to one; measured, that was 2-5 % slower, not faster.)
#define CAT_ISSUE(buf)                                                                     \
    if (tl < ntiles) {                                                                     \
        if (BOUNDS)                                                                        \
            load_chunk<BF16, 1, true>(buf, p, tl, cl, lane, lrow);                         \
        else                                                                               \
            load_chunk<BF16, MODE == MODE_ASSIGN ? (MULTI ? 2 : SPLIT ? 3 : 1) : 0>(buf, p, tl, cl, lane); \
        if (++cl == p.nchunks) {                                                           \
            cl = 0;                                                                        \
            tl += tstride;                                                                 \
            if (BOUNDS) {                                                                  \
                lrow = lrow_nx;                                                            \
                lrow_nx = tile_row(tl + tstride < ntiles ? tl + tstride : 0);              \
            }                                                                              \
        }                                                                                  \
    }
    // prologue: centroids (operand order) and their norms into LDS.  Returns come back in issue order,
    // so the operand copy goes first, in batches of eight independent loads, then the first two chunks
    // of rows are requested, and only then does anything wait.
    {
        // resident operand: all of it; chunked operand (CA): the first chunk into the first of two buffers
        const u32x4* src = (const u32x4*)p.packA;
        u32x4* dst = (u32x4*)smem;
        const uint32_t nvec = CA ? (uint32_t)(4 * KT * P * 1024 / 16) : p.ldsA_bytes / 16;
        const uint32_t nt = blockDim.x;
        uint32_t i = threadIdx.x;
        u32x4 t[8];
        const bool first = i + 7 * nt < nvec;
        if (first) {
#pragma unroll
            for (int u = 0; u < 8; u++) t[u] = src[i + u * nt];
        }
        float cn_mine = 0.f;
        if ((int)threadIdx.x < p.K16) {
            if (p.norm_slices > 0) {
                double nn = 0.0;
                const size_t nstride = SPLIT ? (size_t)p.norm_stride : (size_t)p.K;
                if ((int)threadIdx.x < p.K) {
                    const double* np = p.norm_part + (SPLIT ? p.k_base : 0) + threadIdx.x;
                    int sl = 0;
                    for (; sl + 8 <= p.norm_slices; sl += 8) {  // eight loads in flight, added in slice order
                        double v[8];
#pragma unroll
                        for (int u = 0; u < 8; u++) v[u] = np[(size_t)(sl + u) * nstride];
#pragma unroll
                        for (int u = 0; u < 8; u++) nn += v[u];
                    }
                    for (; sl < p.norm_slices; sl++) nn += np[(size_t)sl * nstride];
                }
                cn_mine = (int)threadIdx.x < p.K ? (float)nn : kPadNorm;
            } else {
                cn_mine = p.cnorm[threadIdx.x];
            }
        }
        CAT_ISSUE(b0)
        CAT_ISSUE(b1)
        if (first) {
#pragma unroll
            for (int u = 0; u < 8; u++) dst[i + u * nt] = t[u];
            i += 8 * nt;
        }
        for (; i + 7 * nt < nvec; i += 8 * nt) {
#pragma unroll
            for (int u = 0; u < 8; u++) t[u] = src[i + u * nt];
#pragma unroll
            for (int u = 0; u < 8; u++) dst[i + u * nt] = t[u];
        }
        for (; i < nvec; i += nt) dst[i] = src[i];
        if (MULTI && (int)threadIdx.x < p.K) {
            // slots past the clusters of their set hold no centroid
            const int t_ = (int)threadIdx.x >> 4;
            int s_ = 0;
            while (s_ + 1 < p.nsets && t_ >= (int)p.set_t0[s_ + 1]) s_++;
            if ((int)threadIdx.x - 16 * (int)p.set_t0[s_] >= (int)p.set_k[s_]) cn_mine = kPadNorm;
        }
        if ((int)threadIdx.x < p.K16) s_cnorm[threadIdx.x] = cn_mine;
        if (MULTI && threadIdx.x < 16) ((double*)(s_misc + 2) + kMaxWaves)[threadIdx.x] = 0.0;
        for (int k = threadIdx.x; k < (SPLIT ? p.k_hist : p.K); k += blockDim.x) {
            s_hist[k] = 0;
            s_rep[k] = ~0ull;
        }
        if (threadIdx.x == 0) s_misc[0] = 0;
        if (VAR == VAR_PLAIN && MODE == MODE_ASSIGN && p.queue_cap > 0 && threadIdx.x == 0) *(int*)(smem + p.off_queue) = 0;
    }
    __syncthreads();
    {
        float cm2 = 0.f;  // largest centroid norm: every wave reduces the table for itself
        for (int k = lane; k < p.K; k += kWave) {
            const float v = s_cnorm[k];
            cm2 = fmaxf(cm2, (MULTI && v == kPadNorm) ? 0.f : v);
        }
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) cm2 = fmaxf(cm2, __shfl_xor(cm2, o, kWave));
        cmax_out = sqrtf(cm2);
        if (SPLIT) {
            // the error bound of a comparison involves the norms of both shares
            if (p.carry_in) cmax_out = fmaxf(cmax_out, *p.cmax_io);
            if (p.carry_out && blockIdx.x == 0 && threadIdx.x == 0) *p.cmax_io = cmax_out;
        }
    }
    const float cmax = cmax_out;

    double in_acc = 0.0;

    // a three-buffer register pipeline keeps two chunks of loads in flight
    // while a third is contracted; the (tile, chunk) cursors run across tile boundaries
    f32x4 acc[KT];
    float nrm = 0.f;
#pragma unroll
    for (int t = 0; t < KT; t++) acc[t] = (f32x4){0.f, 0.f, 0.f, 0.f};
    int tc = tile0, cc = 0;  // compute cursor
#define CAT_STEP(buf)                                                                                          \
    contract_chunk<KT, PASSES, BF16>(buf, acc, nrm, smem + (size_t)cc * 4 * KT * P * 1024, lane, cc, p.D);     \
    if (++cc == p.nchunks) {                                                                                   \
        if (MULTI)                                                                                             \
            finish_tile_multi<KT, BF16>(p, smem, acc, nrm, tc, lane, cmax, buf.prevv);                         \
        else if (BOUNDS)                                                                                       \
            finish_tile<KT, BF16, MODE, true>(p, smem, acc, nrm, tc, lane, cmax, in_acc, buf.prev, buf.row, n_listed, gnow); \
        else if (SPLIT)                                                                                        \
            finish_tile<KT, BF16, MODE, false, true>(p, smem, acc, nrm, tc, lane, cmax, in_acc, buf.prev, -1, 0, 0.0, buf.carry); \
        else                                                                                                   \
            finish_tile<KT, BF16, MODE>(p, smem, acc, nrm, tc, lane, cmax, in_acc, buf.prev);                  \
        cc = 0;                                                                                                \
        tc += tstride;                                                                                         \
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
        int s = 0;
        // the operand chunk of step s + 2 is requested during step s and written to LDS at the end of
        // step s + 1 (into the buffer step s + 1 does not read), so an operand load has two steps to land
        u32x4 ra[AREG], rb[AREG];
        // Loads and LDS writes are unconditional (a lane past the end of the chunk repeats the last
        // vector, a load past the last step fetches a chunk nobody reads): a conditional load would be
        // waited for on the spot.  The workgroup is always kMaxWaves waves here (checked at launch).
        constexpr int NT = kMaxWaves * kWave, NVEC = chunkA / 16;
        int ca_next = 1 % p.nchunks;  // chunk index of the next operand load
#define CAT_CA_LOAD(reg)                                                                                      \
    {                                                                                                         \
        const u32x4* src_ = (const u32x4*)((const unsigned char*)p.packA + (size_t)ca_next * chunkA);         \
        _Pragma("unroll") for (int i_ = 0; i_ < AREG; i_++) {                                                 \
            const int v_ = i_ * NT + (int)threadIdx.x;                                                        \
            reg[i_] = src_[NVEC % NT == 0 ? v_ : (v_ < NVEC ? v_ : NVEC - 1)];                                \
        }                                                                                                     \
        if (++ca_next == p.nchunks) ca_next = 0;                                                              \
    }
#define CAT_CA_STEP(bufcur, bufnext, regw, regl)                                                              \
    {                                                                                                         \
        CAT_CA_LOAD(regl)                                                                                     \
        CAT_ISSUE(bufnext)                                                                                    \
        if (tc < ntiles) {                                                                                    \
            contract_chunk<KT, PASSES, BF16>(bufcur, acc, nrm, smem + (size_t)(s & 1) * chunkA, lane, cc, p.D); \
            if (++cc == p.nchunks) {                                                                          \
                if (MULTI)                                                                                    \
                    finish_tile_multi<KT, BF16>(p, smem, acc, nrm, tc, lane, cmax, bufcur.prevv);             \
                else if (BOUNDS)                                                                              \
                    finish_tile<KT, BF16, MODE, true>(p, smem, acc, nrm, tc, lane, cmax, in_acc, bufcur.prev, bufcur.row, n_listed, gnow); \
                else if (SPLIT)                                                                               \
                    finish_tile<KT, BF16, MODE, false, true>(p, smem, acc, nrm, tc, lane, cmax, in_acc, bufcur.prev, -1, 0, 0.0, bufcur.carry); \
                else                                                                                          \
                    finish_tile<KT, BF16, MODE>(p, smem, acc, nrm, tc, lane, cmax, in_acc, bufcur.prev);      \
                cc = 0;                                                                                       \
                tc += tstride;                                                                                \
            }                                                                                                 \
        }                                                                                                     \
        {                                                                                                     \
            u32x4* dst_ = (u32x4*)(smem + (size_t)((s + 1) & 1) * chunkA);                                    \
            _Pragma("unroll") for (int i_ = 0; i_ < AREG; i_++) {                                             \
                const int v_ = i_ * NT + (int)threadIdx.x;                                                    \
                dst_[NVEC % NT == 0 ? v_ : (v_ < NVEC ? v_ : NVEC - 1)] = regw[i_];                           \
            }                                                                                                 \
        }                                                                                                     \
        __syncthreads();                                                                                      \
        s++;                                                                                                  \
    }
        CAT_CA_LOAD(rb)
        while (s < nsteps) {
            CAT_CA_STEP(b0, b2, rb, ra)
            if (s >= nsteps) break;
            CAT_CA_STEP(b1, b0, ra, rb)
            if (s >= nsteps) break;
            CAT_CA_STEP(b2, b1, rb, ra)
            if (s >= nsteps) break;
            CAT_CA_STEP(b0, b2, ra, rb)
            if (s >= nsteps) break;
            CAT_CA_STEP(b1, b0, rb, ra)
            if (s >= nsteps) break;
            CAT_CA_STEP(b2, b1, ra, rb)
        }
#undef CAT_CA_LOAD
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

    if (VAR == VAR_PLAIN && p.queue_cap > 0) {
        // the rows whose exact re-rank was put off: shared out over the waves, one row at a time
        __syncthreads();
        const int pushed = *(const int*)(smem + p.off_queue);
        const int qn = pushed < p.queue_cap ? pushed : p.queue_cap;
        const DeferredRow* qe = (const DeferredRow*)(smem + p.off_queue + 16);
        for (int e = wave; e < qn; e += p.waves) finish_deferred<BF16>(p, smem, qe[e], lane, in_acc);
    }

    // workgroup epilogue: counts, first rows, objective
    double* s_in = (double*)(s_misc + 2);
    in_acc = wave_sum(in_acc);
    if (lane == 0) s_in[wave] = in_acc;
    __syncthreads();
    for (int k = threadIdx.x; k < (SPLIT ? p.k_hist : p.K); k += blockDim.x) {
        if (p.counts && s_hist[k]) atomicAdd(&p.counts[k], s_hist[k]);
        if (p.rep && s_rep[k] != ~0ull) atomicMin(&p.rep[k], s_rep[k]);
    }
    if (MULTI) {
        if (p.inertia && (int)threadIdx.x < p.nsets) atomicAdd(p.inertia + threadIdx.x, (s_in + kMaxWaves)[threadIdx.x]);
    } else if (p.inertia && threadIdx.x == 0) {
        double tot = 0.0;
        for (int w = 0; w < p.waves; w++) tot += s_in[w];
        atomicAdd(p.inertia, tot);
    }
    if (!p.list) return;

    // the workgroup's changed rows join the global list: one reservation, then a coalesced copy
    const int cnt = s_misc[0] < p.list_cap ? s_misc[0] : p.list_cap;
    if (cnt == 0) return;  // uniform: s_misc[0] is final after the barrier above
    if (threadIdx.x == 0) s_misc[1] = (int)atomicAdd(p.list_count, (uint32_t)cnt);
    __syncthreads();
    const uint32_t base = (uint32_t)s_misc[1];
    const unsigned long long* l_ent = (const unsigned long long*)(smem + p.off_list);
    for (int i = threadIdx.x; i < cnt; i += blockDim.x) p.list[base + i] = l_ent[i];
}

// ---- variant chosen on the host (cat_tile.hip: tile_config) ------------------------------------
struct TileCfg {
    bool ok = false;
    int KT = 0, P = 0, waves = 0, nchunks = 0, mode = MODE_ASSIGN;
    bool chunked = false;  // the centroid operand streams through LDS instead of living there
    uint32_t ldsA = 0, off_cnorm = 0, off_hist = 0, off_rep = 0, off_list = 0, off_misc = 0, off_queue = 0;
    int queue_cap = 0;  // entries of the queue of rows whose exact re-rank is put off (0: the layout has no room for one)
    size_t lds_total = 0;
};

template <int KT, int PASSES, bool BF16, int MODE, bool CA, int VAR = VAR_PLAIN>
static inline cat_status launch_one(const TileParams& p, const TileCfg& c, hipStream_t st) {
    auto kern = k_tile<KT, PASSES, BF16, MODE, CA, VAR>;
    if (CA && c.waves != kMaxWaves) {
        return set_error(CAT_ERR_INVALID_ARG, "k_tile: the chunked-operand variant needs %d waves, got %d", kMaxWaves, c.waves);
    }
    CAT_HIP_TRY(hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)c.lds_total));
    // persistent grid: as many workgroups as are resident at once (registers and LDS decide), each
    // walking its share of the tiles; asked from the runtime once per kernel variant, LDS size and device
    static thread_local int cached_lds = -1, cached_dev = -1, cached_per_cu = 1, ncu = 256;
    int dev = 0;
    CAT_HIP_TRY(hipGetDevice(&dev));
    if (cached_lds != (int)c.lds_total || cached_dev != dev) {
        int nb = 0, v = 0;
        CAT_HIP_TRY(hipOccupancyMaxActiveBlocksPerMultiprocessor(&nb, (const void*)kern, c.waves * kWave, c.lds_total));
        CAT_HIP_TRY(hipDeviceGetAttribute(&v, hipDeviceAttributeMultiprocessorCount, dev));
        cached_per_cu = nb < 1 ? 1 : nb;
        ncu = v > 0 ? v : 256;
        cached_lds = (int)c.lds_total;
        cached_dev = dev;
    }
    int64_t want = (p.ntiles + c.waves - 1) / c.waves;
    int64_t cap = (int64_t)ncu * cached_per_cu;
    unsigned blocks = (unsigned)(want < cap ? want : cap);
    const bool prof = profile_on();
    if (prof) {
        cat_status ps = profile_mark(true, st);
        if (ps != CAT_OK) return ps;
    }
    hipLaunchKernelGGL(kern, dim3(blocks), dim3(c.waves * kWave), c.lds_total, st, p);
    CAT_LAUNCH_CHECK("k_tile");
    if (prof) return profile_mark(false, st);
    return CAT_OK;
}

template <int KT, int PASSES, bool BF16>
static inline cat_status launch_mode(const TileParams& p, const TileCfg& c, hipStream_t st) {
    if (c.chunked) {
        if (c.mode == MODE_ASSIGN) return launch_one<KT, PASSES, BF16, MODE_ASSIGN, true>(p, c, st);
        if (c.mode == MODE_APPLY) return launch_one<KT, PASSES, BF16, MODE_APPLY, true>(p, c, st);
    } else {
        if (c.mode == MODE_ASSIGN) return launch_one<KT, PASSES, BF16, MODE_ASSIGN, false>(p, c, st);
        if (c.mode == MODE_APPLY) return launch_one<KT, PASSES, BF16, MODE_APPLY, false>(p, c, st);
    }
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernel: no instance for this mode");
}

template <int KT, bool BF16>
static inline cat_status launch_kt(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return c.P == 2 ? launch_mode<KT, 3, BF16>(p, c, st) : launch_mode<KT, 1, BF16>(p, c, st);
}

// several centroid sets side by side: assignment passes only
template <int KT, bool BF16>
static inline cat_status launch_kt_multi(const TileParams& p, const TileCfg& c, hipStream_t st) {
    if (c.chunked)
        return c.P == 2 ? launch_one<KT, 3, BF16, MODE_ASSIGN, true, VAR_MULTI>(p, c, st)
                        : launch_one<KT, 1, BF16, MODE_ASSIGN, true, VAR_MULTI>(p, c, st);
    return c.P == 2 ? launch_one<KT, 3, BF16, MODE_ASSIGN, false, VAR_MULTI>(p, c, st)
                    : launch_one<KT, 1, BF16, MODE_ASSIGN, false, VAR_MULTI>(p, c, st);
}

// assignment passes that keep distance bounds (two-part operand only)
template <int KT, bool BF16>
static inline cat_status launch_kt_bounds(const TileParams& p, const TileCfg& c, hipStream_t st) {
    if (c.P != 2) return set_error(CAT_ERR_UNSUPPORTED, "tile kernel with distance bounds: two-part operand only");
    if (c.chunked) return launch_one<KT, 3, BF16, MODE_ASSIGN, true, VAR_BOUNDS>(p, c, st);
    return launch_one<KT, 3, BF16, MODE_ASSIGN, false, VAR_BOUNDS>(p, c, st);
}

// one of the two launches over the halves of a large cluster set (8 cluster tiles each, two-part operand)
template <bool BF16>
static inline cat_status launch_split(const TileParams& p, const TileCfg& c, hipStream_t st) {
    if (c.KT != 8 || c.P != 2) return set_error(CAT_ERR_UNSUPPORTED, "split ranking: 8 cluster tiles and the two-part operand only");
    if (c.chunked) return launch_one<8, 3, BF16, MODE_ASSIGN, true, VAR_SPLIT>(p, c, st);
    return launch_one<8, 3, BF16, MODE_ASSIGN, false, VAR_SPLIT>(p, c, st);
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
// the instantiations for several centroid sets: cat_tile_multi_<dtype>.hip
cat_status launch_multi_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_multi_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);
// the instantiations for the halves of a large cluster set: cat_tile_split.hip
cat_status launch_split_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_split_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);
// the instantiations that keep distance bounds: cat_tile_bounds_<dtype>.hip
cat_status launch_bounds_f32(const TileParams& p, const TileCfg& c, hipStream_t st);
cat_status launch_bounds_bf16(const TileParams& p, const TileCfg& c, hipStream_t st);

}  // namespace cat
