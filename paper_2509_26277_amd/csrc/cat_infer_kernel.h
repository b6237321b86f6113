// Fused CAT Inferencing (Algorithm 2: nearest centroid, then that cluster's affine map) that reads every row
// from memory once.
//
// A workgroup of 8 waves owns a tile of 16 * RGT rows.  Each wave
//   - loads its 2 * RGT rows of the tile with coalesced 16-byte loads and KEEPS them in registers as loaded
//     (the affine map and the exact re-rank work on these registers, so the rows are never fetched again);
//   - writes them once to LDS as bf16 (fp32 rows: a hi part and, with two-part centroids, a lo part), row-major,
//     which is the B-operand layout of v_mfma_f32_16x16x32_bf16: lane (n, g) reads the 8 channels 32 s + 8 g ..
//     of row n with one 16-byte LDS read, no conversion in the contraction;
//   - holds ITS share of the centroid operand in registers for the whole launch: the 8 waves split the cluster
//     tiles (S_k ways) and the channels (S_c ways, S_k * S_c = 8), so LDS carries only the row tile;
//   - contracts all rows of the tile against its share, leaves the partial dot products in LDS;
//   - ranks the centroids of its own rows from the partial products (summed in a fixed order), re-ranks the rows
//     inside the error bound of the split arithmetic with direct-form double-precision distances (same rule as
//     the tile kernel: the exact nearest centroid, lowest index on ties), applies gamma / beta and stores.
// Two barriers per tile: rows staged -> contraction -> scores complete -> ranking.  The rows of the following two or
// three tiles are on their way at any time (one register buffer each, rotating by name), the gamma / beta rows of
// this tile during the contraction of the next.
#pragma once
#include <type_traits>

#include "cat_tile.h"

namespace cat {

typedef __attribute__((ext_vector_type(8))) __bf16 ibf16x8;
typedef __attribute__((ext_vector_type(2))) __bf16 ibf16x2;
typedef __attribute__((ext_vector_type(2))) float if32x2;
typedef __attribute__((ext_vector_type(4))) float if32x4;
typedef __attribute__((ext_vector_type(4))) uint32_t iu32x4;
typedef __attribute__((ext_vector_type(2))) uint32_t iu32x2;

constexpr int kInferWaves = 8;
// row stride (floats) of the partial dot products in LDS for a row of n floats: n rounded up to 16 mod 64
constexpr int infer_dots_stride(int n) { return n + (16 - n % 64 + 64) % 64; }

struct InferParams {
    const void* lq;
    void* out;        // nullable: nothing is written (assignment only; gamma / beta must still be readable K x D arrays)
    int32_t* assign;  // nullable
    double* inertia;  // nullable: the sum of the squared distances to the assigned centroids is added here
    int64_t N, D, ntiles;
    int32_t K, KT;        // clusters; cluster tiles of 16 in packA
    int32_t psteps;       // steps present in packA (4 per 128-channel chunk)
    const uint16_t* packA;  // [step][ktile][part][lane][8] bf16, channels of a step in order (8 per lane group)
    const float* cnorm;     // K16 squared norms (padding clusters: huge)
    const float* cent;      // K x D fp32 (exact re-rank)
    const float* gamma;
    const float* beta;
    float tau, tau2;        // re-rank threshold T = tau |x| cmax + tau2 cmax^2
    uint32_t xstride;       // bytes between rows of one bf16 part in LDS
    uint32_t xpart;         // bytes between the hi and the lo part
    uint32_t off_s, off_cnorm;  // LDS: [0, off_s) row tile, then the partial dot products, then the norms
    unsigned int* counters;     // DYN: 8 x 16 words, zero on entry: the next tile of each group of workgroups
    int32_t out_bf16;           // fp32 rows only: the corrected rows are written as bfloat16 (rounded to nearest even)
};

__device__ __forceinline__ uint32_t ipack_bf16(float a, float b) {  // a -> low half, b -> high half, RNE
    if32x2 v = {a, b};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, ibf16x2));
}
__device__ __forceinline__ float ilo_half(uint32_t w) { return __uint_as_float(w << 16); }
__device__ __forceinline__ float ihi_half(uint32_t w) { return __uint_as_float(w & 0xFFFF0000u); }

// Butterfly reductions whose result every lane holds, on the VALU alone: four steps inside the rows of 16 lanes
// (DPP quad swaps, half mirror, mirror), then the rows of a pair and the two halves of the wave are exchanged with
// v_permlane16_swap / v_permlane32_swap.  No LDS traffic, a few cycles per step.
template <typename Op>
__device__ __forceinline__ float wave_all(float v, Op op) {
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0xB1, 0xF, 0xF, true)));   // lanes ^ 1
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x4E, 0xF, 0xF, true)));   // lanes ^ 2
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x141, 0xF, 0xF, true)));  // 7 - lane in each 8
    v = op(v, __int_as_float(__builtin_amdgcn_update_dpp(0, __float_as_int(v), 0x140, 0xF, 0xF, true)));  // 15 - lane in each 16
    auto r = __builtin_amdgcn_permlane16_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    v = op(__uint_as_float(r[0]), __uint_as_float(r[1]));
    auto q = __builtin_amdgcn_permlane32_swap(__float_as_uint(v), __float_as_uint(v), false, false);
    return op(__uint_as_float(q[0]), __uint_as_float(q[1]));
}
// Scores are ranked as integers: key(x) orders like x for all finite floats and infinities (sign-magnitude to two's
// complement), so the minimum steps are v_min_i32 with the DPP lane pattern folded in, one instruction each (a float
// minimum would quiet its operands first).
__device__ __forceinline__ int score_key(float x) {
    const int b = __float_as_int(x);
    return b ^ ((b >> 31) & 0x7fffffff);
}
__device__ __forceinline__ float key_score(int k) { return __int_as_float(k ^ ((k >> 31) & 0x7fffffff)); }
__device__ __forceinline__ int wave_min_all(int v) {
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0xB1, 0xF, 0xF, true));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x4E, 0xF, 0xF, true));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x141, 0xF, 0xF, true));
    v = min(v, __builtin_amdgcn_update_dpp(0, v, 0x140, 0xF, 0xF, true));
    auto r = __builtin_amdgcn_permlane16_swap((unsigned)v, (unsigned)v, false, false);
    v = min((int)r[0], (int)r[1]);
    auto q = __builtin_amdgcn_permlane32_swap((unsigned)v, (unsigned)v, false, false);
    return min((int)q[0], (int)q[1]);
}
__device__ __forceinline__ float wave_sum_all(float v) {
    return wave_all(v, [](float a, float b) { return a + b; });
}

// BF16: dtype of the rows.  KW: cluster tiles per wave.  SC: channel shares (the 8 waves are 8 / SC cluster shares
// times SC channel shares).  SPW: MFMA steps per wave and tile.  P: parts of the centroid operand (2: hi + lo, 1: hi
// only, wider re-rank bound).  RGT: 16-row groups per tile.  VPR: 16-byte vectors per lane and row
// (ceil(D * b / 1024)).  DYN: tiles handed out in order by counters instead of a fixed stride.
// UA: rows that are not whole 16-byte groups (D not a multiple of 4, of 8 for bf16).  Rows, parameters and outputs
// then move in 4-byte words, and word e of vector v of a lane is word 256 v + 64 e + lane of the row instead of word
// 256 v + 4 lane + e: every wave instruction still reads or writes 256 consecutive bytes, and no access is wider than
// its alignment.  Only the addressing differs: on chip a word is a word, whichever channels it holds.
template <bool BF16, int KW, int SC, int SPW, int P, int RGT, int VPR, bool DYN, bool UA = false>
__global__ __launch_bounds__(kInferWaves * kWave) void k_infer(const InferParams p) {
    extern __shared__ __align__(16) unsigned char smem[];
    constexpr int SK = kInferWaves / SC;           // cluster shares
    constexpr int K16 = 16 * KW * SK;              // padded clusters
    constexpr int RPW = 2 * RGT;                   // rows of the tile a wave loads, ranks and writes
    constexpr int ROWS = 16 * RGT;
    constexpr int EPL = BF16 ? 8 : 4;              // channels per 16-byte vector
    constexpr int XP = (!BF16 && P == 2) ? 2 : 1;  // bf16 parts of a row in LDS
    constexpr int NSLOT = (K16 + kWave - 1) / kWave;  // clusters per lane in the ranking
    // Floats between the rows of the partial dot products: SC * K16 plus a skew that leaves the row stride at 16 mod 64.
    // Lane (n, g) writes four floats at 4 g of row n: with a stride that is a multiple of 64 floats all 16 rows would
    // fall on the same 16 banks; at 16 mod 64 every bank is hit exactly four times, the least a 1 KB write can do
    // (bank-conflict cycles per LDS instruction of the whole kernel 4.2 -> 3.1; the kernel's duration does not
    // change, it is bound by the memory system).
    constexpr int DS = infer_dots_stride(SC * K16);
    constexpr int DEPTH = VPR <= 2 ? 3 : 2;        // tiles requested ahead (a register buffer each)
    typedef typename std::conditional<BF16, bf16_t, float>::type T;
    typedef iu32x4 Rows[RPW][VPR];

    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int n = lane & 15, g = lane >> 4;
    const int ik = wave % SK, ic = wave / SK;
    float* s_dots = (float*)(smem + p.off_s);       // [row][SC][K16], rows DS floats apart
    float* s_cnorm = (float*)(smem + p.off_cnorm);

    // ---- prologue: zero the row tile (its padding channels stay zero for good), norms, operand share ----
    for (uint32_t i = threadIdx.x; i < p.off_s / 16; i += blockDim.x) ((iu32x4*)smem)[i] = (iu32x4){0u, 0u, 0u, 0u};
    for (int k = threadIdx.x; k < K16; k += blockDim.x) s_cnorm[k] = p.cnorm[k];
    ibf16x8 A[KW][SPW][P];
#pragma unroll
    for (int kw = 0; kw < KW; kw++)
#pragma unroll
        for (int sl = 0; sl < SPW; sl++)
#pragma unroll
            for (int part = 0; part < P; part++) {
                const int sg = ic * SPW + sl, kt = ik * KW + kw;
                iu32x4 v = {0u, 0u, 0u, 0u};
                if (sg < p.psteps) v = *(const iu32x4*)(p.packA + ((((size_t)sg * p.KT + kt) * P + part) * 64 + lane) * 8);
                A[kw][sl][part] = __builtin_bit_cast(ibf16x8, v);
            }

    // The tiles of this workgroup, numbered j = 0, 1, ...: a fixed stride, or (DYN) handed out in order: workgroup b
    // belongs to group b % 8 and takes the tiles g + 8 c, c from its group's counter; the numbers of the next tiles wait
    // in a small LDS queue, fetched DEPTH + 1 steps ahead.  Tiles in order keep the rows that the whole chip is reading
    // and writing at any moment within a narrow band of memory, which the memory system rewards; the counters cost a
    // launch to clear and a round trip each, so short launches keep the fixed stride.  A tile number past the last
    // tile is harmless to load (its rows are clamped) and ends the loop.
    __shared__ long long s_queue[8];
    const int grp = blockIdx.x & 7;
    auto fetch = [&]() -> long long { return (long long)grp + 8ll * (long long)atomicAdd(p.counters + grp * 16, 1u); };
    if (DYN) {
        if (threadIdx.x <= DEPTH) s_queue[threadIdx.x] = fetch();
        __syncthreads();
    }
    auto tile_at = [&](int64_t j) -> int64_t {
        if (DYN) return __builtin_amdgcn_readfirstlane((int)s_queue[j & 7]);
        return (int64_t)blockIdx.x + j * (int64_t)gridDim.x;
    };
    // per-lane channel of each vector, and whether it exists
    int ch[VPR];
    bool ch_ok[VPR];
#pragma unroll
    for (int v = 0; v < VPR; v++) {
        ch[v] = (v * kWave + lane) * EPL;
        ch_ok[v] = ch[v] < p.D;
    }
    // UA: the row words of this lane, clamped to the last word of the row (no load is conditional), and which exist
    const int Wx = (int)(BF16 ? p.D / 2 : p.D);
    uint32_t wo[UA ? VPR : 1][4];  // as byte offsets (unsigned 32 bits: base in scalar registers + offset per lane)
    int okm[UA ? VPR : 1];
    if (UA) {
#pragma unroll
        for (int v = 0; v < VPR; v++) {
            okm[v] = 0;
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const int wi = v * 4 * kWave + e * kWave + lane;
                wo[v][e] = 4u * (uint32_t)(wi < Wx ? wi : Wx - 1);
                okm[v] |= (wi < Wx ? 1 : 0) << e;
            }
            ch_ok[v] = okm[v] != 0;
        }
    }
    auto word_ok = [&](int v, int e) { return !UA || ((okm[UA ? v : 0] >> e) & 1) != 0; };
    // the fp32 parameters under the words of vector v of a parameter row (centroids, gamma, beta)
    auto load_params = [&](const float* row, int v, if32x4& lo4, if32x4& hi4) {
        if (!UA) {
            const int cc = ch_ok[v] ? ch[v] : 0;
            lo4 = *(const if32x4*)(row + cc);
            if (BF16) hi4 = *(const if32x4*)(row + cc + 4);
        } else if (BF16) {  // two channels per word: D is even, so the pairs are 8-byte aligned
#pragma unroll
            for (int e = 0; e < 4; e++) {
                const if32x2 t = *(const if32x2*)((const unsigned char*)row + 2u * wo[UA ? v : 0][e]);
                if (e < 2) {
                    lo4[2 * e] = t.x;
                    lo4[2 * e + 1] = t.y;
                } else {
                    hi4[2 * e - 4] = t.x;
                    hi4[2 * e - 3] = t.y;
                }
            }
        } else {
#pragma unroll
            for (int e = 0; e < 4; e++) lo4[e] = *(const float*)((const unsigned char*)row + wo[UA ? v : 0][e]);
        }
    };

    // rows of tile number i of this workgroup as loaded (rows past N repeat the last row, vectors past D the first
    // one, a tile number past the last repeats the last: no load is conditional)
    auto load_rows = [&](Rows& G, int64_t i) {
        const int64_t tile = tile_at(i);
#pragma unroll
        for (int r = 0; r < RPW; r++) {
            int64_t row = tile * ROWS + wave * RPW + r;
            row = row < p.N ? row : p.N - 1;
            const T* x = (const T*)p.lq + row * p.D;
#pragma unroll
            for (int v = 0; v < VPR; v++) {
                if (UA) {
#pragma unroll
                    for (int e = 0; e < 4; e++) G[r][v][e] = *(const uint32_t*)((const unsigned char*)x + wo[UA ? v : 0][e]);
                } else {
                    G[r][v] = *(const iu32x4*)(x + (ch_ok[v] ? ch[v] : 0));
                }
            }
        }
    };
    // bf16 copy of the wave's rows into the LDS tile
    auto stage = [&](const Rows& G) {
#pragma unroll
        for (int r = 0; r < RPW; r++) {
            unsigned char* xr = smem + (size_t)(wave * RPW + r) * p.xstride;
#pragma unroll
            for (int v = 0; v < VPR; v++) {
                if (UA) {
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        if (!word_ok(v, e)) continue;
                        const int wi = v * 4 * kWave + e * kWave + lane;
                        if (BF16) {
                            *(uint32_t*)(xr + 4 * wi) = G[r][v][e];
                        } else {
                            const float x0 = __uint_as_float(G[r][v][e]);
                            const uint32_t h = ipack_bf16(x0, 0.f);
                            *(uint16_t*)(xr + 2 * wi) = (uint16_t)h;
                            if (XP == 2) *(uint16_t*)(xr + p.xpart + 2 * wi) = (uint16_t)ipack_bf16(x0 - ilo_half(h), 0.f);
                        }
                    }
                } else if (ch_ok[v]) {
                    if (BF16) {
                        *(iu32x4*)(xr + ch[v] * 2) = G[r][v];
                    } else {
                        const float x0 = __uint_as_float(G[r][v].x), x1 = __uint_as_float(G[r][v].y);
                        const float x2 = __uint_as_float(G[r][v].z), x3 = __uint_as_float(G[r][v].w);
                        iu32x2 h = {ipack_bf16(x0, x1), ipack_bf16(x2, x3)};
                        *(iu32x2*)(xr + ch[v] * 2) = h;
                        if (XP == 2) {
                            iu32x2 l = {ipack_bf16(x0 - ilo_half(h.x), x1 - ihi_half(h.x)),
                                        ipack_bf16(x2 - ilo_half(h.y), x3 - ihi_half(h.y))};
                            *(iu32x2*)(xr + p.xpart + ch[v] * 2) = l;
                        }
                    }
                }
            }
        }
    };
    // all rows of the tile against this wave's clusters and channels; partial dot products to LDS.  The LDS rows
    // span all SC * SPW steps (zeros past the data), so nothing here is conditional: the operand reads of a tile go
    // out together and the products follow, alternating between two accumulators
    auto contract = [&]() {
        constexpr int NA = SPW > 1 ? 2 : 1;
        if32x4 acc[KW][RGT][NA];
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
#pragma unroll
            for (int rg = 0; rg < RGT; rg++)
#pragma unroll
                for (int a = 0; a < NA; a++) acc[kw][rg][a] = (if32x4){0.f, 0.f, 0.f, 0.f};
        const unsigned char* xbase = smem + (size_t)n * p.xstride + (32 * ic * SPW + 8 * g) * 2;
#pragma unroll
        for (int sl = 0; sl < SPW; sl++) {
#pragma unroll
            for (int rg = 0; rg < RGT; rg++) {
                const unsigned char* xa = xbase + (size_t)(16 * rg) * p.xstride + 64 * sl;
                const ibf16x8 bh = __builtin_bit_cast(ibf16x8, *(const iu32x4*)xa);
                ibf16x8 bl;
                if (XP == 2) bl = __builtin_bit_cast(ibf16x8, *(const iu32x4*)(xa + p.xpart));
#pragma unroll
                for (int kw = 0; kw < KW; kw++) {
                    if32x4& c = acc[kw][rg][sl % NA];
                    c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[kw][sl][0], bh, c, 0, 0, 0);
                    if (P == 2) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[kw][sl][P - 1], bh, c, 0, 0, 0);
                    if (XP == 2) c = __builtin_amdgcn_mfma_f32_16x16x32_bf16(A[kw][sl][0], bl, c, 0, 0, 0);
                }
            }
        }
        // lane (n, g) holds, for row n of a group, the clusters 4 g .. 4 g + 3 of each of its cluster tiles
#pragma unroll
        for (int kw = 0; kw < KW; kw++)
#pragma unroll
            for (int rg = 0; rg < RGT; rg++) {
                if32x4 c = acc[kw][rg][0];
                if (NA == 2) c += acc[kw][rg][NA - 1];
                *(if32x4*)(s_dots + (size_t)(16 * rg + n) * DS + ic * K16 + 16 * (ik * KW + kw) + 4 * g) = c;
            }
    };

    // One step of the pipeline.  On entry: Xc holds this wave's rows of tile i, the partial dot products of tile i
    // are in LDS, the rows of tile i + 1 are on their way into Xn, Xf is free.
    float cmax = 0.f;
    double in_acc = 0.0;  // wave-uniform: this wave's rows
    const int64_t Nst = p.out ? p.N : 0;  // rows to store
    auto step = [&](Rows& Xc, Rows& Xn, Rows& Xf, int64_t i) {
        const int64_t t = tile_at(i);
        long long fetched = 0;
        if (DYN && threadIdx.x == 0) fetched = fetch();  // the tile of step i + DEPTH + 1; queued at the end of the step
        load_rows(Xf, i + DEPTH);  // the rows DEPTH tiles ahead are requested first: nothing below has to precede them
        // ---- rank the centroids of this wave's rows of tile i ----
        int idx[RPW];
#pragma unroll
        for (int r = 0; r < RPW; r++) {
            const int trow = wave * RPW + r;
            const int64_t row = t * ROWS + trow;
            // best score, its cluster (the lowest index among equal scores), and the best of the others
            int sc[NSLOT];  // score keys
            int m1 = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < NSLOT; j++) {
                const int k = lane + kWave * j;
                sc[j] = 0x7fffffff;
                if (K16 % kWave == 0 || k < K16) {
                    const float* sp = s_dots + (size_t)trow * DS + k;
                    float dot = sp[0];
#pragma unroll
                    for (int c = 1; c < SC; c++) dot += sp[c * K16];
                    sc[j] = score_key(fmaf(-2.f, dot, s_cnorm[k]));
                }
                m1 = min(m1, sc[j]);
            }
            const int kb1 = wave_min_all(m1);
            int i1 = 0;
            bool found = false;
            int m2 = 0x7fffffff;
#pragma unroll
            for (int j = 0; j < NSLOT; j++) {
                const unsigned long long hit = __ballot(sc[j] == kb1);
                const int wl = (!found && hit) ? (int)__builtin_ctzll(hit) : -1;  // wave-uniform
                if (wl >= 0) {
                    i1 = wl + kWave * j;
                    found = true;
                }
                m2 = min(m2, lane == wl ? 0x7fffffff : sc[j]);
            }
            const float b1 = key_score(kb1), b2 = key_score(wave_min_all(m2));
            // |x|^2 of the row, from the registers
            float xn2 = 0.f;
#pragma unroll
            for (int v = 0; v < VPR; v++) {
                if (ch_ok[v]) {
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        if (!word_ok(v, e)) continue;
                        if (BF16) {
                            const float x0 = ilo_half(Xc[r][v][e]), x1 = ihi_half(Xc[r][v][e]);
                            xn2 = fmaf(x0, x0, fmaf(x1, x1, xn2));
                        } else {
                            const float x0 = __uint_as_float(Xc[r][v][e]);
                            xn2 = fmaf(x0, x0, xn2);
                        }
                    }
                }
            }
            xn2 = wave_sum_all(xn2);
            // (the hardware square root is good to 1 ulp; the bound only has to err on the large side)
            const float T = p.tau * (1.000001f * __builtin_amdgcn_sqrtf(xn2)) * cmax + p.tau2 * cmax * cmax;
            if (row < p.N && !(b2 - b1 > T)) {  // wave-uniform: every lane holds the row's b1, b2
                // exact re-rank: direct-form double-precision distance to every centroid whose score is inside the bound
                const float thr = b1 + T;
                double dbest = __builtin_inf();
                int kbest = 0x7fffffff;
#pragma unroll
                for (int j = 0; j < NSLOT; j++) {
                    unsigned long long m = __ballot(sc[j] <= score_key(thr) && lane + kWave * j < p.K);
                    while (m) {
                        const int l = __builtin_amdgcn_readfirstlane(__builtin_ctzll(m));
                        m &= m - 1;
                        const int k = l + kWave * j;
                        const float* cr = p.cent + (int64_t)k * p.D;
                        double d = 0.0;
#pragma unroll
                        for (int v = 0; v < VPR; v++) {
                            if (ch_ok[v]) {
                                if32x4 c0, c1;
                                load_params(cr, v, c0, c1);
                                if (BF16) {
#pragma unroll
                                    for (int e = 0; e < 4; e++) {
                                        if (!word_ok(v, e)) continue;
                                        const double d0 = (double)ilo_half(Xc[r][v][e]) - (double)(e < 2 ? c0[2 * e] : c1[2 * e - 4]);
                                        const double d1 = (double)ihi_half(Xc[r][v][e]) - (double)(e < 2 ? c0[2 * e + 1] : c1[2 * e - 3]);
                                        d = fma(d0, d0, d);
                                        d = fma(d1, d1, d);
                                    }
                                } else {
#pragma unroll
                                    for (int e = 0; e < 4; e++) {
                                        if (!word_ok(v, e)) continue;
                                        const double d0 = (double)__uint_as_float(Xc[r][v][e]) - (double)c0[e];
                                        d = fma(d0, d0, d);
                                    }
                                }
                            }
                        }
                        d = wave_sum(d);
                        if (d < dbest || (d == dbest && k < kbest)) {
                            dbest = d;
                            kbest = k;
                        }
                    }
                }
                if (kbest != 0x7fffffff) {
                    i1 = kbest;
                    if (row < p.N) in_acc += dbest - (double)fmaxf(xn2 + b1, 0.f);  // (the score's share is added below)
                }
            }
            if (row < p.N) in_acc += (double)fmaxf(xn2 + b1, 0.f);
            // (non-finite rows have no defined result; whatever they rank first, the index stays inside the tables)
            idx[r] = __builtin_amdgcn_readfirstlane(i1 < p.K ? i1 : p.K - 1);
            if (p.assign && lane == 0 && row < p.N) p.assign[row] = idx[r];
        }

        // ---- gamma / beta rows of tile i: requested now, used after the contraction of the next tile ----
        if32x4 gv[RPW][VPR][BF16 ? 2 : 1], bv[RPW][VPR][BF16 ? 2 : 1];
#pragma unroll
        for (int r = 0; r < RPW; r++) {
            const float* gr = p.gamma + (int64_t)idx[r] * p.D;
            const float* br = p.beta + (int64_t)idx[r] * p.D;
#pragma unroll
            for (int v = 0; v < VPR; v++) {
                load_params(gr, v, gv[r][v][0], gv[r][v][BF16 ? 1 : 0]);
                load_params(br, v, bv[r][v][0], bv[r][v][BF16 ? 1 : 0]);
            }
        }
        // ---- the rows of tile i + 2 are requested, those of tile i + 1 (in flight since the last step) go to LDS ----
        stage(Xn);
        __syncthreads();
        contract();  // tile i + 1 (after the last tile: the last tile once more, to no effect)

        // ---- affine map of this wave's rows of tile i, from the registers ----
#pragma unroll
        for (int r = 0; r < RPW; r++) {
            const int64_t row = t * ROWS + wave * RPW + r;
            T* orow = (T*)p.out + row * p.D;
#pragma unroll
            for (int v = 0; v < VPR; v++) {
                iu32x4 o;
                if (BF16) {
                    const if32x4 g0 = gv[r][v][0], g1 = gv[r][v][BF16 ? 1 : 0], b0 = bv[r][v][0], b1 = bv[r][v][BF16 ? 1 : 0];
                    const iu32x4 w = Xc[r][v];
                    o.x = ipack_bf16(fmaf(g0.x, ilo_half(w.x), b0.x), fmaf(g0.y, ihi_half(w.x), b0.y));
                    o.y = ipack_bf16(fmaf(g0.z, ilo_half(w.y), b0.z), fmaf(g0.w, ihi_half(w.y), b0.w));
                    o.z = ipack_bf16(fmaf(g1.x, ilo_half(w.z), b1.x), fmaf(g1.y, ihi_half(w.z), b1.y));
                    o.w = ipack_bf16(fmaf(g1.z, ilo_half(w.w), b1.z), fmaf(g1.w, ihi_half(w.w), b1.w));
                } else {
                    const if32x4 gg = gv[r][v][0], bb = bv[r][v][0];
                    o.x = __float_as_uint(fmaf(gg.x, __uint_as_float(Xc[r][v].x), bb.x));
                    o.y = __float_as_uint(fmaf(gg.y, __uint_as_float(Xc[r][v].y), bb.y));
                    o.z = __float_as_uint(fmaf(gg.z, __uint_as_float(Xc[r][v].z), bb.z));
                    o.w = __float_as_uint(fmaf(gg.w, __uint_as_float(Xc[r][v].w), bb.w));
                }
                if (!BF16 && p.out_bf16) {  // uniform over the launch
                    const iu32x2 o2 = {ipack_bf16(__uint_as_float(o.x), __uint_as_float(o.y)),
                                       ipack_bf16(__uint_as_float(o.z), __uint_as_float(o.w))};
                    if (UA) {
                        bf16_t* oh = (bf16_t*)p.out + row * p.D + (v * 4 * kWave + lane);
#pragma unroll
                        for (int e = 0; e < 4; e++)
                            if (row < Nst && word_ok(v, e))
                                __builtin_nontemporal_store((bf16_t)(o2[e >> 1] >> (16 * (e & 1))), oh + e * kWave);
                    } else if (row < Nst && ch_ok[v]) {
                        __builtin_nontemporal_store(o2, (iu32x2*)((bf16_t*)p.out + row * p.D + ch[v]));
                    }
                } else if (UA) {
                    uint32_t* ow = (uint32_t*)orow + (v * 4 * kWave + lane);
#pragma unroll
                    for (int e = 0; e < 4; e++)
                        if (row < Nst && word_ok(v, e)) __builtin_nontemporal_store(o[e], ow + e * kWave);
                } else if (row < Nst && ch_ok[v]) {
                    __builtin_nontemporal_store(o, (iu32x4*)(orow + ch[v]));
                }
            }
        }
        if (DYN && threadIdx.x == 0) s_queue[(i + DEPTH + 1) & 7] = fetched;
        __syncthreads();  // the partial dot products of tile i + 1 are complete
    };

    Rows X0, X1, X2, X3;  // X3 only with DEPTH == 3
    load_rows(X0, 0);
    load_rows(X1, 1);
    if (DEPTH == 3) load_rows(X2, 2);
    __syncthreads();  // the zeroed tile and the norms are in place
    {
        float cm2 = 0.f;
        for (int k = lane; k < p.K; k += kWave) cm2 = fmaxf(cm2, s_cnorm[k]);
        cmax = sqrtf(wave_all(cm2, [](float a, float b) { return fmaxf(a, b); }));
    }
    if (tile_at(0) >= p.ntiles) return;  // uniform over the workgroup
    stage(X0);
    __syncthreads();
    contract();
    __syncthreads();
    // the buffers rotate by name: (rows of tile i, rows of tile i + 1, free buffer)
    if (DEPTH == 3) {
        for (int64_t i = 0;;) {
            step(X0, X1, X3, i);
            if (tile_at(++i) >= p.ntiles) break;
            step(X1, X2, X0, i);
            if (tile_at(++i) >= p.ntiles) break;
            step(X2, X3, X1, i);
            if (tile_at(++i) >= p.ntiles) break;
            step(X3, X0, X2, i);
            if (tile_at(++i) >= p.ntiles) break;
        }
    } else {
        for (int64_t i = 0;;) {
            step(X0, X1, X2, i);
            if (tile_at(++i) >= p.ntiles) break;
            step(X1, X2, X0, i);
            if (tile_at(++i) >= p.ntiles) break;
            step(X2, X0, X1, i);
            if (tile_at(++i) >= p.ntiles) break;
        }
    }
    if (p.inertia && lane == 0) atomicAdd(p.inertia, in_acc);
}

}  // namespace cat
