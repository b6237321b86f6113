// MFMA tile kernels of the CAT hot path: host side (variant selection, workspace, the Lloyd
// driver) and the centroid preparation kernel.  The tile kernel itself is in cat_tile_kernel.h.
#include "cat_tile_kernel.h"
#include "cat_infer.h"

namespace cat {

// ---- centroid preparation: (sums -> centroids), split to bf16 (hi, lo), operand order ----
// One workgroup per cluster slot k in [0, K16).  With `base` given: S = base + delta is
// folded back into base, delta is cleared, centroid = S / count (kept if the cluster is
// empty; the counts are those of the pass before, counts_read).  Then the row is split and
// scattered into packA, and its squared norm stored.  Last, the outputs of the following pass are
// reset: its counts (counts_reset, which may be the buffer just read), the objective slot and the
// first-row table.  (KT is not used for the layout any more: KTs, the cluster tiles per operand array, is.)
__global__ __launch_bounds__(256) void k_tile_prep(float* cent, double* base, double* delta,
                                                   const int32_t* counts_read, int32_t* counts_reset,
                                                   int64_t D, int32_t K, int32_t KT, int32_t P, int32_t nchunks, int f32_rows,
                                                   uint16_t* packA, float* cnorm, double* inertia_slot,
                                                   int32_t inertia_n, unsigned long long* rep, int32_t KTs) {
    __shared__ double s_red[256];
    const int k = blockIdx.x;
    const int t = k >> 4, m = k & 15;
    double nn = 0.0;
    const int64_t Dpad = (int64_t)nchunks * kChunk;
    const int cntk = (base && k < K) ? counts_read[k] : 0;
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
        // position of channel ch in the operand: chunk, MFMA step s (32 channels), then the lane group g
        // and the element j of the 8 that lane (m, g) feeds to one MFMA (operand_slot)
        const int cc = (int)(ch / kChunk), r = (int)(ch % kChunk);
        const int s = r >> 5;
        int g, j;
        operand_slot(r & 31, f32_rows != 0, g, j);
        const int lane = g * 16 + m;
        const uint32_t hw = pack_bf16(c, 0.f) & 0xFFFFu;
        // (KTs < KT: the operand is laid out as KT / KTs arrays of KTs cluster tiles each, one after the other)
        const size_t blk = (size_t)(t / KTs) * ((size_t)nchunks * 4 * KTs * P) + ((size_t)(cc * 4 + s) * KTs + t % KTs) * P;
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
            if (counts_reset) counts_reset[k] = 0;
            if (rep) rep[k] = ~0ull;
        }
        if (k < inertia_n && inertia_slot) inertia_slot[k] = 0.0;  // one per centroid set (at most 16 <= gridDim.x)
    }
}

// ---- sums update from the changed-row list + centroid preparation, one launch -------------------
// After a Lloyd pass that listed the rows that changed cluster: grid (G list shares) x (64-channel
// slices) x (cluster ranges).  Every workgroup adds its share of the listed rows to (new cluster) and
// subtracts them from (old cluster) in an LDS panel of doubles, and merges the panel into `delta`.
// The workgroup that finishes a slice last (a counter per slice, no waiting) then does for that
// slice what k_tile_prep does: S = base + delta folded into base, delta cleared, centroid = S /
// count (kept if the cluster is empty), bf16 split into the operand, and the slice's share of
// |c|^2 (the tile kernel adds the shares up in slice order, so the norms do not depend on which
// slice finished first).  Everything the following pass accumulates into is double-buffered
// (counts, list length, the slice counters), so the first workgroup can clear the other buffer at
// once and nothing in this launch waits for anything else.
struct DeltaParams {
    const void* lq;
    int64_t D;
    int32_t K, KT, KTs, P, KC, G, f32_rows;  // KTs: cluster tiles per operand array (KT unless the clusters are split)
    const unsigned long long* list;
    const uint32_t* list_count;  // length of the list of the pass before
    uint32_t* list_count_next;   // cleared: the following pass appends here
    uint32_t* done;              // [slices] finished workgroups per slice, zero on entry
    uint32_t* done_next;         // cleared for the next launch
    double* base;
    double* delta;
    const int32_t* counts;       // of the pass before
    int32_t* counts_next;        // cleared: the following pass counts here
    float* cent;
    uint16_t* packA;
    double* norm_part;           // slices x K
    double* inertia_slot;
    int32_t inertia_n;           // objective entries at inertia_slot (one per centroid set)
    unsigned long long* rep;
    int32_t* skipped;            // nullable: early stop allowed; counts the passes that were not run
    // Loops that skip rows by distance bounds: the passes between the first listed pass and the last do not count the
    // rows of every cluster again, so every slice keeps running counts of its own (slice_counts, slices x K): seeded
    // from `counts` (seed_counts != 0; the pass before counted all rows), afterwards moved along with the listed rows
    // and used instead of `counts`.  move_part (slices x K) receives the slice's share of |c_new - c_old|^2.
    int32_t* slice_counts;
    int32_t seed_counts;
    double* move_part;
    uint32_t* n_rows_clear;      // nullable: cleared (the row selection that follows counts into it)
};

constexpr int kDeltaWaves = 8;
constexpr int kDeltaSW = 64;  // channels per slice: one per lane

template <typename T>
__global__ __launch_bounds__(kDeltaWaves * kWave) void k_delta_prep(const DeltaParams q) {
    extern __shared__ double s_panel[];  // KC x 64
    __shared__ int s_flag;
    __shared__ int s_moved[128];         // KC: rows that joined minus rows that left, per cluster of the range
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int slice = blockIdx.y, nslices = gridDim.y;
    const int64_t ch = (int64_t)slice * kDeltaSW + lane;
    const bool ch_ok = ch < q.D;
    const int k0 = blockIdx.z * q.KC;
    const int kc = (q.K - k0) < q.KC ? (q.K - k0) : q.KC;

    const uint32_t len = *q.list_count;
    if (q.skipped && len == 0u) {
        // No row changed cluster in the pass before: the sums, the centroids and therefore the pass that would
        // follow are what they were.  That pass is not run (its kernel reads the same word); what it would have
        // written is carried forward instead, and the double buffers are left as a pass with an empty list
        // leaves them, so that the next launch of this kernel takes the same branch.
        if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) {
            for (int k = threadIdx.x; k < q.K; k += blockDim.x) q.counts_next[k] = q.counts[k];
            for (int s = threadIdx.x; s < nslices; s += blockDim.x) q.done_next[s] = 0;
            if (threadIdx.x == 0) {
                *q.list_count_next = 0;
                if (q.inertia_slot) q.inertia_slot[0] = q.inertia_slot[-1];
                q.skipped[0] += 1;
            }
        }
        return;
    }
    if (blockIdx.x == 0 && blockIdx.y == 0 && blockIdx.z == 0) {  // the other halves of the double buffers
        for (int k = threadIdx.x; k < q.K; k += blockDim.x) {
            q.counts_next[k] = 0;
            if (q.rep) q.rep[k] = ~0ull;
        }
        for (int s = threadIdx.x; s < nslices; s += blockDim.x) q.done_next[s] = 0;
        if (threadIdx.x == 0) {
            *q.list_count_next = 0;
            if (q.n_rows_clear) *q.n_rows_clear = 0;
        }
        if ((int)threadIdx.x < q.inertia_n && q.inertia_slot) q.inertia_slot[threadIdx.x] = 0.0;
    }
    const uint32_t per = (len + q.G - 1) / q.G;
    const uint32_t e0 = blockIdx.x * per;
    const uint32_t e1 = (e0 + per < len) ? e0 + per : len;
    const bool moving_counts = q.slice_counts && !q.seed_counts;
    if (e0 < e1) {
        for (int i = threadIdx.x; i < kc * kDeltaSW; i += blockDim.x) s_panel[i] = 0.0;
        if (moving_counts)
            for (int i = threadIdx.x; i < kc; i += blockDim.x) s_moved[i] = 0;
        __syncthreads();
        // each wave takes a contiguous run of the share: 64 entries per load, then 8 rows in flight
        const uint32_t pw = (e1 - e0 + kDeltaWaves - 1) / kDeltaWaves;
        const uint32_t ws = e0 + wave * pw;
        const uint32_t we = (ws + pw < e1) ? ws + pw : e1;
        // Long runs (from 24 entries per wave on) keep two rounds of eight rows in flight; short runs load a round and
        // add it up, which measures faster there (65536 x 1000, some 40 entries per wave: 9.1 against 10.3 us per
        // launch; 262144 x 2048 bf16, some 300 per wave: 41.6 against 30 us).
        if (pw >= 24u) {
            // Eight rows per round, two rounds in flight.  Every load is issued by every wave on every path (an entry past
            // the run repeats entry 0 of the batch, a lane past the row reads channel 0, a round past the batch is loaded
            // and dropped): the compiler counts the loads in flight at each use, and a load it cannot prove was issued
            // would make it wait for all of them.
            constexpr int RB = 8;
            const int64_t chc = ch_ok ? ch : 0;
            unsigned long long ent = ws < we ? q.list[ws + lane < we ? ws + lane : we - 1] : 0ull;
            for (uint32_t b = ws; b < we; b += kWave) {
                const uint32_t ent_lo = (uint32_t)ent, ent_hi = (uint32_t)(ent >> 32);
                const int nb = (we - b) < (uint32_t)kWave ? (int)(we - b) : kWave;
                {  // the entries of the next batch, one batch ahead (the last batch: itself again)
                    const uint32_t nb0 = b + kWave < we ? b + kWave : b;
                    ent = q.list[nb0 + lane < we ? nb0 + lane : we - 1];
                }
                if (moving_counts && lane < nb) {  // every lane holds one entry
                    const int a = (int)(ent_lo & 0xFFFu) - k0, c = (int)((ent_lo >> 12) & 0xFFFu) - 1 - k0;
                    if (a >= 0 && a < kc) atomicAdd(&s_moved[a], 1);
                    if (c >= 0 && c < kc) atomicAdd(&s_moved[c], -1);
                }
                auto issue = [&](int i0, float (&x)[RB], int (&nw)[RB], int (&od)[RB]) {
    #pragma unroll
                    for (int u = 0; u < RB; u++) {
                        const bool in = i0 + u < nb;
                        const uint32_t lo = __builtin_amdgcn_readlane(ent_lo, in ? i0 + u : 0);
                        const uint32_t hi = __builtin_amdgcn_readlane(ent_hi, in ? i0 + u : 0);
                        const int64_t row = (int64_t)(((unsigned long long)hi << 8) | (lo >> 24));
                        const int a = (int)(lo & 0xFFFu) - k0, c = (int)((lo >> 12) & 0xFFFu) - 1 - k0;
                        nw[u] = (in && a >= 0 && a < kc && ch_ok) ? a : -1;
                        od[u] = (in && c >= 0 && c < kc && ch_ok) ? c : -1;
                        x[u] = ld_elem((const T*)q.lq + row * q.D + chc);
                    }
                };
                auto consume = [&](const float (&x)[RB], const int (&nw)[RB], const int (&od)[RB]) {
    #pragma unroll
                    for (int u = 0; u < RB; u++) {
                        if (nw[u] >= 0) atomicAdd(s_panel + nw[u] * kDeltaSW + lane, (double)x[u]);
                        if (od[u] >= 0) atomicAdd(s_panel + od[u] * kDeltaSW + lane, -(double)x[u]);
                    }
                };
                float xa[RB], xb[RB];
                int nwa[RB], oda[RB], nwb[RB], odb[RB];
                issue(0, xa, nwa, oda);
                if (nb <= RB) {  // (a short run: one round, nothing to overlap it with)
                    consume(xa, nwa, oda);
                    continue;
                }
                for (int i0 = 0; i0 < nb; i0 += 2 * RB) {
                    issue(i0 + RB, xb, nwb, odb);
                    consume(xa, nwa, oda);
                    if (i0 + RB >= nb) break;
                    issue(i0 + 2 * RB, xa, nwa, oda);
                    consume(xb, nwb, odb);
                }
            }
        } else {
            constexpr int RB = 8;
            for (uint32_t b = ws; b < we; b += kWave) {
                const unsigned long long ent = (b + lane < we) ? q.list[b + lane] : 0ull;
                const uint32_t ent_lo = (uint32_t)ent, ent_hi = (uint32_t)(ent >> 32);
                const int nb = (we - b) < (uint32_t)kWave ? (int)(we - b) : kWave;
                if (moving_counts && lane < nb) {  // every lane holds one entry
                    const int a = (int)(ent_lo & 0xFFFu) - k0, c = (int)((ent_lo >> 12) & 0xFFFu) - 1 - k0;
                    if (a >= 0 && a < kc) atomicAdd(&s_moved[a], 1);
                    if (c >= 0 && c < kc) atomicAdd(&s_moved[c], -1);
                }
                for (int i0 = 0; i0 < nb; i0 += RB) {
                    int nw[RB], od[RB];
                    float x[RB];
    #pragma unroll
                    for (int u = 0; u < RB; u++) {
                        nw[u] = od[u] = -1;
                        x[u] = 0.f;
                        if (i0 + u < nb) {
                            const uint32_t lo = __builtin_amdgcn_readlane(ent_lo, i0 + u);
                            const uint32_t hi = __builtin_amdgcn_readlane(ent_hi, i0 + u);
                            const int64_t row = (int64_t)(((unsigned long long)hi << 8) | (lo >> 24));
                            const int a = (int)(lo & 0xFFFu) - k0, c = (int)((lo >> 12) & 0xFFFu) - 1 - k0;
                            nw[u] = (a >= 0 && a < kc) ? a : -1;
                            od[u] = (c >= 0 && c < kc) ? c : -1;
                            if ((nw[u] >= 0 || od[u] >= 0) && ch_ok) x[u] = ld_elem((const T*)q.lq + row * q.D + ch);
                        }
                    }
    #pragma unroll
                    for (int u = 0; u < RB; u++) {
                        if (nw[u] >= 0) atomicAdd(s_panel + nw[u] * kDeltaSW + lane, (double)x[u]);
                        if (od[u] >= 0) atomicAdd(s_panel + od[u] * kDeltaSW + lane, -(double)x[u]);
                    }
                }
            }
        }
        __syncthreads();
        for (int i = threadIdx.x; i < kc * kDeltaSW; i += blockDim.x) {
            const int k = i / kDeltaSW, c = i - k * kDeltaSW;
            const double v = s_panel[i];
            const int64_t cg = (int64_t)slice * kDeltaSW + c;
            if (v != 0.0 && cg < q.D) atomicAdd(q.delta + (int64_t)(k0 + k) * q.D + cg, v);
        }
        if (moving_counts)
            for (int i = threadIdx.x; i < kc; i += blockDim.x)
                if (s_moved[i]) atomicAdd(q.slice_counts + (size_t)slice * q.K + k0 + i, s_moved[i]);
    }

    // ---- who finishes the slice? ----
    // What crosses workgroups here (delta, the counter) goes through device-scope atomics, which
    // are performed where every XCD sees them; waiting for this wave's own atomics to be
    // acknowledged therefore orders them before the counter.  A device-scope fence would write
    // back and invalidate the whole L2 once per workgroup, at several times the cost of the update.
    __builtin_amdgcn_s_waitcnt(0);
    __syncthreads();
    if (threadIdx.x == 0) {
        const uint32_t total = gridDim.x * gridDim.z;
        s_flag = atomicAdd(q.done + slice, 1u) == total - 1;
    }
    __syncthreads();
    if (!s_flag) return;

    // ---- this slice's centroids, operand parts, norm shares ----
    // eight clusters per wave at a time: all their loads first (a load is not moved above the
    // stores of the cluster before it, so one cluster at a time would cost a round trip each)
    constexpr int KB = 8;
    for (int kb = wave; kb < q.K; kb += kDeltaWaves * KB) {
        double S[KB];
        float cold[KB];
        int n[KB];
#pragma unroll
        for (int u = 0; u < KB; u++) {
            const int k = kb + u * kDeltaWaves;
            S[u] = 0.0;
            cold[u] = 0.f;
            n[u] = 0;
            if (k < q.K && ch_ok) {
                const int64_t i = (int64_t)k * q.D + ch;
                S[u] = q.base[i] + __hip_atomic_load(q.delta + i, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
                cold[u] = q.cent[i];
                n[u] = moving_counts ? __hip_atomic_load(q.slice_counts + (size_t)slice * q.K + k, __ATOMIC_RELAXED,
                                                         __HIP_MEMORY_SCOPE_AGENT)
                                     : q.counts[k];
            }
        }
#pragma unroll
        for (int u = 0; u < KB; u++) {
            const int k = kb + u * kDeltaWaves;
            if (k >= q.K) break;  // wave-uniform
            double nn = 0.0, mv = 0.0;
            if (ch_ok) {
                const int64_t i = (int64_t)k * q.D + ch;
                q.base[i] = S[u];
                q.delta[i] = 0.0;
                float c = cold[u];
                if (n[u] > 0) {
                    c = (float)(S[u] / (double)n[u]);
                    q.cent[i] = c;
                }
                nn = (double)c * (double)c;
                mv = ((double)c - (double)cold[u]) * ((double)c - (double)cold[u]);
                const int t = k >> 4, m = k & 15;
                const int cc = (int)(ch / kChunk), r = (int)(ch % kChunk);
                const int s = r >> 5;
                int g, j;
                operand_slot(r & 31, q.f32_rows != 0, g, j);
                const int ol = g * 16 + m;
                const uint32_t hw = pack_bf16(c, 0.f) & 0xFFFFu;
                const size_t nch = (size_t)((q.D + kChunk - 1) / kChunk);
                const size_t blk = (size_t)(t / q.KTs) * (nch * 4 * q.KTs * q.P) + ((size_t)(cc * 4 + s) * q.KTs + t % q.KTs) * q.P;
                q.packA[(blk * 64 + ol) * 8 + j] = (uint16_t)hw;
                if (q.P == 2) {
                    const uint32_t lw = pack_bf16(c - lo_half(hw), 0.f) & 0xFFFFu;
                    q.packA[((blk + 1) * 64 + ol) * 8 + j] = (uint16_t)lw;
                }
            }
            nn = wave_sum(nn);
            if (lane == 0) q.norm_part[(size_t)slice * q.K + k] = nn;
            if (q.move_part) {
                mv = wave_sum(mv);
                if (lane == 0) {
                    q.move_part[(size_t)slice * q.K + k] = mv;
                    if (q.seed_counts) q.slice_counts[(size_t)slice * q.K + k] = q.counts[k];
                }
            }
        }
    }
}

// ---- which rows does the next pass have to evaluate? (distance bounds; Hamerly, SDM 2010) ----
// The update just done moved centroid k by p(k) = sqrt(sum over the slices of move_part[.][k]).  A row's distance to
// its own centroid grew by at most p(own) and its distance to any other shrank by at most the largest p among the
// others, so the difference of the two shrank by at most the sum of the two largest movements.  That sum is added
// to the running drift G; a row whose bound expire[i] (the drift at its last evaluation plus its margin then) is
// still above G keeps its nearest centroid and is left out.  Every workgroup computes the same G (same data, same
// order); the rows are taken in contiguous pieces and the kept ones appended to `rows` with one reservation per piece.
constexpr int kSelThreads = 256;
constexpr int kSelPerThread = 8;
__global__ __launch_bounds__(kSelThreads) void k_bound_select(const double* __restrict__ move_part, int32_t slices, int32_t K,
                                                              const double* __restrict__ g_prev, double* __restrict__ g_now,
                                                              const double* __restrict__ expire, int64_t N,
                                                              int32_t* __restrict__ rows, uint32_t* __restrict__ n_rows) {
    __shared__ double s_p[256];
    __shared__ double s_g;
    __shared__ uint32_t s_wave[kSelThreads / kWave + 1];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    double pk = 0.0;
    if ((int)threadIdx.x < K) {
        double m2 = 0.0;
        const double* mp = move_part + threadIdx.x;
        int sl = 0;
        for (; sl + 8 <= slices; sl += 8) {  // eight loads in flight, added in slice order
            double v[8];
#pragma unroll
            for (int u = 0; u < 8; u++) v[u] = mp[(size_t)(sl + u) * K];
#pragma unroll
            for (int u = 0; u < 8; u++) m2 += v[u];
        }
        for (; sl < slices; sl++) m2 += mp[(size_t)sl * K];
        pk = sqrt(m2);
    }
    s_p[threadIdx.x] = pk;
    __syncthreads();
    if (threadIdx.x < kWave) {
        // the two largest movements: every lane ranks its four entries, then the wave's largest and, with that one
        // taken out at the lane that holds it, the largest of the rest
        double t1 = 0.0, t2 = 0.0;
#pragma unroll
        for (int j = 0; j < kSelThreads / kWave; j++) {
            const double v = s_p[threadIdx.x + j * kWave];
            if (v > t1) {
                t2 = t1;
                t1 = v;
            } else if (v > t2) {
                t2 = v;
            }
        }
        double w1 = t1;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) w1 = fmax(w1, __shfl_xor(w1, o, kWave));
        const unsigned long long holders = __ballot(t1 == w1);
        const bool mine = lane == (int)__builtin_ctzll(holders);
        double w2 = mine ? t2 : t1;
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) w2 = fmax(w2, __shfl_xor(w2, o, kWave));
        if (threadIdx.x == 0) {
            s_g = *g_prev + (w1 + w2) * (1.0 + 1e-9);
            if (blockIdx.x == 0) *g_now = s_g;
        }
    }
    __syncthreads();
    const double G = s_g;
    constexpr int64_t kPiece = (int64_t)kSelThreads * kSelPerThread;
    for (int64_t r0 = (int64_t)blockIdx.x * kPiece; r0 < N; r0 += (int64_t)gridDim.x * kPiece) {
        // thread t takes rows r0 + t * 8 .. + 7: the kept rows of a piece stay in row order
        const int64_t mine = r0 + (int64_t)threadIdx.x * kSelPerThread;
        uint32_t keep = 0;
        int cnt = 0;
#pragma unroll
        for (int j = 0; j < kSelPerThread; j++) {
            const int64_t i = mine + j;
            const bool k = i < N && !(G < expire[i]);
            keep |= (uint32_t)k << j;
            cnt += k;
        }
        // exclusive prefix over the workgroup: shuffle scan per wave, wave totals through LDS
        int incl = cnt;
#pragma unroll
        for (int o = 1; o < kWave; o <<= 1) {
            const int v = __shfl_up(incl, o, kWave);
            if (lane >= o) incl += v;
        }
        if (lane == kWave - 1) s_wave[wave] = (uint32_t)incl;
        __syncthreads();
        if (threadIdx.x == 0) {
            uint32_t tot = 0;
            for (int w = 0; w < kSelThreads / kWave; w++) {
                const uint32_t v = s_wave[w];
                s_wave[w] = tot;
                tot += v;
            }
            s_wave[kSelThreads / kWave] = tot ? atomicAdd(n_rows, tot) : 0u;
        }
        __syncthreads();
        uint32_t pos = s_wave[kSelThreads / kWave] + s_wave[wave] + (uint32_t)(incl - cnt);
#pragma unroll
        for (int j = 0; j < kSelPerThread; j++)
            if (keep >> j & 1u) rows[pos++] = (int32_t)(mine + j);
        __syncthreads();
    }
}

// ---- host side ----------------------------------------------------------------------------

static inline uint32_t up16(size_t x) { return (uint32_t)((x + 15) & ~(size_t)15); }

static TileCfg tile_config(TileMode mode, int64_t D, int32_t K, cat_dtype dt, bool two_parts_only = false, int32_t hist_k = 0) {
    TileCfg c;
    const int K16 = (K + 15) & ~15;
    int KT = 1;
    while (KT * 16 < K16) KT *= 2;
    if (KT > 16) return c;
    if (D % (dt == CAT_BF16 ? 8 : 4)) return c;  // rows must keep the 16-byte alignment of the operand loads
    if (D > 65536) return c;  // also bounds the fp32 accumulation term of the re-rank threshold
    const int nchunks = (int)((D + kChunk - 1) / kChunk);
    const bool lists = mode == TILE_LLOYD;
    // Order of preference: the two-part operand resident in LDS, the two-part operand in chunks (two chunk buffers),
    // then the one-part operand resident, then in chunks.  The one-part operand ranks with an error bound of 1.6 % of
    // |x||c|: k-means boundaries run through the data, so on anything but widely separated clusters most rows then
    // take the exact re-rank (measured on overlapping mixtures, per Lloyd iteration: 262144 x 512, K = 128: 739 us
    // resident one-part against 328 us chunked two-part; 65536 x 1000, K = 64: 244 against 98 us; on widely separated
    // mixtures 262 against 310 us and 98 against 91 us).
    for (int pass = 0; pass < 4; pass++) {
        const bool chunked = (pass == 1 || pass == 3);
        const int P = pass < 2 ? 2 : 1;
        if (two_parts_only && P != 2) continue;
        const size_t ldsA = chunked ? (size_t)2 * 4 * KT * P * 1024 : (size_t)nchunks * 4 * KT * P * 1024;
        for (int waves = kMaxWaves; waves >= kMaxWaves; waves -= 2) {
            size_t off = ldsA;
            TileCfg t;
            t.off_cnorm = up16(off);
            off = t.off_cnorm + (size_t)KT * 16 * 4;
            const size_t KH = hist_k > K ? hist_k : K;  // clusters the per-cluster tables span
            t.off_hist = up16(off);
            off = t.off_hist + KH * 4;
            t.off_rep = up16(off);
            off = t.off_rep + KH * 8;
            t.off_list = up16(off);
            off = t.off_list + (lists ? (size_t)kListCap * 8 : 0);
            t.off_misc = up16(off);
            off = t.off_misc + 16 + 8 * kMaxWaves + 8 * 16;  // list count, objective per wave, objective per centroid set
            if (off > kLdsLimit) continue;
            // assignment passes: the queue of rows whose exact re-rank waits for the end of the workgroup's tiles,
            // where the layout leaves room for it
            if (mode != TILE_APPLY && up16(off) + 16 + (size_t)kQueueCap * sizeof(DeferredRow) <= kLdsLimit) {
                t.off_queue = up16(off);
                t.queue_cap = kQueueCap;
                off = t.off_queue + 16 + (size_t)kQueueCap * sizeof(DeferredRow);
            }
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

bool tile_supports(TileMode mode, int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    // tile indices are 32-bit in the kernels and a changed-row entry keeps 40 bits of row number
    return N < ((int64_t)1 << 34) && tile_config(mode, D, K, dt).ok;
}

static size_t packA_bytes(int64_t D, int32_t K) {
    const int K16 = (K + 15) & ~15;
    int KT = 1;
    while (KT * 16 < K16) KT *= 2;
    const size_t nchunks = (size_t)((D + kChunk - 1) / kChunk);
    return nchunks * 4 * KT * 2 * 1024;
}
static inline size_t a256(size_t x) { return (x + 255) & ~(size_t)255; }

size_t tile_workspace_bytes(int64_t D, int32_t K, cat_dtype dt) {
    // (the row-tile inference kernel shares this scratch and also takes rows that are not whole 16-byte groups)
    if (!tile_config(TILE_ASSIGN, D, K, dt).ok && !infer_supported(1, D, K, dt)) return 0;
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

static inline int64_t delta_slices(int64_t D) { return (D + kDeltaSW - 1) / kDeltaSW; }
constexpr int kSplitTiles = 8;  // cluster tiles per launch when the clusters of a pass are split over two

static inline size_t lloyd_ctrl_words(int64_t D) { return (size_t)(3 + 2 * delta_slices(D)); }

size_t lloyd_workspace_bytes(int64_t N, int64_t D, int32_t K) {
    return a256((size_t)N * 8) + a256(lloyd_ctrl_words(D) * 4) + a256((size_t)delta_slices(D) * K * 8) +
           a256((size_t)K * 4) + (K > kSplitTiles * 16 ? a256((size_t)N * 8) + 256 : 0);
}
LloydWs lloyd_carve(void* base, int64_t N, int64_t D, int32_t K) {
    LloydWs w;
    w.bytes = lloyd_workspace_bytes(N, D, K);
    if (!base) return w;
    char* b = (char*)base;
    w.list = (unsigned long long*)b;
    b += a256((size_t)N * 8);
    w.ctrl = (uint32_t*)b;
    b += a256(lloyd_ctrl_words(D) * 4);
    w.skipped = (int32_t*)(w.ctrl + lloyd_ctrl_words(D) - 1);
    w.norm_part = (double*)b;
    b += a256((size_t)delta_slices(D) * K * 8);
    w.counts2 = (int32_t*)b;
    b += a256((size_t)K * 4);
    if (K > kSplitTiles * 16) {
        w.carry = (float2*)b;
        b += a256((size_t)N * 8);
        w.carry_cmax = (float*)b;
    }
    return w;
}

// More than 128 clusters need 16 cluster tiles, whose two-part operand fits LDS only for short rows; otherwise the
// clusters are ranked by two launches of 8 tiles each (k_tile<..., VAR_SPLIT>), the first handing its best on.
static bool split_config(int64_t D, int32_t K, cat_dtype dt, TileCfg* out, TileMode mode = TILE_LLOYD) {
    if (K <= kSplitTiles * 16 || K > 2 * kSplitTiles * 16) return false;
    if (tile_config(mode, D, K, dt, true).ok) return false;  // one launch ranks them all with two parts
    TileCfg c = tile_config(mode, D, kSplitTiles * 16, dt, true, K);
    if (!c.ok || c.KT != kSplitTiles) return false;
    if (out) *out = c;
    return true;
}

bool tile_bounds_supports(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    // row numbers in the list of rows are 32-bit; the bounds are derived for the two-part operand
    return N < ((int64_t)1 << 31) && tile_config(TILE_LLOYD, D, K, dt, true).ok;
}
size_t bounds_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t iters) {
    const size_t sk = (size_t)delta_slices(D) * (size_t)K;
    return a256((size_t)N * 8) + a256((size_t)N * 4) + a256(4) + a256(((size_t)iters + 1) * 8) + a256(sk * 8) + a256(sk * 4);
}
BoundsWs bounds_carve(void* base, int64_t N, int64_t D, int32_t K, int32_t iters) {
    BoundsWs w;
    w.bytes = bounds_workspace_bytes(N, D, K, iters);
    if (!base) return w;
    const size_t sk = (size_t)delta_slices(D) * (size_t)K;
    char* b = (char*)base;
    w.expire = (double*)b;
    b += a256((size_t)N * 8);
    w.rows = (int32_t*)b;
    b += a256((size_t)N * 4);
    w.n_rows = (uint32_t*)b;
    b += a256(4);
    w.drift = (double*)b;
    b += a256(((size_t)iters + 1) * 8);
    w.move_part = (double*)b;
    b += a256(sk * 8);
    w.slice_counts = (int32_t*)b;
    return w;
}

__global__ void k_fill_i32(int32_t* p, int64_t n, int32_t v) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < n) p[i] = v;
}
cat_status launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st) {
    hipLaunchKernelGGL(k_fill_i32, dim3((unsigned)((n + 255) / 256)), dim3(256), 0, st, p, n, v);
    CAT_LAUNCH_CHECK("k_fill_i32");
    return CAT_OK;
}

// Sums update from the list of changed rows, then the centroid preparation of the next pass.
// `par` is the parity of the pass that follows: it selects the halves of the double buffers.
static cat_status launch_delta_prep(const void* lq, cat_dtype dt, int64_t D, int32_t K, const TileCfg& c,
                                    const TileWs& ws, const LloydWs& lw, int par, float* cent, double* base,
                                    double* delta, const int32_t* counts_prev, int32_t* counts_next,
                                    double* inertia_slot, unsigned long long* rep, int32_t* skipped, hipStream_t st,
                                    int32_t inertia_n = 1, const BoundsWs* bw = nullptr, bool seed_counts = false,
                                    int32_t split_tiles = 0) {
    DeltaParams q = {};
    q.KTs = split_tiles ? split_tiles : c.KT;
    if (bw) {
        q.slice_counts = bw->slice_counts;
        q.seed_counts = seed_counts ? 1 : 0;
        q.move_part = bw->move_part;
        q.n_rows_clear = bw->n_rows;
    }
    q.lq = lq;
    q.D = D;
    q.K = K;
    q.KT = c.KT;
    q.P = c.P;
    q.f32_rows = dt == CAT_F32;
    q.KC = K < 128 ? K : 128;  // LDS panel: KC x 64 doubles, at most 64 KB
    const int64_t slices = delta_slices(D);
    const int kchunks = (K + q.KC - 1) / q.KC;
    int64_t G = 256 / (slices * kchunks);  // about one workgroup per CU in all: with 1024 the launch itself
                                           // (dispatch, panel clears, counters) cost 10 us more than the work
    q.G = (int32_t)(G < 1 ? 1 : (G > 256 ? 256 : G));
    q.list = lw.list;
    q.list_count = lw.ctrl + (par ^ 1);
    q.list_count_next = lw.ctrl + par;
    q.done = lw.ctrl + 2 + (size_t)par * slices;
    q.done_next = lw.ctrl + 2 + (size_t)(par ^ 1) * slices;
    q.base = base;
    q.delta = delta;
    q.counts = counts_prev;
    q.counts_next = counts_next;
    q.cent = cent;
    q.packA = ws.packA;
    q.norm_part = lw.norm_part;
    q.inertia_slot = inertia_slot;
    q.inertia_n = inertia_n;
    q.rep = rep;
    q.skipped = skipped;
    dim3 grid((unsigned)q.G, (unsigned)slices, (unsigned)kchunks), block(kDeltaWaves * kWave);
    const size_t lds = (size_t)q.KC * kDeltaSW * sizeof(double);
    if (dt == CAT_BF16)
        hipLaunchKernelGGL(k_delta_prep<bf16_t>, grid, block, lds, st, q);
    else
        hipLaunchKernelGGL(k_delta_prep<float>, grid, block, lds, st, q);
    CAT_LAUNCH_CHECK("k_delta_prep");
    return CAT_OK;
}

static cat_status launch_prep(cat_dtype dt, float* cent, double* base, double* delta, const int32_t* counts_read,
                              int32_t* counts_reset, int64_t D, int32_t K, const TileCfg& c, const TileWs& ws,
                              double* inertia_slot, unsigned long long* rep, hipStream_t st, int32_t inertia_n = 1,
                              int32_t split_arrays = 1) {
    dim3 grid(c.KT * 16 * split_arrays), block(256);
    hipLaunchKernelGGL(k_tile_prep, grid, block, 0, st, cent, base, delta, counts_read, counts_reset, D, K, c.KT * split_arrays,
                       c.P, c.nchunks, dt == CAT_F32 ? 1 : 0, ws.packA, ws.cnorm, inertia_slot, inertia_n, rep, c.KT);
    CAT_LAUNCH_CHECK("k_tile_prep");
    return CAT_OK;
}

// Centroids as they are (no sums to fold) -> operand parts and norms, for kernels outside this file that choose
// their own cluster tiling, part count and channel order.
cat_status launch_tile_prep_plain(cat_dtype dt, const float* cent, int64_t D, int32_t K, int32_t KT, int32_t P,
                                  int32_t nchunks, int rows_layout_f32, uint16_t* packA, float* cnorm, hipStream_t st) {
    (void)dt;
    dim3 grid(KT * 16), block(256);
    hipLaunchKernelGGL(k_tile_prep, grid, block, 0, st, const_cast<float*>(cent), (double*)nullptr, (double*)nullptr,
                       (const int32_t*)nullptr, (int32_t*)nullptr, D, K, KT, P, nchunks, rows_layout_f32, packA, cnorm,
                       (double*)nullptr, 0, (unsigned long long*)nullptr, KT);
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
    p.off_queue = c.off_queue;
    p.queue_cap = c.queue_cap < rerank_queue_capacity() ? c.queue_cap : rerank_queue_capacity();
    return p;
}

cat_status tile_assign(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                       int32_t* assign, int32_t* counts, double* inertia, unsigned long long* rep,
                       const float* gamma, const float* beta, void* corrected, const TileWs& ws, hipStream_t st) {
    const TileMode mode = gamma ? TILE_APPLY : TILE_ASSIGN;
    TileCfg c = tile_config(mode, D, K, dt);
    if (!c.ok) return set_error(CAT_ERR_UNSUPPORTED, "tile kernels do not fit D=%lld K=%d", (long long)D, (int)K);
    // The preparation only reads the centroids here (no sums to fold), and the exact re-rank reads them with
    // 16-byte loads: the caller's array serves both as it is when it is aligned, else a copy in the workspace.
    const float* cw = cent;
    cat_status s = CAT_OK;
    if (((uintptr_t)cent & 15u) != 0) {
        s = launch_copy_words(cent, ws.cent, (int64_t)K * D, st);
        if (s != CAT_OK) return s;
        cw = ws.cent;
    }
    s = launch_prep(dt, const_cast<float*>(cw), nullptr, nullptr, nullptr, nullptr, D, K, c, ws, nullptr, nullptr, st);
    if (s != CAT_OK) return s;
    TileParams p = base_params(lq, N, D, K, c, ws, dt);
    p.cent = cw;
    p.assign = assign;
    p.counts = counts;
    p.inertia = inertia;
    p.rep = rep;
    p.gamma = gamma;
    p.beta = beta;
    p.out = corrected;
    return launch_tile(p, c, dt, st);
}

// The two launches of a pass whose clusters are split (p: the parameters of the pass as for one launch).
static cat_status launch_split_pair(const TileParams& p, const TileCfg& c, cat_dtype dt, int32_t K, const TileWs& ws,
                                    float2* carry, float* carry_cmax, hipStream_t st) {
    // first launch: clusters 0 .. 127, no bookkeeping, leaves (best score, nearest centroid) per row
    const int32_t K0 = kSplitTiles * 16;
    TileParams a = p;
    a.K = K0;
    a.k_base = 0;
    a.k_hist = K;
    a.norm_stride = K;
    a.carry_out = carry;
    a.cmax_io = carry_cmax;
    a.counts = nullptr;
    a.inertia = nullptr;
    a.rep = nullptr;
    a.list = nullptr;
    a.delta_mode = 0;
    cat_status s = dt == CAT_BF16 ? launch_split_bf16(a, c, st) : launch_split_f32(a, c, st);
    if (s != CAT_OK) return s;
    // second launch: the other clusters beside that pair, and the bookkeeping of the pass
    TileParams b = p;
    b.K = K - K0;
    b.k_base = K0;
    b.k_hist = K;
    b.norm_stride = K;
    b.packA = ws.packA + (size_t)c.nchunks * 4 * kSplitTiles * c.P * 512;
    b.cnorm = ws.cnorm + K0;
    b.carry_in = carry;
    b.cmax_io = carry_cmax;
    return dt == CAT_BF16 ? launch_split_bf16(b, c, st) : launch_split_f32(b, c, st);
}

size_t tile_split_scratch_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt) {
    return split_config(D, K, dt, nullptr, TILE_ASSIGN) ? a256((size_t)N * 8) + 256 : 0;
}

// tile_assign (assignment only) for more than 128 clusters, ranked by two launches; scratch: tile_split_scratch_bytes.
cat_status tile_assign_split(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent, int32_t* assign,
                             int32_t* counts, double* inertia, unsigned long long* rep, const TileWs& ws, void* scratch,
                             hipStream_t st) {
    TileCfg c;
    if (!scratch || !split_config(D, K, dt, &c, TILE_ASSIGN))
        return set_error(CAT_ERR_UNSUPPORTED, "split ranking does not apply to D=%lld K=%d", (long long)D, (int)K);
    const float* cw = cent;
    cat_status s = CAT_OK;
    if (((uintptr_t)cent & 15u) != 0) {
        s = launch_copy_words(cent, ws.cent, (int64_t)K * D, st);
        if (s != CAT_OK) return s;
        cw = ws.cent;
    }
    s = launch_prep(dt, const_cast<float*>(cw), nullptr, nullptr, nullptr, nullptr, D, K, c, ws, nullptr, nullptr, st, 1, 2);
    if (s != CAT_OK) return s;
    TileParams p = base_params(lq, N, D, K, c, ws, dt);
    p.cent = cw;
    p.assign = assign;
    p.counts = counts;
    p.inertia = inertia;
    p.rep = rep;
    return launch_split_pair(p, c, dt, K, ws, (float2*)scratch, (float*)((char*)scratch + a256((size_t)N * 8)), st);
}

cat_status tile_lloyd(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, int32_t iters,
                      float* cent_io, double* sums, int32_t* assign, int32_t* counts, double* inertia,
                      unsigned long long* rep, int32_t* skipped, const TileWs& ws, const LloydWs& lw, hipStream_t st,
                      const BoundsWs* bw) {
    // rows are left out by their bounds in the passes 3 .. iters - 1
    const bool bounds = bw && bw->expire && iters >= 4 && tile_bounds_supports(N, D, K, dt);
    if (bounds) skipped = nullptr;  // (a pass over an empty list of rows costs next to nothing already)
    TileCfg c = tile_config(TILE_LLOYD, D, K, dt, bounds);
    if (!c.ok) return set_error(CAT_ERR_UNSUPPORTED, "tile kernels do not fit D=%lld K=%d", (long long)D, (int)K);
    const bool split = !bounds && lw.carry && split_config(D, K, dt, &c);  // (c then describes one of the two launches)
    const int32_t arrays = split ? 2 : 1;
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
    if (iters > 2) CAT_T(launch_fill_zero(lw.ctrl, lloyd_ctrl_words(D) * 4, st));
    if (skipped) CAT_T(launch_fill_zero(skipped, sizeof(int32_t), st));
    if (bw && bw->evaluated) CAT_T(launch_fill_i32(bw->evaluated, (int64_t)iters + 1, (int32_t)N, st));
    if (bounds) CAT_T(launch_fill_zero(bw->drift, ((size_t)iters + 1) * sizeof(double), st));
    // Passes 0 and 1 are each followed by a full segmented sum: after the first reassignment most
    // rows still move, and moving them one by one costs several times a fresh sum (measured: 0.97 ms
    // against 0.33 ms on a 262144 x 2048 bf16 matrix).  From pass 2 on a pass lists the rows that
    // changed cluster, and the launch between two passes moves just those rows between the running
    // sums and prepares the next centroids (k_delta_prep).  The last pass only assigns.
    // With `skipped` given, a pass t in kFullPasses < t < iters whose predecessor listed no row is not run: the
    // partition has stopped changing, so it would reproduce its predecessor.  Both of its launches then return at
    // once (they read the list length on the device; nothing waits on the host), and the final pass runs as always.
    // Counts alternate between two buffers so that a pass never accumulates into the buffer the
    // preparation before it reads; the last pass uses the caller's.
    constexpr int32_t kFullPasses = 2;
    int32_t* cb[2] = {counts, lw.counts2};
    for (int32_t t = 0; t <= iters; t++) {
        const bool last = t == iters;
        double* slot = inertia ? inertia + t : nullptr;
        int32_t* cnt_t = cb[(iters - t) & 1];
        const int32_t* cnt_prev = cb[(iters - t + 1) & 1];
        if (t <= kFullPasses)
            CAT_T(launch_prep(dt, cent_io, t ? base : nullptr, t ? delta : nullptr, t ? cnt_prev : nullptr, cnt_t, D, K, c,
                              ws, slot, last ? rep : nullptr, st, 1, arrays));
        else
            CAT_T(launch_delta_prep(lq, dt, D, K, c, ws, lw, t & 1, cent_io, base, delta, cnt_prev, cnt_t, slot,
                                    last ? rep : nullptr, last ? nullptr : skipped, st, 1, bounds ? bw : nullptr,
                                    t == kFullPasses + 1, split ? kSplitTiles : 0));
        // With bounds: pass 2 evaluates every row and leaves its bound; the passes 3 .. iters - 1 evaluate the rows
        // whose bound the drift of the centroids has used up (selected here, after the update that moved them)
        const bool keeps_bounds = bounds && t >= kFullPasses && !last;
        const bool listed = keeps_bounds && t > kFullPasses;
        if (listed) {
            const int64_t piece = (int64_t)kSelThreads * kSelPerThread;
            int64_t blocks = (N + piece - 1) / piece;
            blocks = blocks > 2048 ? 2048 : blocks;
            hipLaunchKernelGGL(k_bound_select, dim3((unsigned)blocks), dim3(kSelThreads), 0, st, bw->move_part,
                               (int32_t)delta_slices(D), K, bw->drift + t - 1, bw->drift + t, bw->expire, N, bw->rows, bw->n_rows);
            CAT_LAUNCH_CHECK("k_bound_select");
        }
        p.expire = keeps_bounds ? bw->expire : nullptr;
        p.gnow = keeps_bounds ? bw->drift + t : nullptr;
        p.rows = listed ? bw->rows : nullptr;
        p.n_rows = listed ? bw->n_rows : nullptr;
        p.evaluated_slot = (keeps_bounds && bw->evaluated) ? bw->evaluated + t : nullptr;
        p.norm_part = t > kFullPasses ? lw.norm_part : nullptr;
        p.norm_slices = t > kFullPasses ? (int32_t)delta_slices(D) : 0;
        p.counts = listed ? nullptr : cnt_t;  // (a pass over listed rows cannot count: the slices keep running counts)
        p.inertia = listed ? nullptr : slot;
        p.rep = last ? rep : nullptr;  // the final pass describes the partition that is returned
        p.list = (t >= kFullPasses && !last) ? lw.list : nullptr;
        p.list_count = lw.ctrl + (t & 1);
        p.list_cap = lloyd_list_capacity();
        p.delta_mode = p.list ? 1 : 0;
        // alternate the scan direction: the rows a pass reads last are the ones most likely still in
        // the memory-side cache when the next pass starts
        p.reverse = listed ? 0 : (t & 1);
        p.skip_when_zero = (skipped && t > kFullPasses && !last) ? lw.ctrl + ((t - 1) & 1) : nullptr;
        if (split) {
            CAT_T(launch_split_pair(p, c, dt, K, ws, lw.carry, lw.carry_cmax, st));
        } else if (keeps_bounds)
            CAT_T(dt == CAT_BF16 ? launch_bounds_bf16(p, c, st) : launch_bounds_f32(p, c, st));
        else
            CAT_T(launch_tile(p, c, dt, st));
        if (t < kFullPasses && !last) {  // full sums of this pass's partition
            CAT_T(launch_fill_zero(sums, (t == 0 ? 2 : 1) * KD * sizeof(double), st));
            if (lw.sort_ws && segsum_sorted_supported(1, N, D, dt))
                CAT_T(launch_segsum_sorted(1, lq, nullptr, dt, assign, cnt_t, N, D, K, nullptr, nullptr, base, lw.sort_ws, st));
            else
                CAT_T(launch_segsum(1, lq, nullptr, dt, assign, N, D, K, nullptr, nullptr, base, st));
        }
    }
    if (bounds && inertia && iters > kFullPasses + 1)  // the objective of a pass over listed rows is not known
        CAT_T(launch_fill_u64((unsigned long long*)(inertia + kFullPasses + 1), iters - kFullPasses - 1, 0x7ff8000000000000ull, st));
#undef CAT_T
    return CAT_OK;
}

// ---- several centroid sets side by side: fits for a grid of cluster counts that share every read of the rows ----
// Column `s` of the N x 16 assignment table of the multi-set passes (slot numbers of the concatenation), as cluster
// numbers of that set.
__global__ __launch_bounds__(256) void k_multi_column(const int32_t* assign16, int64_t N, int32_t s, int32_t slot0,
                                                      int32_t* out) {
    const int64_t i = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < N) out[i] = assign16[i * 16 + s] - slot0;
}

cat_status launch_multi_column(const int32_t* assign16, int64_t N, int32_t s, int32_t slot0, int32_t* out, hipStream_t st) {
    const int64_t blocks = (N + 255) / 256;
    hipLaunchKernelGGL(k_multi_column, dim3((unsigned)blocks), dim3(256), 0, st, assign16, N, s, slot0, out);
    CAT_LAUNCH_CHECK("k_multi_column");
    return CAT_OK;
}

bool tile_multi_supports(int64_t N, int64_t D, int32_t slots, int32_t nsets, cat_dtype dt) {
    // only with the two-part operand: the one-part variants rank with a wide error bound (many exact re-ranks) and
    // leave an objective of a few digits, which a set would not get when fitted alone
    return nsets >= 1 && nsets <= 16 && slots % 16 == 0 && N * (int64_t)nsets < ((int64_t)1 << 32) &&
           N < ((int64_t)1 << 34) && tile_config(TILE_LLOYD, D, slots, dt, true).ok;
}

cat_status tile_lloyd_multi(const void* lq, cat_dtype dt, int64_t N, int64_t D, const MultiSets& ms, int32_t iters,
                            float* cent_io, double* sums, int32_t* assign16, int32_t* counts, double* inertia16,
                            unsigned long long* rep, int32_t* column, const TileWs& ws, const LloydWs& lw, hipStream_t st) {
    const int32_t K = 16 * ms.t0[ms.nsets];  // slots of the concatenation
    if (!tile_multi_supports(N, D, K, ms.nsets, dt))
        return set_error(CAT_ERR_UNSUPPORTED, "tile kernels do not fit D=%lld with %d cluster slots in %d sets", (long long)D,
                         (int)K, (int)ms.nsets);
    TileCfg c = tile_config(TILE_LLOYD, D, K, dt, true);
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
    p.assign = assign16;
    p.nsets = ms.nsets;
    for (int i = 0; i < ms.nsets; i++) p.set_k[i] = (int16_t)ms.k[i];
    for (int i = 0; i <= ms.nsets; i++) p.set_t0[i] = (uint8_t)ms.t0[i];
    if (iters > 2) CAT_T(launch_fill_zero(lw.ctrl, lloyd_ctrl_words(D) * 4, st));
    // The same sequence as tile_lloyd over the concatenated cluster slots (no early stop: the sets settle at
    // different passes).  The full sums after passes 0 and 1 run set by set on that set's column of the table.
    constexpr int32_t kFullPasses = 2;
    int32_t* cb[2] = {counts, lw.counts2};
    for (int32_t t = 0; t <= iters; t++) {
        const bool last = t == iters;
        double* slot = inertia16 ? inertia16 + (size_t)t * 16 : nullptr;
        int32_t* cnt_t = cb[(iters - t) & 1];
        const int32_t* cnt_prev = cb[(iters - t + 1) & 1];
        if (t <= kFullPasses)
            CAT_T(launch_prep(dt, cent_io, t ? base : nullptr, t ? delta : nullptr, t ? cnt_prev : nullptr, cnt_t, D, K, c,
                              ws, slot, last ? rep : nullptr, st, ms.nsets));
        else
            CAT_T(launch_delta_prep(lq, dt, D, K, c, ws, lw, t & 1, cent_io, base, delta, cnt_prev, cnt_t, slot,
                                    last ? rep : nullptr, nullptr, st, ms.nsets));
        p.norm_part = t > kFullPasses ? lw.norm_part : nullptr;
        p.norm_slices = t > kFullPasses ? (int32_t)delta_slices(D) : 0;
        p.counts = cnt_t;
        p.inertia = slot;
        p.rep = last ? rep : nullptr;
        p.list = (t >= kFullPasses && !last) ? lw.list : nullptr;
        p.list_count = lw.ctrl + (t & 1);
        p.list_cap = lloyd_list_capacity();
        p.delta_mode = p.list ? 1 : 0;
        p.reverse = t & 1;
        CAT_T(dt == CAT_BF16 ? launch_multi_bf16(p, c, st) : launch_multi_f32(p, c, st));
        if (t < kFullPasses && !last) {
            CAT_T(launch_fill_zero(sums, (t == 0 ? 2 : 1) * KD * sizeof(double), st));
            for (int i = 0; i < ms.nsets; i++) {
                const int32_t slot0 = 16 * ms.t0[i];
                CAT_T(launch_multi_column(assign16, N, i, slot0, column, st));
                double* acc = base + (size_t)slot0 * D;
                if (lw.sort_ws && segsum_sorted_supported(1, N, D, dt))
                    CAT_T(launch_segsum_sorted(1, lq, nullptr, dt, column, cnt_t + slot0, N, D, ms.k[i], nullptr, nullptr, acc,
                                               lw.sort_ws, st));
                else
                    CAT_T(launch_segsum(1, lq, nullptr, dt, column, N, D, ms.k[i], nullptr, nullptr, acc, st));
            }
        }
    }
#undef CAT_T
    return CAT_OK;
}

}  // namespace cat
