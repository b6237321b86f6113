// Streaming assignment / inference for the shapes the matrix-core kernels do not hold (rows whose length is not a
// whole number of 16-byte groups, more than 256 clusters): any D, any K <= CAT_MAX_K, any row alignment.
//
// Nearest centroid (Algorithm 1 "Cluster-Model fit", Algorithm 2 "predict"): argmin_k |x - c_k|^2, lowest index on
// ties.  A workgroup of 4 waves owns a tile of 256 rows, ONE ROW PER LANE, and walks the channels in chunks of 32:
//   - the chunk of the rows travels global -> registers -> LDS with coalesced element loads (a wave instruction
//     reads 32 consecutive channels of two rows), one chunk ahead of the arithmetic;
//   - the same chunk of up to 64 centroids is staged beside it;
//   - every lane then accumulates x . c_k for its row in fp32 FMAs: one 16-byte LDS read of its row and, per
//     centroid, one 16-byte broadcast read feed four FMAs; the K running dot products stay in registers.
// The scores |c_k|^2 - 2 x . c_k rank the centroids inside the lane: no cross-lane step at all.  A row whose two best
// scores are closer than the rounding bound of the fp32 accumulation (tau |x| max|c| + tau2 max|c|^2,
// tau = 4 (D + 4) 2^-24) is re-ranked with direct-form double-precision distances, the whole wave on the row, over the
// centroids inside the bound (all of them when K > 64), so the result is the exact nearest centroid as in the
// matrix-core kernels.  With more than 64 clusters the tile is walked once per group of 64.
// Inference (APPLY) then maps the 64 rows of each wave four rows at a time, lanes side by side over the channels.
#include "cat_common.h"

namespace cat {

namespace {

constexpr int kLT = 256;     // threads = rows of a tile
constexpr int kLC = 32;      // channels per chunk
constexpr int kLS = 36;      // floats between rows in LDS (16-byte aligned; 9 x 16 bytes: conflict-free 16-byte reads)
constexpr int kLPT = kLC;    // elements of a chunk per thread (256 rows x 32 channels / 256 threads)

typedef __attribute__((ext_vector_type(4))) float lf4;

template <typename T, int KG, bool APPLY>
__global__ __launch_bounds__(kLT, 2) void k_assign_lds(const T* __restrict__ lq, int64_t N, int64_t D, int32_t K,
                                                    const float* __restrict__ cent, int32_t* __restrict__ assign,
                                                    int32_t* counts, double* inertia, unsigned long long* rep,
                                                    const float* __restrict__ gamma, const float* __restrict__ beta,
                                                    T* __restrict__ out, float tau, float tau2) {
    __shared__ __align__(16) float xs[kLT * kLS];
    __shared__ __align__(16) float cs[KG * kLS];
    __shared__ float s_cnorm[CAT_MAX_K];
    __shared__ int s_cnt[CAT_MAX_K];
    __shared__ unsigned long long s_rep[CAT_MAX_K];
    __shared__ double s_in[kLT / kWave];
    const int tid = threadIdx.x;
    const int lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const bool hist = counts != nullptr || rep != nullptr;
    const int ngroups = (K + KG - 1) / KG;
    const int nchunks = (int)((D + kLC - 1) / kLC);

    // ---- prologue: squared norms of the centroids in double (a wave per centroid), tables ----
    for (int k = wave; k < K; k += kLT / kWave) {
        const float* c = cent + (int64_t)k * D;
        double s = 0.0;
        for (int64_t j = lane; j < D; j += kWave) {
            const double v = (double)c[j];
            s = fma(v, v, s);
        }
        s = wave_sum(s);
        if (lane == 0) s_cnorm[k] = (float)s;
    }
    for (int k = tid; k < K; k += kLT) {
        s_cnt[k] = 0;
        s_rep[k] = ~0ull;
    }
    __syncthreads();
    float cmax;
    {
        float m = 0.f;
        for (int k = lane; k < K; k += kWave) m = fmaxf(m, s_cnorm[k]);
#pragma unroll
        for (int o = 32; o > 0; o >>= 1) m = fmaxf(m, __shfl_xor(m, o, kWave));
        cmax = sqrtf(m) * 1.000001f;
    }

    // element e = i * 256 + tid of a chunk: row e / 32 of the tile, channel e % 32 of the chunk
    const int ech = tid & (kLC - 1);
    const int erow = tid / kLC;  // + 8 i
    double in_acc = 0.0;
    const int64_t ntiles = (N + kLT - 1) / kLT;
    for (int64_t tile = blockIdx.x; tile < ntiles; tile += gridDim.x) {
        const int64_t row0 = tile * kLT;
        const int64_t myrow = row0 + tid;
        const bool valid = myrow < N;
        float b1 = __builtin_inff(), b2 = __builtin_inff(), xn2 = 0.f;
        int i1 = 0;
        float acc[KG];
        for (int g = 0; g < ngroups; g++) {
            const int k0 = g * KG;
#pragma unroll
            for (int k = 0; k < KG; k++) acc[k] = 0.f;
            float xr[kLPT];
            // rows past N repeat the last row, channels past D the last channel (valid addresses, no conditional
            // load); the padding is zeroed on its way into LDS
            auto fetch = [&](int c) {
                const int64_t ch = (int64_t)c * kLC + ech;
                const int64_t chc = ch < D ? ch : D - 1;
                const int64_t lastl = N - 1 - row0;  // last valid row of the tile, relative
                const int last = lastl < kLT ? (int)lastl : kLT;
                // (the row length is made opaque so that the 32 row offsets are recomputed per chunk, one multiply-add
                // each, instead of being kept in 64 registers across the chunk loop)
                int64_t Dv = D;
                asm volatile("" : "+s"(Dv));
                const T* base = lq + row0 * Dv + chc;
#pragma unroll
                for (int i = 0; i < kLPT; i++) {
                    const int rr = erow + 8 * i;
                    xr[i] = ld_elem(base + (int64_t)(rr < last ? rr : last) * Dv);
                }
            };
            // the same chunk of the group's centroids, one chunk ahead like the rows (clusters past K repeat the last
            // one, channels past D the last channel; zeroed on the way into LDS)
            float cr[KG * kLC / kLT];
            auto cfetch = [&](int c) {
                const int64_t ch = (int64_t)c * kLC + ech;
                const int64_t chc = ch < D ? ch : D - 1;
#pragma unroll
                for (int i = 0; i < KG * kLC / kLT; i++) {
                    const int k = k0 + erow + 8 * i;
                    cr[i] = cent[(int64_t)(k < K ? k : K - 1) * D + chc];
                }
            };
            fetch(0);
            cfetch(0);
            for (int c = 0; c < nchunks; c++) {
                // chunk c of the rows and of the centroids: registers -> LDS
#pragma unroll
                for (int i = 0; i < kLPT; i++)
                    xs[(erow + 8 * i) * kLS + ech] = (row0 + erow + 8 * i < N && (int64_t)c * kLC + ech < D) ? xr[i] : 0.f;
                {
                    const int64_t ch = (int64_t)c * kLC + ech;
#pragma unroll
                    for (int i = 0; i < KG * kLC / kLT; i++) {
                        const int k = erow + 8 * i;
                        cs[k * kLS + ech] = (k0 + k < K && ch < D) ? cr[i] : 0.f;
                    }
                }
                __syncthreads();
                // chunk c + 1 is requested by every wave on every pass (after the last chunk: the last one again, unused),
                // so that the compiler can count the loads in flight instead of waiting for all of them
                fetch(c + 1 < nchunks ? c + 1 : c);
                cfetch(c + 1 < nchunks ? c + 1 : c);
                const float* xrow = xs + tid * kLS;
#pragma unroll 1
                for (int j = 0; j < kLC; j += 4) {
                    const lf4 x = *(const lf4*)(xrow + j);
                    if (g == 0) xn2 = fmaf(x.x, x.x, fmaf(x.y, x.y, fmaf(x.z, x.z, fmaf(x.w, x.w, xn2))));
                    // the centroid reads go out eight at a time, ahead of their FMAs
#pragma unroll
                    for (int kb = 0; kb < KG; kb += 8) {
                        lf4 cv[8];
#pragma unroll
                        for (int u = 0; u < 8; u++) cv[u] = *(const lf4*)(cs + (kb + u) * kLS + j);
#pragma unroll
                        for (int u = 0; u < 8; u++)
                            acc[kb + u] = fmaf(x.x, cv[u].x, fmaf(x.y, cv[u].y, fmaf(x.z, cv[u].z, fmaf(x.w, cv[u].w, acc[kb + u]))));
                    }
                }
                __syncthreads();
            }
            // scores of this group into the running best / second best (ascending k: the lowest index keeps a tie)
#pragma unroll
            for (int k = 0; k < KG; k++) {
                const float s = k0 + k < K ? fmaf(-2.f, acc[k], s_cnorm[k0 + k < K ? k0 + k : 0]) : __builtin_inff();
                acc[k] = s;
                if (s < b1) {
                    b2 = b1;
                    b1 = s;
                    i1 = k0 + k;
                } else if (s < b2) {
                    b2 = s;
                }
            }
        }
        // ---- exact re-rank of the rows inside the rounding bound ----
        const float Tb = tau * sqrtf(xn2) * cmax + tau2 * cmax * cmax;
        float dmin = fmaxf(xn2 + b1, 0.f);
        unsigned long long mask = __ballot(valid && !(b2 - b1 > Tb));
        while (mask) {
            const int r = __builtin_amdgcn_readfirstlane(__builtin_ctzll(mask));
            mask &= mask - 1;
            const int64_t row = row0 + wave * kWave + r;
            const float thr = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(b1 + Tb), r));
            const T* x = lq + row * D;
            double dbest = __builtin_inf();
            int kbest = 0x7fffffff;
            auto measure = [&](int k) {
                const float* c = cent + (int64_t)k * D;
                double s = 0.0;
                for (int64_t j = lane; j < D; j += kWave) {
                    const double d = (double)ld_elem(x + j) - (double)c[j];
                    s = fma(d, d, s);
                }
                s = wave_sum(s);
                if (s < dbest || (s == dbest && k < kbest)) {
                    dbest = s;
                    kbest = k;
                }
            };
            if (ngroups == 1) {
                // the candidates: one per lane, then measured (acc[] holds the scores of the only group)
                int cand = 0, cnt = 0;
#pragma unroll
                for (int k = 0; k < KG; k++) {
                    const float s = __int_as_float(__builtin_amdgcn_readlane(__float_as_int(acc[k]), r));
                    if (s <= thr && k < K) {  // wave-uniform
                        if (lane == cnt) cand = k;
                        cnt++;
                    }
                }
                for (int c = 0; c < cnt; c++) measure(__builtin_amdgcn_readlane(cand, c));
            } else {
                for (int k = 0; k < K; k++) measure(k);
            }
            if (lane == r && kbest != 0x7fffffff) {
                i1 = kbest;
                dmin = (float)dbest;
            }
        }
        const int idx = i1 < K ? i1 : K - 1;  // non-finite rows: unspecified result, index inside the tables
        if (valid) {
            if (assign) assign[myrow] = idx;
            if (hist) {
                atomicAdd(&s_cnt[idx], 1);
                atomicMin(&s_rep[idx], (unsigned long long)myrow);
            }
            in_acc += (double)dmin;
        }
        if (APPLY) {
            // four rows at a time, lanes side by side over the channels: twelve independent loads per lane and step
            for (int r0 = 0; r0 < kWave; r0 += 4) {
                if (row0 + wave * kWave + r0 >= N) break;  // wave-uniform
                const T* x[4];
                T* o[4];
                const float* gr[4];
                const float* br[4];
                bool on[4];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    const int64_t row = row0 + wave * kWave + r0 + u;
                    on[u] = row < N;
                    const int64_t rc = on[u] ? row : N - 1;
                    const int a = __builtin_amdgcn_readlane(idx, (r0 + u) & (kWave - 1));
                    x[u] = lq + rc * D;
                    o[u] = out + rc * D;
                    gr[u] = gamma + (int64_t)(on[u] ? a : 0) * D;
                    br[u] = beta + (int64_t)(on[u] ? a : 0) * D;
                }
                // four steps of 64 channels at a time: 48 independent loads per lane before the first store (channels
                // past D repeat the lane's first channel of the step group and are not stored)
                for (int64_t j0 = lane; j0 < D; j0 += 4 * kWave) {
                    float xv[4][4], gv[4][4], bv[4][4];
#pragma unroll
                    for (int v = 0; v < 4; v++) {
                        const int64_t j = j0 + v * kWave < D ? j0 + v * kWave : j0;
#pragma unroll
                        for (int u = 0; u < 4; u++) {
                            xv[v][u] = ld_elem(x[u] + j);
                            gv[v][u] = gr[u][j];
                            bv[v][u] = br[u][j];
                        }
                    }
#pragma unroll
                    for (int v = 0; v < 4; v++) {
                        const int64_t j = j0 + v * kWave;
#pragma unroll
                        for (int u = 0; u < 4; u++)
                            if (on[u] && j < D) st_elem(o[u] + j, fmaf(gv[v][u], xv[v][u], bv[v][u]));
                    }
                }
            }
        }
    }
    if (hist || inertia) {
        in_acc = wave_sum(in_acc);
        if (lane == 0) s_in[wave] = in_acc;
        __syncthreads();
        if (hist)
            for (int k = tid; k < K; k += kLT) {
                if (counts && s_cnt[k]) atomicAdd(&counts[k], s_cnt[k]);
                if (rep && s_rep[k] != ~0ull) atomicMin(&rep[k], s_rep[k]);
            }
        if (inertia && tid == 0) {
            double tot = 0.0;
            for (int w = 0; w < kLT / kWave; w++) tot += s_in[w];
            atomicAdd(inertia, tot);
        }
    }
}

template <typename T, int KG>
cat_status launch_kg(const void* lq, int64_t N, int64_t D, int32_t K, const float* cent, int32_t* assign, int32_t* counts,
                     double* inertia, unsigned long long* rep, const float* gamma, const float* beta, void* corrected,
                     hipStream_t st) {
    const int64_t ntiles = (N + kLT - 1) / kLT;
    const unsigned blocks = (unsigned)(ntiles < 512 ? ntiles : 512);
    // rounding bound of a score difference as a fraction of |x| |c|: two dot products of D fp32 FMAs each, doubled in
    // the score, plus the roundings of the norm, of the score and of |x|^2 itself
    const float du = (float)(D + 4) * 5.9604645e-8f;
    const float tau = (1.01f + du) * 4.f * du, tau2 = 4.0e-7f;
    if (gamma)
        hipLaunchKernelGGL((k_assign_lds<T, KG, true>), dim3(blocks), dim3(kLT), 0, st, (const T*)lq, N, D, K, cent, assign,
                           counts, inertia, rep, gamma, beta, (T*)corrected, tau, tau2);
    else
        hipLaunchKernelGGL((k_assign_lds<T, KG, false>), dim3(blocks), dim3(kLT), 0, st, (const T*)lq, N, D, K, cent, assign,
                           counts, inertia, rep, gamma, beta, (T*)corrected, tau, tau2);
    CAT_LAUNCH_CHECK("k_assign_lds");
    return CAT_OK;
}

}  // namespace

cat_status launch_assign_lds(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                             int32_t* assign, int32_t* counts, double* inertia, unsigned long long* rep,
                             const float* gamma, const float* beta, void* corrected, hipStream_t st) {
#define CAT_LDS(T)                                                                                                         \
    (K <= 16 ? launch_kg<T, 16>(lq, N, D, K, cent, assign, counts, inertia, rep, gamma, beta, corrected, st)              \
     : K <= 32 ? launch_kg<T, 32>(lq, N, D, K, cent, assign, counts, inertia, rep, gamma, beta, corrected, st)            \
               : launch_kg<T, 64>(lq, N, D, K, cent, assign, counts, inertia, rep, gamma, beta, corrected, st))
    return dt == CAT_F32 ? CAT_LDS(float) : CAT_LDS(bf16_t);
#undef CAT_LDS
}

}  // namespace cat
