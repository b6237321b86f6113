// D^2-weighted seeding of the centroids ("k-means++", Arthur and Vassilvitskii, SODA 2007): an alternative
// to the seeded distinct rows; the paper fixes no k-means initialisation (Sec. 4, Setup).
//
// Round t (1 <= t < K) is two launches.  k_pp_update reads every row once: squared distance to the row
// chosen last (direct form, doubles), d2 = min(d2, that), and the sum of d2 over every 64 consecutive rows.
// k_pp_pick (one workgroup) adds those sums in index order, draws u_t from the SplitMix64 counter stream and
// walks to the first row whose running sum exceeds u_t times the total.  Every sum has a fixed order, so
// a seed always gives the same rows.  HBM-bound: K - 1 reads of the matrix.
#include "cat_common.h"

namespace cat {

constexpr int kPpWaves = 4;
constexpr int kPpRowsPerWave = 16;
constexpr int kPpGroup = kPpWaves * kPpRowsPerWave;  // rows per partial sum
constexpr int kPickThreads = 1024;

__device__ __forceinline__ double pp_uniform(uint64_t seed, uint64_t t) {
    return (double)(splitmix64_at(seed, t) >> 11) * 0x1.0p-53;  // [0, 1)
}

__global__ void k_pp_first(int64_t N, uint64_t seed, int64_t* idx) {
    if (threadIdx.x != 0) return;
    int64_t pick = (int64_t)(pp_uniform(seed, 0) * (double)N);
    idx[0] = pick > N - 1 ? N - 1 : pick;
}

// 16 bytes of a row as floats: 4 (fp32) or 8 (bf16) channels
__device__ __forceinline__ void ld16(const float* p, float (&o)[8]) {
    const float4 v = *(const float4*)p;
    o[0] = v.x, o[1] = v.y, o[2] = v.z, o[3] = v.w;
}
__device__ __forceinline__ void ld16(const bf16_t* p, float (&o)[8]) {
    const uint4 v = *(const uint4*)p;
    o[0] = __uint_as_float(v.x << 16), o[1] = __uint_as_float(v.x & 0xFFFF0000u);
    o[2] = __uint_as_float(v.y << 16), o[3] = __uint_as_float(v.y & 0xFFFF0000u);
    o[4] = __uint_as_float(v.z << 16), o[5] = __uint_as_float(v.z & 0xFFFF0000u);
    o[6] = __uint_as_float(v.w << 16), o[7] = __uint_as_float(v.w & 0xFFFF0000u);
}

// GROUP lanes per row (64, or 16 for short rows: four rows per wave at a time), 16 rows per wave, 64 rows per
// workgroup and partial sum.  WIDE: 16-byte loads, two per operand in flight (D a multiple of the 16-byte
// group, aligned base); else one channel per lane.  Rows past the end are clamped to the last row and dropped
// at the end, so that the shuffles below always run with all lanes.
template <typename T, bool WIDE, int GROUP>
__global__ __launch_bounds__(kPpWaves* kWave) void k_pp_update(const T* __restrict__ x, int64_t N, int64_t D,
                                                               const int64_t* __restrict__ idx, int t,
                                                               double* __restrict__ d2, double* __restrict__ part) {
    __shared__ double s_sum[kPpWaves];
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int sub = lane & (GROUP - 1), grp = lane / GROUP;
    constexpr int RPI = kWave / GROUP;  // rows per iteration of a wave
    constexpr int EPL = (int)(16 / sizeof(T));
    const T* c = x + idx[t - 1] * D;  // the row chosen last
    const int64_t row0 = (int64_t)blockIdx.x * kPpGroup + (int64_t)wave * kPpRowsPerWave;
    double run = 0.0;  // lane 0: the wave's rows, in row order
    // RU row groups at a time: all their loads are requested before the first sum, and the chosen row is read once for
    // all of them.  Every load is unconditional (rows past the end repeat the last row, a second vector past the row
    // repeats the first), so that they overlap; what a row adds up, and in which order, does not depend on RU.
    constexpr int RU = 4;
    for (int r = 0; r < kPpRowsPerWave; r += RPI * RU) {
        if (row0 + r >= N) break;  // wave-uniform
        bool row_ok[RU];
        int64_t row[RU];
        const T* xr[RU];
        double old[RU], s[RU];
#pragma unroll
        for (int u = 0; u < RU; u++) {
            const int64_t rr = row0 + r + u * RPI + grp;
            row_ok[u] = rr < N;
            row[u] = row_ok[u] ? rr : N - 1;
            xr[u] = x + row[u] * D;
            // the row's distance so far, requested ahead of the row itself (its leader lane needs it at the end)
            old[u] = d2[row[u]];
            s[u] = 0.0;
        }
        if (WIDE) {
            const int64_t step = (int64_t)GROUP * EPL;
            for (int64_t j0 = (int64_t)sub * EPL; j0 < D; j0 += 2 * step) {
                const int64_t j1 = j0 + step;
                const bool two = j1 < D;
                float xa[RU][8], xb[RU][8], ca[8], cb[8];
                ld16(c + j0, ca);
                ld16(c + (two ? j1 : j0), cb);
#pragma unroll
                for (int u = 0; u < RU; u++) {
                    ld16(xr[u] + j0, xa[u]);
                    ld16(xr[u] + (two ? j1 : j0), xb[u]);
                }
#pragma unroll
                for (int u = 0; u < RU; u++) {
#pragma unroll
                    for (int e = 0; e < EPL; e++) {
                        const double d = (double)xa[u][e] - (double)ca[e];
                        s[u] = fma(d, d, s[u]);
                    }
                    if (two) {
#pragma unroll
                        for (int e = 0; e < EPL; e++) {
                            const double d = (double)xb[u][e] - (double)cb[e];
                            s[u] = fma(d, d, s[u]);
                        }
                    }
                }
            }
        } else {
            for (int64_t j = sub; j < D; j += GROUP) {
                const double cj = (double)ld_elem(c + j);
#pragma unroll
                for (int u = 0; u < RU; u++) {
                    const double d = (double)ld_elem(xr[u] + j) - cj;
                    s[u] = fma(d, d, s[u]);
                }
            }
        }
#pragma unroll
        for (int u = 0; u < RU; u++) {
            double su = s[u];
#pragma unroll
            for (int o = GROUP / 2; o > 0; o >>= 1) su += __shfl_xor(su, o, kWave);
            double v = su;
            if (t > 1) v = su < old[u] ? su : old[u];
            if (sub == 0 && row_ok[u]) d2[row[u]] = v;
            if (!row_ok[u]) v = 0.0;
#pragma unroll
            for (int g = 0; g < RPI; g++) {  // the group leaders' values reach lane 0 in row order
                const double vg = __shfl(v, g * GROUP, kWave);
                run += vg;
            }
        }
    }
    if (lane == 0) s_sum[wave] = run;
    __syncthreads();
    if (threadIdx.x == 0) {
        double tot = 0.0;
        for (int w = 0; w < kPpWaves; w++) tot += s_sum[w];
        part[blockIdx.x] = tot;
    }
}

// ---- the pick: one workgroup of 1024 threads --------------------------------------------------
// Inclusive prefix sums over the threads of the workgroup in a fixed association (a shuffle scan inside
// each wave, the wave totals added in wave order).  s_incl receives every thread's result, `total` the last one.
struct PickShared {
    double incl[kPickThreads];
    double wave_tot[kPickThreads / kWave];
    int first;
};
__device__ __forceinline__ double pick_scan(double v, PickShared& sh, double& total) {
    const int tid = threadIdx.x, lane = tid & (kWave - 1), wave = tid / kWave;
#pragma unroll
    for (int o = 1; o < kWave; o <<= 1) {
        const double u = __shfl_up(v, o, kWave);
        if (lane >= o) v += u;
    }
    __syncthreads();  // the previous use of the shared arrays is over
    if (lane == kWave - 1) sh.wave_tot[wave] = v;
    if (tid == 0) sh.first = kPickThreads;
    __syncthreads();
    double off = 0.0, tot = 0.0;
    for (int w = 0; w < kPickThreads / kWave; w++) {
        if (w == wave) off = tot;
        tot += sh.wave_tot[w];
    }
    total = tot;
    const double r = wave == 0 ? v : off + v;
    sh.incl[tid] = r;
    return r;
}
// the lowest thread whose flag is set (kPickThreads if none); every thread gets the answer
__device__ __forceinline__ int pick_first(bool flag, PickShared& sh) {
    const unsigned long long m = __ballot(flag);
    if (m && (threadIdx.x & (kWave - 1)) == 0) atomicMin(&sh.first, (int)(threadIdx.x + __builtin_ctzll(m)));
    __syncthreads();
    return sh.first;
}

// Running sums are taken level by level: over the 1024 contiguous shares of the partial sums, over the
// partial sums of the share in which the target is crossed, over the rows from there on; at every level the
// first element whose running sum exceeds the target is taken.  With a total of zero (every row coincides
// with a chosen one) the lowest row not chosen yet is taken.
__global__ __launch_bounds__(kPickThreads) void k_pp_pick(const double* __restrict__ d2, const double* __restrict__ part,
                                                          int64_t npart, int64_t N, uint64_t seed, int t,
                                                          int64_t* __restrict__ idx) {
    __shared__ PickShared sh;
    const int tid = threadIdx.x;
    const int64_t per = (npart + kPickThreads - 1) / kPickThreads;
    double v = 0.0;
    {
        const int64_t p0 = (int64_t)tid * per;
        const int64_t p1 = p0 + per < npart ? p0 + per : npart;
        for (int64_t p = p0; p < p1; p++) v += part[p];
    }
    double S;
    double incl = pick_scan(v, sh, S);
    int64_t pick = -1;
    if (S > 0.0) {  // uniform: every thread holds the same S
        const double target = pp_uniform(seed, (uint64_t)t) * S;
        const int share = pick_first(incl > target, sh);  // < kPickThreads: the last running sum is S > target
        const double run_share = share > 0 ? sh.incl[share - 1] : 0.0;  // running sum in front of the share
        double run = run_share;
        // partial sums of that share
        const int64_t pbeg = (int64_t)share * per;
        const int64_t pend = pbeg + per < npart ? pbeg + per : npart;
        int64_t row_beg = pbeg * kPpGroup;  // if rounding lets no partial sum cross: all rows of the share
        for (int64_t base = pbeg; base < pend; base += kPickThreads) {
            const int64_t n = pend - base < kPickThreads ? pend - base : kPickThreads;
            double tot;
            incl = pick_scan(tid < n ? part[base + tid] : 0.0, sh, tot);
            const int i = pick_first(tid < n && run + incl > target, sh);
            if (i < kPickThreads) {
                row_beg = (base + i) * kPpGroup;
                if (i > 0) run += sh.incl[i - 1];
                break;
            }
            if (base + kPickThreads < pend) run += tot;  // on to the next stage; after the last one `run` restarts below
        }
        if (row_beg == pbeg * kPpGroup) run = run_share;
        // rows from there on; rounding may carry the crossing past the end of the partial sum
        for (int64_t base = row_beg; base < N; base += kPickThreads) {
            const int64_t n = N - base < kPickThreads ? N - base : kPickThreads;
            double tot;
            incl = pick_scan(tid < n ? d2[base + tid] : 0.0, sh, tot);
            const int i = pick_first(tid < n && run + incl > target, sh);
            if (i < kPickThreads) {
                pick = base + i;
                break;
            }
            run += tot;
        }
    }
    if (tid != 0) return;
    if (pick < 0) {  // no weight (or u_t S rounded up to S itself): the lowest row not chosen yet
        for (int64_t c = 0; c < N && pick < 0; c++) {
            bool taken = false;
            for (int q = 0; q < t; q++) taken = taken || idx[q] == c;
            if (!taken) pick = c;
        }
    }
    idx[t] = pick;
}

static inline size_t pad256s(size_t v) { return (v + 255) & ~(size_t)255; }

}  // namespace cat

using namespace cat;

extern "C" {

size_t cat_init_kmeanspp_workspace_bytes(int64_t N, int32_t K) {
    if (N < 1 || K < 1) return 0;
    const size_t npart = (size_t)((N + kPpGroup - 1) / kPpGroup);
    return pad256s((size_t)N * 8) + pad256s(npart * 8) + pad256s((size_t)K * 8);
}

cat_status cat_init_kmeanspp(const void* lq, int64_t N, int64_t D, int32_t K, uint64_t seed, cat_dtype dt,
                             float* centroids, int64_t* indices, void* workspace, size_t workspace_bytes,
                             void* hip_stream) {
    if ((dt != CAT_F32 && dt != CAT_BF16) || N < 1 || D < 1 || K < 1 || K > CAT_MAX_K || (int64_t)K > N)
        return set_error(CAT_ERR_INVALID_ARG, "cat_init_kmeanspp: need 1 <= K <= min(N, %d), D >= 1 (N=%lld D=%lld K=%d dt=%d)",
                         CAT_MAX_K, (long long)N, (long long)D, (int)K, (int)dt);
    if (!lq || !centroids) return set_error(CAT_ERR_INVALID_ARG, "cat_init_kmeanspp: null argument");
    if (!workspace || ((uintptr_t)workspace & 255u) || workspace_bytes < cat_init_kmeanspp_workspace_bytes(N, K))
        return set_error(CAT_ERR_WORKSPACE, "cat_init_kmeanspp: workspace of %zu bytes, 256-byte aligned, needed",
                         cat_init_kmeanspp_workspace_bytes(N, K));
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t npart = (N + kPpGroup - 1) / kPpGroup;
    char* b = (char*)workspace;
    double* d2 = (double*)b;
    b += pad256s((size_t)N * 8);
    double* part = (double*)b;
    b += pad256s((size_t)npart * 8);
    int64_t* idx = (int64_t*)b;
    const size_t esz = dt == CAT_F32 ? 4 : 2;
    const bool wide = (D * esz) % 16 == 0 && ((uintptr_t)lq & 15u) == 0;
    // 16 lanes per row, four rows of a wave in flight: rows of at most 1 KB (wide) or 64 channels (narrow), which
    // would leave most of a wave idle otherwise, and fp32 rows up to 4 KB (measured: 44.9 against 50.1 us per
    // launch on 65,536 x 1000 fp32; bf16 rows of 4 KB are 3 % slower that way)
    const bool narrow_rows = wide ? D * esz <= (dt == CAT_F32 ? 4096 : 1024) : D <= 64;

    hipLaunchKernelGGL(k_pp_first, dim3(1), dim3(kWave), 0, st, N, seed, idx);
    CAT_LAUNCH_CHECK("k_pp_first");
    dim3 g((unsigned)npart), blk(kPpWaves * kWave);
    for (int t = 1; t < K; t++) {
#define CAT_PP(T, W, G) \
    hipLaunchKernelGGL((k_pp_update<T, W, G>), g, blk, 0, st, (const T*)lq, N, D, idx, t, d2, part)
        if (dt == CAT_F32) {
            if (wide && narrow_rows) CAT_PP(float, true, 16);
            else if (wide) CAT_PP(float, true, 64);
            else if (narrow_rows) CAT_PP(float, false, 16);
            else CAT_PP(float, false, 64);
        } else {
            if (wide && narrow_rows) CAT_PP(bf16_t, true, 16);
            else if (wide) CAT_PP(bf16_t, true, 64);
            else if (narrow_rows) CAT_PP(bf16_t, false, 16);
            else CAT_PP(bf16_t, false, 64);
        }
#undef CAT_PP
        CAT_LAUNCH_CHECK("k_pp_update");
        hipLaunchKernelGGL(k_pp_pick, dim3(1), dim3(kPickThreads), 0, st, d2, part, npart, N, seed, t, idx);
        CAT_LAUNCH_CHECK("k_pp_pick");
    }
    cat_status s = launch_gather_rows(lq, dt, D, K, idx, centroids, st);
    if (s != CAT_OK) return s;
    if (indices) return launch_copy_words(idx, indices, (int64_t)K * 2, st);
    return CAT_OK;
}

}  // extern "C"
