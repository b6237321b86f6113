// Sweep of the blending coefficient (the alpha display of Sec. 3.1; the ablation on alpha, Sec. 5):
// one pass over the rows evaluates a fitted transformation at a whole list of alpha values.
//
// With t = (gamma_a - 1) x + beta_a, the corrected entry is x + alpha t.  Per alpha the pass keeps the
// position of the largest corrected entry of the row (Top-1) and counts the rows where it equals a given
// label.  The squared error to fp is a parabola in alpha, sum (x - f)^2 + 2 alpha sum (x - f) t +
// alpha^2 sum t^2, so three sums cover every alpha.  HBM-bound: each row of lq (and fp) is read once,
// whatever the length of the list; gamma and beta rows come from L2.
#include <limits.h>

#include <type_traits>

#include "cat_common.h"

namespace cat {

struct SweepAlphas {
    float v[CAT_MAX_ALPHAS];
};

constexpr int kSweepWaves = 4;
constexpr int kSweepMaxGrid = 2048;  // 8 workgroups of 4 waves per CU walk the rows

// What the workgroups of the sweep leave behind: quantity-major, one slot per workgroup, so that the
// launch that adds them reads consecutive words.  Quantities 0..2 are the three sums (doubles), 3 + s the
// Top-1 hits of alpha s (64-bit counts).
constexpr int kSweepQuantities = 3 + CAT_MAX_ALPHAS;
struct SweepPartial {
    unsigned long long slot[kSweepQuantities][kSweepMaxGrid];
};

__device__ __forceinline__ void ld_vec4(const float* p, float (&o)[4]) {
    const float4 v = *(const float4*)p;
    o[0] = v.x, o[1] = v.y, o[2] = v.z, o[3] = v.w;
}
__device__ __forceinline__ void ld_vec4(const bf16_t* p, float (&o)[4]) {
    const uint2 v = *(const uint2*)p;
    o[0] = __uint_as_float(v.x << 16), o[1] = __uint_as_float(v.x & 0xFFFF0000u);
    o[2] = __uint_as_float(v.y << 16), o[3] = __uint_as_float(v.y & 0xFFFF0000u);
}
template <int VEC, typename T>
__device__ __forceinline__ void ld_vec(const T* p, float (&o)[4]) {
    if (VEC == 4)
        ld_vec4(p, o);
    else
        o[0] = ld_elem(p);
}

// ---- reductions over the 16 lanes of a DPP row: quad swaps, then the mirror of 8 and of 16 lanes.  Each
// step is a lane permutation inside the row, so every lane ends with the result of its own row.
// All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ int row_perm(int v) {
    return __builtin_amdgcn_update_dpp(0, v, CTRL, 0xF, 0xF, true);
}
constexpr int kQuadSwap1 = 0xB1;    // quad_perm [1, 0, 3, 2]
constexpr int kQuadSwap2 = 0x4E;    // quad_perm [2, 3, 0, 1]
constexpr int kHalfMirror = 0x141;  // lane i <-> 7 - i within 8 lanes
constexpr int kRowMirror = 0x140;   // lane i <-> 15 - i within 16 lanes
__device__ __forceinline__ float row16_max(float v) {
    v = fmaxf(v, __int_as_float(row_perm<kQuadSwap1>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(row_perm<kQuadSwap2>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(row_perm<kHalfMirror>(__float_as_int(v))));
    v = fmaxf(v, __int_as_float(row_perm<kRowMirror>(__float_as_int(v))));
    return v;
}
__device__ __forceinline__ int row16_min(int v) {
    v = min(v, row_perm<kQuadSwap1>(v));
    v = min(v, row_perm<kQuadSwap2>(v));
    v = min(v, row_perm<kHalfMirror>(v));
    v = min(v, row_perm<kRowMirror>(v));
    return v;
}

constexpr int kGroup = 16;              // lanes that share one matrix row
constexpr int kRowsPerWave = kWave / kGroup;

// Running Top-1 per alpha and the three sums of the parabola, over VEC consecutive entries.  Top-1 needs
// no mask: an entry loaded again from the clamped position carries a position past the end of the row
// and the value of its original, so the original (lower position) wins the tie; the same holds for a
// clamped row, whose results are dropped anyway.  Updates are selects, not branches.
template <int NA, int VEC, bool ARG, bool ERR, bool MASKED>
__device__ __forceinline__ void sweep_entries(const float (&x)[4], const float (&f)[4], const float (&g)[4],
                                              const float (&b)[4], bool inside, bool valid, int j,
                                              const SweepAlphas& al, float (&best)[NA], int (&bidx)[NA],
                                              float& saa, float& sab, float& sbb) {
#pragma unroll
    for (int e = 0; e < VEC; e++) {
        const float t = inside ? fmaf(x[e], g[e] - 1.f, b[e]) : 0.f;
        if (ARG) {
            const int pos = j + e;
#pragma unroll
            for (int s = 0; s < NA; s++) {
                const float y = fmaf(al.v[s], t, x[e]);
                const bool up = y > best[s];  // strict: a lane keeps the first of equal entries
                best[s] = up ? y : best[s];
                bidx[s] = up ? pos : bidx[s];
            }
        }
        if (ERR) {
            const bool use = !MASKED || valid;
            const float a = use ? x[e] - f[e] : 0.f, te = use ? t : 0.f;
            saa = fmaf(a, a, saa);
            sab = fmaf(a, te, sab);
            sbb = fmaf(te, te, sbb);
        }
    }
}

// Sixteen lanes per matrix row, four rows per wave at a time; a lane takes VEC consecutive entries per
// step, so the Top-1 reduction of a row stays inside one DPP row.  The part of a row that fills whole
// steps runs without masks; the rest is one more step that loads from a clamped position (always inside
// the row) where it would leave the row and masks what it must not count.  Rows past the end are clamped to the last row and masked the same
// way, so that no load, and no lane of a reduction, is conditional.
template <typename T, int NA, int VEC, bool ARG, bool ERR>
__global__ __launch_bounds__(kSweepWaves* kWave) void k_alpha_sweep(
    const T* __restrict__ x, const T* __restrict__ fp, const int32_t* __restrict__ labels,
    const int32_t* __restrict__ assign, int64_t N, int64_t D, int32_t K, const float* __restrict__ gamma,
    const float* __restrict__ beta, const SweepAlphas al, int n_alpha, SweepPartial* __restrict__ part,
    int32_t* __restrict__ top1) {
    __shared__ double s_mom[kSweepWaves][3];
    __shared__ unsigned s_hit[kSweepWaves][CAT_MAX_ALPHAS];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = threadIdx.x / kWave;
    const int sub = lane & (kGroup - 1), grp = lane / kGroup;
    const int64_t gw = (int64_t)blockIdx.x * kSweepWaves + threadIdx.x / kWave;
    const int64_t nw = (int64_t)gridDim.x * kSweepWaves;
    constexpr int STEP = kGroup * VEC;
    constexpr int U = NA <= 4 ? 4 : 2;  // vectors per lane and step; short lists leave registers for more
    const int64_t Dfull = D / (U * STEP) * (U * STEP);
    const int64_t jlast = D - VEC;  // last position a whole vector fits at

    unsigned hit[NA];
#pragma unroll
    for (int s = 0; s < NA; s++) hit[s] = 0u;
    double maa = 0.0, mab = 0.0, mbb = 0.0;

    for (int64_t row0 = gw * kRowsPerWave; row0 < N; row0 += nw * kRowsPerWave) {
        const bool row_ok = row0 + grp < N;
        const int64_t row = row_ok ? row0 + grp : N - 1;
        const int a = assign[row];
        const bool inside = a >= 0 && a < K;  // a label outside [0, K) leaves the row as it is
        const float* gr = gamma + (int64_t)(inside ? a : 0) * D;
        const float* br = beta + (int64_t)(inside ? a : 0) * D;
        const T* xr = x + row * D;
        const T* fr = ERR ? fp + row * D : xr;
        float best[NA];
        int bidx[NA];
#pragma unroll
        for (int s = 0; s < NA; s++) best[s] = -INFINITY, bidx[s] = INT_MAX;
        float saa = 0.f, sab = 0.f, sbb = 0.f;

        // U vectors of every operand are requested before the first is used
        auto step = [&](int64_t j0, auto masked_tag) {
            constexpr bool MASKED = decltype(masked_tag)::value;
            float xv[U][4], fv[U][4], gv[U][4], bv[U][4];
            int64_t jj[U];
            bool ok[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                jj[u] = j0 + (int64_t)(u * kGroup + sub) * VEC;
                ok[u] = !MASKED || jj[u] < D;  // D is a multiple of VEC: a vector is inside the row or wholly outside
            }
#pragma unroll
            for (int u = 0; u < U; u++) ld_vec<VEC>(xr + (ok[u] ? jj[u] : jlast), xv[u]);
            if (ERR) {
#pragma unroll
                for (int u = 0; u < U; u++) ld_vec<VEC>(fr + (ok[u] ? jj[u] : jlast), fv[u]);
            }
#pragma unroll
            for (int u = 0; u < U; u++) ld_vec<VEC>(gr + (ok[u] ? jj[u] : jlast), gv[u]);
#pragma unroll
            for (int u = 0; u < U; u++) ld_vec<VEC>(br + (ok[u] ? jj[u] : jlast), bv[u]);
#pragma unroll
            for (int u = 0; u < U; u++)
                sweep_entries<NA, VEC, ARG, ERR, MASKED>(xv[u], fv[u], gv[u], bv[u], inside, ok[u], (int)jj[u], al, best, bidx,
                                                         saa, sab, sbb);
        };
        for (int64_t j0 = 0; j0 < Dfull; j0 += U * STEP) step(j0, std::false_type{});
        if (Dfull < D) step(Dfull, std::true_type{});  // the rest of the row is less than one such step

        if (ARG) {
            const int lab = labels ? labels[row] : -1;
            int mine = 0;
#pragma unroll
            for (int s = 0; s < NA; s++) {
                // largest entry of the row, then the lowest position among the lanes that hold it
                const float m = row16_max(best[s]);
                int arg = row16_min(best[s] == m ? bidx[s] : INT_MAX);
                if (arg == INT_MAX) arg = 0;  // nothing above -inf in the row: the first entry
                hit[s] += (labels && row_ok && arg == lab) ? 1u : 0u;
                if (sub == s) mine = arg;
            }
            if (top1 && row_ok && sub < n_alpha) top1[row * n_alpha + sub] = mine;
        }
        if (ERR && row_ok) {  // a clamped row repeats the last one: its sums are dropped
            maa += (double)saa;
            mab += (double)sab;
            mbb += (double)sbb;
        }
    }

    // The workgroup's sums go to its own record; a second launch adds the records in a fixed order
    // (thousands of atomic additions to the same few addresses would take longer than the pass itself).
#pragma unroll
    for (int s = 0; s < NA; s++) {
        unsigned h = hit[s];  // equal on the 16 lanes of a group: add the four groups
        h += __shfl_xor(h, 16, kWave);
        h += __shfl_xor(h, 32, kWave);
        if (lane == 0) s_hit[wave][s] = h;
    }
    maa = wave_sum(maa);
    mab = wave_sum(mab);
    mbb = wave_sum(mbb);
    if (lane == 0) s_mom[wave][0] = maa, s_mom[wave][1] = mab, s_mom[wave][2] = mbb;
    __syncthreads();
    if (threadIdx.x < 3) {
        double v = 0.0;
        for (int w = 0; w < kSweepWaves; w++) v += s_mom[w][threadIdx.x];
        part->slot[threadIdx.x][blockIdx.x] = (unsigned long long)__double_as_longlong(v);
    }
    if (threadIdx.x < CAT_MAX_ALPHAS) {
        unsigned long long v = 0ull;
        if ((int)threadIdx.x < NA)
            for (int w = 0; w < kSweepWaves; w++) v += s_hit[w][threadIdx.x];
        part->slot[3 + threadIdx.x][blockIdx.x] = v;
    }
}

__device__ __forceinline__ float wave_max(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = fmaxf(v, __shfl_xor(v, o, kWave));
    return v;
}
__device__ __forceinline__ int wave_min(int v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v = min(v, __shfl_xor(v, o, kWave));
    return v;
}

// position of the largest entry of each row (the first one on ties): one wave per row at a time
template <typename T, int VEC>
__global__ __launch_bounds__(kSweepWaves* kWave) void k_row_top1(const T* __restrict__ x, int64_t N, int64_t D,
                                                                 int32_t* __restrict__ top1) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t gw = (int64_t)blockIdx.x * kSweepWaves + threadIdx.x / kWave;
    const int64_t nw = (int64_t)gridDim.x * kSweepWaves;
    for (int64_t row = gw; row < N; row += nw) {
        const T* xr = x + row * D;
        float best = -INFINITY;
        int bidx = INT_MAX;
        for (int64_t j = (int64_t)lane * VEC; j < D; j += kWave * VEC) {
            float v[4];
            ld_vec<VEC>(xr + j, v);
#pragma unroll
            for (int e = 0; e < VEC; e++)
                if (v[e] > best) best = v[e], bidx = (int)j + e;
        }
        const float m = wave_max(best);
        int arg = wave_min(best == m ? bidx : INT_MAX);
        if (arg == INT_MAX) arg = 0;
        if (lane == 0) top1[row] = arg;
    }
}

// Adds what the workgroups left, in a fixed order (lane-strided, then a butterfly over the wave).  Workgroup 0
// (one wave): the three sums and the squared error per alpha from them; workgroup 1 + s: the hits of alpha s.
// a lane's share of one quantity: every slot is requested before the first is used (a slot past the
// last record is read from slot 0 and not counted)
__device__ __forceinline__ void sweep_slots(const unsigned long long* q, int nrec, int lane,
                                            unsigned long long (&v)[kSweepMaxGrid / kWave]) {
#pragma unroll
    for (int i = 0; i < kSweepMaxGrid / kWave; i++) {
        const int r = i * kWave + lane;
        v[i] = q[r < nrec ? r : 0];
    }
}
__global__ __launch_bounds__(kWave) void k_sweep_finish(const SweepPartial* part, int nrec, const SweepAlphas al, int n_alpha,
                                                         unsigned long long* hits, double* sq_err, double* moments) {
    const int lane = threadIdx.x;
    unsigned long long v[kSweepMaxGrid / kWave];
    if (blockIdx.x == 0) {
        if (!sq_err && !moments) return;
        double m[3];
#pragma unroll
        for (int q = 0; q < 3; q++) {
            sweep_slots(part->slot[q], nrec, lane, v);
            double t = 0.0;
#pragma unroll
            for (int i = 0; i < kSweepMaxGrid / kWave; i++)
                t += i * kWave + lane < nrec ? __longlong_as_double((long long)v[i]) : 0.0;
            m[q] = wave_sum(t);
        }
        if (moments && lane < 3) moments[lane] = lane == 0 ? m[0] : (lane == 1 ? m[1] : m[2]);
        if (sq_err && lane < n_alpha) {
            const double a = (double)al.v[lane];
            sq_err[lane] = m[0] + 2.0 * a * m[1] + a * a * m[2];
        }
        return;
    }
    if (!hits) return;
    const int s = (int)blockIdx.x - 1;
    sweep_slots(part->slot[3 + s], nrec, lane, v);
    unsigned long long t = 0ull;
#pragma unroll
    for (int i = 0; i < kSweepMaxGrid / kWave; i++) t += i * kWave + lane < nrec ? v[i] : 0ull;
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) t += __shfl_xor(t, o, kWave);
    if (lane == 0) hits[s] = t;
}

template <typename T, int VEC, bool ERR>
static void launch_sweep_arg(int na_inst, dim3 g, hipStream_t st, const T* x, const T* fp, const int32_t* labels,
                             const int32_t* assign, int64_t N, int64_t D, int32_t K, const float* gamma,
                             const float* beta, const SweepAlphas& al, int n_alpha, SweepPartial* part,
                             int32_t* top1) {
    dim3 b(kSweepWaves * kWave);
#define CAT_SWEEP(NA)                                                                                              \
    hipLaunchKernelGGL((k_alpha_sweep<T, NA, VEC, true, ERR>), g, b, 0, st, x, fp, labels, assign, N, D, K, gamma, \
                       beta, al, n_alpha, part, top1)
    switch (na_inst) {
        case 1: CAT_SWEEP(1); break;
        case 2: CAT_SWEEP(2); break;
        case 4: CAT_SWEEP(4); break;
        case 8: CAT_SWEEP(8); break;
        case 10: CAT_SWEEP(10); break;
        case 12: CAT_SWEEP(12); break;
        default: CAT_SWEEP(16); break;
    }
#undef CAT_SWEEP
}

template <typename T>
static cat_status launch_sweep(const void* lq, const void* fp, const int32_t* labels, const int32_t* assign, int64_t N,
                               int64_t D, int32_t K, const float* gamma, const float* beta, const SweepAlphas& al,
                               int n_alpha, SweepPartial* part, int* nrec, int32_t* top1, bool vec4, hipStream_t st) {
    const T* x = (const T*)lq;
    const T* f = (const T*)fp;
    const bool arg = labels || top1;
    int na_inst = 16;
    for (int c : {12, 10, 8, 4, 2, 1})
        if (n_alpha <= c) na_inst = c;
    const int64_t rows_per_wg = (int64_t)kSweepWaves * kRowsPerWave;
    const int64_t want = (N + rows_per_wg - 1) / rows_per_wg;
    dim3 g((unsigned)(want < kSweepMaxGrid ? want : kSweepMaxGrid));
    *nrec = (int)g.x;
    dim3 b(kSweepWaves * kWave);
    if (arg) {
        if (vec4) {
            if (f)
                launch_sweep_arg<T, 4, true>(na_inst, g, st, x, f, labels, assign, N, D, K, gamma, beta, al, n_alpha, part, top1);
            else
                launch_sweep_arg<T, 4, false>(na_inst, g, st, x, f, labels, assign, N, D, K, gamma, beta, al, n_alpha, part, top1);
        } else {
            if (f)
                launch_sweep_arg<T, 1, true>(na_inst, g, st, x, f, labels, assign, N, D, K, gamma, beta, al, n_alpha, part, top1);
            else
                launch_sweep_arg<T, 1, false>(na_inst, g, st, x, f, labels, assign, N, D, K, gamma, beta, al, n_alpha, part, top1);
        }
    } else {  // the three sums only
        if (vec4)
            hipLaunchKernelGGL((k_alpha_sweep<T, 1, 4, false, true>), g, b, 0, st, x, f, labels, assign, N, D, K, gamma, beta, al,
                               n_alpha, part, top1);
        else
            hipLaunchKernelGGL((k_alpha_sweep<T, 1, 1, false, true>), g, b, 0, st, x, f, labels, assign, N, D, K, gamma, beta, al,
                               n_alpha, part, top1);
    }
    CAT_LAUNCH_CHECK("k_alpha_sweep");
    return CAT_OK;
}

static inline bool aligned16(const void* p) { return ((uintptr_t)p & 15u) == 0; }

}  // namespace cat

using namespace cat;

extern "C" {

size_t cat_alpha_sweep_workspace_bytes(void) { return sizeof(SweepPartial); }

cat_status cat_alpha_sweep(const void* lq, const void* fp, const int32_t* labels, const int32_t* assignments, int64_t N,
                           int64_t D, int32_t K, cat_dtype dt, const float* gamma, const float* beta,
                           const float* alphas_host, int32_t n_alpha, int64_t* hits, double* sq_err, double* moments,
                           int32_t* top1, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if ((dt != CAT_F32 && dt != CAT_BF16) || N < 1 || D < 1 || D > INT_MAX - 8 || K < 1 || K > CAT_MAX_K)
        return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: bad shape (N=%lld D=%lld K=%d dt=%d)", (long long)N,
                         (long long)D, (int)K, (int)dt);
    if (n_alpha < 1 || n_alpha > CAT_MAX_ALPHAS || !alphas_host)
        return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: need 1 <= n_alpha <= %d and the list (got %d)",
                         CAT_MAX_ALPHAS, (int)n_alpha);
    if (!lq || !assignments || !gamma || !beta) return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: null argument");
    if ((labels != nullptr) != (hits != nullptr))
        return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: labels and hits go together");
    if (!fp && (sq_err || moments))
        return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: sq_err and moments need fp");
    if (fp && !sq_err && !moments)
        return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: fp given but neither sq_err nor moments asked for");
    if (!labels && !top1 && !fp) return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: nothing to compute");
    if (!workspace || workspace_bytes < cat_alpha_sweep_workspace_bytes() || ((uintptr_t)workspace & 255u))
        return set_error(CAT_ERR_WORKSPACE, "cat_alpha_sweep: workspace of %zu bytes, 256-byte aligned, needed",
                         cat_alpha_sweep_workspace_bytes());
    SweepAlphas al;
    for (int s = 0; s < CAT_MAX_ALPHAS; s++) {
        const float a = alphas_host[s < n_alpha ? s : n_alpha - 1];  // unused slots repeat the last value
        if (!(a == a) || a - a != 0.f) return set_error(CAT_ERR_INVALID_ARG, "cat_alpha_sweep: alpha %d is not finite", s);
        al.v[s] = a;
    }
    hipStream_t st = (hipStream_t)hip_stream;
    SweepPartial* part = (SweepPartial*)workspace;
    int nrec = 0;
    // whole 16-byte (fp32) or 8-byte (bf16) vectors need D % 4 == 0 and aligned bases
    const bool vec4 = D % 4 == 0 && aligned16(lq) && aligned16(gamma) && aligned16(beta) && (!fp || aligned16(fp));
    cat_status s = dt == CAT_F32 ? launch_sweep<float>(lq, fp, labels, assignments, N, D, K, gamma, beta, al, n_alpha, part,
                                                       &nrec, top1, vec4, st)
                                 : launch_sweep<bf16_t>(lq, fp, labels, assignments, N, D, K, gamma, beta, al, n_alpha, part,
                                                        &nrec, top1, vec4, st);
    if (s != CAT_OK) return s;
    if (fp || hits) {
        hipLaunchKernelGGL(k_sweep_finish, dim3(1 + (hits ? n_alpha : 0)), dim3(kWave), 0, st, part, nrec, al, (int)n_alpha, (unsigned long long*)hits,
                           sq_err, moments);
        CAT_LAUNCH_CHECK("k_sweep_finish");
    }
    return CAT_OK;
}

cat_status cat_top1(const void* x, int64_t N, int64_t D, cat_dtype dt, int32_t* top1, void* hip_stream) {
    if ((dt != CAT_F32 && dt != CAT_BF16) || N < 1 || D < 1 || D > INT_MAX - 8)
        return set_error(CAT_ERR_INVALID_ARG, "cat_top1: bad shape (N=%lld D=%lld dt=%d)", (long long)N, (long long)D, (int)dt);
    if (!x || !top1) return set_error(CAT_ERR_INVALID_ARG, "cat_top1: null argument");
    hipStream_t st = (hipStream_t)hip_stream;
    const bool vec4 = D % 4 == 0 && aligned16(x);
    const int64_t want = (N + kSweepWaves - 1) / kSweepWaves;
    dim3 g((unsigned)(want < 4096 ? want : 4096)), b(kSweepWaves * kWave);
    if (dt == CAT_F32) {
        if (vec4)
            hipLaunchKernelGGL((k_row_top1<float, 4>), g, b, 0, st, (const float*)x, N, D, top1);
        else
            hipLaunchKernelGGL((k_row_top1<float, 1>), g, b, 0, st, (const float*)x, N, D, top1);
    } else {
        if (vec4)
            hipLaunchKernelGGL((k_row_top1<bf16_t, 4>), g, b, 0, st, (const bf16_t*)x, N, D, top1);
        else
            hipLaunchKernelGGL((k_row_top1<bf16_t, 1>), g, b, 0, st, (const bf16_t*)x, N, D, top1);
    }
    CAT_LAUNCH_CHECK("k_row_top1");
    return CAT_OK;
}

}  // extern "C"
