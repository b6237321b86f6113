// PCA front-end of CAT (Sec. 3.1; first step of Algorithms 1 and 2): the LQ vectors are reduced to
// their p leading principal components before clustering, and the affine correction is then applied
// by the cluster found in that space.  Everything here runs on the device in double precision
// except the projection (fp32 accumulation) and the labelled affine map:
//
//   cat_pca_fit       column means -> population covariance (D x D) -> symmetric eigendecomposition
//                     (one-sided Jacobi on the rows) -> the p leading directions
//   cat_pca_project   z = (x - mean) W^T
//   cat_apply_assigned   corrected = x + alpha ((gamma_a x + beta_a) - x) for given labels a
#include "cat_common.h"

namespace cat {

typedef __attribute__((ext_vector_type(4))) float f32x4_t;

constexpr int kPcaMaxD = 2048;  // eigen workspace is 2 (D+1)^2 doubles; the selection kernel keeps D values in LDS
static_assert(kPcaMaxD % 2 == 0 && kPcaMaxD <= 8 * 256, "a Jacobi step keeps a row in 8 x 256 registers at most");

// ---- column sums ---------------------------------------------------------------------------------
template <typename T>
__global__ __launch_bounds__(256) void k_pca_colsum(const T* __restrict__ x, int64_t N, int64_t D, int64_t rows_per_block,
                                                    double* __restrict__ sum) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < N ? r0 + rows_per_block : N;
    if (j >= D) return;
    double s = 0.0;
    constexpr int U = 8;  // loads in flight per thread; the adds stay in row order
    int64_t i = r0;
    for (; i + U <= r1; i += U) {
        float v[U];
#pragma unroll
        for (int u = 0; u < U; u++) v[u] = ld_elem(x + (i + u) * D + j);
#pragma unroll
        for (int u = 0; u < U; u++) s += (double)v[u];
    }
    for (; i < r1; i++) s += (double)ld_elem(x + i * D + j);
    atomicAdd(sum + j, s);
}

__global__ void k_pca_mean(const double* __restrict__ sum, int64_t N, int64_t D, double* __restrict__ mean_d,
                           float* __restrict__ mean_f) {
    const int64_t j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= D) return;
    const double m = sum[j] / (double)N;
    mean_d[j] = m;
    mean_f[j] = (float)m;
}

// ---- covariance: one workgroup per (32 x 32 tile of the upper triangle, row range) ----------------
// 256 threads, each owns a 2 x 2 block of the tile; 64 centred rows of both column blocks are staged
// in LDS as doubles per round.  W (ld = ldw) receives sum (x_a - m_a)(x_b - m_b); scaled and mirrored
// afterwards.
constexpr int kCovTile = 32, kCovRows = 64;
template <typename T>
__global__ __launch_bounds__(256) void k_pca_cov(const T* __restrict__ x, int64_t N, int64_t D, const double* __restrict__ mean,
                                                 int64_t rows_per_block, int32_t ntile, double* __restrict__ W, int64_t ldw) {
    __shared__ double sa[kCovRows][kCovTile + 1], sb[kCovRows][kCovTile + 1];
    // tile index -> (ta <= tb)
    int t = blockIdx.x, ta = 0;
    while (t >= ntile - ta) {
        t -= ntile - ta;
        ta++;
    }
    const int tb = ta + t;
    const int64_t a0 = (int64_t)ta * kCovTile, b0 = (int64_t)tb * kCovTile;
    const int64_t r0 = (int64_t)blockIdx.y * rows_per_block;
    const int64_t r1 = r0 + rows_per_block < N ? r0 + rows_per_block : N;
    const int ty = threadIdx.x >> 4, tx = threadIdx.x & 15;  // 16 x 16 threads, 2 x 2 outputs each
    double c00 = 0.0, c01 = 0.0, c10 = 0.0, c11 = 0.0;
    for (int64_t rb = r0; rb < r1; rb += kCovRows) {
        __syncthreads();
        for (int i = threadIdx.x; i < kCovRows * kCovTile; i += blockDim.x) {
            const int r = i / kCovTile, c = i - r * kCovTile;
            const int64_t row = rb + r;
            double va = 0.0, vb = 0.0;
            if (row < r1) {
                if (a0 + c < D) va = (double)ld_elem(x + row * D + a0 + c) - mean[a0 + c];
                if (b0 + c < D) vb = (double)ld_elem(x + row * D + b0 + c) - mean[b0 + c];
            }
            sa[r][c] = va;
            sb[r][c] = vb;
        }
        __syncthreads();
#pragma unroll 8
        for (int r = 0; r < kCovRows; r++) {
            const double a_0 = sa[r][2 * ty], a_1 = sa[r][2 * ty + 1];
            const double b_0 = sb[r][2 * tx], b_1 = sb[r][2 * tx + 1];
            c00 = fma(a_0, b_0, c00);
            c01 = fma(a_0, b_1, c01);
            c10 = fma(a_1, b_0, c10);
            c11 = fma(a_1, b_1, c11);
        }
    }
    const int64_t ia = a0 + 2 * ty, ib = b0 + 2 * tx;
    if (ia < D && ib < D) atomicAdd(W + ia * ldw + ib, c00);
    if (ia < D && ib + 1 < D) atomicAdd(W + ia * ldw + ib + 1, c01);
    if (ia + 1 < D && ib < D) atomicAdd(W + (ia + 1) * ldw + ib, c10);
    if (ia + 1 < D && ib + 1 < D) atomicAdd(W + (ia + 1) * ldw + ib + 1, c11);
}

// The same sums on the fp64 matrix cores (v_mfma_f64_16x16x4_f64), used from D = 64 on.  One wave per
// (64 x 64 tile of the upper triangle, row range): lane (m, k) = (lane & 15, lane >> 4) loads entry m of a
// 16-column piece of row i0 + k, centres and widens it, and that is at once the A operand (for the piece of the
// tile's rows) and the B operand (for the piece of its columns) of a 16 x 16 x 4 product; 4 + 4 pieces feed 16
// products per step of four rows, 16 rows are requested ahead of their use.  No LDS, no barriers; the 64 x 64
// doubles of a wave stay in registers until they are added to W with atomics.
typedef double f64x4_t __attribute__((ext_vector_type(4)));
constexpr int kCovM = 64;     // tile edge of a wave
constexpr int kCovAhead = 4;  // steps of four rows requested together
template <typename T>
__global__ __launch_bounds__(256) void k_pca_cov_mfma(const T* __restrict__ x, int64_t N, int64_t D, const double* __restrict__ mean,
                                                      int64_t rows_per_wave, int32_t ntile, double* __restrict__ W, int64_t ldw) {
    int t = blockIdx.x, ta = 0;  // tile index -> (ta <= tb)
    while (t >= ntile - ta) {
        t -= ntile - ta;
        ta++;
    }
    const int tb = ta + t;
    const int64_t a0 = (int64_t)ta * kCovM, b0 = (int64_t)tb * kCovM;
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    const int m = lane & 15, kk = lane >> 4;
    const int64_t range = (int64_t)blockIdx.y * (blockDim.x / kWave) + wave;
    const int64_t r0 = range * rows_per_wave;
    const int64_t r1 = r0 + rows_per_wave < N ? r0 + rows_per_wave : N;
    if (r0 >= N) return;  // wave-uniform
    // this lane's eight columns (four of the tile's rows, four of its columns), clamped to valid positions
    int64_t col[8];
    double mu[8];
    bool ok[8];
#pragma unroll
    for (int s = 0; s < 8; s++) {
        const int64_t c = (s < 4 ? a0 : b0) + 16 * (s & 3) + m;
        ok[s] = c < D;
        col[s] = ok[s] ? c : 0;
        mu[s] = mean[col[s]];
    }
    f64x4_t acc[4][4];
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++) acc[i][j] = (f64x4_t){0.0, 0.0, 0.0, 0.0};
    for (int64_t rb = r0; rb < r1; rb += 4 * kCovAhead) {
        float raw[kCovAhead][8];
#pragma unroll
        for (int u = 0; u < kCovAhead; u++) {
            const int64_t i = rb + 4 * u + kk;
            const T* xr = x + (i < r1 ? i : r0) * D;  // past the range: a valid row, its values dropped below
#pragma unroll
            for (int s = 0; s < 8; s++) raw[u][s] = ld_elem(xr + col[s]);
        }
#pragma unroll
        for (int u = 0; u < kCovAhead; u++) {
            const bool in = rb + 4 * u + kk < r1;
            double v[8];
#pragma unroll
            for (int s = 0; s < 8; s++) v[s] = (in && ok[s]) ? (double)raw[u][s] - mu[s] : 0.0;
#pragma unroll
            for (int i = 0; i < 4; i++)
#pragma unroll
                for (int j = 0; j < 4; j++) acc[i][j] = __builtin_amdgcn_mfma_f64_16x16x4f64(v[i], v[4 + j], acc[i][j], 0, 0, 0);
        }
    }
    // entry r of acc[i][j]: row a0 + 16 i + 4 r + (lane >> 4) of W, column b0 + 16 j + (lane & 15) (the fp64
    // product interleaves its result rows over the lane groups, unlike the fp32 one)
#pragma unroll
    for (int i = 0; i < 4; i++)
#pragma unroll
        for (int j = 0; j < 4; j++)
#pragma unroll
            for (int r = 0; r < 4; r++) {
                const int64_t ia = a0 + 16 * i + 4 * r + kk, ib = b0 + 16 * j + m;
                if (ia < D && ib < D && ia <= ib) atomicAdd(W + ia * ldw + ib, acc[i][j][r]);
            }
}

// scale the upper triangle by 1/N, set the padding row / column (an eigenvalue below every eigenvalue
// of a covariance, so it is never selected), start Vt as the identity; then mirror into the lower
// triangle (a second launch, so that it reads finished values)
__global__ void k_pca_cov_finish(double* __restrict__ W, double* __restrict__ Vt, int64_t D, int64_t Dp, int64_t N) {
    const int64_t i = (int64_t)blockIdx.y, j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (j >= Dp) return;
    Vt[i * Dp + j] = (i == j) ? 1.0 : 0.0;
    if (i >= D || j >= D)
        W[i * Dp + j] = (i == j) ? -1.0 : 0.0;
    else if (i <= j)
        W[i * Dp + j] = W[i * Dp + j] / (double)N;
}
__global__ void k_pca_mirror(double* __restrict__ W, int64_t D, int64_t Dp) {
    const int64_t i = (int64_t)blockIdx.y, j = (int64_t)blockIdx.x * blockDim.x + threadIdx.x;
    if (i < D && j < i) W[i * Dp + j] = W[j * Dp + i];
}

// ---- one-sided Jacobi on the rows of W (= the symmetric matrix at the start) ------------------------
// A rotation of rows p and q makes them orthogonal; the same rotation is applied to Vt.  When all rows
// are orthogonal, W = Lambda Q^T and Vt = Q^T for the eigendecomposition Q Lambda Q^T of the start
// matrix: row i of Vt is the eigenvector, w_i . vt_i its eigenvalue.  A sweep visits every pair of rows
// once; disjoint pairs are rotated side by side.  Rows are contiguous, so every access is coalesced.
//
// k_pca_jacobi_step: one workgroup per pair, Dp / 2 pairs per launch.  With step >= 0 the pairs are
// those of step `step` of the round-robin (tournament) schedule over the rows (Dp - 1 steps make a sweep);
// with step < 0 they are the neighbours (2k, 2k + 1), which is how the sweeps below use it (the pairs
// inside the blocks of k_pca_jacobi_block).
template <int NI>  // elements per thread and row: Dp <= 256 NI
__global__ __launch_bounds__(256) void k_pca_jacobi_step(double* __restrict__ W, double* __restrict__ Vt, int32_t Dp, int32_t step) {
    __shared__ double s_red[3][4];
    __shared__ double s_cs[2];
    const int k = blockIdx.x, m = Dp - 1;
    int p, q;
    if (step < 0) {  // the two rows of every block of two (see k_pca_jacobi_quad)
        p = 2 * k;
        q = 2 * k + 1;
    } else if (k == 0) {
        p = step;
        q = m;
    } else {
        p = (step + k) % m;
        q = (step - k + m) % m;
    }
    double* wp = W + (int64_t)p * Dp;
    double* wq = W + (int64_t)q * Dp;
    double* vp = Vt + (int64_t)p * Dp;
    double* vq = Vt + (int64_t)q * Dp;
    // The four rows are requested at once and stay in registers (NI elements per thread and row), so the step
    // has one memory latency in front of the reduction instead of one before and one after it.
    constexpr int MAXI = NI;
    double x[MAXI], y[MAXI], u[MAXI], v[MAXI];
#pragma unroll
    for (int i = 0; i < MAXI; i++) {
        const int j = threadIdx.x + i * 256;
        const int jc = j < Dp ? j : 0;  // past the end: element 0 again, dropped below
        x[i] = wp[jc];
        y[i] = wq[jc];
        u[i] = vp[jc];
        v[i] = vq[jc];
    }
    double a = 0.0, b = 0.0, g = 0.0;
#pragma unroll
    for (int i = 0; i < MAXI; i++) {
        if (threadIdx.x + i * 256 < Dp) {
            a = fma(x[i], x[i], a);
            b = fma(y[i], y[i], b);
            g = fma(x[i], y[i], g);
        }
    }
    a = wave_sum(a);
    b = wave_sum(b);
    g = wave_sum(g);
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    if (lane == 0) {
        s_red[0][wave] = a;
        s_red[1][wave] = b;
        s_red[2][wave] = g;
    }
    __syncthreads();
    if (threadIdx.x == 0) {
        a = s_red[0][0] + s_red[0][1] + s_red[0][2] + s_red[0][3];
        b = s_red[1][0] + s_red[1][1] + s_red[1][2] + s_red[1][3];
        g = s_red[2][0] + s_red[2][1] + s_red[2][2] + s_red[2][3];
        double c = 1.0, s = 0.0;
        if (fabs(g) > 1e-15 * sqrt(a * b) && g != 0.0) {
            const double zeta = (b - a) / (2.0 * g);
            const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
            c = 1.0 / sqrt(1.0 + t * t);
            s = c * t;
        }
        s_cs[0] = c;
        s_cs[1] = s;
    }
    __syncthreads();
    const double c = s_cs[0], s = s_cs[1];
    if (s == 0.0) return;  // uniform
#pragma unroll
    for (int i = 0; i < MAXI; i++) {
        const int j = threadIdx.x + i * 256;
        if (j < Dp) {
            wp[j] = c * x[i] - s * y[i];
            wq[j] = s * x[i] + c * y[i];
            vp[j] = c * u[i] - s * v[i];
            vq[j] = s * u[i] + c * v[i];
        }
    }
}

// Sum of a double over the wave, valid in lane 0: four steps inside each row of 16 lanes as lane permutations
// fused into the moves (no LDS round trip as with a butterfly of shuffles), then the four row sums from lanes
// 0, 16, 32 and 48.  All 64 lanes must be active.
template <int CTRL>
__device__ __forceinline__ double dpp_move(double v) {
    const long long b = __double_as_longlong(v);
    const int lo = __builtin_amdgcn_update_dpp(0, (int)(b & 0xFFFFFFFFll), CTRL, 0xF, 0xF, true);
    const int hi = __builtin_amdgcn_update_dpp(0, (int)(b >> 32), CTRL, 0xF, 0xF, true);
    return __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
}
__device__ __forceinline__ double wave_sum_lane0(double v) {
    v += dpp_move<0xB1>(v);   // quad_perm [1, 0, 3, 2]
    v += dpp_move<0x4E>(v);   // quad_perm [2, 3, 0, 1]
    v += dpp_move<0x141>(v);  // row_half_mirror
    v += dpp_move<0x140>(v);  // row_mirror
    const long long b = __double_as_longlong(v);
    double r[4];
#pragma unroll
    for (int q = 0; q < 4; q++) {
        const int lo = __builtin_amdgcn_readlane((int)(b & 0xFFFFFFFFll), 16 * q);
        const int hi = __builtin_amdgcn_readlane((int)(b >> 32), 16 * q);
        r[q] = __longlong_as_double(((long long)hi << 32) | (unsigned int)lo);
    }
    return (r[0] + r[1]) + (r[2] + r[3]);
}

// BR tournament steps per launch.  Rows are taken in blocks of BR (2 or 4); a round of the tournament over the
// Dp / BR blocks pairs block bp with block bq, and one workgroup holds the 2 BR rows of both matrices in
// registers and rotates, in BR steps of BR disjoint pairs, every row of bp against every row of bq: one load and
// one store of the rows for BR steps.  A launch is bound by its memory latencies (load, store and drain) and by
// the barriers and square roots of a step, not by bandwidth or arithmetic, so fewer, longer launches shorten a
// sweep.  A sweep: the pairs inside the blocks (k_pca_jacobi_step with step < 0 for the blocks of two, and for
// BR = 4 this kernel with BR = 2 and round < 0 for the two halves of every block), then Dp / BR - 1 rounds.
// Dp is a multiple of 2 BR.
template <int NI, int BR, int T>  // T threads, NI elements per thread and row: Dp <= T NI
__global__ __launch_bounds__(T) void k_pca_jacobi_block(double* __restrict__ W, double* __restrict__ Vt, int32_t Dp, int32_t round) {
    __shared__ double s_part[3 * BR][T];  // every thread's share of the three sums of each pair
    __shared__ double s_cs[2 * BR];
    const int k = blockIdx.x, m = Dp / BR - 1;  // tournament over Dp / BR blocks
    int bp, bq;
    if (round < 0) {  // neighbouring blocks: the two halves of a block of 2 BR rows
        bp = 2 * k;
        bq = 2 * k + 1;
    } else if (k == 0) {
        bp = round;
        bq = m;
    } else {
        bp = (round + k) % m;
        bq = (round - k + m) % m;
    }
    double w[2 * BR][NI], v[2 * BR][NI];
#pragma unroll
    for (int r = 0; r < 2 * BR; r++) {
        const int64_t row = (int64_t)(r < BR ? bp : bq) * BR + (r % BR);
#pragma unroll
        for (int i = 0; i < NI; i++) {
            const int j = threadIdx.x + i * T;
            const int jc = j < Dp ? j : 0;  // past the end: element 0 again, never used
            w[r][i] = W[row * Dp + jc];
            v[r][i] = Vt[row * Dp + jc];
        }
    }
    const int lane = threadIdx.x & (kWave - 1), wave = threadIdx.x / kWave;
    bool any = false;
#pragma unroll
    for (int st = 0; st < BR; st++) {
        // step st: row i of bp against row (i + st) mod BR of bq, i = 0 .. BR - 1.  Every thread leaves its
        // share of the sums in LDS; wave i adds the shares of pair i (T values per sum: T / 64 per lane, then one
        // butterfly), so a step costs three butterflies per wave instead of 3 BR, and two barriers.
#pragma unroll
        for (int i = 0; i < BR; i++) {
            const int q = BR + (i + st) % BR;
            double a = 0.0, b = 0.0, g = 0.0;
#pragma unroll
            for (int e = 0; e < NI; e++) {
                if ((int)threadIdx.x + e * T < Dp) {
                    a = fma(w[i][e], w[i][e], a);
                    b = fma(w[q][e], w[q][e], b);
                    g = fma(w[i][e], w[q][e], g);
                }
            }
            s_part[3 * i][threadIdx.x] = a;
            s_part[3 * i + 1][threadIdx.x] = b;
            s_part[3 * i + 2][threadIdx.x] = g;
        }
        __syncthreads();
        if (wave < BR) {  // BR <= 4 <= T / 64 waves
            const int i = wave;
            double a = 0.0, b = 0.0, g = 0.0;
#pragma unroll
            for (int h = 0; h < T / kWave; h++) {
                a += s_part[3 * i][lane + h * kWave];
                b += s_part[3 * i + 1][lane + h * kWave];
                g += s_part[3 * i + 2][lane + h * kWave];
            }
            a = wave_sum_lane0(a);
            b = wave_sum_lane0(b);
            g = wave_sum_lane0(g);
            if (lane == 0) {
                double c = 1.0, sn = 0.0;
                if (g * g > 1e-30 * (a * b) && g != 0.0) {  // |g| > 1e-15 sqrt(a b)
                    const double zeta = (b - a) / (2.0 * g);
                    const double t = (zeta >= 0.0 ? 1.0 : -1.0) / (fabs(zeta) + sqrt(1.0 + zeta * zeta));
                    c = 1.0 / sqrt(1.0 + t * t);
                    sn = c * t;
                }
                s_cs[2 * i] = c;
                s_cs[2 * i + 1] = sn;
            }
        }
        __syncthreads();
        // (the shares of the next step are written after this barrier and read before the next one; the
        // angles are read here, before the next step's first barrier, and written after it)
#pragma unroll
        for (int i = 0; i < BR; i++) {
            const int q = BR + (i + st) % BR;
            const double c = s_cs[2 * i], sn = s_cs[2 * i + 1];
            if (sn != 0.0) {  // uniform
                any = true;
#pragma unroll
                for (int e = 0; e < NI; e++) {
                    const double x = w[i][e], y = w[q][e], u = v[i][e], z = v[q][e];
                    w[i][e] = c * x - sn * y;
                    w[q][e] = sn * x + c * y;
                    v[i][e] = c * u - sn * z;
                    v[q][e] = sn * u + c * z;
                }
            }
        }
    }
    if (!any) return;  // uniform
#pragma unroll
    for (int r = 0; r < 2 * BR; r++) {
        const int64_t row = (int64_t)(r < BR ? bp : bq) * BR + (r % BR);
#pragma unroll
        for (int i = 0; i < NI; i++) {
            const int j = threadIdx.x + i * T;
            if (j < Dp) {
                W[row * Dp + j] = w[r][i];
                Vt[row * Dp + j] = v[r][i];
            }
        }
    }
}

// eigenvalue of row i: w_i . vt_i
__global__ __launch_bounds__(256) void k_pca_rayleigh(const double* __restrict__ W, const double* __restrict__ Vt, int32_t Dp,
                                                      double* __restrict__ lambda) {
    __shared__ double s_red[4];
    const int i = blockIdx.x;
    double a = 0.0;
    for (int j = threadIdx.x; j < Dp; j += blockDim.x) a = fma(W[(int64_t)i * Dp + j], Vt[(int64_t)i * Dp + j], a);
    a = wave_sum(a);
    if ((threadIdx.x & (kWave - 1)) == 0) s_red[threadIdx.x / kWave] = a;
    __syncthreads();
    if (threadIdx.x == 0) lambda[i] = s_red[0] + s_red[1] + s_red[2] + s_red[3];
}

// the p largest eigenvalues in descending order (lowest row index first among equals), their rows of Vt
// as unit directions whose entry of largest magnitude (the first such) is positive.  Workgroup c finds the
// entry with exactly c entries ahead of it in that order (a count per entry against all others, the values
// in LDS) and writes direction c.
__global__ __launch_bounds__(256) void k_pca_select(const double* __restrict__ lambda, const double* __restrict__ Vt, int32_t D,
                                                    int32_t Dp, float* __restrict__ comps, double* __restrict__ evals) {
    __shared__ double s_lam[kPcaMaxD + 16];
    __shared__ double s_val[256];
    __shared__ int s_idx[256];
    __shared__ int s_row;
    const int c = blockIdx.x;
    for (int i = threadIdx.x; i < Dp; i += blockDim.x) s_lam[i] = lambda[i];
    if (threadIdx.x == 0) s_row = 0;  // stays in range even if no entry qualifies (NaN input)
    __syncthreads();
    for (int i = threadIdx.x; i < Dp; i += blockDim.x) {
        const double v = s_lam[i];
        int ahead = 0;
        for (int j = 0; j < Dp; j++) {
            const double u = s_lam[j];
            ahead += (u > v || (u == v && j < i)) ? 1 : 0;
        }
        if (ahead == c) s_row = i;  // the order is total: exactly one entry
    }
    __syncthreads();
    const int row = s_row;
    // sign: first entry of largest magnitude among the D real coordinates
    double am = -1.0;
    int aj = 0x7fffffff;
    for (int j = threadIdx.x; j < D; j += blockDim.x) {
        const double v = fabs(Vt[(int64_t)row * Dp + j]);
        if (v > am || (v == am && j < aj)) {
            am = v;
            aj = j;
        }
    }
    s_val[threadIdx.x] = am;
    s_idx[threadIdx.x] = aj;
    __syncthreads();
    for (int o = 128; o > 0; o >>= 1) {
        if ((int)threadIdx.x < o) {
            const double v = s_val[threadIdx.x + o];
            const int j = s_idx[threadIdx.x + o];
            if (v > s_val[threadIdx.x] || (v == s_val[threadIdx.x] && j < s_idx[threadIdx.x])) {
                s_val[threadIdx.x] = v;
                s_idx[threadIdx.x] = j;
            }
        }
        __syncthreads();
    }
    const int jmax = s_idx[0] < D ? s_idx[0] : 0;
    const double sgn = Vt[(int64_t)row * Dp + jmax] < 0.0 ? -1.0 : 1.0;
    for (int j = threadIdx.x; j < D; j += blockDim.x) comps[(int64_t)c * D + j] = (float)(sgn * Vt[(int64_t)row * Dp + j]);
    if (threadIdx.x == 0 && evals) evals[c] = s_lam[row];
}

// ---- projection: z[i][c] = sum_j (x[i][j] - mean[j]) comps[c][j] -----------------------------------
// A skinny GEMM in fp32 on the fp32 matrix cores (v_mfma_f32_16x16x4_f32: exact products, fp32
// accumulation), one wave per tile of 16 rows, 8 waves per workgroup.  Directions are the M dimension
// and rows the N dimension, so a lane ends up with 4 consecutive scores of one row (one 16-byte store).
// The k index of the MFMA is free to be any channel as long as both operands agree: lane (n, g) loads
// the four channels 16 s + 4 g .. + 3 of row n in one 16-byte load (64 contiguous bytes per row and
// instruction) and feeds them to four MFMAs; the directions are staged per 128-channel chunk in LDS
// in exactly that order ([step][tile][lane][4]), so their reads are 16 bytes per lane, conflict-free.
// NT = 16-direction tiles per pass (p <= 16 NT per pass; more directions take more passes over the rows).
constexpr int kProjWaves = 8, kProjChunk = 128;
template <typename T, int NT>
__global__ __launch_bounds__(kProjWaves * kWave) void k_pca_project(const T* __restrict__ x, int64_t N, int64_t D, int32_t p,
                                                                    const float* __restrict__ mean, const float* __restrict__ comps,
                                                                    float* __restrict__ z, int32_t ldz) {
    __shared__ __align__(16) float s_w[(kProjChunk / 16) * NT * kWave * 4];  // 8 steps x NT tiles x 64 lanes x 4
    __shared__ __align__(16) float s_m[kProjChunk];
    const int lane = threadIdx.x & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(threadIdx.x / kWave);
    const int n = lane & 15, g = lane >> 4;
    const int64_t ntiles = (N + 15) / 16;
    const int64_t tile = (int64_t)blockIdx.x * kProjWaves + wave;
    const int64_t row = tile * 16 + n;
    const int64_t rowc = row < N ? row : N - 1;  // rows past the end repeat the last row; never stored
    const T* xr = x + rowc * D;
    for (int c0 = 0; c0 < p; c0 += 16 * NT) {
        f32x4_t acc[NT];
#pragma unroll
        for (int t = 0; t < NT; t++) acc[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        for (int64_t j0 = 0; j0 < D; j0 += kProjChunk) {
            __syncthreads();
            // directions of this chunk into operand order; zero outside p x D
            for (int i = threadIdx.x; i < 16 * NT * (kProjChunk / 4); i += blockDim.x) {
                const int r = i / (kProjChunk / 4), q = i - r * (kProjChunk / 4);  // direction in pass, 4-channel group
                const int64_t ch = j0 + 4 * q;
                f32x4_t v = (f32x4_t){0.f, 0.f, 0.f, 0.f};
                if (c0 + r < p) {
                    const float* src = comps + (int64_t)(c0 + r) * D + ch;
                    if (ch + 3 < D && ((D & 3) == 0)) {
                        v = *(const f32x4_t*)src;
                    } else {
                        if (ch < D) v.x = src[0];
                        if (ch + 1 < D) v.y = src[1];
                        if (ch + 2 < D) v.z = src[2];
                        if (ch + 3 < D) v.w = src[3];
                    }
                }
                const int s_ = q >> 2, gg = q & 3, t = r >> 4, m = r & 15;
                *(f32x4_t*)&s_w[(((s_ * NT + t) * kWave) + gg * 16 + m) * 4] = v;
            }
            for (int i = threadIdx.x; i < kProjChunk; i += blockDim.x) s_m[i] = j0 + i < D ? mean[j0 + i] : 0.f;
            __syncthreads();
            if (tile < ntiles) {
                f32x4_t xv[kProjChunk / 16];
#pragma unroll
                for (int s_ = 0; s_ < kProjChunk / 16; s_++) {
                    const int64_t ch = j0 + 16 * s_ + 4 * g;
                    float e[4];
                    if ((D & 3) == 0) {  // rows keep 16-byte (bf16: 8-byte) alignment: one load per group
                        if (ch < D) {
                            if (sizeof(T) == 4) {
                                const f32x4_t v4 = *(const f32x4_t*)(xr + ch);
                                e[0] = v4.x; e[1] = v4.y; e[2] = v4.z; e[3] = v4.w;
                            } else {
                                const uint2 w2 = *(const uint2*)(xr + ch);
                                e[0] = __uint_as_float(w2.x << 16); e[1] = __uint_as_float(w2.x & 0xFFFF0000u);
                                e[2] = __uint_as_float(w2.y << 16); e[3] = __uint_as_float(w2.y & 0xFFFF0000u);
                            }
                        } else {
                            e[0] = e[1] = e[2] = e[3] = 0.f;
                        }
                    } else {
#pragma unroll
                        for (int u = 0; u < 4; u++) e[u] = ch + u < D ? ld_elem(xr + ch + u) : 0.f;
                    }
                    const f32x4_t mv = *(const f32x4_t*)&s_m[16 * s_ + 4 * g];
                    xv[s_] = (f32x4_t){ch < D ? e[0] - mv.x : 0.f, ch + 1 < D ? e[1] - mv.y : 0.f, ch + 2 < D ? e[2] - mv.z : 0.f,
                                       ch + 3 < D ? e[3] - mv.w : 0.f};
                }
#pragma unroll
                for (int s_ = 0; s_ < kProjChunk / 16; s_++) {
#pragma unroll
                    for (int t = 0; t < NT; t++) {
                        const f32x4_t wv = *(const f32x4_t*)&s_w[(((s_ * NT + t) * kWave) + lane) * 4];
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.x, xv[s_].x, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.y, xv[s_].y, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.z, xv[s_].z, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.w, xv[s_].w, acc[t], 0, 0, 0);
                    }
                }
            }
        }
        if (row < N) {
#pragma unroll
            for (int t = 0; t < NT; t++) {
                const int c = c0 + 16 * t + 4 * g;
                // rows of z are ldz >= p floats apart; columns p .. ldz - 1 receive the zeros the padded directions give
                float* o = z + row * ldz + c;
                if (c + 3 < ldz && ((ldz & 3) == 0)) {
                    *(f32x4_t*)o = acc[t];
                } else {
                    if (c < ldz) o[0] = acc[t].x;
                    if (c + 1 < ldz) o[1] = acc[t].y;
                    if (c + 2 < ldz) o[2] = acc[t].z;
                    if (c + 3 < ldz) o[3] = acc[t].w;
                }
            }
        }
    }
}

// The same projection with the staging of the directions software-pipelined, for rows of whole 16-byte groups (D a
// multiple of 4, aligned bases): while chunk j is contracted, the directions and the means of chunk j + 1 are
// already on their way into registers; they then go into the LDS buffer chunk j does not use, and one barrier per
// chunk separates the two.  Registers are capped at 128 so that two workgroups share a CU (four waves per SIMD).  Every load is unconditional (a position past the end is
// clamped to a valid one and its value dropped), so none is waited for where it is issued.
//
// FUSED: Algorithm 2 with the PCA front-end in one kernel (p <= 16 NT, K <= 256).  The scores of a tile stay
// in registers; the centroids of score space go into the LDS the directions no longer need; every row takes the
// centroid of smallest squared distance (direct form, doubles, lowest index on ties), and the wave then reads its
// 16 rows once more, four at a time with 16-byte (bf16: 8-byte) loads, and writes the blended affine map.
struct ProjFuse {
    const float* cz;     // K x p centroids in score space
    const float* gamma;  // K x D
    const float* beta;
    void* out;           // N x D of the row type
    int32_t* assign;     // nullable
    int32_t K;
    float alpha;
};
template <typename T, int NT, bool FUSED>
__global__ __launch_bounds__(kProjWaves * kWave, 4) void k_pca_project_pipe(const T* __restrict__ x, int64_t N, int64_t D, int32_t p,
                                                                         const float* __restrict__ mean,
                                                                         const float* __restrict__ comps, float* __restrict__ z,
                                                                         int32_t ldz, const ProjFuse f) {
    constexpr int SW = (kProjChunk / 16) * NT * kWave * 4;  // floats of directions per chunk
    constexpr int XS = kProjChunk / 16;                     // 16-channel steps per chunk
    __shared__ __align__(16) float s_w[2][SW];
    __shared__ __align__(16) float s_m[2][kProjChunk];
    const int tid = threadIdx.x, lane = tid & (kWave - 1);
    const int wave = __builtin_amdgcn_readfirstlane(tid / kWave);
    const int n = lane & 15, g = lane >> 4;
    const int64_t ntiles = (N + 15) / 16;
    const int64_t tile = (int64_t)blockIdx.x * kProjWaves + wave;
    const int64_t row = tile * 16 + n;
    const int64_t rowc = row < N ? row : N - 1;  // rows past the end repeat the last row; never stored
    const T* xr = x + rowc * D;
    const int nch = (int)((D + kProjChunk - 1) / kProjChunk);
    // this thread's share of the staging: direction m of every tile, 4-channel group q of the chunk
    const int sm = tid >> 5, sq = tid & 31;
    const int s_slot = (((sq >> 2) * NT) * kWave + (sq & 3) * 16 + sm) * 4;  // + t * kWave * 4 for tile t

    typedef uint32_t __attribute__((ext_vector_type(sizeof(T) == 4 ? 4 : 2))) xraw_t;
    auto load_w = [&](int c0, int jc, f32x4_t (&w)[NT]) {
        const int64_t ch = (int64_t)jc * kProjChunk + 4 * sq;
        const int64_t chc = ch < D ? ch : 0;
#pragma unroll
        for (int t = 0; t < NT; t++) {
            const int r = c0 + 16 * t + sm;
            const f32x4_t v = *(const f32x4_t*)(comps + (int64_t)(r < p ? r : 0) * D + chc);
            const bool ok = r < p && ch < D;
            w[t] = (f32x4_t){ok ? v.x : 0.f, ok ? v.y : 0.f, ok ? v.z : 0.f, ok ? v.w : 0.f};
        }
    };
    auto load_m = [&](int jc) {
        const int64_t ch = (int64_t)jc * kProjChunk + (tid & (kProjChunk - 1));
        const float v = mean[ch < D ? ch : 0];
        return ch < D ? v : 0.f;
    };
    auto load_x = [&](int jc, xraw_t (&xv)[XS]) {
#pragma unroll
        for (int s_ = 0; s_ < XS; s_++) {
            const int64_t ch = (int64_t)jc * kProjChunk + 16 * s_ + 4 * g;
            xv[s_] = *(const xraw_t*)(xr + (ch < D ? ch : 0));
        }
    };

    for (int c0 = 0; c0 < p; c0 += 16 * NT) {
        f32x4_t acc[NT];
#pragma unroll
        for (int t = 0; t < NT; t++) acc[t] = (f32x4_t){0.f, 0.f, 0.f, 0.f};
        f32x4_t wreg[NT];
        xraw_t xcur[XS];
        __syncthreads();  // the buffers of the previous pass are no longer read
        load_w(c0, 0, wreg);
        float mreg = load_m(0);
#pragma unroll
        for (int t = 0; t < NT; t++) *(f32x4_t*)&s_w[0][s_slot + t * kWave * 4] = wreg[t];
        if (tid < kProjChunk) s_m[0][tid] = mreg;
        __syncthreads();
        for (int jc = 0; jc < nch; jc++) {
            const int cur = jc & 1;
            const int jn = jc + 1 < nch ? jc + 1 : jc;  // past the last chunk: loaded again, never used
            load_x(jc, xcur);  // this chunk's rows first (the other waves of the SIMD cover their latency), then the next chunk's directions
            load_w(c0, jn, wreg);
            mreg = load_m(jn);
            if (tile < ntiles) {
#pragma unroll
                for (int s_ = 0; s_ < XS; s_++) {
                    const int64_t ch = (int64_t)jc * kProjChunk + 16 * s_ + 4 * g;
                    float e[4];
                    if (sizeof(T) == 4) {
                        e[0] = __uint_as_float(xcur[s_][0]), e[1] = __uint_as_float(xcur[s_][1]);
                        e[2] = __uint_as_float(xcur[s_][sizeof(T) == 4 ? 2 : 0]), e[3] = __uint_as_float(xcur[s_][sizeof(T) == 4 ? 3 : 1]);
                    } else {
                        e[0] = __uint_as_float(xcur[s_][0] << 16), e[1] = __uint_as_float(xcur[s_][0] & 0xFFFF0000u);
                        e[2] = __uint_as_float(xcur[s_][1] << 16), e[3] = __uint_as_float(xcur[s_][1] & 0xFFFF0000u);
                    }
                    const f32x4_t mv = *(const f32x4_t*)&s_m[cur][16 * s_ + 4 * g];
                    const bool in = ch < D;  // D is a multiple of 4: a group is inside the row or wholly outside
                    const f32x4_t xv = (f32x4_t){in ? e[0] - mv.x : 0.f, in ? e[1] - mv.y : 0.f, in ? e[2] - mv.z : 0.f,
                                                 in ? e[3] - mv.w : 0.f};
#pragma unroll
                    for (int t = 0; t < NT; t++) {
                        const f32x4_t wv = *(const f32x4_t*)&s_w[cur][(((s_ * NT + t) * kWave) + lane) * 4];
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.x, xv.x, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.y, xv.y, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.z, xv.z, acc[t], 0, 0, 0);
                        acc[t] = __builtin_amdgcn_mfma_f32_16x16x4f32(wv.w, xv.w, acc[t], 0, 0, 0);
                    }
                }
            }
            // the other buffer was last read one chunk ago, before the barrier that ended that chunk
#pragma unroll
            for (int t = 0; t < NT; t++) *(f32x4_t*)&s_w[cur ^ 1][s_slot + t * kWave * 4] = wreg[t];
            if (tid < kProjChunk) s_m[cur ^ 1][tid] = mreg;
            __syncthreads();
        }
        if (!FUSED) {
            if (row < N) {
#pragma unroll
                for (int t = 0; t < NT; t++) {
                    const int c = c0 + 16 * t + 4 * g;
                    float* o = z + row * ldz + c;
                    if (c + 3 < ldz && ((ldz & 3) == 0)) {
                        *(f32x4_t*)o = acc[t];
                    } else {
                        if (c < ldz) o[0] = acc[t].x;
                        if (c + 1 < ldz) o[1] = acc[t].y;
                        if (c + 2 < ldz) o[2] = acc[t].z;
                        if (c + 3 < ldz) o[3] = acc[t].w;
                    }
                }
            }
            continue;
        }
        // ---- FUSED (one pass: c0 = 0).  Centroids of score space into LDS, padded to 16 NT columns of zeros.
        constexpr int CW = 16 * NT;
        float* s_cz = &s_w[0][0];  // 2 SW floats: room for 256 centroids; the last barrier of the loop has passed
        for (int i = tid; i < f.K * CW; i += kProjWaves * kWave) {
            const int k = i / CW, c = i - k * CW;
            s_cz[i] = c < p ? f.cz[(int64_t)k * p + c] : 0.f;
        }
        __syncthreads();
        if (tile >= ntiles) continue;
        double dbest = __builtin_inf();
        int kbest = 0;
        for (int k = 0; k < f.K; k++) {
            double d = 0.0;
#pragma unroll
            for (int t = 0; t < NT; t++) {
                const f32x4_t cv = *(const f32x4_t*)&s_cz[k * CW + 16 * t + 4 * g];
                const double d0 = (double)acc[t].x - (double)cv.x, d1 = (double)acc[t].y - (double)cv.y;
                const double d2 = (double)acc[t].z - (double)cv.z, d3 = (double)acc[t].w - (double)cv.w;
                d = fma(d0, d0, d);
                d = fma(d1, d1, d);
                d = fma(d2, d2, d);
                d = fma(d3, d3, d);
            }
            d += __shfl_xor(d, 16, kWave);  // the four lanes of a row end with the same bits (addition commutes)
            d += __shfl_xor(d, 32, kWave);
            if (d < dbest) {
                dbest = d;
                kbest = k;
            }
        }
        if (f.assign && g == 0 && row < N) f.assign[row] = kbest;
        // the affine map of the 16 rows, four rows at a time: the whole wave on each row
        T* outp = (T*)f.out;
        const int64_t tile_row0 = tile * 16;
        for (int r0 = 0; r0 < 16; r0 += 4) {
            if (tile_row0 + r0 >= N) break;  // wave-uniform
            int a[4];
            int64_t rr[4];
            bool ok[4];
#pragma unroll
            for (int u = 0; u < 4; u++) {
                a[u] = __builtin_amdgcn_readlane(kbest, r0 + u);
                ok[u] = tile_row0 + r0 + u < N;
                rr[u] = ok[u] ? tile_row0 + r0 + u : N - 1;  // past the end: the last row again, not stored
            }
            for (int64_t j = (int64_t)lane * 4; j < D; j += kWave * 4) {
                xraw_t xv[4];
                f32x4_t gv[4], bv[4];
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    xv[u] = *(const xraw_t*)(x + rr[u] * D + j);
                    gv[u] = *(const f32x4_t*)(f.gamma + (int64_t)a[u] * D + j);
                    bv[u] = *(const f32x4_t*)(f.beta + (int64_t)a[u] * D + j);
                }
#pragma unroll
                for (int u = 0; u < 4; u++) {
                    float e[4], r[4];
                    if (sizeof(T) == 4) {
                        e[0] = __uint_as_float(xv[u][0]), e[1] = __uint_as_float(xv[u][1]);
                        e[2] = __uint_as_float(xv[u][sizeof(T) == 4 ? 2 : 0]), e[3] = __uint_as_float(xv[u][sizeof(T) == 4 ? 3 : 1]);
                    } else {
                        e[0] = __uint_as_float(xv[u][0] << 16), e[1] = __uint_as_float(xv[u][0] & 0xFFFF0000u);
                        e[2] = __uint_as_float(xv[u][1] << 16), e[3] = __uint_as_float(xv[u][1] & 0xFFFF0000u);
                    }
#pragma unroll
                    for (int c = 0; c < 4; c++) {
                        const float gg = 1.f + f.alpha * (gv[u][c] - 1.f), bb = f.alpha * bv[u][c];
                        r[c] = fmaf(gg, e[c], bb);
                    }
                    if (ok[u]) {
                        xraw_t o;
                        if (sizeof(T) == 4) {
                            o[0] = __float_as_uint(r[0]), o[1] = __float_as_uint(r[1]);
                            o[sizeof(T) == 4 ? 2 : 0] = __float_as_uint(r[2]), o[sizeof(T) == 4 ? 3 : 1] = __float_as_uint(r[3]);
                        } else {
                            o[0] = (uint32_t)f32_to_bf16(r[0]) | ((uint32_t)f32_to_bf16(r[1]) << 16);
                            o[1] = (uint32_t)f32_to_bf16(r[2]) | ((uint32_t)f32_to_bf16(r[3]) << 16);
                        }
                        *(xraw_t*)(outp + rr[u] * D + j) = o;
                    }
                }
            }
        }
    }
}

// ---- affine map by given labels ------------------------------------------------------------------
// One wave per row.  WIDE: 16-byte loads and stores, all of a lane's requests for the row issued before the
// first is used (rows of whole 16-byte groups, aligned bases); else one channel per lane and step.
template <typename T, bool WIDE>
__global__ __launch_bounds__(256) void k_apply_assigned(const T* __restrict__ x, const int32_t* __restrict__ assign, int64_t N,
                                                        int64_t D, int32_t K, const float* __restrict__ gamma,
                                                        const float* __restrict__ beta, float alpha, T* __restrict__ out) {
    const int lane = threadIdx.x & (kWave - 1);
    const int64_t row = (int64_t)blockIdx.x * (blockDim.x / kWave) + threadIdx.x / kWave;
    if (row >= N) return;
    const int a = assign[row];
    const bool ok = a >= 0 && a < K;  // a label outside [0, K) leaves the row as it is
    const float* gr = gamma + (int64_t)(ok ? a : 0) * D;
    const float* br = beta + (int64_t)(ok ? a : 0) * D;
    const T* xr = x + row * D;
    T* orow = out + row * D;
    if (WIDE) {
        constexpr int EPL = (int)(16 / sizeof(T));  // channels per 16-byte group: 4 (fp32) or 8 (bf16)
        constexpr int U = 4;                        // groups per lane in flight
        for (int64_t j0 = (int64_t)lane * EPL; j0 < D; j0 += (int64_t)U * kWave * EPL) {
            uint4 xv[U];
            f32x4_t gv[U][EPL / 4], bv[U][EPL / 4];
            int64_t j[U];
#pragma unroll
            for (int u = 0; u < U; u++) {
                const int64_t jj = j0 + (int64_t)u * kWave * EPL;
                j[u] = jj < D ? jj : j0;  // past the end: the first group again, not stored
                xv[u] = *(const uint4*)(xr + j[u]);
#pragma unroll
                for (int h = 0; h < EPL / 4; h++) {
                    gv[u][h] = *(const f32x4_t*)(gr + j[u] + 4 * h);
                    bv[u][h] = *(const f32x4_t*)(br + j[u] + 4 * h);
                }
            }
#pragma unroll
            for (int u = 0; u < U; u++) {
                if (j0 + (int64_t)u * kWave * EPL >= D) break;
                float v[EPL];
                if (sizeof(T) == 4) {
                    v[0] = __uint_as_float(xv[u].x), v[1] = __uint_as_float(xv[u].y);
                    v[2] = __uint_as_float(xv[u].z), v[3] = __uint_as_float(xv[u].w);
                } else {
                    const uint32_t w[4] = {xv[u].x, xv[u].y, xv[u].z, xv[u].w};
#pragma unroll
                    for (int e = 0; e < 4; e++) {
                        v[2 * e] = __uint_as_float(w[e] << 16);
                        v[(2 * e + 1) % EPL] = __uint_as_float(w[e] & 0xFFFF0000u);
                    }
                }
                float r[EPL];
#pragma unroll
                for (int e = 0; e < EPL; e++) {
                    const float g = 1.f + alpha * (gv[u][e / 4][e % 4] - 1.f), b = alpha * bv[u][e / 4][e % 4];
                    r[e] = ok ? fmaf(g, v[e], b) : v[e];
                }
                uint4 o;
                if (sizeof(T) == 4) {
                    o = make_uint4(__float_as_uint(r[0]), __float_as_uint(r[1]), __float_as_uint(r[2]), __float_as_uint(r[3]));
                } else {
                    uint32_t w[4];
#pragma unroll
                    for (int e = 0; e < 4; e++)
                        w[e] = (uint32_t)f32_to_bf16(r[2 * e]) | ((uint32_t)f32_to_bf16(r[(2 * e + 1) % EPL]) << 16);
                    o = make_uint4(w[0], w[1], w[2], w[3]);
                }
                *(uint4*)(orow + j[u]) = o;
            }
        }
    } else {
        for (int64_t j = lane; j < D; j += kWave) {
            const float v = ld_elem(xr + j);
            float r = v;
            if (ok) {
                const float g = 1.f + alpha * (gr[j] - 1.f), b = alpha * br[j];
                r = fmaf(g, v, b);
            }
            st_elem(orow + j, r);
        }
    }
}

// ---- host side ---------------------------------------------------------------------------------
static inline size_t pad256(size_t x) { return (x + 255) & ~(size_t)255; }
static inline int64_t even_up(int64_t D) { return (D + 7) & ~(int64_t)7; }  // rows of the eigen workspace: a multiple of 8

struct PcaWs {
    double* sum;     // D
    double* mean;    // D
    double* lambda;  // Dp
    double* W;       // Dp x Dp
    double* Vt;      // Dp x Dp
    size_t bytes;
};
static PcaWs pca_carve(void* base, int64_t D) {
    const int64_t Dp = even_up(D);
    PcaWs w;
    char* b = (char*)base;
    size_t off = 0;
    w.sum = (double*)(b + off);
    off += pad256((size_t)D * 8);
    w.mean = (double*)(b + off);
    off += pad256((size_t)D * 8);
    w.lambda = (double*)(b + off);
    off += pad256((size_t)Dp * 8);
    w.W = (double*)(b + off);
    off += pad256((size_t)Dp * Dp * 8);
    w.Vt = (double*)(b + off);
    off += pad256((size_t)Dp * Dp * 8);
    w.bytes = off;
    return w;
}

static bool pca_shape_ok(int64_t N, int64_t D, int32_t p, cat_dtype dt) {
    return (dt == CAT_F32 || dt == CAT_BF16) && N >= 1 && D >= 1 && D <= kPcaMaxD && p >= 1 && (int64_t)p <= D &&
           N <= ((int64_t)1 << 40);
}

// scores with rows ldz >= p floats apart (the padding columns are written as zeros); ldz < p + 16
cat_status pca_project_ld(const void* lq, int64_t N, int64_t D, int32_t p, cat_dtype dt, const float* mean,
                          const float* components, float* z, int32_t ldz, hipStream_t st) {
    if ((dt != CAT_F32 && dt != CAT_BF16) || N < 1 || D < 1 || p < 1 || (int64_t)p > D || ldz < p || ldz > ((p + 15) & ~15))
        return set_error(CAT_ERR_INVALID_ARG, "cat_pca_project: need N >= 1, 1 <= p <= D (N=%lld D=%lld p=%d dt=%d ld=%d)", (long long)N,
                         (long long)D, (int)p, (int)dt, (int)ldz);
    if (!lq || !mean || !components || !z) return set_error(CAT_ERR_INVALID_ARG, "cat_pca_project: null argument");
    const int64_t rows_per_block = kProjWaves * 16;
    dim3 g((unsigned)((N + rows_per_block - 1) / rows_per_block)), b(kProjWaves * kWave);
    // rows of whole 16-byte groups (bf16: 8-byte) on aligned bases take the software-pipelined kernel
    const bool pipe = (D & 3) == 0 && (((uintptr_t)lq | (uintptr_t)components | (uintptr_t)mean) & 15u) == 0;
#define CAT_PROJ(T, NT)                                                                                                         \
    do {                                                                                                                        \
        if (pipe)                                                                                                               \
            hipLaunchKernelGGL((k_pca_project_pipe<T, NT, false>), g, b, 0, st, (const T*)lq, N, D, p, mean, components, z, ldz, \
                               ProjFuse{});                                                                                    \
        else                                                                                                                    \
            hipLaunchKernelGGL((k_pca_project<T, NT>), g, b, 0, st, (const T*)lq, N, D, p, mean, components, z, ldz);           \
    } while (0)
    if (dt == CAT_F32) {
        if (p <= 16) CAT_PROJ(float, 1); else if (p <= 32) CAT_PROJ(float, 2); else CAT_PROJ(float, 4);
    } else {
        if (p <= 16) CAT_PROJ(bf16_t, 1); else if (p <= 32) CAT_PROJ(bf16_t, 2); else CAT_PROJ(bf16_t, 4);
    }
#undef CAT_PROJ
    CAT_LAUNCH_CHECK("k_pca_project");
    return CAT_OK;
}

// Algorithm 2 with the PCA front-end in one kernel, where the shape allows it (see k_pca_project_pipe).
bool apply_pca_fused_supported(const void* lq, int64_t D, int32_t K, int32_t p, const float* mean, const float* components,
                               const float* gamma, const float* beta, const void* corrected) {
    const uintptr_t bases = (uintptr_t)lq | (uintptr_t)components | (uintptr_t)mean | (uintptr_t)gamma | (uintptr_t)beta |
                            (uintptr_t)corrected;
    return (D & 3) == 0 && (bases & 15u) == 0 && p <= 64 && K <= 256;
}
cat_status launch_apply_pca_fused(const void* lq, int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt, const float* mean,
                                  const float* components, const float* centroids_z, const float* gamma, const float* beta,
                                  float alpha, void* corrected, int32_t* assignments, hipStream_t st) {
    if (!apply_pca_fused_supported(lq, D, K, p, mean, components, gamma, beta, corrected))
        return set_error(CAT_ERR_UNSUPPORTED, "fused PCA inference does not take D=%lld K=%d p=%d", (long long)D, (int)K, (int)p);
    ProjFuse f{centroids_z, gamma, beta, corrected, assignments, K, alpha};
    const int64_t rows_per_block = kProjWaves * 16;
    dim3 g((unsigned)((N + rows_per_block - 1) / rows_per_block)), b(kProjWaves * kWave);
#define CAT_FUSE(T, NT) \
    hipLaunchKernelGGL((k_pca_project_pipe<T, NT, true>), g, b, 0, st, (const T*)lq, N, D, p, mean, components, nullptr, 0, f)
    if (dt == CAT_F32) {
        if (p <= 16) CAT_FUSE(float, 1); else if (p <= 32) CAT_FUSE(float, 2); else CAT_FUSE(float, 4);
    } else {
        if (p <= 16) CAT_FUSE(bf16_t, 1); else if (p <= 32) CAT_FUSE(bf16_t, 2); else CAT_FUSE(bf16_t, 4);
    }
#undef CAT_FUSE
    CAT_LAUNCH_CHECK("k_pca_project_pipe (fused inference)");
    return CAT_OK;
}

}  // namespace cat

using namespace cat;

extern "C" {

size_t cat_pca_workspace_bytes(int64_t N, int64_t D, int32_t p, cat_dtype dt) {
    if (!pca_shape_ok(N, D, p, dt)) return 0;
    return pca_carve(nullptr, D).bytes;
}

cat_status cat_pca_fit(const void* lq, int64_t N, int64_t D, int32_t p, cat_dtype dt, int32_t sweeps, float* mean,
                       float* components, double* eigenvalues, void* workspace, size_t workspace_bytes, void* hip_stream) {
    if (!pca_shape_ok(N, D, p, dt))
        return set_error(CAT_ERR_INVALID_ARG, "cat_pca_fit: need 1 <= p <= D <= %d, N >= 1 (N=%lld D=%lld p=%d dt=%d)", kPcaMaxD,
                         (long long)N, (long long)D, (int)p, (int)dt);
    if (!lq || !mean || !components) return set_error(CAT_ERR_INVALID_ARG, "cat_pca_fit: null argument");
    if (sweeps < 0 || sweeps > 64) return set_error(CAT_ERR_INVALID_ARG, "cat_pca_fit: sweeps must be in 0 .. 64");
    if (sweeps == 0) sweeps = 12;
    PcaWs w = pca_carve(workspace, D);
    if (!workspace || workspace_bytes < w.bytes)
        return set_error(CAT_ERR_WORKSPACE, "cat_pca_fit: workspace of %zu bytes needed, %zu given", w.bytes, workspace_bytes);
    hipStream_t st = (hipStream_t)hip_stream;
    const int64_t Dp = even_up(D);
    cat_status s;
    if ((s = launch_fill_zero(w.sum, (size_t)D * 8, st)) != CAT_OK) return s;
    if ((s = launch_fill_zero(w.W, (size_t)Dp * Dp * 8, st)) != CAT_OK) return s;
    // about 64 row ranges: enough workgroups for the covariance without drowning it in atomics
    int64_t rpb = (N + 63) / 64;
    rpb = (rpb + kCovRows - 1) / kCovRows * kCovRows;
    const unsigned nrb = (unsigned)((N + rpb - 1) / rpb);
    {
        // about 1024 workgroups: 256 or more row ranges (256 atomics per column at most)
        const int64_t cblocks = (D + 255) / 256;
        int64_t ranges = (1024 + cblocks - 1) / cblocks;
        ranges = ranges < 256 ? 256 : ranges;
        int64_t rps = (N + ranges - 1) / ranges;
        rps = (rps + 7) & ~(int64_t)7;
        dim3 g((unsigned)cblocks, (unsigned)((N + rps - 1) / rps)), b(256);
        if (dt == CAT_F32)
            hipLaunchKernelGGL(k_pca_colsum<float>, g, b, 0, st, (const float*)lq, N, D, rps, w.sum);
        else
            hipLaunchKernelGGL(k_pca_colsum<bf16_t>, g, b, 0, st, (const bf16_t*)lq, N, D, rps, w.sum);
        CAT_LAUNCH_CHECK("k_pca_colsum");
        hipLaunchKernelGGL(k_pca_mean, dim3((unsigned)((D + 255) / 256)), dim3(256), 0, st, w.sum, N, D, w.mean, mean);
        CAT_LAUNCH_CHECK("k_pca_mean");
    }
    {
        if (D >= kCovM) {
            // matrix cores: 64 x 64 tiles, the rows split so that about 6144 waves are at work, four per workgroup
            const int ntile = (int)((D + kCovM - 1) / kCovM);
            const int ntri = ntile * (ntile + 1) / 2;
            int64_t split = (6144 + ntri - 1) / ntri;
            split = (split + 3) / 4 * 4;
            int64_t rpw = (N + split - 1) / split;
            rpw = (rpw + 15) / 16 * 16;
            const int64_t nranges = (N + rpw - 1) / rpw;
            dim3 g((unsigned)ntri, (unsigned)((nranges + 3) / 4)), b(256);
            if (dt == CAT_F32)
                hipLaunchKernelGGL(k_pca_cov_mfma<float>, g, b, 0, st, (const float*)lq, N, D, w.mean, rpw, ntile, w.W, Dp);
            else
                hipLaunchKernelGGL(k_pca_cov_mfma<bf16_t>, g, b, 0, st, (const bf16_t*)lq, N, D, w.mean, rpw, ntile, w.W, Dp);
        } else {
            const int ntile = (int)((D + kCovTile - 1) / kCovTile);
            dim3 g((unsigned)(ntile * (ntile + 1) / 2), nrb), b(256);
            if (dt == CAT_F32)
                hipLaunchKernelGGL(k_pca_cov<float>, g, b, 0, st, (const float*)lq, N, D, w.mean, rpb, ntile, w.W, Dp);
            else
                hipLaunchKernelGGL(k_pca_cov<bf16_t>, g, b, 0, st, (const bf16_t*)lq, N, D, w.mean, rpb, ntile, w.W, Dp);
        }
        CAT_LAUNCH_CHECK("k_pca_cov");
        dim3 g2((unsigned)((Dp + 255) / 256), (unsigned)Dp);
        hipLaunchKernelGGL(k_pca_cov_finish, g2, dim3(256), 0, st, w.W, w.Vt, D, Dp, N);
        CAT_LAUNCH_CHECK("k_pca_cov_finish");
        hipLaunchKernelGGL(k_pca_mirror, g2, dim3(256), 0, st, w.W, D, Dp);
        CAT_LAUNCH_CHECK("k_pca_mirror");
    }
    {
        const int ni = (int)((Dp + 255) / 256);
        const dim3 jb(256), gpair((unsigned)(Dp / 2)), gquad((unsigned)(Dp / 4)), goct((unsigned)(Dp / 8));
#define CAT_JACOBI_CASES(KERNEL, GRID, ARG, FROM)                                                              \
        case FROM: hipLaunchKernelGGL(KERNEL<FROM>, GRID, jb, 0, st, w.W, w.Vt, (int32_t)Dp, ARG); break;
#define CAT_STEP(NI_) CAT_JACOBI_CASES(k_pca_jacobi_step, gpair, -1, NI_)
        // rows in registers: 4 BR NI doubles per thread with blocks of BR = 4 rows: 256 threads up to Dp = 512,
        // 512 beyond (NI <= 4; twice the waves to issue the loads and stores of a launch: 3 % faster at Dp = 1000)
        const bool wide = ni > 2;
        const int nb = wide ? (int)((Dp + 511) / 512) : ni;
        const dim3 jbb(wide ? 512 : 256);
        for (int sw = 0; sw < sweeps; sw++) {
            switch (ni) { CAT_STEP(1) CAT_STEP(2) CAT_STEP(3) CAT_STEP(4) CAT_STEP(5) CAT_STEP(6) CAT_STEP(7) default: CAT_STEP(8) }
            CAT_LAUNCH_CHECK("k_pca_jacobi_step");
            // the two halves of every block of four, then every pair of blocks of four
            for (int round = -1; round < (int)(Dp / 4) - 1; round++) {
                const bool halves = round < 0;
#define CAT_B(NI_, T_)                                                                                                      \
    if (halves)                                                                                                             \
        hipLaunchKernelGGL((k_pca_jacobi_block<NI_, 2, T_>), gquad, jbb, 0, st, w.W, w.Vt, (int32_t)Dp, -1);                 \
    else                                                                                                                    \
        hipLaunchKernelGGL((k_pca_jacobi_block<NI_, 4, T_>), goct, jbb, 0, st, w.W, w.Vt, (int32_t)Dp, round);
                if (wide) {
                    if (nb <= 2) { CAT_B(2, 512) } else if (nb == 3) { CAT_B(3, 512) } else { CAT_B(4, 512) }
                } else if (nb == 1) { CAT_B(1, 256) } else if (nb == 2) { CAT_B(2, 256) } else if (nb == 3) { CAT_B(3, 256) } else { CAT_B(4, 256) }
#undef CAT_B
                CAT_LAUNCH_CHECK("k_pca_jacobi_block");
            }
        }
#undef CAT_STEP
#undef CAT_JACOBI_CASES
    }
    hipLaunchKernelGGL(k_pca_rayleigh, dim3((unsigned)Dp), dim3(256), 0, st, w.W, w.Vt, (int32_t)Dp, w.lambda);
    CAT_LAUNCH_CHECK("k_pca_rayleigh");
    hipLaunchKernelGGL(k_pca_select, dim3((unsigned)p), dim3(256), 0, st, w.lambda, w.Vt, (int32_t)D, (int32_t)Dp, components, eigenvalues);
    CAT_LAUNCH_CHECK("k_pca_select");
    return CAT_OK;
}

cat_status cat_pca_project(const void* lq, int64_t N, int64_t D, int32_t p, cat_dtype dt, const float* mean,
                           const float* components, float* z, void* hip_stream) {
    return pca_project_ld(lq, N, D, p, dt, mean, components, z, p, (hipStream_t)hip_stream);
}

cat_status cat_apply_assigned(const void* lq, const int32_t* assignments, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                              const float* gamma, const float* beta, float alpha, void* corrected, void* hip_stream) {
    if ((dt != CAT_F32 && dt != CAT_BF16) || N < 1 || D < 1 || K < 1 || K > CAT_MAX_K)
        return set_error(CAT_ERR_INVALID_ARG, "cat_apply_assigned: bad shape (N=%lld D=%lld K=%d dt=%d)", (long long)N, (long long)D,
                         (int)K, (int)dt);
    if (!lq || !assignments || !gamma || !beta || !corrected || corrected == lq)
        return set_error(CAT_ERR_INVALID_ARG, "cat_apply_assigned: null or aliased argument");
    if (!(alpha == alpha) || alpha - alpha != 0.f) return set_error(CAT_ERR_INVALID_ARG, "cat_apply_assigned: alpha must be finite");
    hipStream_t st = (hipStream_t)hip_stream;
    dim3 g((unsigned)((N + 3) / 4)), b(256);
    const size_t esz = dt == CAT_F32 ? 4 : 2;
    const bool wide = (D * esz) % 16 == 0 && (((uintptr_t)lq | (uintptr_t)corrected | (uintptr_t)gamma | (uintptr_t)beta) & 15u) == 0 &&
                      (D * 4) % 16 == 0;
#define CAT_AA(T, W) \
    hipLaunchKernelGGL((k_apply_assigned<T, W>), g, b, 0, st, (const T*)lq, assignments, N, D, K, gamma, beta, alpha, (T*)corrected)
    if (dt == CAT_F32) {
        if (wide) CAT_AA(float, true); else CAT_AA(float, false);
    } else {
        if (wide) CAT_AA(bf16_t, true); else CAT_AA(bf16_t, false);
    }
#undef CAT_AA
    CAT_LAUNCH_CHECK("k_apply_assigned");
    return CAT_OK;
}

}  // extern "C"
