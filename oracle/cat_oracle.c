/*
 * CPU oracle for CAT (Cluster-based Affine Transformation), arXiv 2509.26277.
 *
 * TEST INFRASTRUCTURE ONLY.  This file is the slow, plain, double-precision
 * statement of what the hot path computes.  It shares no code with the GPU
 * library, includes none of its headers, and must never be called from the
 * product path.  Only the test-suite, the smoke check and the benchmark's
 * CPU-baseline leg use it.
 *
 * What it follows:
 *   - clustering: the paper names k-means as its clustering model (Sec. 4,
 *     Setup; Algorithm 1, the Cluster-Model fit step) and fixes no variant,
 *     so this is textbook Lloyd: squared Euclidean distance in the direct form
 *     sum_j (x_j - c_j)^2, the lowest cluster index wins a tie, a cluster that
 *     loses all its rows keeps its centroid, exactly `iters` iterations.
 *   - affine fit: the cluster means, the LQ variance, the LQ/FP covariance
 *     (Sec. 3.1, the three unnumbered displays before Eq. (gamma-beta)), all
 *     with the 1/|C_k| normalisation, two-pass; gamma = cov / max(var, 1e-8)
 *     and beta = mu_FP - gamma * mu_LQ (Eq. (gamma-beta) with the variance
 *     floor of Algorithm 1); an empty cluster gets gamma = 1, beta = 0
 *     (Algorithm 1, the empty-index branch).
 *   - inference: nearest centroid, then q + alpha * ((q * gamma + beta) - q)
 *     (Algorithm 2; the alpha-blend display at the end of Sec. 3.1).
 *   - seeded initialisation: K distinct row indices drawn with SplitMix64
 *     (Steele, Lea, Flood, OOPSLA 2014) used as a counter-based generator,
 *     re-implemented here from its published definition.
 *   - PCA front-end (Sec. 3.1; first step of Algorithms 1 and 2): column means,
 *     population covariance, projection (near the end of this file); pinned in
 *     tests/test_oracle_pca_pins.py.
 *   - sweep of the blending coefficient (Sec. 3.1 alpha display; the ablation on
 *     alpha, Sec. 5): Top-1 index, Top-1 hits and squared error per alpha (the
 *     sweep function near the end of this file); pinned in tests/test_oracle_sweep_pins.py.
 *   - D^2-weighted seeding (k-means++, Arthur and Vassilvitskii 2007) as an
 *     alternative initialisation (last function); pinned in
 *     tests/test_oracle_seeding_pins.py.
 *
 * Inputs are float arrays (bf16 data is widened exactly by the caller); every
 * sum, mean, distance and quotient below is IEEE double, accumulated
 * sequentially in row order.  OpenMP is used only where iterations are
 * independent (rows in the assignment/inference steps, channels in the
 * reductions), so the thread count never changes a single bit of the result.
 *
 * Pins (tests/test_oracle_*.py): SplitMix64 published vectors; the K=1 case
 * against a library least-squares fit; normal equations; a hand example that
 * is exact in binary; planted-mixture recovery; brute-force enumeration of
 * all labelings on tiny inputs; monotone objective; invariances.
 */
#include <math.h>
#include <stdint.h>
#include <stdlib.h>
#include <string.h>
#ifdef _OPENMP
#include <omp.h>
#endif

#define VAR_FLOOR 1e-8 /* Algorithm 1: sigma_Q^2 <- max(Var(Q), 1e-8) */
#define CH_BLOCK 32    /* channels handed to one thread at a time; no effect on results */

int cat_oracle_threads(void) {
#ifdef _OPENMP
    return omp_get_max_threads();
#else
    return 1;
#endif
}

/* ------------------------------------------------------------------ */
/* SplitMix64 as a counter-based generator: output t (t = 0, 1, ...)   */
/* is the SplitMix64 finaliser applied to seed + (t + 1) * golden.     */
/* This equals the t-th output of the sequential generator started at  */
/* state = seed.                                                       */
/* ------------------------------------------------------------------ */
uint64_t cat_oracle_splitmix64(uint64_t seed, uint64_t t) {
    uint64_t z = seed + (t + 1u) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}

/* K distinct row indices: walk the counter t = 0, 1, 2, ...; candidate =
 * output mod N; a candidate equal to an index already taken is skipped. */
void cat_oracle_init_indices(int64_t N, int32_t K, uint64_t seed, int64_t *idx) {
    int32_t have = 0;
    uint64_t t = 0;
    while (have < K) {
        int64_t cand = (int64_t)(cat_oracle_splitmix64(seed, t) % (uint64_t)N);
        t++;
        int dup = 0;
        for (int32_t q = 0; q < have; q++)
            if (idx[q] == cand) { dup = 1; break; }
        if (!dup) idx[have++] = cand;
    }
}

/* ------------------------------------------------------------------ */
/* Assignment step: a_i = argmin_k sum_j (x_ij - c_kj)^2, lowest k on  */
/* ties.  d1 = the minimum, d2 = the second smallest (over k != a_i;   */
/* +inf when K == 1); either may be NULL.                              */
/* ------------------------------------------------------------------ */
void cat_oracle_assign(const float *lq, int64_t N, int64_t D, int32_t K,
                       const double *cent, int32_t *assign, double *d1, double *d2) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; i++) {
        const float *x = lq + i * D;
        double best = INFINITY, second = INFINITY;
        int32_t arg = 0;
        for (int32_t k = 0; k < K; k++) {
            const double *c = cent + (int64_t)k * D;
            double s = 0.0;
            for (int64_t j = 0; j < D; j++) {
                double diff = (double)x[j] - c[j];
                s += diff * diff;
            }
            if (s < best) { /* strict: an equal later k never replaces an earlier one */
                second = best;
                best = s;
                arg = k;
            } else if (s < second) {
                second = s;
            }
        }
        assign[i] = arg;
        if (d1) d1[i] = best;
        if (d2) d2[i] = second;
    }
}

/* Distances of every row to every centroid (N x K), for tests on small inputs. */
void cat_oracle_distances(const float *lq, int64_t N, int64_t D, int32_t K,
                          const double *cent, double *dist) {
    for (int64_t i = 0; i < N; i++)
        for (int32_t k = 0; k < K; k++) {
            double s = 0.0;
            for (int64_t j = 0; j < D; j++) {
                double diff = (double)lq[i * D + j] - cent[(int64_t)k * D + j];
                s += diff * diff;
            }
            dist[i * K + k] = s;
        }
}

/* ------------------------------------------------------------------ */
/* Update step: c_k <- mean of the rows assigned to k; a cluster with  */
/* no rows keeps its centroid.                                         */
/* ------------------------------------------------------------------ */
void cat_oracle_update(const float *lq, const int32_t *assign, int64_t N, int64_t D,
                       int32_t K, double *cent, int64_t *counts) {
    int64_t *n = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    double *sum = (double *)calloc((size_t)K * (size_t)D, sizeof(double));
    for (int64_t i = 0; i < N; i++) n[assign[i]]++;
    /* channels are independent; each (k, j) sum runs over rows in row order */
#pragma omp parallel for schedule(static)
    for (int64_t j0 = 0; j0 < D; j0 += CH_BLOCK) {
        int64_t j1 = j0 + CH_BLOCK < D ? j0 + CH_BLOCK : D;
        for (int64_t i = 0; i < N; i++)
            for (int64_t j = j0; j < j1; j++)
                sum[(int64_t)assign[i] * D + j] += (double)lq[i * D + j];
    }
    for (int32_t k = 0; k < K; k++) {
        if (n[k] > 0)
            for (int64_t j = 0; j < D; j++)
                cent[(int64_t)k * D + j] = sum[(int64_t)k * D + j] / (double)n[k];
        if (counts) counts[k] = n[k];
    }
    free(sum);
    free(n);
}

/* ------------------------------------------------------------------ */
/* Per-cluster, per-channel affine parameters (two passes).            */
/* ------------------------------------------------------------------ */
void cat_oracle_affine(const float *lq, const float *fp, const int32_t *assign,
                       int64_t N, int64_t D, int32_t K,
                       double *gamma, double *beta, int64_t *counts) {
    size_t KD = (size_t)K * (size_t)D;
    int64_t *n = (int64_t *)calloc((size_t)K, sizeof(int64_t));
    double *mu_q = (double *)calloc(KD, sizeof(double));
    double *mu_f = (double *)calloc(KD, sizeof(double));
    double *var = (double *)calloc(KD, sizeof(double));
    double *cov = (double *)calloc(KD, sizeof(double));
    for (int64_t i = 0; i < N; i++) n[assign[i]]++;

    /* pass 1: cluster means of LQ and FP */
#pragma omp parallel for schedule(static)
    for (int64_t j0 = 0; j0 < D; j0 += CH_BLOCK) {
        int64_t j1 = j0 + CH_BLOCK < D ? j0 + CH_BLOCK : D;
        for (int64_t i = 0; i < N; i++)
            for (int64_t j = j0; j < j1; j++) {
                int64_t kj = (int64_t)assign[i] * D + j;
                mu_q[kj] += (double)lq[i * D + j];
                mu_f[kj] += (double)fp[i * D + j];
            }
        for (int32_t k = 0; k < K; k++)
            if (n[k] > 0)
                for (int64_t j = j0; j < j1; j++) {
                    mu_q[(int64_t)k * D + j] /= (double)n[k];
                    mu_f[(int64_t)k * D + j] /= (double)n[k];
                }
    }
    /* pass 2: centred second moments, 1/|C_k| normalisation */
#pragma omp parallel for schedule(static)
    for (int64_t j0 = 0; j0 < D; j0 += CH_BLOCK) {
        int64_t j1 = j0 + CH_BLOCK < D ? j0 + CH_BLOCK : D;
        for (int64_t i = 0; i < N; i++)
            for (int64_t j = j0; j < j1; j++) {
                int64_t kj = (int64_t)assign[i] * D + j;
                double dq = (double)lq[i * D + j] - mu_q[kj];
                double df = (double)fp[i * D + j] - mu_f[kj];
                var[kj] += dq * dq;
                cov[kj] += dq * df;
            }
        for (int32_t k = 0; k < K; k++)
            for (int64_t j = j0; j < j1; j++) {
                int64_t kj = (int64_t)k * D + j;
                if (n[k] == 0) {
                    gamma[kj] = 1.0;
                    beta[kj] = 0.0;
                } else {
                    double v = var[kj] / (double)n[k];
                    double c = cov[kj] / (double)n[k];
                    if (v < VAR_FLOOR) v = VAR_FLOOR;
                    gamma[kj] = c / v;
                    beta[kj] = mu_f[kj] - gamma[kj] * mu_q[kj];
                }
            }
    }
    if (counts) memcpy(counts, n, (size_t)K * sizeof(int64_t));
    free(cov); free(var); free(mu_f); free(mu_q); free(n);
}

/* ------------------------------------------------------------------ */
/* CAT Fitting: init, `iters` Lloyd iterations, a final assignment     */
/* against the final centroids, then the affine fit on that partition. */
/* inertia[t] (t = 0..iters) is the k-means objective of the t-th      */
/* assignment pass; may be NULL.  init may be NULL (seeded rows).       */
/* ------------------------------------------------------------------ */
void cat_oracle_fit(const float *lq, const float *fp, int64_t N, int64_t D, int32_t K,
                    int32_t iters, uint64_t seed, const double *init,
                    double *cent, double *gamma, double *beta, int32_t *assign,
                    int64_t *counts, double *inertia) {
    if (init) {
        memcpy(cent, init, (size_t)K * (size_t)D * sizeof(double));
    } else {
        int64_t *idx = (int64_t *)malloc((size_t)K * sizeof(int64_t));
        cat_oracle_init_indices(N, K, seed, idx);
        for (int32_t k = 0; k < K; k++)
            for (int64_t j = 0; j < D; j++)
                cent[(int64_t)k * D + j] = (double)lq[idx[k] * D + j];
        free(idx);
    }
    double *d1 = (double *)malloc((size_t)N * sizeof(double));
    for (int32_t t = 0; t <= iters; t++) {
        cat_oracle_assign(lq, N, D, K, cent, assign, d1, NULL);
        if (inertia) {
            double J = 0.0;
            for (int64_t i = 0; i < N; i++) J += d1[i];
            inertia[t] = J;
        }
        if (t < iters) cat_oracle_update(lq, assign, N, D, K, cent, NULL);
    }
    free(d1);
    cat_oracle_affine(lq, fp, assign, N, D, K, gamma, beta, counts);
}

/* ------------------------------------------------------------------ */
/* CAT Inferencing.                                                    */
/* ------------------------------------------------------------------ */
void cat_oracle_apply(const float *lq, int64_t N, int64_t D, int32_t K,
                      const double *cent, const double *gamma, const double *beta,
                      double alpha, double *out, int32_t *assign) {
    int32_t *a = assign ? assign : (int32_t *)malloc((size_t)N * sizeof(int32_t));
    cat_oracle_assign(lq, N, D, K, cent, a, NULL, NULL);
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; i++) {
        const double *g = gamma + (int64_t)a[i] * D;
        const double *b = beta + (int64_t)a[i] * D;
        for (int64_t j = 0; j < D; j++) {
            double q = (double)lq[i * D + j];
            double affine = q * g[j] + b[j];
            out[i * D + j] = q + alpha * (affine - q);
        }
    }
    if (!assign) free(a);
}

/* ---------------------------------------------------------------------------
 * PCA front-end (Sec. 3.1: the LQ vectors are reduced by a principal component
 * analysis before clustering; Alg. 1 and Alg. 2, first step).  Written out as
 * the textbook definition: column means, the D x D covariance of the centred
 * data with the 1/N normalisation used everywhere else here (the directions do
 * not depend on the divisor), and the projection of centred rows on given
 * directions.  The symmetric eigendecomposition in between is a library
 * routine called from the Python wrapper.  Sums are sequential in double;
 * OpenMP only splits independent outputs.
 * ------------------------------------------------------------------------- */
void cat_oracle_colmean(const float *x, int64_t N, int64_t D, double *mean) {
#pragma omp parallel for schedule(static)
    for (int64_t j = 0; j < D; j++) {
        double s = 0.0;
        for (int64_t i = 0; i < N; i++) s += (double)x[i * D + j];
        mean[j] = s / (double)N;
    }
}

/* cov[a][b] = (1/N) sum_i (x[i][a] - mean[a]) (x[i][b] - mean[b]), full D x D */
void cat_oracle_covariance(const float *x, int64_t N, int64_t D, const double *mean, double *cov) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int64_t a = 0; a < D; a++) {
        for (int64_t b = a; b < D; b++) {
            double s = 0.0;
            for (int64_t i = 0; i < N; i++)
                s += ((double)x[i * D + a] - mean[a]) * ((double)x[i * D + b] - mean[b]);
            cov[a * D + b] = s / (double)N;
        }
    }
    for (int64_t a = 0; a < D; a++)
        for (int64_t b = 0; b < a; b++) cov[a * D + b] = cov[b * D + a];
}

/* z[i][c] = sum_j (x[i][j] - mean[j]) comps[c][j],  comps is p x D */
void cat_oracle_project(const float *x, int64_t N, int64_t D, int32_t p, const double *mean,
                        const double *comps, double *z) {
#pragma omp parallel for schedule(static)
    for (int64_t i = 0; i < N; i++) {
        for (int32_t c = 0; c < p; c++) {
            double s = 0.0;
            for (int64_t j = 0; j < D; j++) s += ((double)x[i * D + j] - mean[j]) * comps[(int64_t)c * D + j];
            z[i * p + c] = s;
        }
    }
}

/* ---------------------------------------------------------------------------
 * Sweep of the blending coefficient (the alpha display of Sec. 3.1; the ablation
 * on alpha in Sec. 5 and its appendix evaluates one fitted transformation at a
 * list of alpha values).  For every alpha in the list and every row i with
 * cluster label a_i:
 *     c_i(alpha) = q_i + alpha * (gamma_a q_i + beta_a - q_i)
 * (a label outside [0, K) leaves the row uncorrected, c_i = q_i).  Reported per
 * alpha: top1[i] = the position of the largest entry of c_i(alpha), the first
 * one on ties; margin[i] = that entry minus the second largest (0 on a tie,
 * +inf for D = 1); hits = the number of rows whose top1 equals labels[i]; sq_err =
 * sum over all entries of (c - fp)^2.  Layouts: top1 and margin are N x n_alpha.
 * fp, labels, top1, margin are optional (NULL).  Sums are sequential in row
 * order, in double; OpenMP only splits the independent alpha values.
 * ------------------------------------------------------------------------- */
void cat_oracle_alpha_sweep(const float *lq, const float *fp, const int32_t *labels,
                            const int32_t *assign, int64_t N, int64_t D, int32_t K,
                            const double *gamma, const double *beta, const double *alphas,
                            int32_t n_alpha, int64_t *hits, double *sq_err, int32_t *top1,
                            double *margin) {
#pragma omp parallel for schedule(dynamic, 1)
    for (int32_t s = 0; s < n_alpha; s++) {
        const double alpha = alphas[s];
        int64_t h = 0;
        double err = 0.0;
        for (int64_t i = 0; i < N; i++) {
            const int32_t a = assign[i];
            const int inside = a >= 0 && a < K;
            const double *g = inside ? gamma + (int64_t)a * D : NULL;
            const double *b = inside ? beta + (int64_t)a * D : NULL;
            double best = 0.0, second = 0.0;
            int64_t arg = -1;
            for (int64_t j = 0; j < D; j++) {
                const double q = (double)lq[i * D + j];
                double c = q;
                if (inside) {
                    const double affine = g[j] * q + b[j];
                    c = q + alpha * (affine - q);
                }
                if (fp) {
                    const double e = c - (double)fp[i * D + j];
                    err += e * e;
                }
                if (arg < 0) {
                    best = c;
                    arg = j;
                    second = -HUGE_VAL;
                } else if (c > best) {
                    second = best;
                    best = c;
                    arg = j;
                } else if (c > second) {
                    second = c;
                }
            }
            if (labels && (int64_t)labels[i] == arg) h++;
            if (top1) top1[i * n_alpha + s] = (int32_t)arg;
            if (margin) margin[i * n_alpha + s] = best - second;
        }
        if (hits) hits[s] = h;
        if (sq_err) sq_err[s] = fp ? err : 0.0;
    }
}

/* ---------------------------------------------------------------------------
 * D^2-weighted seeding ("k-means++", Arthur and Vassilvitskii, SODA 2007), an
 * alternative to the seeded distinct rows above; the paper fixes no k-means
 * initialisation (Sec. 4, Setup).  The published procedure: the first centre is a
 * row drawn uniformly; every further centre is a row drawn with probability
 * proportional to its squared distance to the nearest centre chosen so far.
 * The draws: u_t = (SplitMix64 output t of the seed >> 11) * 2^-53 in [0, 1),
 * t = 0 .. K-1.  First row: floor(u_0 * N).  Row t >= 1: with d2[i] the current
 * squared distance of row i to its nearest centre and S the sum of all d2 in row
 * order, the row is the first i whose running sum d2[0] + .. + d2[i] exceeds
 * u_t * S.  If S = 0 (every row coincides with a centre) the row is the lowest
 * index not chosen yet.  Distances are direct-form sums over the channels in
 * double.  idx receives the K row indices in the order drawn.
 * ------------------------------------------------------------------------- */
void cat_oracle_kmeanspp(const float *lq, int64_t N, int64_t D, int32_t K, uint64_t seed,
                         int64_t *idx) {
    double *d2 = (double *)malloc((size_t)N * sizeof(double));
    for (int32_t t = 0; t < K; t++) {
        const double u = (double)(cat_oracle_splitmix64(seed, (uint64_t)t) >> 11) * 0x1.0p-53;
        int64_t pick = -1;
        if (t == 0) {
            pick = (int64_t)(u * (double)N);
            if (pick > N - 1) pick = N - 1;
        } else {
            double S = 0.0;
            for (int64_t i = 0; i < N; i++) S += d2[i];
            if (S > 0.0) {
                const double target = u * S;
                double run = 0.0;
                for (int64_t i = 0; i < N; i++) {
                    run += d2[i];
                    if (run > target) { pick = i; break; }
                }
            }
            if (pick < 0) { /* S = 0: lowest index not chosen yet */
                for (int64_t c = 0; c < N && pick < 0; c++) {
                    int taken = 0;
                    for (int32_t q = 0; q < t; q++)
                        if (idx[q] == c) { taken = 1; break; }
                    if (!taken) pick = c;
                }
            }
        }
        idx[t] = pick;
        const float *cr = lq + pick * D;
#pragma omp parallel for schedule(static)
        for (int64_t i = 0; i < N; i++) {
            double s = 0.0;
            for (int64_t j = 0; j < D; j++) {
                const double d = (double)lq[i * D + j] - (double)cr[j];
                s += d * d;
            }
            if (t == 0 || s < d2[i]) d2[i] = s;
        }
    }
    free(d2);
}
