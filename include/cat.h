/*
 * cat.h -- C ABI of the MI355X (gfx950) hot path of CAT, the Cluster-based
 * Affine Transformation of arXiv 2509.26277.
 *
 * Two phases (Sec. 3.1; Appendix B, Algorithms 1 and 2):
 *   CAT Fitting      k-means over the low-bit-quantised (LQ) output vectors, then,
 *                    per cluster and per channel, gamma = cov(LQ,FP) / var(LQ) and
 *                    beta = mean(FP) - gamma * mean(LQ).
 *   CAT Inferencing  nearest centroid, then  q + alpha * (gamma_k * q + beta_k - q).
 * The paper reduces the LQ vectors with PCA before clustering.  cat_fit and
 * cat_apply cluster in the full dimension D (the pca_dim = D case: a full-rank
 * PCA is a rigid motion and leaves every distance unchanged); cat_fit_pca and
 * cat_apply_pca are the same two phases with the PCA front-end (further down).
 *
 * Conventions, valid for every entry point unless stated otherwise
 *   - Every data pointer is a DEVICE pointer owned by the caller.  The library
 *     allocates and frees nothing; scratch memory comes from `workspace`
 *     (device, 256-byte aligned, at least the size the matching
 *     *_workspace_bytes() returns; its contents on entry do not matter and are
 *     garbage on return).
 *   - Matrices are row-major and contiguous: lq, fp, corrected are N x D of
 *     `dt` (CAT_F32: float, CAT_BF16: bfloat16 stored as uint16); centroids,
 *     gamma, beta are K x D float.  Row starts must be 4-byte aligned (for
 *     CAT_BF16 this means D even); the base pointers 16-byte aligned.
 *   - 1 <= K <= N, 1 <= D, K <= CAT_MAX_K.  Element offsets are 64-bit.
 *   - Work is enqueued on `hip_stream` (a hipStream_t; NULL = the default
 *     stream); calls return without synchronising.  The status covers argument
 *     checks and launch errors; an asynchronous fault shows at the caller's
 *     next synchronisation.
 *   - Inputs are never modified; outputs are fully overwritten.  Nullable
 *     outputs are marked.  No exception crosses the ABI.
 *   - Non-finite input values give unspecified results (no crash, no hang).
 *   - Calls are re-entrant across distinct streams and workspaces, also from
 *     several host threads (what the library caches between calls is per thread).
 *
 * Distances are squared Euclidean.  A tie goes to the LOWEST cluster index.
 * The assignment is exact up to rounding: a fast bf16-split MFMA pass ranks the
 * centroids, and every row whose two best scores are closer than the pass's
 * error bound is re-ranked with direct-form double-precision distances.
 */
#ifndef CAT_H
#define CAT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

#define CAT_MAX_K 1024
#define CAT_MAX_ALPHAS 16 /* longest list of blending coefficients one cat_alpha_sweep call takes */

typedef enum {
    CAT_OK = 0,
    CAT_ERR_INVALID_ARG = 1, /* null pointer, bad size, bad alignment, bad enum      */
    CAT_ERR_UNSUPPORTED = 2, /* a valid request this build has no kernel for         */
    CAT_ERR_WORKSPACE = 3,   /* workspace null, misaligned or too small              */
    CAT_ERR_DEVICE = 4       /* a HIP call (launch, query) failed; see cat_last_error */
} cat_status;

typedef enum { CAT_F32 = 0, CAT_BF16 = 1 } cat_dtype;

/* Kernel family used for the assignment-type steps.  CAT_PATH_AUTO picks the
 * MFMA tile kernels whenever the shape fits them and the streaming kernels
 * otherwise; the other two values force one family (tests use this to cover
 * both on any shape).  Forcing CAT_PATH_TILE on a shape it cannot run makes the
 * call return CAT_ERR_UNSUPPORTED.  Process-wide; default CAT_PATH_AUTO. */
typedef enum { CAT_PATH_AUTO = 0, CAT_PATH_STREAM = 1, CAT_PATH_TILE = 2 } cat_path;

/* How cat_fit_restarts seeds the centroids of a run: the distinct rows of cat_init_indices, or the
 * D^2-weighted seeding of cat_init_kmeanspp. */
typedef enum { CAT_SEED_ROWS = 0, CAT_SEED_KMEANSPP = 1 } cat_seeding;
#define CAT_MAX_RESTARTS 1024
cat_status cat_select_path(cat_path p);

/* Bytes of device scratch cat_fit / cat_assign / cat_update / cat_stats need
 * (one size covers all four) and cat_apply needs.  Returns 0 for invalid
 * arguments.
 *
 * Rows that are not a whole number of 16-byte groups (D not a multiple of 4, of 8
 * for bf16) do not fit the MFMA tile kernels as they lie.  A fit reads lq once per
 * Lloyd pass, so with CAT_PATH_AUTO and iters >= 2 the fits (cat_fit, cat_fit_early_stop,
 * cat_fit_bounds, cat_fit_restarts, cat_fit_multi_k) copy lq once into rows padded
 * with zero channels up to the next such multiple, which leave every distance as it
 * is, and run their Lloyd loops on the copy wherever the tile kernels take the padded
 * shape; the statistics read the original rows.  For those shapes the scratch sizes
 * of the fits include the copy (N rows of the padded length).
 * cat_debug_padded_fit(on): 0 keeps such fits on the streaming kernels; process-wide,
 * default 1, for measurements and tests (results agree to rounding).
 * Single passes over such rows (cat_apply, cat_apply_lp, cat_apply_static, cat_assign,
 * fits of fewer than two iterations) run the fused row-tile inference kernel in a form
 * that moves rows, parameters and outputs in 4-byte words (K <= 128; rows of at most
 * 4 KB for fp32, 2 KB for bf16; for 33 .. 64 clusters at most 2 KB), and the LDS
 * streaming kernel beyond that. */
size_t cat_fit_workspace_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt);
cat_status cat_debug_padded_fit(int on);
size_t cat_apply_workspace_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt);

/*
 * CAT Fitting (Algorithm 1 with pca_dim = D; Sec. 3.1 for the statistics).
 *
 *   init      centroids <- init_centroids if given, else the K distinct rows of
 *             lq picked by cat_init_indices(N, K, seed).
 *   Lloyd     `iters` times: assign every row to its nearest centroid, then move
 *             each centroid to the mean of its rows (a centroid with no rows
 *             stays where it is).  No early stop.
 *   final     one more assignment against the final centroids: this is what
 *             `assignments`, `counts` and the last inertia entry describe, and
 *             what cat_apply reproduces on the same rows.
 *   affine    per cluster k and channel j, over the rows of cluster k:
 *             var = mean((x - mean x)^2), cov = mean((x - mean x)(y - mean y)),
 *             gamma = cov / max(var, 1e-8), beta = mean y - gamma * mean x
 *             (x = lq, y = fp).  An empty cluster gets gamma = 1, beta = 0.
 *
 * lq, fp          in,  N x D of dt
 * iters           >= 0 (0: centroids = init, then final + affine)
 * init_centroids  in,  K x D float, or NULL
 * centroids, gamma, beta   out, K x D float each
 * assignments     out, N int32
 * counts          out, K int32, nullable: rows per cluster of `assignments`
 * inertia         out, iters + 1 doubles, nullable: k-means objective (sum of
 *                 squared distances to the assigned centroid) of each of the
 *                 iters + 1 assignment passes.  On the tile kernels a row's term is
 *                 |x|^2 plus its best score in single precision (exact only for the rows
 *                 that go through the double-precision re-rank), so its error is the error
 *                 bound of a score, about 1e-4 |x||c| (3e-5 for bfloat16 rows): far below
 *                 1e-4 of the sum where the rows are as far from their centroid as from the
 *                 origin, a larger share of it where the data sit far from the origin
 *                 compared with their spread.  The assignments do not depend on it.
 */
cat_status cat_fit(const void *lq, const void *fp, int64_t N, int64_t D, int32_t K,
                   int32_t iters, uint64_t seed, cat_dtype dt,
                   const float *init_centroids,
                   float *centroids, float *gamma, float *beta,
                   int32_t *assignments, int32_t *counts, double *inertia,
                   void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * cat_fit with the Lloyd loop allowed to stop early.  The paper names k-means without a stopping
 * rule (Sec. 4, Setup); the rule here changes the work done, not the result: once a pass assigns
 * every row to the cluster it already had, the means and so every later pass repeat themselves,
 * and the passes between that one and the final one are not run.  All outputs are those of
 * cat_fit with the same arguments (the inertia entries of the passes not run repeat the entry
 * before them).  The decision is taken on the device from the number of rows that changed
 * cluster; nothing waits on the host, and the call can be captured in a HIP graph.
 *
 * passes_skipped  out, 1 int32: the number of assignment passes not run, between 0 and
 *                 iters - 3.  The library starts to look from pass 2 on: if pass t >= 1 is the
 *                 first whose assignments equal those of pass t - 1, this is
 *                 max(0, iters - 1 - max(t, 2)); 0 if there is none.  Loops that run on the
 *                 streaming kernels (K > 256, the streaming path selected, rows that are not
 *                 whole 16-byte groups where no padded copy is made) run every pass and report 0.
 * Other arguments, workspace and errors: as cat_fit.
 *
 * cat_allow_early_stop(on != 0) lets every Lloyd loop the library runs stop in the same way
 * (cat_fit, each run of cat_fit_restarts, the clustering of the scores in cat_fit_pca), without
 * the count of passes left out; their outputs do not change.  Process-wide, default off; returns
 * CAT_OK.
 */
cat_status cat_allow_early_stop(int on);
cat_status cat_fit_early_stop(const void *lq, const void *fp, int64_t N, int64_t D, int32_t K,
                              int32_t iters, uint64_t seed, cat_dtype dt,
                              const float *init_centroids,
                              float *centroids, float *gamma, float *beta,
                              int32_t *assignments, int32_t *counts, double *inertia,
                              int32_t *passes_skipped,
                              void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * CAT Inferencing (Algorithm 2; the alpha-blend at the end of Sec. 3.1), fused:
 * corrected_i = x_i + alpha * (gamma_a * x_i + beta_a - x_i),  a = nearest centroid
 * of x_i.  alpha is folded once into gamma' = 1 + alpha * (gamma - 1), beta' =
 * alpha * beta (K x D, in the workspace), so alpha = 0 returns the input values
 * unchanged and alpha = 1 is the pure affine map.  alpha must be finite.
 *
 * corrected     out, N x D of dt (may not alias lq)
 * assignments   out, N int32, nullable
 */
cat_status cat_apply(const void *lq, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                     const float *centroids, const float *gamma, const float *beta,
                     float alpha, void *corrected, int32_t *assignments,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * cat_apply for callers that cannot allocate device memory or carry a workspace around: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and errors as cat_apply, without the workspace: the scratch memory (the alpha-folded gamma / beta,
 * the centroids in matrix-core operand order and their norms) lives in a device array built into the
 * library, CAT_APPLY_STATIC_SCRATCH_BYTES long, one copy per GPU, held until the process ends.  The
 * call allocates and frees nothing.  A shape whose cat_apply_workspace_bytes() exceeds the array
 * returns CAT_ERR_UNSUPPORTED (K * D up to about 500,000 fits; cat_apply_static_max_workspace_bytes()
 * returns the limit).  Every call on a GPU uses that GPU's one array: calls that overlap in time on
 * the same GPU (different streams or threads) race and give unspecified results; calls on one stream
 * are ordered and safe.  The array keeps the last call's contents; nothing in it has to be cleared
 * (every byte the inference pass reads is written earlier in the same call).
 */
#define CAT_APPLY_STATIC_SCRATCH_BYTES (8u << 20)
size_t cat_apply_static_max_workspace_bytes(void);
cat_status cat_apply_static(const void *lq, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                            const float *centroids, const float *gamma, const float *beta,
                            float alpha, void *corrected, int32_t *assignments, void *hip_stream);

/* ---- step-level entry points (the pieces cat_fit is made of) ------------- */

/* Assignment step (the Cluster-Model "predict" of Algorithms 1 and 2).
 * assignments out N int32; counts out K int32, nullable; inertia out 1 double,
 * nullable. */
cat_status cat_assign(const void *lq, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                      const float *centroids, int32_t *assignments, int32_t *counts,
                      double *inertia, void *workspace, size_t workspace_bytes,
                      void *hip_stream);

/* Centroid update step of Lloyd's iteration: centroids[k] = mean of the rows with
 * assignments == k, or prev_centroids[k] if there is none.  assignments in, N
 * int32, each in [0, K).  centroids out (may alias prev_centroids); counts out,
 * nullable. */
cat_status cat_update(const void *lq, const int32_t *assignments, int64_t N, int64_t D,
                      int32_t K, cat_dtype dt, const float *prev_centroids,
                      float *centroids, int32_t *counts,
                      void *workspace, size_t workspace_bytes, void *hip_stream);

/* Per-cluster affine fit (Sec. 3.1 statistics, Eq. (gamma-beta), Algorithm 1's
 * variance floor and empty-cluster rule) for a given partition.  `centroids` is
 * an optional hint (K x D float, nullable): values near the cluster means of lq
 * used as the shift of the one-pass moment accumulation; it never changes what
 * is computed.  gamma, beta out; counts out, nullable. */
cat_status cat_stats(const void *lq, const void *fp, const int32_t *assignments,
                     int64_t N, int64_t D, int32_t K, cat_dtype dt, const float *centroids,
                     float *gamma, float *beta, int32_t *counts,
                     void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Seeded initial rows (the paper does not fix the k-means initialisation; this
 * is the rule).  SplitMix64 (Steele, Lea, Flood 2014) as a counter-based
 * generator: output t = mix(seed + (t + 1) * 0x9E3779B97F4A7C15) with
 *   mix(z): z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9;
 *           z = (z ^ (z >> 27)) * 0x94D049BB133111EB;  return z ^ (z >> 31);
 * all in 64-bit unsigned arithmetic.  Walk t = 0, 1, 2, ...; the candidate is
 * output mod N; a candidate already taken is skipped; stop at K indices.
 * idx_out is a HOST array of K int64.  Pure host code, no GPU needed.
 */
cat_status cat_init_indices(int64_t N, int32_t K, uint64_t seed, int64_t *idx_out);

/* ---- PCA front-end (Sec. 3.1; the first step of Algorithms 1 and 2) --------
 *
 * The paper clusters the p leading principal components of the LQ vectors rather
 * than the vectors themselves, and applies the affine correction of the cluster
 * found there to the full vector.  With these three calls that pipeline is
 *   fit:    cat_pca_fit -> cat_pca_project -> cat_fit on z (its assignments and
 *           centroids) -> cat_stats(lq, fp, assignments)
 *   apply:  cat_pca_project -> cat_assign on z -> cat_apply_assigned
 *
 * cat_pca_fit: column means of lq, the D x D covariance with the 1/N
 * normalisation, its eigendecomposition (one-sided Jacobi rotations in double
 * precision, `sweeps` sweeps over all pairs; 0 picks the default, 12), and the p
 * directions of largest eigenvalue in descending order, each a unit vector whose
 * entry of largest magnitude (the first such entry) is positive.  1 <= p <= D <=
 * 2048.
 *   mean         out, D float
 *   components   out, p x D float, row c = direction c
 *   eigenvalues  out, p doubles, nullable
 * cat_pca_project: z[i][c] = sum_j (lq[i][j] - mean[j]) components[c][j];
 *   z out, N x p float (fp32 accumulation).  No workspace.
 * cat_apply_assigned: corrected_i = x_i + alpha (gamma_a x_i + beta_a - x_i) with
 *   a = assignments[i] given by the caller; a label outside [0, K) copies the row.
 *   corrected out, N x D of dt, may not alias lq.  No workspace.
 */
/*
 * Algorithm 1 and Algorithm 2 with pca_dim = p as single calls, composed of the steps above:
 *   cat_fit_pca    PCA of lq -> scores -> init (seeded rows of the scores), `iters` Lloyd iterations and
 *                  the final assignment in score space -> gamma, beta on the full vectors.
 *                  mean (D), components (p x D), centroids_z (K x p), gamma, beta (K x D) out, float;
 *                  assignments out N int32; counts (K) and inertia (iters + 1, of the score-space
 *                  clustering) out, nullable.
 *   cat_apply_pca  scores -> nearest centroid in score space -> affine map of the full vector with
 *                  the alpha-blend.  corrected out (may not alias lq); assignments out, nullable.
 *                  One kernel when D is a multiple of 4, p <= 64 and K <= 256 (the scores never leave
 *                  the chip); the three steps one after the other otherwise, with identical results.
 */
size_t cat_fit_pca_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt);
cat_status cat_fit_pca(const void *lq, const void *fp, int64_t N, int64_t D, int32_t K, int32_t p,
                       int32_t iters, uint64_t seed, cat_dtype dt,
                       float *mean, float *components, float *centroids_z, float *gamma, float *beta,
                       int32_t *assignments, int32_t *counts, double *inertia,
                       void *workspace, size_t workspace_bytes, void *hip_stream);
size_t cat_apply_pca_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt);
cat_status cat_apply_pca(const void *lq, int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt,
                         const float *mean, const float *components, const float *centroids_z,
                         const float *gamma, const float *beta, float alpha,
                         void *corrected, int32_t *assignments,
                         void *workspace, size_t workspace_bytes, void *hip_stream);

size_t cat_pca_workspace_bytes(int64_t N, int64_t D, int32_t p, cat_dtype dt);
cat_status cat_pca_fit(const void *lq, int64_t N, int64_t D, int32_t p, cat_dtype dt, int32_t sweeps,
                       float *mean, float *components, double *eigenvalues,
                       void *workspace, size_t workspace_bytes, void *hip_stream);
cat_status cat_pca_project(const void *lq, int64_t N, int64_t D, int32_t p, cat_dtype dt,
                           const float *mean, const float *components, float *z, void *hip_stream);
cat_status cat_apply_assigned(const void *lq, const int32_t *assignments, int64_t N, int64_t D,
                              int32_t K, cat_dtype dt, const float *gamma, const float *beta,
                              float alpha, void *corrected, void *hip_stream);

/* ---- sweep of the blending coefficient (the alpha display of Sec. 3.1; the ablation on
 * alpha of Sec. 5 evaluates one fitted transformation at a list of alpha values) ----
 *
 * cat_alpha_sweep reads every row once and evaluates, for each of the n_alpha values,
 *     c_i(alpha) = x_i + alpha (gamma_a x_i + beta_a - x_i),   a = assignments[i]
 * (a label outside [0, K) leaves the row as it is), without writing c anywhere:
 *   top1     out, nullable, N x n_alpha int32 (row-major): the position of the largest entry of
 *            c_i(alpha), the first such position on ties.  The comparison is made on fp32 values
 *            fma(alpha, fma(x, gamma - 1, beta), x), also for bf16 rows (no rounding to bf16).
 *   labels   in, nullable, N int32; hits out, n_alpha int64: the number of rows whose top1 equals
 *            labels[i] (a label outside [0, D) never matches).  Both or neither.
 *   fp       in, nullable, N x D of dt.  sq_err out, nullable, n_alpha doubles: the sum over all
 *            entries of (c - fp)^2.  moments out, nullable, 3 doubles S_aa, S_ab, S_bb with
 *            a = x - fp and b = (gamma_a - 1) x + beta_a, so that the squared error at any alpha is
 *            S_aa + 2 alpha S_ab + alpha^2 S_bb (its minimum is at alpha = -S_ab / S_bb); sq_err is
 *            evaluated from them in double.  fp needs at least one of the two outputs.
 *   alphas   HOST array of n_alpha finite floats, 1 <= n_alpha <= CAT_MAX_ALPHAS; read before
 *            the call returns.
 * All other pointers are device memory.  Inputs are taken as finite.  workspace: at least
 * cat_alpha_sweep_workspace_bytes() bytes, 256-byte aligned, caller-owned.  Errors:
 * CAT_ERR_INVALID_ARG (shape, null or mismatched optional arguments, non-finite alpha),
 * CAT_ERR_WORKSPACE, CAT_ERR_DEVICE.
 *
 * cat_top1: top1[i] = the position of the largest entry of row i of x (N x D of dt), the first
 * on ties; the Top-1 prediction of a logit vector, e.g. of the FP rows as `labels` above.
 */
size_t cat_alpha_sweep_workspace_bytes(void);
cat_status cat_alpha_sweep(const void *lq, const void *fp, const int32_t *labels,
                           const int32_t *assignments, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                           const float *gamma, const float *beta,
                           const float *alphas, int32_t n_alpha,
                           int64_t *hits, double *sq_err, double *moments, int32_t *top1,
                           void *workspace, size_t workspace_bytes, void *hip_stream);
cat_status cat_top1(const void *x, int64_t N, int64_t D, cat_dtype dt, int32_t *top1, void *hip_stream);

/* ---- CAT Fitting whose Lloyd loop leaves out distance evaluations by bounds ----
 * The paper names k-means without fixing a variant (Sec. 4, Setup).  cat_fit_bounds returns what cat_fit returns and
 * does less work: after Hamerly ("Making k-means even faster", SDM 2010) every row carries a bound on how far the
 * centroids may move before its nearest centroid can change.  When a pass evaluates a row it records the gap
 * between the distances to its nearest and second nearest centroid (a lower bound of it, given the rounding of the
 * scores); every update adds the two largest centroid movements to a running drift; a row whose gap exceeds the drift
 * accumulated since its evaluation keeps its centroid (its distance to its own centroid grew by at most one movement,
 * its distance to any other shrank by at most another) and is neither read nor ranked in that pass.  Coarser than the
 * published algorithm (one gap per row instead of separate upper and lower bounds, no centre-to-centre test, no
 * tightening step): a pass reads a row or it does not.  Passes 0, 1, 2 and the last evaluate every row.
 *
 * rows_evaluated  out, device, iters + 1 int32, nullable: rows read and ranked by each pass
 * inertia         as cat_fit, but only the entries of the passes that evaluate every row (0, 1, 2, iters) are
 *                 defined; the others are NaN where rows were left out
 * workspace       cat_fit_bounds_workspace_bytes(N, D, K, iters, dt) bytes
 * Other arguments and errors: as cat_fit.  N below 2^31.  Shapes the matrix-core kernels do not take, more than 128
 * clusters on rows of more than 128 channels (their passes rank in two launches, which keep no bounds), the streaming
 * path selected, or iters < 4: the plain loop runs and every pass reports N rows.  centroids, assignments and counts
 * are those of cat_fit bit for bit, gamma and beta as from one call of cat_fit to the next (their sums are
 * accumulated with atomics, whose order moves the last bits). */
size_t cat_fit_bounds_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t iters, cat_dtype dt);
cat_status cat_fit_bounds(const void *lq, const void *fp, int64_t N, int64_t D, int32_t K,
                          int32_t iters, uint64_t seed, cat_dtype dt,
                          const float *init_centroids,
                          float *centroids, float *gamma, float *beta,
                          int32_t *assignments, int32_t *counts, double *inertia, int32_t *rows_evaluated,
                          void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- low-precision deployment ----
 * Sec. 3.1 of the paper remarks that the clustering yields gamma and beta of low precision and gives no mechanism.
 * The reading taken here: the fitted parameters (centroids, gamma, beta) are stored as bfloat16, rounded to nearest
 * with ties to the even significand, and CAT Inferencing (Algorithm 2) runs on the stored values as it stands:
 * nearest stored centroid (exact, lowest index on ties), x + alpha ((gamma - 1) x + beta) with the stored gamma,
 * beta in fp32 arithmetic.  The corrected rows of fp32 inputs may be written as bfloat16 (one more rounding to
 * nearest even), which takes a quarter off the bytes of the pass.
 *
 * cat_params_to_bf16: dst[i] = bfloat16 nearest to src[i] (device arrays of n elements; finite values).
 * cat_apply_lp:
 *   centroids, gamma, beta   in, device, K x D bfloat16 each (uint16 storage, 2-byte aligned)
 *   out_dt                   type of `corrected`: dt, or CAT_BF16 for fp32 rows
 *   corrected                out, device, N x D of out_dt, 16-byte aligned, not aliasing lq
 *   workspace                cat_apply_lp_workspace_bytes(N, D, K, dt) bytes
 * Other arguments and errors: as cat_apply. */
cat_status cat_params_to_bf16(const float *src, int64_t n, uint16_t *dst, void *hip_stream);
size_t cat_apply_lp_workspace_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt);
cat_status cat_apply_lp(const void *lq, int64_t N, int64_t D, int32_t K, cat_dtype dt,
                        const uint16_t *centroids, const uint16_t *gamma, const uint16_t *beta, float alpha,
                        cat_dtype out_dt, void *corrected, int32_t *assignments,
                        void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- fits for a grid of cluster counts ----
 * The paper's ablation on the number of clusters (Sec. 5 and the appendix on the number of clusters) fits CAT for
 * a list of cluster counts on the same calibration rows.  cat_fit_multi_k returns, for every K in the list, what
 * cat_fit(lq, fp, N, D, K, iters, seed, dt, NULL, ...) returns: the fits are independent and every one starts from
 * the rows cat_init_indices(N, K, seed) picks.  Where the shape fits the matrix-core kernels, consecutive entries of
 * the list whose clusters fill at most 64 slots together (128 for rows of at most 1 KB; each K rounded up to a multiple
 * of 16) run their Lloyd loops side by side, so that one read of lq per pass serves all of them; other entries run one after the other.
 *
 * Ks           in, HOST array of nK cluster counts, 1 <= nK <= CAT_MAX_MULTI_K, each 1 <= K <= min(N, CAT_MAX_K)
 * centroids, gamma, beta
 *              out, device, (sum of Ks) x D floats each: the K rows of entry i start at row Ks[0] + .. + Ks[i-1]
 * assignments  out, device, nK x N int32: row i holds the assignments of entry i
 * counts       out, device, (sum of Ks) int32, nullable, laid out as the rows of centroids
 * inertia      out, device, nK x (iters + 1) doubles, nullable
 * workspace    cat_fit_multi_k_workspace_bytes(N, D, Ks, nK, iters, dt) bytes (0 for invalid arguments)
 * Other arguments and errors: as cat_fit.  Enqueues on the stream; no allocation, no synchronisation.
 * cat_debug_multi_group_tiles(t), t in {0, 1, 2, 4, 8}: at most t 16-cluster tiles per group (0, the default: 4, or 8 for
 * rows of at most 1 KB; 1 runs
 * every entry on its own); process-wide, for measurements and tests; results do not depend on it. */
#define CAT_MAX_MULTI_K 64
size_t cat_fit_multi_k_workspace_bytes(int64_t N, int64_t D, const int32_t *Ks, int32_t nK, int32_t iters, cat_dtype dt);
cat_status cat_fit_multi_k(const void *lq, const void *fp, int64_t N, int64_t D, const int32_t *Ks, int32_t nK,
                           int32_t iters, uint64_t seed, cat_dtype dt,
                           float *centroids, float *gamma, float *beta,
                           int32_t *assignments, int32_t *counts, double *inertia,
                           void *workspace, size_t workspace_bytes, void *hip_stream);
cat_status cat_debug_multi_group_tiles(int tiles);

/* ---- D^2-weighted seeding ("k-means++", Arthur and Vassilvitskii, SODA 2007) ----
 * An alternative to the seeded distinct rows of cat_init_indices; the paper fixes no k-means
 * initialisation (Sec. 4, Setup).  Use: cat_init_kmeanspp -> cat_fit(..., init_centroids = centroids).
 *
 * The draws are u_t = (SplitMix64 output t of `seed` >> 11) * 2^-53, t = 0 .. K-1 (the counter
 * stream documented at cat_init_indices).  Row 0 of the result is row floor(u_0 N) of lq.  For
 * t >= 1, with d2[i] the squared distance (direct form, double) of row i to the nearest row chosen
 * so far and S the sum of all d2, the row chosen is the first i whose running sum
 * d2[0] + .. + d2[i] exceeds u_t S; if S = 0 it is the lowest row not chosen yet.  All sums are
 * taken in a fixed order (rows in groups of 64, groups in index order), so a seed always gives the
 * same rows; they equal those of the same rule with one sequential running sum unless u_t S falls
 * within rounding of a running sum.
 *   centroids  out, K x D float: the chosen rows, in the order drawn
 *   indices    out, nullable, K int64 (device): their row numbers
 * 1 <= K <= min(N, CAT_MAX_K).  K - 1 reads of lq.  workspace: cat_init_kmeanspp_workspace_bytes(N, K)
 * bytes, 256-byte aligned, caller-owned.  Errors: CAT_ERR_INVALID_ARG, CAT_ERR_WORKSPACE, CAT_ERR_DEVICE.
 */
size_t cat_init_kmeanspp_workspace_bytes(int64_t N, int32_t K);
cat_status cat_init_kmeanspp(const void *lq, int64_t N, int64_t D, int32_t K, uint64_t seed, cat_dtype dt,
                             float *centroids, int64_t *indices,
                             void *workspace, size_t workspace_bytes, void *hip_stream);

/* ---- several runs, the best kept (the paper gives neither the k-means initialisation nor a number
 * of restarts, Sec. 4 Setup; this is the usual remedy for Lloyd's dependence on its start) ----
 *
 * cat_fit_restarts runs the clustering part of cat_fit `restarts` times, run r with the seed
 * `seed + r` (seeding CAT_SEED_ROWS: the rows of cat_init_indices; CAT_SEED_KMEANSPP: those of
 * cat_init_kmeanspp), keeps the run whose final objective (the sum of squared distances of the final
 * assignment, as reported in `inertia`) is lowest, the first such run on ties, and fits gamma and
 * beta on its partition.  With restarts = 1 and CAT_SEED_ROWS it is cat_fit without init_centroids.
 * Outputs as cat_fit, all of the kept run, plus
 *   best_run       out, nullable, 1 int32 (device): r of the kept run
 *   final_inertia  out, nullable, `restarts` doubles (device): the final objective of every run
 * The comparison between runs is made on the device, on the objective as the library computes it
 * (fp32 scores summed in double, about 1e-6 relative): runs closer than that may be ordered
 * differently than by their exact objectives.  1 <= restarts <= CAT_MAX_RESTARTS.  workspace:
 * cat_fit_restarts_workspace_bytes(N, D, K, iters, dt).
 */
size_t cat_fit_restarts_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t iters, cat_dtype dt);
cat_status cat_fit_restarts(const void *lq, const void *fp, int64_t N, int64_t D, int32_t K,
                            int32_t iters, uint64_t seed, int32_t restarts, cat_seeding seeding, cat_dtype dt,
                            float *centroids, float *gamma, float *beta,
                            int32_t *assignments, int32_t *counts, double *inertia,
                            int32_t *best_run, double *final_inertia,
                            void *workspace, size_t workspace_bytes, void *hip_stream);

/*
 * Timing of the dominant kernel, for benchmarks.  While enabled, every launch of the tile
 * kernel (the assignment / Lloyd / inference pass) made by the calling process is bracketed by
 * two HIP events recorded on the launch stream.  cat_profile_read waits for those events and
 * copies up to `cap` durations (milliseconds, launch order) to the HOST array ms_out; it
 * returns the number of launches recorded since cat_profile_enable(1) (which also clears the
 * record), or -1 on a HIP error.  Event objects are created on first use and kept; nothing is
 * recorded, created or waited for while profiling is disabled (the default).  Not thread-safe.
 */
cat_status cat_profile_enable(int on);
int cat_profile_read(float *ms_out, int cap);

/*
 * What the memory system gives a kernel that does nothing else, for benchmarks: the yardstick beside the 8 TB/s
 * peak for the passes above, which are bound by one read (assignment, sums) or by a read and a write (inference) of
 * the rows.  One launch streams `bytes` bytes from src: dst == NULL reads them and keeps nothing, else copies them to
 * dst.  Blocks of 256 lanes walk contiguous spans, 16 bytes per lane, four loads in flight per lane.
 *
 * src    in,  device, bytes (a multiple of 16), 16-byte aligned
 * dst    out, device, bytes, 16-byte aligned, or NULL
 * Enqueues on the stream; no allocation, no synchronisation.  CAT_ERR_INVALID_ARG for a null or misaligned
 * pointer or a size that is zero or not a multiple of 16.
 */
cat_status cat_stream_probe(const void *src, void *dst, size_t bytes, void *hip_stream);

/*
 * Test hook.  In the fused Lloyd loop (cat_fit on the tile path) every workgroup collects the rows
 * that changed cluster in a list in fast memory before appending them to the device-wide list; a
 * workgroup whose list is full appends tile by tile instead.  This call sets the capacity of that
 * list for later cat_fit calls of the process (1 .. 1024 entries; 0 restores the default, 1024),
 * so that the tile-by-tile path can be reached on small inputs.  Results never depend on it.
 * CAT_ERR_INVALID_ARG outside that range.  Not thread-safe.
 */
cat_status cat_debug_list_capacity(int entries);

/*
 * Test hook.  In the assignment passes of the tile path (cat_assign, the passes of cat_fit without distance
 * bounds), a row whose two best scores are within the error bound of the split arithmetic is measured exactly,
 * in double precision.  A workgroup does not do that where it finds the row: it queues the row in fast memory
 * and its waves share the queued rows out when the workgroup has no tiles left; a row that finds the queue
 * full, or has more than 8 candidates, is measured on the spot.  This call sets the capacity of the queue for
 * later calls of the process (1 .. 256 entries; 0 restores the default, 256; -1: no queue, every such row is
 * measured on the spot), so that both ways can be reached on small inputs.  Results never depend on it.
 * CAT_ERR_INVALID_ARG outside that range.  Not thread-safe.
 */
cat_status cat_debug_rerank_queue(int entries);

/*
 * Test hook.  cat_apply (and cat_apply_static) on the fused path has two kernels: one that keeps a tile of rows
 * on the chip between the ranking and the affine map (used whenever it has an instance for the shape), and the
 * tile kernel shared with cat_assign.  0 = automatic (default), 1 = never the row-tile kernel, 2 = only the
 * row-tile kernel (CAT_ERR_UNSUPPORTED on a shape it has no instance for).  Results never depend on it beyond
 * rounding-equivalent ties.  Process-wide.  CAT_ERR_INVALID_ARG for other values.
 */
cat_status cat_debug_apply_kernel(int which);

/* Message of the last non-OK status on the calling thread ("" if none).  The
 * pointer stays valid until the next failing call on the same thread. */
const char *cat_last_error(void);

#ifdef __cplusplus
}
#endif
#endif /* CAT_H */
