// Shared declarations of the CAT HIP library (gfx950 only).
#pragma once
#include <hip/hip_runtime.h>
#include <stdint.h>
#include <stddef.h>

#include "cat.h"

namespace cat {

constexpr int kWave = 64;            // CDNA wavefront
constexpr double kVarFloor = 1e-8;   // Algorithm 1: variance floor of the affine fit

// ---- element access: float, or bfloat16 stored as uint16 -------------------
typedef uint16_t bf16_t;

__device__ __forceinline__ float bf16_to_f32(bf16_t u) { return __uint_as_float(((uint32_t)u) << 16); }
// round-to-nearest-even; non-finite inputs are outside the contract
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
    uint32_t b = __float_as_uint(f);
    return (bf16_t)((b + 0x7FFFu + ((b >> 16) & 1u)) >> 16);
}
__device__ __forceinline__ float ld_elem(const float* p) { return *p; }
__device__ __forceinline__ float ld_elem(const bf16_t* p) { return bf16_to_f32(*p); }
__device__ __forceinline__ void st_elem(float* p, float v) { *p = v; }
__device__ __forceinline__ void st_elem(bf16_t* p, float v) { *p = f32_to_bf16(v); }

// ---- wave-level reductions (64 lanes, butterfly) ---------------------------
__device__ __forceinline__ double wave_sum(double v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}
__device__ __forceinline__ float wave_sum(float v) {
#pragma unroll
    for (int o = 32; o > 0; o >>= 1) v += __shfl_xor(v, o, kWave);
    return v;
}

// ---- SplitMix64 (Steele, Lea, Flood 2014) as a counter-based generator -----
__host__ __device__ __forceinline__ uint64_t splitmix64_at(uint64_t seed, uint64_t t) {
    uint64_t z = seed + (t + 1ull) * 0x9E3779B97F4A7C15ull;
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
}
// the seeded walk is cut after this many draws (never reached in practice: the
// expected number is below N (ln N + 1))
__host__ __device__ __forceinline__ uint64_t init_draw_cap(int64_t N) {
    int lg = 1;
    while ((1ll << lg) < N && lg < 62) lg++;
    return 32ull * (uint64_t)N * (uint64_t)(lg + 1) + 1024ull;
}

// ---- error reporting ---------------------------------------------------------
cat_status set_error(cat_status st, const char* fmt, ...);
#define CAT_HIP_TRY(expr)                                                                  \
    do {                                                                                   \
        hipError_t _e = (expr);                                                            \
        if (_e != hipSuccess)                                                              \
            return cat::set_error(CAT_ERR_DEVICE, "%s failed: %s", #expr, hipGetErrorString(_e)); \
    } while (0)
#define CAT_LAUNCH_CHECK(name)                                                             \
    do {                                                                                   \
        hipError_t _e = hipGetLastError();                                                 \
        if (_e != hipSuccess)                                                              \
            return cat::set_error(CAT_ERR_DEVICE, "launch of %s failed: %s", name, hipGetErrorString(_e)); \
    } while (0)

// ---- streaming kernels (cat_stream.hip) ------------------------------------------
// Every launcher enqueues on `st` and returns a status; none synchronises.
cat_status launch_fill_zero(void* p, size_t bytes, hipStream_t st);
cat_status launch_init_indices(int64_t N, int32_t K, uint64_t seed, int64_t* idx, hipStream_t st);
cat_status launch_gather_rows(const void* lq, cat_dtype dt, int64_t D, int32_t K, const int64_t* idx,
                              float* out, hipStream_t st);
// Nearest centroid per row, direct-form double precision.  counts (K), inertia (1 double, added to),
// rep (K, smallest row index per cluster, min-combined) are optional and must be pre-initialised
// (zero / zero / ~0ull).  If gamma != NULL also writes corrected = gamma[a] * x + beta[a].
cat_status launch_assign_stream(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K,
                                const float* cent, int32_t* assign, int32_t* counts, double* inertia,
                                unsigned long long* rep, const float* gamma, const float* beta,
                                void* corrected, hipStream_t st);
// The same contract on the LDS streaming kernel (cat_lds.hip): fp32 scores with the centroids staged in LDS, exact
// double-precision re-rank of the rows inside the rounding bound.  Any D, K and row alignment.
cat_status launch_assign_lds(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                             int32_t* assign, int32_t* counts, double* inertia, unsigned long long* rep,
                             const float* gamma, const float* beta, void* corrected, hipStream_t st);
// counts[k] and rep[k] from given assignments (both pre-initialised as above)
cat_status launch_count_rep(const int32_t* assign, int64_t N, int32_t K, int32_t* counts,
                            unsigned long long* rep, hipStream_t st);
// Segmented sums over the rows of each cluster.  NQ = 1: acc[0] += x.  NQ = 4: with x' = x - pivx[k],
// y' = y - pivy[k]: acc[0] += x', acc[1] += y', acc[2] += x'^2, acc[3] += x'y'.  acc is NQ x K x D
// doubles, pre-zeroed.
cat_status launch_segsum(int nq, const void* lq, const void* fp, cat_dtype dt, const int32_t* assign,
                         int64_t N, int64_t D, int32_t K, const float* pivx, const float* pivy,
                         double* acc, hipStream_t st);
// The same sums over rows that were first ordered by cluster (a counting sort on the assignments,
// given the cluster sizes): each wave then keeps its sums in registers and touches memory only when
// the cluster changes.  Scratch: N + 2 K + 2 words (sort_workspace_words).  segsum_sorted_supported
// says whether the shape qualifies (16-byte channel groups, N below 2^31) and gains; otherwise use launch_segsum.
bool segsum_sorted_supported(int nq, int64_t N, int64_t D, cat_dtype dt);
// cat_select_path(CAT_PATH_TILE) is in force: take the tile / sorted kernels wherever they can run,
// whatever the size heuristics say (this is how the tests reach them on small shapes)
bool fast_paths_forced();
size_t sort_workspace_words(int64_t N, int32_t K);
cat_status launch_segsum_sorted(int nq, const void* lq, const void* fp, cat_dtype dt, const int32_t* assign,
                                const int32_t* counts, int64_t N, int64_t D, int32_t K, const float* pivx,
                                const float* pivy, double* acc, uint32_t* sort_ws, hipStream_t st);
cat_status launch_finalize_centroids(const double* sums, const int32_t* counts, const float* prev,
                                     float* cent, int64_t D, int32_t K, hipStream_t st);
// pivx = hint (if given) else lq[rep[k]]; pivy = fp[rep[k]]; rows of empty clusters are zero
cat_status launch_gather_pivots(const void* lq, const void* fp, cat_dtype dt, int64_t D, int32_t K,
                                const unsigned long long* rep, const float* hint, float* pivx, float* pivy,
                                hipStream_t st);
cat_status launch_finalize_affine(const double* acc, const int32_t* counts, const float* pivx,
                                  const float* pivy, float* gamma, float* beta, int64_t D, int32_t K,
                                  hipStream_t st);
cat_status launch_fold_alpha(const float* gamma, const float* beta, float alpha, float* g_eff, float* b_eff,
                             int64_t KD, hipStream_t st);
// device-to-device copy of 32-bit words (any 4-byte-aligned buffers)
cat_status launch_copy_words(const void* src, void* dst, int64_t nwords, hipStream_t st);
cat_status launch_fill_u64(unsigned long long* p, int64_t n, unsigned long long v, hipStream_t st);
// dst (rows x dst_ld) <- the first `cols` columns of src (rows x src_ld), zeros in the columns from `cols` on
cat_status launch_copy_cols(const float* src, int64_t rows, int32_t src_ld, float* dst, int32_t dst_ld, int32_t cols,
                            hipStream_t st);
// cat_stream_probe: a pure read of `bytes` bytes (dst == nullptr) or a pure copy
cat_status launch_stream_probe(const void* src, void* dst, size_t bytes, hipStream_t st);
// dst (rows x dst_ld) <- the first dst_ld columns of src (rows x src_ld), zeros where src has none; elements of dtype dt
cat_status launch_pad_rows(const void* src, cat_dtype dt, int64_t rows, int64_t src_ld, int64_t dst_ld, void* dst, hipStream_t st);
// inference with the PCA front-end in one kernel (cat_pca.hip), where the shape allows it
bool apply_pca_fused_supported(const void* lq, int64_t D, int32_t K, int32_t p, const float* mean, const float* components,
                               const float* gamma, const float* beta, const void* corrected);
cat_status launch_apply_pca_fused(const void* lq, int64_t N, int64_t D, int32_t K, int32_t p, cat_dtype dt, const float* mean,
                                  const float* components, const float* centroids_z, const float* gamma, const float* beta,
                                  float alpha, void* corrected, int32_t* assignments, hipStream_t st);
// best-of-several bookkeeping on the device: state[0] = 1 if `cur` beats `best` (or run == 0), state[1] = best run;
// finals (nullable) receives cur at index run.  launch_copy_words_if copies only while *flag != 0.
cat_status launch_keep_best(const double* cur, double* best, int32_t* state, int32_t run, double* finals, hipStream_t st);
cat_status launch_copy_words_if(const int32_t* flag, const void* src, void* dst, int64_t nwords, hipStream_t st);
// low-precision deployment (cat_lp.hip): fp32 -> bfloat16 (round to nearest even); stored parameters back to fp32 with
// the blending coefficient folded into gamma / beta; rows with given labels -> corrected rows (in the type of the rows, or
// bfloat16 for fp32 rows)
cat_status launch_to_bf16(const float* src, int64_t n, uint16_t* dst, hipStream_t st);
cat_status launch_expand_params(const uint16_t* cent, const uint16_t* gamma, const uint16_t* beta, float alpha, int64_t n,
                                float* c, float* g, float* b, hipStream_t st);
cat_status launch_affine_by_labels(const void* x, cat_dtype dt, const int32_t* assign, int64_t N, int64_t D, const float* g,
                                   const float* b, void* out, bool out_bf16, hipStream_t st);
// PCA scores (cat_pca.hip) with rows ldz >= p floats apart; the padding columns are written as zeros
cat_status pca_project_ld(const void* lq, int64_t N, int64_t D, int32_t p, cat_dtype dt, const float* mean,
                          const float* components, float* z, int32_t ldz, hipStream_t st);

}  // namespace cat
