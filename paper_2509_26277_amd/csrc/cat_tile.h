// MFMA tile kernels of the CAT hot path (cat_tile.hip): interface to the host driver.
#pragma once
#include "cat_common.h"

namespace cat {

enum TileMode { TILE_ASSIGN = 0, TILE_LLOYD = 1, TILE_APPLY = 2 };

// Device scratch of the tile kernels, carved from the caller's workspace.
struct TileWs {
    uint16_t* packA = nullptr;  // centroids as bf16 (hi, lo) in MFMA operand order
    float* cnorm = nullptr;     // K16 squared centroid norms (padding clusters: huge)
    float* cent = nullptr;      // K x D fp32 working centroids (cat_assign / cat_apply copy theirs here)
    size_t bytes = 0;
};

size_t tile_workspace_bytes(int64_t D, int32_t K, cat_dtype dt);
TileWs tile_carve(void* base, int64_t D, int32_t K, cat_dtype dt);

// Whether the tile kernels can run `mode` on this shape (LDS and register budgets, index widths).
bool tile_supports(TileMode mode, int64_t N, int64_t D, int32_t K, cat_dtype dt);

// Assignment pass (gamma == NULL) or fused inference (gamma, beta, corrected given).
// counts / inertia / rep are optional and pre-initialised by the caller.
cat_status tile_assign(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                       int32_t* assign, int32_t* counts, double* inertia, unsigned long long* rep,
                       const float* gamma, const float* beta, void* corrected, const TileWs& ws, hipStream_t st);

// More than 128 clusters whose two-part operand does not fit LDS in one piece: the same assignment pass as two launches
// over the halves of the clusters (assignment only: no inference).  tile_split_scratch_bytes is 0 where that does not apply.
size_t tile_split_scratch_bytes(int64_t N, int64_t D, int32_t K, cat_dtype dt);
cat_status tile_assign_split(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent, int32_t* assign,
                             int32_t* counts, double* inertia, unsigned long long* rep, const TileWs& ws, void* scratch,
                             hipStream_t st);

// Extra device scratch of tile_lloyd: the list of rows that changed cluster in a pass (worst case
// all N), the counters of the update kernel and the per-slice shares of the centroid norms.
struct LloydWs {
    unsigned long long* list = nullptr;  // N entries
    uint32_t* ctrl = nullptr;            // [0..1] list length (two halves), then 2 x slices finished-workgroup counters,
    int32_t* skipped = nullptr;          //   then one word: passes left out, for callers that bring no word of their own
    double* norm_part = nullptr;         // slices x K
    int32_t* counts2 = nullptr;          // K: the second half of the counts double buffer
    float2* carry = nullptr;             // N pairs, only for more than 128 clusters: what the first of two launches that
    float* carry_cmax = nullptr;         //   split the clusters hands to the second (per row; the largest centroid norm)
    uint32_t* sort_ws = nullptr;         // not carved here: the caller's scratch for launch_segsum_sorted
    size_t bytes = 0;
};
size_t lloyd_workspace_bytes(int64_t N, int64_t D, int32_t K);
LloydWs lloyd_carve(void* base, int64_t N, int64_t D, int32_t K);

// Scratch of the loops that leave rows out by distance bounds (Hamerly, SDM 2010): see tile_lloyd.
struct BoundsWs {
    double* expire = nullptr;         // N        per row: the drift at which it has to be evaluated again
    int32_t* rows = nullptr;          // N        the rows of the coming pass
    uint32_t* n_rows = nullptr;       // 1        their number
    double* drift = nullptr;          // iters+1  accumulated centroid drift up to each pass
    double* move_part = nullptr;      // slices x K
    int32_t* slice_counts = nullptr;  // slices x K
    int32_t* evaluated = nullptr;     // iters+1  out: rows evaluated by each pass (the caller's array, nullable)
    size_t bytes = 0;
};
size_t bounds_workspace_bytes(int64_t N, int64_t D, int32_t K, int32_t iters);
BoundsWs bounds_carve(void* base, int64_t N, int64_t D, int32_t K, int32_t iters);
bool tile_bounds_supports(int64_t N, int64_t D, int32_t K, cat_dtype dt);
cat_status launch_fill_i32(int32_t* p, int64_t n, int32_t v, hipStream_t st);

// `iters` Lloyd iterations from cent0 plus the final assignment.  cent_io holds the initial
// centroids on entry and the final ones on return; sums is 2 x K x D doubles of scratch.
// Writes assignments, counts (K), inertia (iters + 1, nullable) and rep (K).  skipped (one device int32,
// nullable) allows the early stop: passes after the partition has stopped changing are not run, and their
// number is written there; every other output is what the full loop gives.
// With bw given (and tile_bounds_supports, iters >= 4): from the first pass that lists the rows that changed cluster
// on, a pass also leaves every row's distance bound, and the passes between that one and the last evaluate only the
// rows whose bound the centroid drift has used up.  Same centroids, assignments, counts and rep; of the objective
// only the entries of the passes that evaluate every row (0, 1, 2 and the last) are written, the others are NaN.
cat_status tile_lloyd(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, int32_t iters,
                      float* cent_io, double* sums, int32_t* assign, int32_t* counts, double* inertia,
                      unsigned long long* rep, int32_t* skipped, const TileWs& ws, const LloydWs& lw, hipStream_t st,
                      const BoundsWs* bw = nullptr);

// Several independent centroid sets side by side: Lloyd loops for a grid of cluster counts that share every read of
// the rows.  Set s owns the 16-cluster tiles t0[s] .. t0[s + 1] - 1 of the concatenation, of whose slots the first
// k[s] hold centroids (the others stay empty).
struct MultiSets {
    int32_t nsets = 0;
    int32_t k[16] = {};
    int32_t t0[17] = {};
};
bool tile_multi_supports(int64_t N, int64_t D, int32_t slots, int32_t nsets, cat_dtype dt);
// tile_lloyd over the concatenated slots.  cent_io, counts, rep are indexed by slot (empty slots: zero rows, zero
// counts); sums is 2 x slots x D doubles; assign16 is the N x 16 table of slot numbers (set s in column s);
// inertia16 (nullable) takes (iters + 1) x 16 doubles, set s in column s; `column` is N int32 of scratch; the
// changed-row list of lw holds N x nsets entries.
cat_status tile_lloyd_multi(const void* lq, cat_dtype dt, int64_t N, int64_t D, const MultiSets& ms, int32_t iters,
                            float* cent_io, double* sums, int32_t* assign16, int32_t* counts, double* inertia16,
                            unsigned long long* rep, int32_t* column, const TileWs& ws, const LloydWs& lw, hipStream_t st);
// column s of the N x 16 table as cluster numbers of the set (slot number minus slot0)
cat_status launch_multi_column(const int32_t* assign16, int64_t N, int32_t s, int32_t slot0, int32_t* out, hipStream_t st);

// Capacity of the per-workgroup changed-row list (cat_debug_list_capacity in cat.h).
int lloyd_list_capacity();
// Capacity of the per-workgroup queue of rows whose exact re-rank is put off (cat_debug_rerank_queue in cat.h).
int rerank_queue_capacity();

// Kernel timing hooks (see cat_profile_enable in cat.h): bracket one launch with events.
bool profile_on();
cat_status profile_mark(bool begin, hipStream_t st);

}  // namespace cat
