// Row-tile inference kernel (cat_infer.hip): interface to the host driver.
#pragma once
#include "cat_tile.h"

namespace cat {

// Whether the row-tile kernel has an instance for this shape (rows of whole 16-byte groups, the 8 waves' shares of the
// centroid operand within their registers, the row tile within LDS).
bool infer_supported(int64_t N, int64_t D, int32_t K, cat_dtype dt);

// corrected = gamma[a] * x + beta[a], a = nearest centroid of x; assign nullable.  Scratch: the tile kernels' (ws).
cat_status infer_apply(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                       const float* gamma, const float* beta, void* corrected, int32_t* assign, const TileWs& ws,
                       hipStream_t st);

// The same kernel as the assignment pass of a Lloyd iteration.  rowtile_assign_config says whether an instance holds the
// shape (lists: the pass collects the rows that change cluster) and which cluster tiling and part count the centroid
// preparation must use; rowtile_assign takes the tile kernel's parameter block.
struct TileParams;
bool rowtile_assign_config(bool lists, int64_t N, int64_t D, int32_t K, cat_dtype dt, int* KT, int* P);
cat_status rowtile_assign(const TileParams& tp, cat_dtype dt, float* cnorm_ws, hipStream_t st);
// cat_debug_apply_kernel(1) is in force: the tile kernel everywhere
bool rowtile_disabled();

}  // namespace cat
