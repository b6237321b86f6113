// Row-tile inference kernel (cat_infer.hip): interface to the host driver.
#pragma once
#include "cat_tile.h"

namespace cat {

// Whether the row-tile kernel has an instance for this shape (rows of whole 16-byte groups, the 8 waves' shares of the
// centroid operand within their registers, the row tile within LDS).
bool infer_supported(int64_t N, int64_t D, int32_t K, cat_dtype dt);

// corrected = gamma[a] * x + beta[a], a = nearest centroid of x; assign nullable.  Scratch: the tile kernels' (ws).
// out_bf16 (fp32 rows only): corrected is written as bfloat16.  corrected == nullptr: assignment only (gamma and beta
// are not read).  inertia (nullable): the sum of the squared distances to the assigned centroids is ADDED to *inertia.
cat_status infer_apply(const void* lq, cat_dtype dt, int64_t N, int64_t D, int32_t K, const float* cent,
                       const float* gamma, const float* beta, void* corrected, int32_t* assign, const TileWs& ws,
                       hipStream_t st, bool out_bf16 = false, double* inertia = nullptr);

}  // namespace cat
