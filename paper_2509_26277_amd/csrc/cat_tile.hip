// MFMA tile kernels (placeholder until the first kernels land: nothing is supported,
// so the host driver always takes the streaming kernels).
#include "cat_tile.h"

namespace cat {

size_t tile_workspace_bytes(int64_t, int32_t, cat_dtype) { return 0; }
TileWs tile_carve(void* base, int64_t, int32_t, cat_dtype) {
    TileWs w;
    w.base = base;
    return w;
}
bool tile_supports(TileMode, int64_t, int32_t, cat_dtype) { return false; }
cat_status tile_assign(const void*, cat_dtype, int64_t, int64_t, int32_t, const float*, int32_t*, int32_t*, double*,
                       unsigned long long*, const float*, const float*, void*, const TileWs&, hipStream_t) {
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernels are not built");
}
cat_status tile_lloyd(const void*, cat_dtype, int64_t, int64_t, int32_t, int32_t, const float*, float*, int32_t*,
                      int32_t*, double*, unsigned long long*, const TileWs&, hipStream_t) {
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernels are not built");
}

}  // namespace cat
