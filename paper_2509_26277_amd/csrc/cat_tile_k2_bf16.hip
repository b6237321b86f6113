// Instantiations of the tile kernel: 32 padded clusters (KT = 2), bf16 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt2_bf16(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<2, true>(p, c, st);
}

}  // namespace cat
