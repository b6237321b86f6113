// Instantiations of the tile kernel: 32 padded clusters (KT = 2), f32 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt2_f32(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<2, false>(p, c, st);
}

}  // namespace cat
