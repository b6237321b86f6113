// Instantiations of the tile kernel: 16 padded clusters (KT = 1), f32 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt1_f32(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<1, false>(p, c, st);
}

}  // namespace cat
