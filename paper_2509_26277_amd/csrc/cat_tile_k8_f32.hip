// Instantiations of the tile kernel: 128 padded clusters (KT = 8), f32 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt8_f32(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<8, false>(p, c, st);
}

}  // namespace cat
