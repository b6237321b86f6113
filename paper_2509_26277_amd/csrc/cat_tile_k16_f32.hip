// Instantiations of the tile kernel: 256 padded clusters (KT = 16), f32 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt16_f32(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<16, false>(p, c, st);
}

}  // namespace cat
