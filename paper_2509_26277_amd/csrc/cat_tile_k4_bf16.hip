// Instantiations of the tile kernel: 64 padded clusters (KT = 4), bf16 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt4_bf16(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<4, true>(p, c, st);
}

}  // namespace cat
