// Instantiations of the tile kernel: 16 padded clusters (KT = 1), bf16 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt1_bf16(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<1, true>(p, c, st);
}

}  // namespace cat
