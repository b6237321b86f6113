// Instantiations of the tile kernel: 128 padded clusters (KT = 8), bf16 rows.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt8_bf16(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_kt<8, true>(p, c, st);
}

}  // namespace cat
