// Instantiations of the tile kernel: 256 padded clusters (KT = 16), bf16 rows, the one-part operand.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt16_bf16_one_part(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return launch_mode<16, 1, true>(p, c, st);
}

}  // namespace cat
