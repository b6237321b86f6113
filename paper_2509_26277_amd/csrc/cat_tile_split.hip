// Instantiations of the tile kernel for the two launches over the halves of a large cluster set, one translation unit.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_split_f32(const TileParams& p, const TileCfg& c, hipStream_t st) { return launch_split<false>(p, c, st); }
cat_status launch_split_bf16(const TileParams& p, const TileCfg& c, hipStream_t st) { return launch_split<true>(p, c, st); }

}  // namespace cat
