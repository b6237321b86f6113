// Instantiations of the tile kernel: 256 padded clusters (KT = 16), bf16 rows, the two-part operand; the one-part
// operand's instances are compiled in a file of their own (these are the largest instances: two files build side by side).
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_kt16_bf16_one_part(const TileParams& p, const TileCfg& c, hipStream_t st);

cat_status launch_kt16_bf16(const TileParams& p, const TileCfg& c, hipStream_t st) {
    return c.P == 2 ? launch_mode<16, 3, true>(p, c, st) : launch_kt16_bf16_one_part(p, c, st);
}

}  // namespace cat
