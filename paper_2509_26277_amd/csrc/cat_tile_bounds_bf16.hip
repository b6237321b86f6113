// Instantiations of the tile kernel that keep distance bounds and walk listed rows (bf16 rows), one translation unit.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_bounds_bf16(const TileParams& p, const TileCfg& c, hipStream_t st) {
    switch (c.KT) {
        case 1: return launch_kt_bounds<1, true>(p, c, st);
        case 2: return launch_kt_bounds<2, true>(p, c, st);
        case 4: return launch_kt_bounds<4, true>(p, c, st);
        case 8: return launch_kt_bounds<8, true>(p, c, st);
        case 16: return launch_kt_bounds<16, true>(p, c, st);
    }
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernel: K tile count %d", c.KT);
}

}  // namespace cat
