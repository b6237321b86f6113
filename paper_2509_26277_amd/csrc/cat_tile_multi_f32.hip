// Instantiations of the tile kernel for several centroid sets side by side (f32 rows), one translation unit.
#include "cat_tile_kernel.h"

namespace cat {

cat_status launch_multi_f32(const TileParams& p, const TileCfg& c, hipStream_t st) {
    switch (c.KT) {
        case 1: return launch_kt_multi<1, false>(p, c, st);
        case 2: return launch_kt_multi<2, false>(p, c, st);
        case 4: return launch_kt_multi<4, false>(p, c, st);
        case 8: return launch_kt_multi<8, false>(p, c, st);
    }
    return set_error(CAT_ERR_UNSUPPORTED, "tile kernel for several centroid sets: K tile count %d (at most 8)", c.KT);
}

}  // namespace cat
