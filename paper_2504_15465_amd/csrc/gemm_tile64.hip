// 64x64-tile instances of the LDS-staged MFMA GEMM.
#include "gemm_tile.hpp"

namespace lithos {

gemm_fn gemm_tile64_fn(bool ta, bool tb, bool split, bool st)
{
    if (split) return LITHOS_TILE_PICK_SPLIT(64);
    return LITHOS_TILE_PICK(64, 2, 2);
}

} // namespace lithos
