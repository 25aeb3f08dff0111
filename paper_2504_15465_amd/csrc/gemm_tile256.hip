// 256x256-tile instances (8 wavefronts, 2x4) of the LDS-staged MFMA GEMM.
#include "gemm_tile.hpp"

namespace lithos {

gemm_fn gemm_tile256_fn(bool ta, bool tb, bool st)
{
    return LITHOS_TILE_PICK(256, 2, 4);
}

} // namespace lithos
