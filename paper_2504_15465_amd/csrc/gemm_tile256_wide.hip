// 256x256-tile instances (8 wavefronts, 2x4) of the register-staged MFMA GEMM with the wide epilogue.
#include "gemm_tile.hpp"

namespace lithos {

gemm_fn gemm_tile256_wide_fn(bool ta, bool tb) { return LITHOS_TILE_PICK4(256, 2, 4, true); }

} // namespace lithos
