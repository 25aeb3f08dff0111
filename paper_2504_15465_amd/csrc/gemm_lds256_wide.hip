// Direct-to-LDS 256x256 GEMM, instances with the wide epilogue (full tiles through LDS / 16 bytes per lane).
#include "gemm_lds256.hpp"

namespace lithos {

gemm_fn gemm_lds256_wide_fn(bool ta, bool tb) { return LITHOS_LDS256_PICK(true); }

} // namespace lithos
