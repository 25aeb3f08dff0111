// Direct-to-LDS 256x256 GEMM, instances that store element by element (C rows not 16-byte addressable).
#include "gemm_lds256.hpp"

namespace lithos {

gemm_fn gemm_lds256_elem_fn(bool ta, bool tb) { return LITHOS_LDS256_PICK(false); }

} // namespace lithos
