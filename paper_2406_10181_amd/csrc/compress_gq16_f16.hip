// Kernel A of the compress path for fp16 storage (see compress_gq16.h).
#include "compress_gq16.h"

namespace lsp {
hipError_t launch_gq16_f16(const CompressGroup& g, int32_t r, int32_t d, int blocks_per_wg, hipStream_t st) {
    return launch_gq16<F16>(g, r, d, blocks_per_wg, st);
}
}  // namespace lsp
