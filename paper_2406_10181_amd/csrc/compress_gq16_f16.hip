// Kernel A of the compress path for fp16 storage (see compress_gq16.h).
#include "compress_gq16.h"

namespace lsp {
hipError_t launch_gq16_f16(const CompressGroup& g, int32_t r, int32_t d, uint32_t* counter, hipStream_t st) {
    return launch_gq16<F16>(g, r, d, counter, st);
}
}  // namespace lsp
